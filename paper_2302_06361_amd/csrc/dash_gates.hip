// dash_gates.hip -- gate-level kernels over LabelTensors.
//
//   k_draw        : PRG labels (fresh zero labels of gate outputs, input wires, masks)
//   k_affine      : free gates: out = sum_t coef_t * term_t mod m   (Sec. Arithmetic Garbled Circuits)
//   k_proj_garble : one lane per ciphertext row: hash the label of value a, add the payload, store
//                   the row at the position its colour names            (projection gates, point-and-permute)
//   k_proj_eval   : one lane per gate: hash the active label, fetch the row its colour names, subtract
//   k_hg_finish   : evaluator side of the mixed-modulus half gate       (Appendix)
//
// A launch carries up to 16 homogeneous gate batches ("jobs", blockIdx.y); every lane of a block
// works on the same pair of moduli, so all modulus-dependent control flow is wave-uniform.  The
// moduli that carry nearly all of the work (the CRT primes and the accumulation moduli of the
// default digit sets, under the ceil label-length rule) run through compile-time descriptions; any
// other modulus takes the same code with run-time constants.
#include "dash_bodies.h"
#include "dash_internal.h"

namespace dash {

struct LdsTab {
    const uint32_t* t;
    __device__ __forceinline__ uint32_t operator()(int r, uint32_t x) const { return t[r * 256 + x]; }
};

__device__ __forceinline__ void load_ttab(uint32_t* lds, const uint32_t* g) {
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) lds[i] = g[i];
    __syncthreads();
}

// ------------------------------------------------------------------------------------------ draw
__global__ __launch_bounds__(kThreads) void k_draw(const DrawLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    draw_body(L, blockIdx.x, blockIdx.y, threadIdx.x, T);
}

int launch_draw(const dash_ctx* c, DrawLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->seed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    dim3 grid((L.n_elem + kThreads - 1) / kThreads, njobs);
    hipLaunchKernelGGL(k_draw, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ---------------------------------------------------------------------------------------- affine
__global__ __launch_bounds__(kThreads) void k_affine(const AffineLaunch L) {
    affine_body(L, blockIdx.x, blockIdx.y, threadIdx.x);
}

int launch_affine(const dash_ctx* c, AffineLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.mods = c->d_mods;
    dim3 grid((L.n_elem + kThreads - 1) / kThreads, njobs);
    hipLaunchKernelGGL(k_affine, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ---------------------------------------------------------------------------------------- garble
// One instantiation per output-modulus description: QD = ModInfo (any modulus, run-time constants) or
// CMod<m, lam> for the hot moduli.  The input modulus is dispatched inside (its code is small).
template <class QD>
__global__ __launch_bounds__(kThreads) void k_proj_garble(const GateLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    garble_body<QD>(L, blockIdx.x, blockIdx.y, threadIdx.x, T);
}

typedef void (*GateKernel)(const GateLaunch);
#define DASH_GARBLE_K(MOD, LAM) k_proj_garble<CMod<MOD, LAM>>,
static const GateKernel kGarbleKernels[] = {k_proj_garble<ModInfo>, DASH_HOT_MODS(DASH_GARBLE_K)};
#undef DASH_GARBLE_K

// every job of a gate launch must have the same output modulus; returns it (0 if they differ)
static uint32_t common_q(const GateLaunch& L, int njobs) {
    for (int j = 1; j < njobs; j++) if (L.jobs[j].q != L.jobs[0].q) return 0;
    return L.jobs[0].q;
}

int launch_garble(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    uint32_t pmax = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table) return DASH_EINVAL;
        pmax = J.p > pmax ? J.p : pmax;
    }
    uint64_t rows = (uint64_t)L.n_elem * pmax;
    uint64_t blocks = (rows + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffull) return DASH_ESIZE;
    dim3 grid((uint32_t)blocks, njobs);
    double units = 0, bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        double lp = c->mods[J.p].lam, lq = J.mode == PAY_SHORT ? 1 : c->mods[J.q].lam;
        units += (double)L.n_elem * J.p;
        bytes += (double)L.n_elem * (lp + (J.phi_stride ? J.p : 0) + lq + J.p * lq + (J.mode == PAY_EHALF ? lq : 0));
    }
    const uint32_t q = common_q(L, njobs);
    if (!q) return DASH_EINVAL;
    ProfScope ps(c->prof, DASH_PROF_GARBLE, s, units, bytes);
    hipLaunchKernelGGL(kGarbleKernels[hot_mod_index(c->mods[q])], grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------------------------------ eval
template <class QD>
__global__ __launch_bounds__(kThreads) void k_proj_eval(const GateLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    eval_body<QD>(L, blockIdx.x, blockIdx.y, threadIdx.x, T);
}
#define DASH_EVAL_K(MOD, LAM) k_proj_eval<CMod<MOD, LAM>>,
static const GateKernel kEvalKernels[] = {k_proj_eval<ModInfo>, DASH_HOT_MODS(DASH_EVAL_K)};
#undef DASH_EVAL_K

int launch_eval(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table || !J.out.p) return DASH_EINVAL;
    }
    dim3 grid((L.n_elem + kThreads - 1) / kThreads, njobs);
    double bytes = 0;
    for (int j = 0; j < njobs; j++) bytes += (double)L.n_elem * (c->mods[L.jobs[j].p].lam + 2.0 * c->mods[L.jobs[j].q].lam);
    const uint32_t q = common_q(L, njobs);
    if (!q) return DASH_EINVAL;
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * njobs, bytes);
    hipLaunchKernelGGL(kEvalKernels[hot_mod_index(c->mods[q])], grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ----------------------------------------------------------------------------- half gate, evaluator
__global__ __launch_bounds__(kThreads) void k_hg_finish(const HgLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    hg_finish_body(L, blockIdx.x, blockIdx.y, threadIdx.x, T);
}

int launch_hg_finish(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    dim3 grid((L.n_elem + kThreads - 1) / kThreads, njobs);
    hipLaunchKernelGGL(k_hg_finish, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
