// dash_gates_eval.hip -- the evaluator's gate kernels over LabelTensors.
//
//   k_proj_eval   : one lane per gate: hash the active label, fetch the row its colour names, subtract
//                   (Sec. Arithmetic Garbled Circuits, projection gates)
//   k_hg_finish   : evaluator side of the mixed-modulus half gate       (Appendix)
//   (the sign gadget's digit gates and carry chain: dash_gates_digits_eval.hip; the scaling gadget's cast step:
//   dash_gates_cast.hip -- separate files so that their many instantiations compile side by side)
//
// Jobs, table layouts and compile-time moduli as in dash_gates.hip.
#include "dash_tabs.h"

namespace dash {

// ------------------------------------------------------------------------------------------ eval
template <class QD, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads, Banked ? 8 : 1) void k_proj_eval(const GateLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.jobs[blockIdx.y].n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) eval_body<QD>(L, tile, blockIdx.y, tx, T);
}
#define DASH_EVAL_K(MOD, LAM) k_proj_eval<CMod<MOD, LAM>, false>,
static const GateKernel kEvalKernels[] = {k_proj_eval<ModInfo, false>, DASH_HOT_MODS(DASH_EVAL_K)};
#undef DASH_EVAL_K
#define DASH_EVAL_KB(MOD, LAM) k_proj_eval<CMod<MOD, LAM>, true>,
static const GateKernel kEvalKernelsBanked[] = {k_proj_eval<ModInfo, true>, DASH_HOT_MODS(DASH_EVAL_KB)};
#undef DASH_EVAL_KB

int launch_eval(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    uint64_t lanes = 0;
    uint32_t nmax = 0;
    double bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
        if (J.n_elem == 0) continue;
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table || !J.out.p) return DASH_EINVAL;
        lanes += J.n_elem;
        nmax = J.n_elem > nmax ? J.n_elem : nmax;
        bytes += (double)J.n_elem * (c->mods[J.p].lam + 2.0 * c->mods[J.q].lam);
    }
    if (nmax == 0) return DASH_OK;
    const bool banked = lanes >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((nmax + kThreads - 1) / kThreads, njobs, banked), njobs);
    const uint32_t q = common_q(L, njobs);
    L.njobs = (uint32_t)njobs;
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)lanes, bytes);
    const int ki = q ? hot_mod_index(c->mods[q]) : 0;
    hipLaunchKernelGGL(banked ? kEvalKernelsBanked[ki] : kEvalKernels[ki], grid, dim3(banked ? kBigThreads : kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ----------------------------------------------------------------------------- half gate, evaluator
__global__ __launch_bounds__(kThreads) void k_hg_finish(const HgLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) hg_finish_body(L, tile, blockIdx.y, threadIdx.x, T);
}

// the half gate's two projection gates and its finish in one launch, four lanes per (element, prime): layers of few elements
__global__ __launch_bounds__(kThreads) void k_hg_eval_quad(const HgLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (uint32_t)(((uint64_t)L.n_elem * 4 + kThreads - 1) / kThreads);
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) hg_eval_quad_body(L, tile, blockIdx.y, threadIdx.x, T);
}

// whether launch_hg_eval_quad serves this layer: few elements, every prime with a compile-time description
bool hg_eval_quad_wanted(const dash_ctx* c, uint32_t n_elem) {
    if ((uint64_t)n_elem * 4 * c->k > c->quad_max_lanes) return false;
    for (int i = 0; i < c->k; i++) if (!hot_mod_index(c->mods[c->prime[i]])) return false;
    return true;
}

int launch_hg_eval_quad(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 26)) return DASH_ESIZE;
    double bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const HgJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || !hot_mod_index(c->mods[J.p]) || J.slot < 2) return DASH_EINVAL;
        if (!J.x.p || !J.y.p || !J.z.p || !J.S || !J.G || !J.Eh) return DASH_EINVAL;
        bytes += (double)L.n_elem * (2.0 * c->mods[2].lam + 4.0 * c->mods[J.p].lam + 4);
    }
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    dim3 grid(grid_x_for(((uint64_t)L.n_elem * 4 + kThreads - 1) / kThreads, njobs), njobs);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * njobs * 2, bytes);
    hipLaunchKernelGGL(k_hg_eval_quad, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

int launch_hg_finish(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, njobs), njobs);
    hipLaunchKernelGGL(k_hg_finish, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
