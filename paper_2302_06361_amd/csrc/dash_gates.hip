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
// works on the same pair of moduli, so all modulus-dependent control flow is wave-uniform.
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

// dword i (digits 4i..4i+3) of element e of a label view
__device__ __forceinline__ uint32_t ld_dw(const LView& v, uint32_t e, int i) {
    return *(const uint32_t*)(v.p + (int64_t)(i >> 2) * v.cs + (uint64_t)e * v.es + (i & 3) * 4);
}
__device__ __forceinline__ void st_dw(const LView& v, uint32_t e, int i, uint32_t w) {
    *(uint32_t*)(v.p + (int64_t)(i >> 2) * v.cs + (uint64_t)e * v.es + (i & 3) * 4) = w;
}

// packed digits 4i..4i+3 of sum_t coef_t * term_t[e] mod m
__device__ __forceinline__ uint32_t combine_dw(const Term* terms, uint32_t first, uint32_t count, const ModInfo& M,
                                               uint32_t e, int i) {
    if (count == 1 && terms[first].coef == 1) return ld_dw(terms[first].v, e, i);
    uint32_t acc[4] = {0, 0, 0, 0};
    for (uint32_t t = 0; t < count; t++) {
        uint32_t w = ld_dw(terms[first + t].v, e, i), c = terms[first + t].coef;
        for (int b = 0; b < 4; b++) acc[b] += c * byte_of(w, b);      // <= 16 * 254 * 254 < 2^24
    }
    return mod_m(acc[0], M) | (mod_m(acc[1], M) << 8) | (mod_m(acc[2], M) << 16) | (mod_m(acc[3], M) << 24);
}

// ------------------------------------------------------------------------------------------ draw
__global__ __launch_bounds__(kThreads) void k_draw(const DrawLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    const DrawJob& J = L.jobs[blockIdx.y];
    uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= L.n_elem) return;
    const ModInfo M = L.mods[J.m];
    U128 h = prg_block(L.elem_base + e, J.slot, L.layer, J.domain, J.m, L.key.rk, T);
    if (J.digit0_only) { J.out.p[e] = (uint8_t)mod_u128(h, M); return; }
    decompress(M, h, [&](int i, uint32_t w) { st_dw(J.out, e, i, w); });
    for (int i = (int)M.ndw; i < (int)M.nchunk * 4; i++) st_dw(J.out, e, i, 0);
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
    const AffineJob& J = L.jobs[blockIdx.y];
    uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= L.n_elem) return;
    const ModInfo M = L.mods[J.m];
    for (int i = 0; i < (int)M.nchunk * 4; i++) {
        uint32_t acc[4] = {0, 0, 0, 0};
        for (uint32_t t = 0; t < J.term_count; t++) {
            uint32_t w = ld_dw(L.terms[J.term_first + t].v, e, i), cf = L.terms[J.term_first + t].coef;
            for (int b = 0; b < 4; b++) acc[b] += cf * byte_of(w, b);
        }
        st_dw(J.out, e, i, mod_m(acc[0], M) | (mod_m(acc[1], M) << 8) | (mod_m(acc[2], M) << 16) | (mod_m(acc[3], M) << 24));
    }
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
__global__ __launch_bounds__(kThreads) void k_proj_garble(const GateLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    const GateJob& J = L.jobs[blockIdx.y];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    // one lane per row: r = gate * p + a
    uint64_t r = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (r >= (uint64_t)L.n_elem * Mp.m) return;
    uint32_t g = (uint32_t)(r / Mp.m), a = (uint32_t)(r - (uint64_t)g * Mp.m);

    // label of value a on the input wire: zero label + a * R_p (table row a of the offset multiples)
    const uint32_t* da = Mp.dtab + (size_t)a * Mp.ndw;
    uint32_t colour;
    U128 K = compress(Mp, [&](int i) {
        return addmod4(combine_dw(L.terms, J.term_first, J.term_count, Mp, g, i), da[i], Mp);
    }, &colour);
    U128 h = hash_block(K, L.elem_base + g, J.slot, L.layer, L.key.rk, T);

    if (J.mode == PAY_SHORT) {
        uint32_t v = mod_m(a + J.r[g] + mod_u128(h, Mq), Mq);
        *(uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * 4) = v;
        return;
    }
    uint32_t* row = (uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * (Mq.ndw * 4));
    if (J.mode == PAY_EHALF) {
        uint32_t cf = mod_m(a + J.r[g], Mq);
        cf = cf ? Mq.m - cf : 0;                         // minus (a + r) * x0
        decompress(Mq, h, [&](int i, uint32_t hd) {
            uint32_t pay = axpymod4(ld_dw(J.out, g, i), cf, ld_dw(J.x0, g, i), Mq);
            row[i] = addmod4(pay, hd, Mq);
        });
        return;
    }
    uint32_t f = (J.mode == PAY_MULR) ? mod_m(a * J.r[g], Mq) : J.phi[(size_t)g * J.phi_stride + a];
    const uint32_t* df = Mq.dtab + (size_t)f * Mq.ndw;
    decompress(Mq, h, [&](int i, uint32_t hd) {
        row[i] = addmod4(addmod4(ld_dw(J.out, g, i), df[i], Mq), hd, Mq);
    });
}

int launch_garble(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    uint32_t pmax = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (J.term_first + J.term_count > (uint32_t)kMaxTerms || J.term_count == 0) return DASH_EINVAL;
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
        bytes += (double)L.n_elem * (J.term_count * lp + (J.phi_stride ? J.p : 0) + lq + J.p * lq + (J.mode == PAY_EHALF ? lq : 0));
    }
    ProfScope ps(c->prof, DASH_PROF_GARBLE, s, units, bytes);
    hipLaunchKernelGGL(k_proj_garble, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------------------------------ eval
__global__ __launch_bounds__(kThreads) void k_proj_eval(const GateLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    const GateJob& J = L.jobs[blockIdx.y];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    uint32_t g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= L.n_elem) return;
    uint32_t colour;
    U128 K = compress(Mp, [&](int i) { return combine_dw(L.terms, J.term_first, J.term_count, Mp, g, i); }, &colour);
    U128 h = hash_block(K, L.elem_base + g, J.slot, L.layer, L.key.rk, T);
    const uint32_t* row = (const uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * (Mq.ndw * 4));
    decompress(Mq, h, [&](int i, uint32_t hd) { st_dw(J.out, g, i, submod4(row[i], hd, Mq)); });
    for (int i = (int)Mq.ndw; i < (int)Mq.nchunk * 4; i++) st_dw(J.out, g, i, 0);
}

int launch_eval(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (J.term_first + J.term_count > (uint32_t)kMaxTerms || J.term_count == 0) return DASH_EINVAL;
    }
    dim3 grid((L.n_elem + kThreads - 1) / kThreads, njobs);
    double bytes = 0;
    for (int j = 0; j < njobs; j++) bytes += (double)L.n_elem * (L.jobs[j].term_count * c->mods[L.jobs[j].p].lam + 2.0 * c->mods[L.jobs[j].q].lam);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * njobs, bytes);
    hipLaunchKernelGGL(k_proj_eval, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ----------------------------------------------------------------------------- half gate, evaluator
__global__ __launch_bounds__(kThreads) void k_hg_finish(const HgLaunch L) {
    __shared__ uint32_t tt[1024];
    load_ttab(tt, L.ttab);
    LdsTab T{tt};
    const HgJob& J = L.jobs[blockIdx.y];
    const ModInfo M2 = L.mods[2], Mp = L.mods[J.p];
    uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= L.n_elem) return;
    uint32_t colour;
    U128 K = compress(M2, [&](int i) { return ld_dw(J.y, e, i); }, &colour);
    U128 h = hash_block(K, L.elem_base + e, J.slot, L.layer, L.key.rk, T);
    uint32_t s = *(const uint32_t*)(J.S + ((size_t)e * 2 + colour) * 4);
    uint32_t beta = mod_m(s + Mp.m - mod_u128(h, Mp), Mp);
    for (int i = 0; i < (int)Mp.nchunk * 4; i++) {
        uint32_t v = axpymod4(ld_dw(J.V, e, i), beta, ld_dw(J.x, e, i), Mp);
        st_dw(J.z, e, i, submod4(v, ld_dw(J.U, e, i), Mp));
    }
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
