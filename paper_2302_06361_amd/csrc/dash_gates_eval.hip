// dash_gates_eval.hip -- the evaluator's gate kernels over LabelTensors.
//
//   k_proj_eval   : one lane per gate: hash the active label, fetch the row its colour names, subtract
//                   (Sec. Arithmetic Garbled Circuits, projection gates)
//   k_digits_eval : the k n digit gates of a sign gadget, one lane per (element, residue): one compress, n gates
//   k_chain_eval  : the n dependent gates of the mixed-radix addition of a sign gadget, one lane per element
//   k_cast_halve  : scaling gadget: cast of the mod-2 wire into an odd prime and the halving that uses it
//                   (Sec. The Scaling Operation)
//   k_hg_finish   : evaluator side of the mixed-modulus half gate       (Appendix)
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

// ------------------------------------------------------------------- digit gates of the sign gadget, evaluator
// One launch for the k n digit gates of a sign gadget (four launches of k_proj_eval before), lane = (element,
// residue): the label is loaded and compressed once for its n gates.
template <class MC, class M1, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads, Banked ? 8 : 1) void k_digits_eval(const DigitsLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles)
        digits_eval_body<MC, M1>(L, tile, blockIdx.y, tx, T);
}

// one lane per (element, residue, digit): blockIdx.y = residue, blockIdx.z = digit - 1
template <class MC, class M1>
__global__ __launch_bounds__(kThreads) void k_digits_eval_wide(const DigitsLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x)
        digits_eval_wide_body<MC, M1>(L, tile, blockIdx.y, blockIdx.z + 1, threadIdx.x, T);
}

static int check_digits(const dash_ctx* c, DigitsLaunch& L, bool* uniform, double* bytes) {
    if (L.n < 1 || L.n > (uint32_t)kMaxChain || L.nres < 1 || L.nres > 16) return DASH_EINVAL;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    *uniform = L.n >= 2;
    for (uint32_t j = 1; j <= L.n; j++) {
        if (L.m[j] < 2 || L.m[j] > 255 || !c->mods[L.m[j]].dtab) return DASH_EINVAL;
        if (j >= 3 && L.m[j] != L.m[2]) *uniform = false;
    }
    for (uint32_t i = 0; i < L.nres; i++) {
        const DigitsRes& R = L.res[i];
        if (R.p < 2 || R.p > 255 || !c->mods[R.p].dtab || !R.in.p || !R.table || !R.out) return DASH_EINVAL;
        for (uint32_t j = 1; j <= L.n; j++) *bytes += (double)L.n_elem * (c->mods[R.p].lam + 2.0 * c->mods[L.m[j]].lam);
    }
    return DASH_OK;
}

// Which digit sets have kernels with compile-time moduli: 1 = (26; 96 ...), 2 = (46; 204 ...), 0 = none
static int typed_digits(const dash_ctx* c, const DigitsLaunch& L, bool uniform) {
    auto is = [](const ModInfo& M, uint32_t m, uint32_t lam) { return M.m == m && M.lam == lam; };
    const ModInfo &M1 = c->mods[L.m[1]], &Mc = c->mods[L.m[L.n >= 2 ? 2 : 1]];
    if (uniform && is(Mc, 96, 20) && is(M1, 26, 28)) return 1;
    if (uniform && is(Mc, 204, 17) && is(M1, 46, 24)) return 2;
    return 0;
}

int launch_digits_eval(const dash_ctx* c, DigitsLaunch& L, hipStream_t s) {
    bool uniform = false;
    double bytes = 0;
    const int st = check_digits(c, L, &uniform, &bytes);
    if (st) return st;
    if (L.n_elem == 0) return DASH_OK;
    const int typed = typed_digits(c, L, uniform);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.nres * L.n, bytes);
    if ((uint64_t)L.n_elem * L.nres * L.n <= c->wide_max_lanes) {
        // few elements: the launch does not fill the chip, its time is the chain of hashes of one lane
        dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)(L.nres * L.n)), L.nres, L.n);
        if (typed == 1) hipLaunchKernelGGL((k_digits_eval_wide<CMod<96, 20>, CMod<26, 28>>), grid, dim3(kThreads), 0, s, L);
        else if (typed == 2) hipLaunchKernelGGL((k_digits_eval_wide<CMod<204, 17>, CMod<46, 24>>), grid, dim3(kThreads), 0, s, L);
        else hipLaunchKernelGGL((k_digits_eval_wide<ModInfo, ModInfo>), grid, dim3(kThreads), 0, s, L);
        DASH_HIP(hipGetLastError());
        return DASH_OK;
    }
    // (by lanes, not by hashes: with n hashes per lane the 64 KB tables were still measured slower below this size)
    const bool banked = (uint64_t)L.n_elem * L.nres >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)L.nres, banked), L.nres);
    const dim3 block(banked ? kBigThreads : kThreads);
    if (typed == 1) {
        if (banked) hipLaunchKernelGGL((k_digits_eval<CMod<96, 20>, CMod<26, 28>, true>), grid, block, 0, s, L);
        else hipLaunchKernelGGL((k_digits_eval<CMod<96, 20>, CMod<26, 28>, false>), grid, block, 0, s, L);
    } else if (typed == 2) {
        if (banked) hipLaunchKernelGGL((k_digits_eval<CMod<204, 17>, CMod<46, 24>, true>), grid, block, 0, s, L);
        else hipLaunchKernelGGL((k_digits_eval<CMod<204, 17>, CMod<46, 24>, false>), grid, block, 0, s, L);
    } else {
        if (banked) hipLaunchKernelGGL((k_digits_eval<ModInfo, ModInfo, true>), grid, block, 0, s, L);
        else hipLaunchKernelGGL((k_digits_eval<ModInfo, ModInfo, false>), grid, block, 0, s, L);
    }
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------- carry chain of the sign gadget, evaluator
// One launch for the n dependent gates of the mixed-radix addition (a launch per digit costs about 10 us each,
// whatever the layer size, and they cannot overlap).  Instantiations for the two default digit sets; any
// other set takes the body with run-time constants.
template <class MC, class M1>
__global__ __launch_bounds__(kThreads) void k_chain_eval(const ChainLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) chain_eval_body<MC, M1>(L, tile, threadIdx.x, T);
}
__global__ __launch_bounds__(kThreads) void k_chain_eval_generic(const ChainLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) chain_eval_generic_body(L, tile, threadIdx.x, T);
}

int launch_chain_eval(const dash_ctx* c, ChainLaunch& L, hipStream_t s) {
    if (L.n < 2 || L.n > (uint32_t)kMaxChain) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    bool uniform = true;
    double bytes = 0;
    for (uint32_t j = 1; j <= L.n; j++) {
        if (L.m[j] < 2 || L.m[j] > 255 || !L.table[j] || !L.sum[j].p || (j < L.n && !L.carry[j].p)) return DASH_EINVAL;
        if (j >= 3 && L.m[j] != L.m[2]) uniform = false;
        bytes += (double)L.n_elem * (c->mods[L.m[j]].lam + (j >= 2 ? c->mods[L.m[j - 1]].lam : 128));
    }
    if ((uint64_t)L.n_elem * 255 >= (1ull << 32)) return DASH_ESIZE;
    const ModInfo &Mc = c->mods[L.m[2]], &M1 = c->mods[L.m[1]];
    auto is = [](const ModInfo& M, uint32_t m, uint32_t lam) { return M.m == m && M.lam == lam; };
    dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, 1));
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.n, bytes);
    const bool bit128 = c->mods[2].lam == 128;      // the fused bodies write the 128 digits of the sign wire
    if (bit128 && uniform && is(Mc, 96, 20) && is(M1, 26, 28))
        hipLaunchKernelGGL((k_chain_eval<CMod<96, 20>, CMod<26, 28>>), grid, dim3(kThreads), 0, s, L);
    else if (bit128 && uniform && is(Mc, 204, 17) && is(M1, 46, 24))
        hipLaunchKernelGGL((k_chain_eval<CMod<204, 17>, CMod<46, 24>>), grid, dim3(kThreads), 0, s, L);
    else
        hipLaunchKernelGGL(k_chain_eval_generic, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ----------------------------------------------------------------------------- scaling gadget, evaluator
// cast of the mod-2 residue into every odd prime and the halving, one launch (a gate launch and a free-gate launch
// before), blockIdx.y = odd prime.  (One lane per element that walks over the primes, compressing the 128-digit label
// once, was measured three times slower: too few lanes.)
__global__ __launch_bounds__(kThreads) void k_cast_halve(const CastLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) cast_halve_body(L, tile, blockIdx.y, threadIdx.x, T);
}

int launch_cast_halve(const dash_ctx* c, CastLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    if (!L.y.p) return DASH_EINVAL;
    double bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const CastJob& J = L.jobs[j];
        if (J.p < 3 || J.p > 255 || !(J.p & 1) || !c->mods[J.p].dtab || J.addc >= J.p) return DASH_EINVAL;
        if (!J.table || !J.x.p || !J.out.p || (J.addc && !J.one.p)) return DASH_EINVAL;
        bytes += (double)L.n_elem * (128 + 2.0 * c->mods[J.p].lam);
    }
    dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, njobs), njobs);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * njobs, bytes);
    hipLaunchKernelGGL(k_cast_halve, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// Scaling gadget, evaluator: the cast-and-halve step and the digit gates of the sign gadget that follows it in ONE
// launch.  Both give a lane the same (element, odd prime): the lane writes its halved label b and reads it back for
// its n digit gates (its own store, then its own loads), so no other lane is waited for, and a launch and its gap
// are saved per repetition of the gadget.
static_assert(sizeof(CastLaunch) + sizeof(DigitsLaunch) <= 4096, "kernel arguments");
template <class MC, class M1, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_cast_digits_eval(const CastLaunch C, const DigitsLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) {
        cast_halve_body(C, tile, blockIdx.y, tx, T);
        digits_eval_body<MC, M1>(L, tile, blockIdx.y, tx, T);
    }
}

// the same with one lane per (element, odd prime, digit): blockIdx.y = prime, blockIdx.z = digit - 1
template <class MC, class M1>
__global__ __launch_bounds__(kThreads) void k_cast_digit_wide(const CastLaunch C, const DigitsLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x)
        cast_digit_wide_body<MC, M1>(C, L, tile, blockIdx.y, blockIdx.z + 1, threadIdx.x, T);
}

static int check_cast(const dash_ctx* c, const CastLaunch& L, int njobs, double* bytes) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    if (!L.y.p) return DASH_EINVAL;
    for (int j = 0; j < njobs; j++) {
        const CastJob& J = L.jobs[j];
        if (J.p < 3 || J.p > 255 || !(J.p & 1) || !c->mods[J.p].dtab || J.addc >= J.p) return DASH_EINVAL;
        if (!J.table || !J.x.p || !J.out.p || (J.addc && !J.one.p)) return DASH_EINVAL;
        *bytes += (double)L.n_elem * (128 + 2.0 * c->mods[J.p].lam);
    }
    return DASH_OK;
}

int launch_cast_digits_eval(const dash_ctx* c, CastLaunch& C, int njobs, DigitsLaunch& L, hipStream_t s) {
    if (L.n < 1 || L.n > (uint32_t)kMaxChain || L.nres < 1 || L.nres > 16 || (int)L.nres != njobs) return DASH_EINVAL;
    if (C.n_elem != L.n_elem || C.layer != L.layer || C.elem_base != L.elem_base) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if ((uint64_t)L.n_elem * L.nres * L.n <= c->wide_max_lanes) {
        // few elements: a lane per digit gate that repeats the cast step of its residue (primes with compile-time label
        // lengths), else the cast step in a launch of its own before the digit gates
        bool hot = true;
        for (int j = 0; j < njobs; j++) if (C.jobs[j].p > 255 || !hot_mod_index(c->mods[C.jobs[j].p])) hot = false;
        if (!hot) {
            const int st = launch_cast_halve(c, C, njobs, s);
            return st ? st : launch_digits_eval(c, L, s);
        }
        bool uniform = false;
        double bytes = 0;
        int st = check_cast(c, C, njobs, &bytes);
        if (st) return st;
        st = check_digits(c, L, &uniform, &bytes);
        if (st) return st;
        for (uint32_t i = 0; i < L.nres; i++) {
            const DigitsRes& R = L.res[i];
            const CastJob& J = C.jobs[i];
            if (R.p != J.p || R.in.p != J.out.p || R.in.cs != J.out.cs || R.in.es != J.out.es) return DASH_EINVAL;
        }
        C.key = c->fixed; C.ttab = c->d_ttab; C.mods = c->d_mods;
        const int typed = typed_digits(c, L, uniform);
        ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.nres * (L.n + 1), bytes);
        dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)(L.nres * L.n)), L.nres, L.n);
        if (typed == 1) hipLaunchKernelGGL((k_cast_digit_wide<CMod<96, 20>, CMod<26, 28>>), grid, dim3(kThreads), 0, s, C, L);
        else if (typed == 2) hipLaunchKernelGGL((k_cast_digit_wide<CMod<204, 17>, CMod<46, 24>>), grid, dim3(kThreads), 0, s, C, L);
        else hipLaunchKernelGGL((k_cast_digit_wide<ModInfo, ModInfo>), grid, dim3(kThreads), 0, s, C, L);
        DASH_HIP(hipGetLastError());
        return DASH_OK;
    }
    double bytes = 0;
    int st = check_cast(c, C, njobs, &bytes);
    if (st) return st;
    C.key = c->fixed; C.ttab = c->d_ttab; C.mods = c->d_mods;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    bool uniform = L.n >= 2;
    for (uint32_t j = 1; j <= L.n; j++) {
        if (L.m[j] < 2 || L.m[j] > 255 || !c->mods[L.m[j]].dtab) return DASH_EINVAL;
        if (j >= 3 && L.m[j] != L.m[2]) uniform = false;
    }
    for (uint32_t i = 0; i < L.nres; i++) {
        const DigitsRes& R = L.res[i];
        const CastJob& J = C.jobs[i];
        if (!R.table || !R.out) return DASH_EINVAL;
        // lane (element, i) of the digit gates reads what lane (element, i) of the cast step wrote
        if (R.p != J.p || R.in.p != J.out.p || R.in.cs != J.out.cs || R.in.es != J.out.es) return DASH_EINVAL;
        for (uint32_t j = 1; j <= L.n; j++) bytes += (double)L.n_elem * (c->mods[R.p].lam + 2.0 * c->mods[L.m[j]].lam);
    }
    const bool banked = (uint64_t)L.n_elem * L.nres >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)L.nres, banked), L.nres);
    const dim3 block(banked ? kBigThreads : kThreads);
    auto is = [](const ModInfo& M, uint32_t m, uint32_t lam) { return M.m == m && M.lam == lam; };
    const ModInfo &M1 = c->mods[L.m[1]], &Mc = c->mods[L.m[L.n >= 2 ? 2 : 1]];
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.nres * (L.n + 1), bytes);
    if (uniform && is(Mc, 96, 20) && is(M1, 26, 28)) {
        if (banked) hipLaunchKernelGGL((k_cast_digits_eval<CMod<96, 20>, CMod<26, 28>, true>), grid, block, 0, s, C, L);
        else hipLaunchKernelGGL((k_cast_digits_eval<CMod<96, 20>, CMod<26, 28>, false>), grid, block, 0, s, C, L);
    } else if (uniform && is(Mc, 204, 17) && is(M1, 46, 24)) {
        if (banked) hipLaunchKernelGGL((k_cast_digits_eval<CMod<204, 17>, CMod<46, 24>, true>), grid, block, 0, s, C, L);
        else hipLaunchKernelGGL((k_cast_digits_eval<CMod<204, 17>, CMod<46, 24>, false>), grid, block, 0, s, C, L);
    } else {
        if (banked) hipLaunchKernelGGL((k_cast_digits_eval<ModInfo, ModInfo, true>), grid, block, 0, s, C, L);
        else hipLaunchKernelGGL((k_cast_digits_eval<ModInfo, ModInfo, false>), grid, block, 0, s, C, L);
    }
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
