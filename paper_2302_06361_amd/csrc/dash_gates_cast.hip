// dash_gates_cast.hip -- the evaluator's kernels for the cast step of the scaling gadget (Sec. The Scaling Operation).
//
//   k_cast_halve  : cast of the mod-2 wire into an odd prime and the halving that uses it
//   k_cast_digits_eval, k_cast_digit_wide : that step and the digit gates of the sign gadget behind it in one launch
//
// Jobs, table layouts and compile-time moduli as in dash_gates.hip.
#include "dash_tabs.h"

namespace dash {

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

// the same with the digit gates adding up their outputs themselves (digits_sum_phase1/2): block = 64 elements x the odd
// primes (a wave each), blockIdx.y = digit - 1
template <class MC, class M1>
__global__ __launch_bounds__(1024) void k_cast_digits_sum_wide(const CastLaunch C, const DigitsLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    __shared__ uint32_t acc[kSumElems * kSumDw * 2];
    for (int i = threadIdx.x; i < kSumElems * kSumDw * 2; i += blockDim.x) acc[i] = 0;
    const LdsTab T = load_ttab(tt, L.ttab);                  // (ends with a barrier: the accumulator is clear after it)
    // (the wave's number through a scalar register: the residue's record is then read with scalar loads, like a blockIdx)
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), el = threadIdx.x & 63u, j = blockIdx.y + 1;
    if constexpr (cmod_m<MC>::value != 0) {
        digits_sum_phase1<MC, M1>(C, L, blockIdx.x, wave, j, el, T, acc);
        __syncthreads();                                     // every lane of the block gets here: phase 1 returns, it does not exit
        if (wave == 0) digits_sum_phase2<MC, M1>(L, blockIdx.x, j, el, acc);
    }
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
        if (digits_sum_wanted(L, typed) && c->sum_in_launch) {
            L.sums_in_launch = 1;
            dim3 sgrid((L.n_elem + kSumElems - 1) / kSumElems, L.n);
            with_digit_set(typed, [&](auto ds) {
                typedef decltype(ds) DS;
                hipLaunchKernelGGL((k_cast_digits_sum_wide<typename DS::MC, typename DS::M1>), sgrid, dim3(kSumElems * L.nres), 0, s, C, L);
            });
            DASH_HIP(hipGetLastError());
            return DASH_OK;
        }
        dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)(L.nres * L.n)), L.nres, L.n);
        with_digit_set(typed, [&](auto ds) {
            typedef decltype(ds) DS;
            hipLaunchKernelGGL((k_cast_digit_wide<typename DS::MC, typename DS::M1>), grid, dim3(kThreads), 0, s, C, L);
        });
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
    const int typed = typed_digits(c, L, uniform);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.nres * (L.n + 1), bytes);
    with_digit_set(typed, [&](auto ds) {
        typedef decltype(ds) DS;
        if (banked) hipLaunchKernelGGL((k_cast_digits_eval<typename DS::MC, typename DS::M1, true>), grid, block, 0, s, C, L);
        else hipLaunchKernelGGL((k_cast_digits_eval<typename DS::MC, typename DS::M1, false>), grid, block, 0, s, C, L);
    });
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
