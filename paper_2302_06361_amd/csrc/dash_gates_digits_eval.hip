// dash_gates_digits_eval.hip -- the evaluator's kernels for the sign gadget (Appendix, Approximated Garbled Sign and
// Garbled Mixed-Radix Addition).
//
//   k_digits_eval : the k n digit gates of a sign gadget, one lane per (element, residue): one compress, n gates
//   k_digits_eval_wide : the same gates one per lane, for gadgets over few elements
//   k_chain_eval  : the n dependent gates of the mixed-radix addition of a sign gadget, one lane per element
//
// Jobs, table layouts and compile-time moduli as in dash_gates.hip.
#include "dash_tabs.h"

namespace dash {

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

// few elements, digit sets with compile-time moduli: the digit gates add up their outputs themselves (digits_sum_phase1/2).
// Block = 64 elements x the residues (a wave each), blockIdx.y = digit - 1.
template <class MC, class M1>
__global__ __launch_bounds__(1024) void k_digits_sum_wide(const DigitsLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    __shared__ uint32_t acc[kSumElems * kSumDw * 2];
    for (int i = threadIdx.x; i < kSumElems * kSumDw * 2; i += blockDim.x) acc[i] = 0;
    const LdsTab T = load_ttab(tt, L.ttab);                  // (ends with a barrier: the accumulator is clear after it)
    // (the wave's number through a scalar register: the residue's record is then read with scalar loads, like a blockIdx)
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), el = threadIdx.x & 63u, j = blockIdx.y + 1;
    if constexpr (cmod_m<MC>::value != 0) {
        digits_sum_phase1<MC, M1>(NoCast{}, L, blockIdx.x, wave, j, el, T, acc);
        __syncthreads();                                     // every lane of the block gets here: phase 1 returns, it does not exit
        if (wave == 0) digits_sum_phase2<MC, M1>(L, blockIdx.x, j, el, acc);
    }
}
// whether a wide launch can take that form
bool digits_sum_wanted(const DigitsLaunch& L, int typed) {
    return typed != 0 && L.n >= 2 && L.sum1 != nullptr && L.nres * kSumElems <= 1024;
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
        if (digits_sum_wanted(L, typed) && c->sum_in_launch) {
            L.sums_in_launch = 1;
            dim3 sgrid((L.n_elem + kSumElems - 1) / kSumElems, L.n);
            with_digit_set(typed, [&](auto ds) {
                typedef decltype(ds) DS;
                hipLaunchKernelGGL((k_digits_sum_wide<typename DS::MC, typename DS::M1>), sgrid, dim3(kSumElems * L.nres), 0, s, L);
            });
            DASH_HIP(hipGetLastError());
            return DASH_OK;
        }
        dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)(L.nres * L.n)), L.nres, L.n);
        with_digit_set(typed, [&](auto ds) {
            typedef decltype(ds) DS;
            hipLaunchKernelGGL((k_digits_eval_wide<typename DS::MC, typename DS::M1>), grid, dim3(kThreads), 0, s, L);
        });
        DASH_HIP(hipGetLastError());
        return DASH_OK;
    }
    // (by lanes, not by hashes: with n hashes per lane the 64 KB tables were still measured slower below this size)
    const bool banked = (uint64_t)L.n_elem * L.nres >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((L.n_elem + kThreads - 1) / kThreads, (int)L.nres, banked), L.nres);
    const dim3 block(banked ? kBigThreads : kThreads);
    with_digit_set(typed, [&](auto ds) {
        typedef decltype(ds) DS;
        if (banked) hipLaunchKernelGGL((k_digits_eval<typename DS::MC, typename DS::M1, true>), grid, block, 0, s, L);
        else hipLaunchKernelGGL((k_digits_eval<typename DS::MC, typename DS::M1, false>), grid, block, 0, s, L);
    });
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------- carry chain of the sign gadget, evaluator
// One launch for the n dependent gates of the mixed-radix addition (a launch per digit costs about 10 us each,
// whatever the layer size, and they cannot overlap).  Instantiations for the digit sets with compile-time moduli (DASH_DIGIT_SETS); any
// other set takes the body with run-time constants.
// QUAD: four lanes per element, which share the AES of each gate (layers of few elements).
template <class MC, class M1, bool QUAD>
__global__ __launch_bounds__(kThreads) void k_chain_eval(const ChainLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (uint32_t)(((uint64_t)L.n_elem * (QUAD ? 4 : 1) + kThreads - 1) / kThreads);
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) chain_eval_body<MC, M1, QUAD>(L, tile, threadIdx.x, T);
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
    const bool quad = (uint64_t)L.n_elem * 4 <= c->quad_max_lanes;
    dim3 grid(grid_x_for(((uint64_t)L.n_elem * (quad ? 4 : 1) + kThreads - 1) / kThreads, 1));
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.n, bytes);
    const bool bit128 = c->mods[2].lam == 128;      // the fused bodies write the 128 digits of the sign wire
    const int typed = bit128 && uniform ? digit_set_index(c->mods[L.m[2]], c->mods[L.m[1]]) : 0;
    with_digit_set(typed, [&](auto ds) {
        typedef decltype(ds) DS;
        if constexpr (cmod_m<typename DS::MC>::value != 0) {
            if (quad) hipLaunchKernelGGL((k_chain_eval<typename DS::MC, typename DS::M1, true>), grid, dim3(kThreads), 0, s, L);
            else hipLaunchKernelGGL((k_chain_eval<typename DS::MC, typename DS::M1, false>), grid, dim3(kThreads), 0, s, L);
        } else hipLaunchKernelGGL(k_chain_eval_generic, grid, dim3(kThreads), 0, s, L);
    });
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
