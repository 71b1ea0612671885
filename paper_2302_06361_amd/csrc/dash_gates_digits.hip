// dash_gates_digits.hip -- the garbler's fused kernels for the digit gates of a sign gadget (Appendix, Approximated
// Garbled Sign).
//
//   k_digits_garble : the k n digit gates of a sign gadget: one lane per (element, value a) of a residue, which forms
//                   and compresses the label once for its n rows
//   k_digits_garble_wide : the same rows, one per lane, for gadgets of few rows
//
// Jobs, table layouts and compile-time moduli as in dash_gates.hip.
#include "dash_tabs.h"

namespace dash {

// --------------------------------------------------------------------- digit gates of the sign gadget, garbler
// One launch for the k n digit gates of a sign gadget: lane = (element, value a) of a residue, which forms and
// compresses the label of a once for the n rows it garbles.  The residues differ in length (n_elem * p rows):
// the blocks share the concatenation of their tiles (one-dimensional grid).
template <class MC, class M1, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads, Banked ? 8 : 1) void k_digits_garble(const DigitsLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    auto tiles_of = [&](uint32_t i) { return (uint32_t)(((uint64_t)L.n_elem * L.res[i].p + kThreads - 1) / kThreads); };
    uint32_t total = 0;
    for (uint32_t i = 0; i < L.nres; i++) total += tiles_of(i);
    uint32_t res = 0, base = 0, next = tiles_of(0);
    for (uint32_t t = blockIdx.x * kGateTiles + sub; t < total; t += gridDim.x * kGateTiles) {
        while (t >= next) { res++; base = next; next += tiles_of(res); }
        digits_garble_body<MC, M1>(L, t - base, __builtin_amdgcn_readfirstlane(res), tx, T);
    }
}

// the same with one lane per ciphertext row: blockIdx.y = digit - 1 (gadgets over few elements)
template <class MC, class M1>
__global__ __launch_bounds__(kThreads) void k_digits_garble_wide(const DigitsLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    auto tiles_of = [&](uint32_t i) { return (uint32_t)(((uint64_t)L.n_elem * L.res[i].p + kThreads - 1) / kThreads); };
    uint32_t total = 0;
    for (uint32_t i = 0; i < L.nres; i++) total += tiles_of(i);
    uint32_t res = 0, base = 0, next = tiles_of(0);
    for (uint32_t t = blockIdx.x; t < total; t += gridDim.x) {
        while (t >= next) { res++; base = next; next += tiles_of(res); }
        digits_garble_body<MC, M1>(L, t - base, __builtin_amdgcn_readfirstlane(res), threadIdx.x, T, blockIdx.y + 1);
    }
}

int launch_digits_garble(const dash_ctx* c, DigitsLaunch& L, hipStream_t s) {
    if (L.n < 1 || L.n > (uint32_t)kMaxChain || L.nres < 1 || L.nres > 16) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    bool uniform = L.n >= 2;
    for (uint32_t j = 1; j <= L.n; j++) {
        if (L.m[j] < 2 || L.m[j] > 255 || !c->mods[L.m[j]].dtab) return DASH_EINVAL;
        if (j >= 3 && L.m[j] != L.m[2]) uniform = false;
    }
    double units = 0, bytes = 0;
    uint64_t tiles = 0;
    for (uint32_t i = 0; i < L.nres; i++) {
        const DigitsRes& R = L.res[i];
        if (R.p < 2 || R.p > 255 || !c->mods[R.p].dtab || !R.in.p || !R.table || !R.out || !R.phi) return DASH_EINVAL;
        const uint64_t rows = (uint64_t)L.n_elem * R.p;
        if (rows >= (1ull << 32)) return DASH_ESIZE;
        tiles += (rows + kThreads - 1) / kThreads;
        units += (double)rows * L.n;
        for (uint32_t j = 1; j <= L.n; j++) bytes += (double)L.n_elem * (c->mods[R.p].lam + (1.0 + R.p) * c->mods[L.m[j]].lam);
    }
    if (tiles > 0x7fffffffull) return DASH_ESIZE;
    const int typed = uniform ? digit_set_index(c->mods[L.m[L.n >= 2 ? 2 : 1]], c->mods[L.m[1]]) : 0;
    ProfScope ps(c->prof, DASH_PROF_GARBLE_DIGITS, s, units, bytes);
    if ((uint64_t)units <= c->few_rows_max) {      // few rows: a lane per row, so that a lane's chain is one hash
        dim3 grid(grid_x_for(tiles, (int)L.n), L.n);
        with_digit_set(typed, [&](auto ds) {
            typedef decltype(ds) DS;
            hipLaunchKernelGGL((k_digits_garble_wide<typename DS::MC, typename DS::M1>), grid, dim3(kThreads), 0, s, L);
        });
        DASH_HIP(hipGetLastError());
        return DASH_OK;
    }
    const bool banked = (uint64_t)(units / L.n) >= c->digits_banked_min_lanes;
    dim3 grid(gate_grid_x_for(tiles, 1, banked));
    const dim3 block(banked ? kBigThreads : kThreads);
    with_digit_set(typed, [&](auto ds) {
        typedef decltype(ds) DS;
        if (banked) hipLaunchKernelGGL((k_digits_garble<typename DS::MC, typename DS::M1, true>), grid, block, 0, s, L);
        else hipLaunchKernelGGL((k_digits_garble<typename DS::MC, typename DS::M1, false>), grid, block, 0, s, L);
    });
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
