// dash_tabs.h -- the AES tables in LDS and the grid shapes shared by the gate kernels (device code,
// included by dash_gates.hip and dash_gates_eval.hip).
#pragma once
#include "dash_bodies.h"
#include "dash_internal.h"

namespace dash {

// AES tables in LDS, two layouts.
//
// LdsTab: T0..T3 once, 4 KB, shared by the block.  A wave's 64 look-ups fall on the 32 banks at random
// (bank = index mod 32): two thirds of the LDS cycles are bank collisions (SQ_LDS_BANK_CONFLICT /
// SQ_LDS_IDX_ACTIVE = 0.68), and AES alone runs at 3.8e10 blocks/s on the chip, exactly what 160 look-ups of
// 6.4 LDS cycles each allow.
//
// BankTab: every entry of T0 and T1 once per bank, 64 KB, for blocks of 1024 lanes (two blocks per CU, eight
// waves per SIMD); T2 and T3 are T0 and T1 rotated by 16 bits, one rotation per column for both.  Byte address
// of entry x of table R (0 or 1) for a lane that owns bank b:  x * 256 + R * 128 + b * 4,  so a look-up never
// collides, and the address still costs ONE instruction, a byte permute: byte 0 <- 4b (from the lane's
// constant), byte 1 <- the state byte; R * 128 goes into the instruction's offset.
//
// Measured on the LeNet batch-16 step: BankTab garbles 3.4e10 rows/s against 2.9e10, but launches that do not
// fill the chip get slower (64 KB to fill per block, fewer and larger blocks), so each kernel exists in both
// forms and the launcher takes BankTab from kBankedMinLanes lanes up.
constexpr int kTabWords = 1024;
constexpr int kBankTabWords = 16384;
constexpr int kBigThreads = 1024;                               // lanes per block with BankTab


struct LdsTab {
    const uint32_t* t;
    template <int R, int B> __device__ __forceinline__ uint32_t at(uint32_t w) const { return t[R * 256 + ((w >> (8 * B)) & 0xffu)]; }
};

__device__ __forceinline__ LdsTab load_ttab(uint32_t* lds, const uint32_t* g) {
    for (int i = threadIdx.x; i < kTabWords; i += blockDim.x) lds[i] = g[i];
    __syncthreads();
    return LdsTab{lds};
}

struct BankTab {
    static constexpr bool two_tables = true;
    const uint8_t* t;
    uint32_t lane;       // byte 0: 4 * bank
    template <int R, int B> __device__ __forceinline__ uint32_t at(uint32_t w) const {
        static_assert(R < 2, "T0 and T1 only");
        // v_perm_b32(hi = w, lo = lane): selector 0..3 bytes of lane, 4..7 bytes of w, 0x0c zero
        constexpr uint32_t sel = 0x0c0c0000u | ((4u + B) << 8);
        const uint32_t a = __builtin_amdgcn_perm(w, lane, sel);
        return *(const uint32_t*)(t + a + R * 128);
    }
};

__device__ __forceinline__ BankTab load_banktab(uint32_t* lds, const uint32_t* g) {
    // one global load per lane (entry x of table R), then its 32 copies as 8 16-byte LDS writes
    for (int e = threadIdx.x; e < 512; e += blockDim.x) {
        const uint32_t v = g[e];
        const int R = e >> 8, x = e & 255;
        uint4* dst = (uint4*)(lds + x * 64 + R * 32);
        const uint4 v4 = make_uint4(v, v, v, v);
#pragma unroll
        for (int i = 0; i < 8; i++) dst[i] = v4;
    }
    __syncthreads();
    return BankTab{(const uint8_t*)lds, (threadIdx.x & 31u) << 2};
}

template <bool Banked> struct gate_tab {
    typedef LdsTab type;
    static constexpr int threads = kThreads, words = kTabWords;
    static __device__ __forceinline__ type load(uint32_t* lds, const uint32_t* g) { return load_ttab(lds, g); }
};
template <> struct gate_tab<true> {
    typedef BankTab type;
    static constexpr int threads = kBigThreads, words = kBankTabWords;
    static __device__ __forceinline__ type load(uint32_t* lds, const uint32_t* g) { return load_banktab(lds, g); }
};

// Blocks walk over tiles of kThreads lanes with a grid stride, so that the table copy in LDS is paid
// once per block and not once per tile.
__host__ inline uint32_t grid_x_for(uint64_t tiles, int njobs) {
    uint64_t cap = 2560 / (uint64_t)njobs;           // about two resident rounds of blocks on 256 CUs
    if (cap < 1) cap = 1;
    return (uint32_t)(tiles < cap ? tiles : cap);
}
// the same for blocks of kBigThreads lanes (kBigThreads / kThreads tiles at a time)
__host__ inline uint32_t gate_grid_x_for(uint64_t tiles, int njobs, bool banked) {
    if (!banked) return grid_x_for(tiles, njobs);
    constexpr int kGateTiles = kBigThreads / kThreads;
    uint64_t blocks = (tiles + kGateTiles - 1) / kGateTiles;
    uint64_t cap = 1024 / (uint64_t)njobs;           // two blocks per CU, two rounds
    if (cap < 1) cap = 1;
    return (uint32_t)(blocks < cap ? blocks : cap);
}

typedef void (*GateKernel)(const GateLaunch);

// every job of a gate launch has the same output modulus: returns it (0 if they differ)
inline uint32_t common_q(const GateLaunch& L, int njobs) {
    for (int j = 1; j < njobs; j++) if (L.jobs[j].q != L.jobs[0].q) return 0;
    return L.jobs[0].q;
}

// argument checks shared by the evaluator's digit-gate launchers; sets the launch's key and table pointers
inline int check_digits(const dash_ctx* c, DigitsLaunch& L, bool* uniform, double* bytes) {
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

// index of the digit set's kernels with compile-time moduli (digit_set_index), 0 = none
inline int typed_digits(const dash_ctx* c, const DigitsLaunch& L, bool uniform) {
    return uniform ? digit_set_index(c->mods[L.m[L.n >= 2 ? 2 : 1]], c->mods[L.m[1]]) : 0;
}

}  // namespace dash
