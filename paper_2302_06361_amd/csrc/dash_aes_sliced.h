// dash_aes_sliced.h -- AES-128 encryption (FIPS-197) on bit planes: a lane works on 32 blocks at once, one bit
// of each per register, and needs no table.  This is the table-free alternative to the T-table code in
// dash_core.h; it exists to be measured against it (dash_profile.h), the gate kernels use the tables.
//
// Layout: the 128 registers S[8 i + b] hold bit b of state byte i (i = 4 c + r: column c, row r; byte i of the
// block in memory), bit j of a register belonging to block j.  SubBytes is the generated Boolean circuit of
// dash_sbox_circuit.h; ShiftRows only renames registers; MixColumns works on planes (doubling in GF(2^8) moves
// plane b to b + 1 and folds plane 7 into planes 0, 1, 3, 4); the round keys enter as masks of all ones or all
// zeros that the caller prepares (sliced_key_masks), with the S-box's constant 0x63 folded into them.
#pragma once
#include "dash_core.h"
#include "dash_sbox_circuit.h"

namespace dash {

// three-input bit operation with truth table TT = f(0xF0, 0xCC, 0xAA)
struct Bop3 {
    template <int TT> static DASH_HD uint32_t op(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__) && __has_builtin(__builtin_amdgcn_bitop3_b32)
        return __builtin_amdgcn_bitop3_b32(a, b, c, TT);
#else
        uint32_t r = 0;
        for (int m = 0; m < 8; m++)
            if ((TT >> m) & 1) r |= ((m & 4) ? a : ~a) & ((m & 2) ? b : ~b) & ((m & 1) ? c : ~c);
        return r;
#endif
    }
};

// bytes of (hi:lo) picked by the four selector bytes (0..3 from lo, 4..7 from hi)
DASH_HD uint32_t pick_bytes(uint32_t hi, uint32_t lo, uint32_t sel) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_perm(hi, lo, sel);
#else
    const uint64_t v = ((uint64_t)hi << 32) | lo;
    uint32_t r = 0;
    for (int k = 0; k < 4; k++) r |= (uint32_t)((v >> (8 * ((sel >> (8 * k)) & 7u))) & 0xffu) << (8 * k);
    return r;
#endif
}

// One stage of the 32 x 32 bit transposition: the bits of a whose index has bit J set change places with the bits
// of b whose index has it clear.
template <int J> DASH_HD void swap_stage(uint32_t& a, uint32_t& b) {
    uint32_t na, nb;
    if constexpr (J == 16) {
        na = pick_bytes(b, a, 0x05040100u);
        nb = pick_bytes(b, a, 0x07060302u);
    } else if constexpr (J == 8) {
        na = pick_bytes(b, a, 0x06020400u);
        nb = pick_bytes(b, a, 0x07030501u);
    } else {
        constexpr uint32_t m = J == 4 ? 0x0f0f0f0fu : J == 2 ? 0x33333333u : 0x55555555u;
        na = Bop3::op<0xE4>(a, b << J, m);          // (a & m) | ((b << J) & ~m)
        nb = Bop3::op<0xE4>(a >> J, b, m);          // ((a >> J) & m) | (b & ~m)
    }
    a = na;
    b = nb;
}
template <int J> DASH_HD void transpose_stage(uint32_t* a) {
#pragma unroll
    for (int k = 0; k < 32; k++)
        if ((k & J) == 0) swap_stage<J>(a[k], a[k + J]);
}
// a[t] bit j  <->  a[j] bit t  (its own inverse)
DASH_HD void transpose32(uint32_t* a) {
    transpose_stage<16>(a);
    transpose_stage<8>(a);
    transpose_stage<4>(a);
    transpose_stage<2>(a);
    transpose_stage<1>(a);
}

// SubBytes (without the constant) and ShiftRows: N[4c + r] = S-box(S[4((c + r) mod 4) + r])
DASH_HD void sliced_sub_shift(const uint32_t* S, uint32_t* N) {
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const int c = i >> 2, r = i & 3, s = 8 * (4 * ((c + r) & 3) + r);
        sbox_planes(S[s + 0], S[s + 1], S[s + 2], S[s + 3], S[s + 4], S[s + 5], S[s + 6], S[s + 7],
                    N[8 * i + 0], N[8 * i + 1], N[8 * i + 2], N[8 * i + 3], N[8 * i + 4], N[8 * i + 5], N[8 * i + 6], N[8 * i + 7], Bop3());
    }
}

// MixColumns and AddRoundKey: out_r = 2 (a_r + a_{r+1}) + a_{r+1} + (a_{r+2} + a_{r+3}) + key, per column
DASH_HD void sliced_mix_key(const uint32_t* N, uint32_t* S, const uint32_t* km) {
#pragma unroll
    for (int c = 0; c < 4; c++) {
        uint32_t t[4][8];
#pragma unroll
        for (int r = 0; r < 4; r++)
#pragma unroll
            for (int b = 0; b < 8; b++) t[r][b] = N[8 * (4 * c + r) + b] ^ N[8 * (4 * c + ((r + 1) & 3)) + b];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const uint32_t* a1 = N + 8 * (4 * c + ((r + 1) & 3));
            const uint32_t* u = t[(r + 2) & 3];
            const uint32_t* k = km + 8 * (4 * c + r);
            uint32_t* o = S + 8 * (4 * c + r);
            const uint32_t t7 = t[r][7];
            o[0] = xor3(t7, a1[0], u[0]) ^ k[0];
            o[1] = xor3(xor3(t[r][0], a1[1], u[1]), t7, k[1]);
            o[2] = xor3(t[r][1], a1[2], u[2]) ^ k[2];
            o[3] = xor3(xor3(t[r][2], a1[3], u[3]), t7, k[3]);
            o[4] = xor3(xor3(t[r][3], a1[4], u[4]), t7, k[4]);
            o[5] = xor3(t[r][4], a1[5], u[5]) ^ k[5];
            o[6] = xor3(t[r][5], a1[6], u[6]) ^ k[6];
            o[7] = xor3(t[r][6], a1[7], u[7]) ^ k[7];
        }
    }
}

// Key masks of rounds 1..9 for sliced_mix_key: km[(round - 1) * 128 + 8 i + b] = all ones iff bit b of byte i of
// (round key xor 0x63 in every byte) is set.  rk: the 44 round-key words of expand_key.
inline void sliced_key_masks(const uint32_t* rk, uint32_t* km) {
    for (int round = 1; round <= 9; round++)
        for (int i = 0; i < 16; i++)
            for (int b = 0; b < 8; b++) {
                const uint32_t byte = ((rk[4 * round + i / 4] >> (8 * (i % 4))) & 0xffu) ^ 0x63u;
                km[(round - 1) * 128 + 8 * i + b] = ((byte >> b) & 1u) ? 0xffffffffu : 0u;
            }
}

// 32 blocks: on entry and on exit X[32 w + j] is word w (little endian, as in aes128_encrypt) of block j.
DASH_HD void aes128_encrypt_sliced(uint32_t* X, const uint32_t* rk, const uint32_t* km) {
#pragma unroll
    for (int w = 0; w < 4; w++) {
#pragma unroll
        for (int j = 0; j < 32; j++) X[32 * w + j] ^= rk[w];
        transpose32(X + 32 * w);            // now X[32 w + 8 y + b] = X[8 (4 w + y) + b]: plane b of byte 4 w + y
    }
    uint32_t N[128];
#pragma unroll 1
    for (int round = 0; round < 9; round++) {
        sliced_sub_shift(X, N);
        sliced_mix_key(N, X, km + round * 128);
    }
    sliced_sub_shift(X, N);
#pragma unroll
    for (int w = 0; w < 4; w++) {
        transpose32(N + 32 * w);
#pragma unroll
        for (int j = 0; j < 32; j++) X[32 * w + j] = N[32 * w + j] ^ rk[40 + w] ^ 0x63636363u;
    }
}

}  // namespace dash
