// dash_core.h -- per-lane arithmetic of the garbling hash: modulus constants, packed-digit
// arithmetic, label compression (Horner, Sec. Implementation), AES-128 on little-endian column
// words with T-tables (FIPS-197; the paper's fixed-key permutation, Sec. Garbled Circuit
// Optimizations) and base-q digit extraction (label decompression, Sec. LabelTensors).
//
// Everything here is a forceinline host+device function with no memory access of its own except
// through the functors it is given, so the same code is exercised by a host self-check.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define DASH_HD __host__ __device__ __forceinline__
#else
#define DASH_HD inline
#endif

namespace dash {

// Constants of one modulus m (2..255), computed on the host (dash_ctx.hip).
struct ModInfo {
    uint32_t m;       // modulus
    uint32_t lam;     // digits per label
    uint32_t nchunk;  // ceil(lam / 16): 16-digit chunks of a LabelTensor
    uint32_t ndw;     // ceil(lam / 4): dwords of a table row (pitch / 4)
    uint32_t mmagic;  // ceil(2^32 / m): floor(n / m) = mulhi(n, mmagic) for n < 2^24
    uint32_t m4;      // m replicated in 4 bytes
    uint32_t c4;      // (128 - m) replicated (m <= 128), else 0
    uint32_t gc;      // digits per 32-bit super-digit of compress: m^(gc-1) <= 2^24, m^gc < 2^32
    uint32_t Qc;      // m^gc
    uint32_t gd;      // digits per super-digit of decompress: m^gd <= 2^15
    uint32_t Qd;      // m^gd
    uint32_t Qdmagic; // ceil(2^(31+L) / Qd), L = ceil(log2 Qd): floor(n / Qd) = mulhi(n, Qdmagic) >> (L-1), n < 2^31
    uint32_t Qdshift; // L - 1
    uint32_t pad_;
    const uint32_t* dtab;  // device: [a = 0..m-1][ndw] packed digits of a * R_m mod m
};

struct U128 { uint32_t w[4]; };

DASH_HD uint32_t mulhi(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }
DASH_HD uint32_t div_m(uint32_t n, const ModInfo& M) { return mulhi(n, M.mmagic); }          // n < 2^24
DASH_HD uint32_t mod_m(uint32_t n, const ModInfo& M) { return n - div_m(n, M) * M.m; }       // n < 2^24
DASH_HD uint32_t byte_of(uint32_t w, int b) { return (w >> (8 * b)) & 0xffu; }

// (a + b) mod m on 4 packed digits, a, b < m per byte.
DASH_HD uint32_t addmod4(uint32_t a, uint32_t b, const ModInfo& M) {
    if (M.m <= 128) {
        uint32_t t = a + b;                                       // bytes <= 2m-2 <= 254
        uint32_t ge = ((t + M.c4) & 0x80808080u) >> 7;            // 1 where byte >= m
        return t - (((ge << 8) - ge) & M.m4);
    }
    uint32_t r = 0;
    for (int b8 = 0; b8 < 4; b8++) {
        uint32_t t = byte_of(a, b8) + byte_of(b, b8);
        t = t >= M.m ? t - M.m : t;
        r |= t << (8 * b8);
    }
    return r;
}
// (a - b) mod m on 4 packed digits.
DASH_HD uint32_t submod4(uint32_t a, uint32_t b, const ModInfo& M) {
    if (M.m <= 128) {
        uint32_t t = a + (M.m4 - b);                              // bytes in [1, 2m-1] <= 255
        uint32_t ge = ((t + M.c4) & 0x80808080u) >> 7;
        return t - (((ge << 8) - ge) & M.m4);
    }
    uint32_t r = 0;
    for (int b8 = 0; b8 < 4; b8++) {
        uint32_t t = byte_of(a, b8) + M.m - byte_of(b, b8);
        t = t >= M.m ? t - M.m : t;
        r |= t << (8 * b8);
    }
    return r;
}
// (a + c * b) mod m on 4 packed digits, c < m.
DASH_HD uint32_t axpymod4(uint32_t a, uint32_t c, uint32_t b, const ModInfo& M) {
    uint32_t r = 0;
    for (int b8 = 0; b8 < 4; b8++) r |= mod_m(byte_of(a, b8) + c * byte_of(b, b8), M) << (8 * b8);
    return r;
}

// acc = acc * mul + add  (mod 2^128)
DASH_HD void muladd128(U128& a, uint32_t mul, uint32_t add) {
    uint64_t t = (uint64_t)a.w[0] * mul + add;
    a.w[0] = (uint32_t)t; t >>= 32;
    t += (uint64_t)a.w[1] * mul; a.w[1] = (uint32_t)t; t >>= 32;
    t += (uint64_t)a.w[2] * mul; a.w[2] = (uint32_t)t; t >>= 32;
    t += (uint64_t)a.w[3] * mul; a.w[3] = (uint32_t)t;
}

// compress(l) = sum_j l[j] m^j mod 2^128 (Horner from the top digit).  dw(i) returns packed digits
// 4i..4i+3 of the label (digits >= lam ignored).  *colour receives digit 0.
template <class LoadDw>
DASH_HD U128 compress(const ModInfo& M, LoadDw dw, uint32_t* colour) {
    U128 acc = {{0, 0, 0, 0}};
    uint32_t S = 0;
    uint32_t left = M.lam % M.gc;           // digits still to take into the current super-digit;
    if (left == 0) left = M.gc;             // the first (top) group may be short: acc is still 0
    uint32_t d = 0;
    for (int i = (int)M.ndw - 1; i >= 0; i--) {
        uint32_t w = dw(i);
        for (int b = 3; b >= 0; b--) {
            if ((uint32_t)(4 * i + b) >= M.lam) continue;
            d = byte_of(w, b);
            S = S * M.m + d;
            if (--left == 0) { muladd128(acc, M.Qc, S); S = 0; left = M.gc; }
        }
    }
    *colour = d;
    return acc;
}

// ---------------------------------------------------------------------------------------------
// AES-128 encryption.  The state is four little-endian column words: word c holds bytes
// in[4c..4c+3], which are exactly the four 32-bit limbs of the 128-bit block read as a little-endian
// integer.  T[r][x] = column r of MixColumns times S[x]; T[r] = T[0] rotated left by 8r bits.
// rk: 44 round-key words in the same byte order.
// ---------------------------------------------------------------------------------------------
template <class Tab>
DASH_HD void aes128_encrypt(uint32_t s[4], const uint32_t* rk, const Tab& T) {
    uint32_t a0 = s[0] ^ rk[0], a1 = s[1] ^ rk[1], a2 = s[2] ^ rk[2], a3 = s[3] ^ rk[3];
    for (int r = 1; r < 10; r++) {
        uint32_t b0 = T(0, a0 & 0xff) ^ T(1, (a1 >> 8) & 0xff) ^ T(2, (a2 >> 16) & 0xff) ^ T(3, a3 >> 24) ^ rk[4 * r + 0];
        uint32_t b1 = T(0, a1 & 0xff) ^ T(1, (a2 >> 8) & 0xff) ^ T(2, (a3 >> 16) & 0xff) ^ T(3, a0 >> 24) ^ rk[4 * r + 1];
        uint32_t b2 = T(0, a2 & 0xff) ^ T(1, (a3 >> 8) & 0xff) ^ T(2, (a0 >> 16) & 0xff) ^ T(3, a1 >> 24) ^ rk[4 * r + 2];
        uint32_t b3 = T(0, a3 & 0xff) ^ T(1, (a0 >> 8) & 0xff) ^ T(2, (a1 >> 16) & 0xff) ^ T(3, a2 >> 24) ^ rk[4 * r + 3];
        a0 = b0; a1 = b1; a2 = b2; a3 = b3;
    }
    // last round: SubBytes + ShiftRows only.  S[x] sits in byte 0 of T2, byte 1 of T3, byte 2 of T0, byte 3 of T1.
    s[0] = ((T(2, a0 & 0xff) & 0xffu) | (T(3, (a1 >> 8) & 0xff) & 0xff00u) | (T(0, (a2 >> 16) & 0xff) & 0xff0000u) | (T(1, a3 >> 24) & 0xff000000u)) ^ rk[40];
    s[1] = ((T(2, a1 & 0xff) & 0xffu) | (T(3, (a2 >> 8) & 0xff) & 0xff00u) | (T(0, (a3 >> 16) & 0xff) & 0xff0000u) | (T(1, a0 >> 24) & 0xff000000u)) ^ rk[41];
    s[2] = ((T(2, a2 & 0xff) & 0xffu) | (T(3, (a3 >> 8) & 0xff) & 0xff00u) | (T(0, (a0 >> 16) & 0xff) & 0xff0000u) | (T(1, a1 >> 24) & 0xff000000u)) ^ rk[42];
    s[3] = ((T(2, a3 & 0xff) & 0xffu) | (T(3, (a0 >> 8) & 0xff) & 0xff00u) | (T(0, (a1 >> 16) & 0xff) & 0xff0000u) | (T(1, a2 >> 24) & 0xff000000u)) ^ rk[43];
}

// h = AES(X) xor X with X = K xor tweak; tweak = elem:u64 | slot:u32 | layer:u16 | 0:u16.
template <class Tab>
DASH_HD U128 hash_block(const U128& K, uint64_t elem, uint32_t slot, uint32_t layer, const uint32_t* rk, const Tab& T) {
    uint32_t x[4] = {K.w[0] ^ (uint32_t)elem, K.w[1] ^ (uint32_t)(elem >> 32), K.w[2] ^ slot, K.w[3] ^ (layer & 0xffffu)};
    uint32_t s[4] = {x[0], x[1], x[2], x[3]};
    aes128_encrypt(s, rk, T);
    U128 h = {{s[0] ^ x[0], s[1] ^ x[1], s[2] ^ x[2], s[3] ^ x[3]}};
    return h;
}
// PRG block: AES_seed(elem:u64 | slot:u32 | layer:u16 | domain:u8 | m:u8), no feed-forward.
template <class Tab>
DASH_HD U128 prg_block(uint64_t elem, uint32_t slot, uint32_t layer, uint32_t domain, uint32_t m, const uint32_t* rk, const Tab& T) {
    uint32_t s[4] = {(uint32_t)elem, (uint32_t)(elem >> 32), slot, (layer & 0xffffu) | (domain << 16) | (m << 24)};
    aes128_encrypt(s, rk, T);
    U128 h = {{s[0], s[1], s[2], s[3]}};
    return h;
}

// ---------------------------------------------------------------------------------------------
// decompress: digits floor(h / m^j) mod m, j = 0..lam-1, delivered as packed dwords emit(i, w)
// for i = 0..ndw-1.  Long division of eight 16-bit limbs by the super-digit base Qd = m^gd <= 2^15
// (every partial dividend r * 2^16 + limb is below 2^31, where the magic division is exact), then
// gd digits out of every remainder.
// ---------------------------------------------------------------------------------------------
struct Limbs { uint32_t l[8]; };

DASH_HD Limbs to_limbs(const U128& h) {
    Limbs x;
    for (int i = 0; i < 4; i++) { x.l[2 * i] = h.w[i] & 0xffffu; x.l[2 * i + 1] = h.w[i] >> 16; }
    return x;
}
// x = floor(x / Qd), returns x mod Qd
DASH_HD uint32_t divrem_Qd(Limbs& x, const ModInfo& M) {
    uint32_t r = 0;
    for (int i = 7; i >= 0; i--) {
        uint32_t cur = (r << 16) | x.l[i];
        uint32_t q = mulhi(cur, M.Qdmagic) >> M.Qdshift;
        r = cur - q * M.Qd;
        x.l[i] = q;
    }
    return r;
}

template <class Emit>
DASH_HD void decompress(const ModInfo& M, const U128& h, Emit emit) {
    Limbs x = to_limbs(h);
    uint32_t S = 0, have = 0;     // digits left in the current super-digit
    uint32_t w = 0;
    for (uint32_t j = 0; j < M.lam; j++) {
        if (have == 0) { S = divrem_Qd(x, M); have = M.gd; }
        uint32_t q = div_m(S, M);
        uint32_t d = S - q * M.m;
        S = q; have--;
        w |= d << (8 * (j & 3));
        if ((j & 3) == 3) { emit((int)(j >> 2), w); w = 0; }
    }
    if (M.lam & 3) emit((int)(M.lam >> 2), w);
}

// digit 0 alone: h mod m
DASH_HD uint32_t mod_u128(const U128& h, const ModInfo& M) {
    Limbs x = to_limbs(h);
    uint32_t r = 0;
    for (int i = 7; i >= 0; i--) r = mod_m((r << 16) | x.l[i], M);    // r < 256, (r<<16)|limb < 2^24
    return r;
}

}  // namespace dash
