// dash_hostconst.h -- host-side constant generation: AES S-box / T-tables / key schedule from FIPS-197,
// label lengths (Sec. LabelTensors) and the per-modulus division constants used by the kernels.
#pragma once
#include <stdint.h>
#include <string.h>

#include "dash_core.h"

namespace dash {
namespace hostconst {

typedef unsigned __int128 u128;

// FIPS-197: GF(2^8) arithmetic, S-box = affine map of the multiplicative inverse
inline uint8_t gmul(uint8_t a, uint8_t b) {
    uint8_t r = 0;
    for (int i = 0; i < 8; i++) {
        if (b & 1) r ^= a;
        bool hi = a & 0x80;
        a <<= 1;
        if (hi) a ^= 0x1b;
        b >>= 1;
    }
    return r;
}
inline void make_sbox(uint8_t S[256]) {
    // inverse via x^254
    for (int x = 0; x < 256; x++) {
        uint8_t inv = 0;
        if (x) {
            uint8_t y = (uint8_t)x, acc = 1;
            for (int e = 254; e; e >>= 1) { if (e & 1) acc = gmul(acc, y); y = gmul(y, y); }
            inv = acc;
        }
        uint8_t s = inv;
        for (int i = 1; i <= 4; i++) s ^= (uint8_t)((inv << i) | (inv >> (8 - i)));
        S[x] = s ^ 0x63;
    }
}
// T[r][x]: little-endian word whose byte j is MixColumns[j][r] * S[x]
inline void make_ttab(const uint8_t S[256], uint32_t T[1024]) {
    for (int x = 0; x < 256; x++) {
        uint32_t s = S[x], s2 = gmul(S[x], 2), s3 = gmul(S[x], 3);
        uint32_t t0 = s2 | (s << 8) | (s << 16) | (s3 << 24);
        for (int r = 0; r < 4; r++) T[r * 256 + x] = r ? ((t0 << (8 * r)) | (t0 >> (32 - 8 * r))) : t0;
    }
}
// FIPS-197 key expansion into little-endian words (word w = bytes 4w..4w+3 of the key schedule)
inline void expand_key(const uint8_t key[16], const uint8_t S[256], uint32_t out_rk[44]) {
    uint8_t rk[176];
    memcpy(rk, key, 16);
    uint8_t rcon = 1;
    for (int w = 4; w < 44; w++) {
        uint8_t t[4] = {rk[4 * w - 4], rk[4 * w - 3], rk[4 * w - 2], rk[4 * w - 1]};
        if (w % 4 == 0) {
            uint8_t t0 = t[0];
            t[0] = S[t[1]] ^ rcon; t[1] = S[t[2]]; t[2] = S[t[3]]; t[3] = S[t0];
            rcon = gmul(rcon, 2);
        }
        for (int b = 0; b < 4; b++) rk[4 * w + b] = rk[4 * (w - 4) + b] ^ t[b];
    }
    for (int w = 0; w < 44; w++)
        out_rk[w] = rk[4 * w] | (rk[4 * w + 1] << 8) | (rk[4 * w + 2] << 16) | ((uint32_t)rk[4 * w + 3] << 24);
}

// label length: integer powers against 2^128
inline int label_length(int m, int rule) {
    u128 limit = (~(u128)0) / (u128)m, v = 1;
    int lam = 0;
    while (v <= limit) { v *= (u128)m; lam++; }      // m^lam < 2^128 <= m^(lam+1)
    bool exact = (m == 2 || m == 4 || m == 16);       // m^(lam+1) == 2^128
    return (exact || rule == 0 /* ceil */) ? lam + 1 : lam;
}

inline uint32_t ceil_log2(uint32_t v) { uint32_t l = 0; while ((1ull << l) < v) l++; return l; }

inline void fill_modinfo(ModInfo& M, int m, int rule) {
    memset(&M, 0, sizeof(M));
    M.m = m;
    M.lam = label_length(m, rule);
    M.nchunk = (M.lam + 15) / 16;
    M.ndw = (M.lam + 3) / 4;
    M.mmagic = (uint32_t)(((1ull << 32) + m - 1) / m);
    M.m4 = (uint32_t)m * 0x01010101u;
    M.c4 = m <= 128 ? (uint32_t)(128 - m) * 0x01010101u : 0;
    // the compile-time descriptions (CMod) use the same formulas
    M.gc = cm::gc_of(m); M.Qc = (uint32_t)cm::ipow(m, 4 * M.gc);
    M.tw = cm::twos_of(m);
    const uint32_t mo = (uint32_t)m >> M.tw;
    M.omagic = (uint32_t)(((1ull << 32) + mo - 1) / mo);
    M.gd = cm::gd_of(m); M.dsh = M.tw * M.gd; M.Qd = (uint32_t)cm::ipow(mo, M.gd);
    if (M.Qd > 1) {
        uint32_t L = ceil_log2(M.Qd);
        M.Qdmagic = (uint32_t)((((u128)1 << (31 + L)) + M.Qd - 1) / M.Qd);
        M.Qdshift = L - 1;
    }
    M.Qdbits = M.dsh + cm::floor_log2(M.Qd);
}

}  // namespace hostconst
}  // namespace dash
