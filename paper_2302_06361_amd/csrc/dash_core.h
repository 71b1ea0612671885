// dash_core.h -- per-lane arithmetic of the garbling hash: modulus constants, packed-digit
// arithmetic, label compression (Horner, Sec. Implementation), AES-128 on little-endian column
// words with T-tables (FIPS-197; the paper's fixed-key permutation, Sec. Garbled Circuit
// Optimizations) and base-q digit extraction (label decompression, Sec. LabelTensors).
//
// Everything here is a forceinline host+device function with no memory access of its own except
// through the functors it is given, so the same code is exercised by a host self-check.
//
// Every routine is a template over the modulus description: either the runtime ModInfo (any
// modulus 2..255, loops with wave-uniform trip counts) or CMod<m, lam> whose fields are
// compile-time constants, so that the same source unrolls completely and all divisions become
// multiplications by literals.
#pragma once
#include <stdint.h>

#include <type_traits>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define DASH_HD __host__ __device__ __forceinline__
#else
#define DASH_HD inline
#endif

namespace dash {

// Constants of one modulus m (2..255), computed on the host (dash_hostconst.h).
struct ModInfo {
    uint32_t m;       // modulus
    uint32_t lam;     // digits per label
    uint32_t nchunk;  // ceil(lam / 16): 16-digit chunks of a LabelTensor
    uint32_t ndw;     // ceil(lam / 4): dwords of a table row (pitch / 4)
    uint32_t mmagic;  // ceil(2^32 / m): floor(n / m) = mulhi(n, mmagic) for n < 2^24
    uint32_t m4;      // m replicated in 4 bytes
    uint32_t c4;      // (128 - m) replicated (m <= 128), else 0
    uint32_t gc;      // dwords (4 digits each) per 32-bit super-digit of compress: m^(4 gc) < 2^32
    uint32_t Qc;      // m^(4 gc)
    // decompress: m = 2^tw * mo (mo odd).  A super-digit of gd digits is h mod m^gd; dividing by
    // m^gd = 2^(tw gd) * mo^gd is a shift by dsh = tw*gd bits and a long division by Qd = mo^gd <= 2^15.
    uint32_t tw;      // number of factors 2 in m
    uint32_t omagic;  // ceil(2^32 / mo): floor(n / mo) = mulhi(n, omagic) for n < 2^24; 0 when mo = 1
    uint32_t gd;      // digits per super-digit
    uint32_t dsh;     // tw * gd
    uint32_t Qd;      // mo^gd
    uint32_t Qdmagic; // ceil(2^(31+L) / Qd), L = ceil(log2 Qd): floor(n / Qd) = mulhi(n, Qdmagic) >> (L-1), n < 2^31
    uint32_t Qdshift; // L - 1
    uint32_t Qdbits;  // dsh + floor(log2 Qd): every super-digit shortens the dividend by at least this many bits
    const uint32_t* dtab;  // device: [a = 0..m-1][ndw] packed digits of a * R_m mod m
};

// ---- the same constants at compile time ---------------------------------------------------------
namespace cm {
constexpr uint32_t ceil_log2(uint64_t v) { uint32_t l = 0; while ((1ull << l) < v) l++; return l; }
constexpr uint32_t floor_log2(uint64_t v) { uint32_t l = 0; while ((2ull << l) <= v) l++; return l; }
constexpr uint64_t ipow(uint64_t b, uint32_t e) { uint64_t r = 1; for (uint32_t i = 0; i < e; i++) r *= b; return r; }
constexpr uint32_t gc_of(uint32_t m) { uint32_t g = 0; while (g < 8 && ipow(m, 4 * (g + 1)) < (1ull << 32)) g++; return g; }
constexpr uint32_t twos_of(uint32_t m) { uint32_t t = 0; while (!(m & 1)) { m >>= 1; t++; } return t; }
constexpr uint32_t bits_of(uint64_t v) { uint32_t b = 0; while (v) { b++; v >>= 1; } return b; }   // v < 2^bits_of(v)
// largest g with mo^g <= 2^15, the super-digit (mo^g - 1) * 2^(tw g) + ... below 2^32 and, for the digit
// extraction, (m^g >> tw) below 2^24 (powers of two: at most 24 bits per super-digit)
constexpr bool gd_ok(uint32_t m, uint32_t g) {
    const uint32_t tw = twos_of(m);
    const uint64_t mo = m >> tw, qo = ipow(mo, g);
    if (qo > (1ull << 15)) return false;
    if (tw * g + ceil_log2(qo) > 32) return false;
    if (mo == 1 && tw * g > 24) return false;
    return (ipow(m, g) >> tw) < (1ull << 24);
}
constexpr uint32_t gd_of(uint32_t m) { uint32_t g = 1; while (gd_ok(m, g + 1)) g++; return g; }
}  // namespace cm

template <uint32_t MOD, uint32_t LAM>
struct CMod {
    static constexpr uint32_t m = MOD, lam = LAM, nchunk = (LAM + 15) / 16, ndw = (LAM + 3) / 4;
    static constexpr uint32_t mmagic = (uint32_t)(((1ull << 32) + MOD - 1) / MOD);
    static constexpr uint32_t m4 = MOD * 0x01010101u, c4 = MOD <= 128 ? (128 - MOD) * 0x01010101u : 0;
    static constexpr uint32_t gc = cm::gc_of(MOD), Qc = (uint32_t)cm::ipow(MOD, 4 * gc);
    static constexpr uint32_t tw = cm::twos_of(MOD), mo = MOD >> tw;
    static constexpr uint32_t omagic = (uint32_t)(((1ull << 32) + mo - 1) / mo);
    static constexpr uint32_t gd = cm::gd_of(MOD), dsh = tw * gd, Qd = (uint32_t)cm::ipow(mo, gd);
    static constexpr uint32_t Qdshift = Qd > 1 ? cm::ceil_log2(Qd) - 1 : 0;
    static constexpr uint32_t Qdmagic = Qd > 1 ? (uint32_t)(((1ull << (32 + Qdshift)) + Qd - 1) / Qd) : 0;
    static constexpr uint32_t Qdbits = dsh + cm::floor_log2(Qd);
    const uint32_t* dtab;
};

// the modulus of a compile-time description, 0 for the run-time one
template <class T> struct cmod_m { static constexpr uint32_t value = 0; };
template <uint32_t MOD, uint32_t LAM> struct cmod_m<CMod<MOD, LAM>> { static constexpr uint32_t value = MOD; };
// dwords per label of a compile-time description, 1 for the run-time one (array sizes)
template <class T> struct cmod_ndw { static constexpr uint32_t value = 1; };
template <uint32_t MOD, uint32_t LAM> struct cmod_ndw<CMod<MOD, LAM>> { static constexpr uint32_t value = (LAM + 3) / 4; };

struct U128 { uint32_t w[4]; };

DASH_HD uint32_t mulhi(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }
// 24-bit multiply (both operands below 2^24, product below 2^32).
// Measured issue cost of a wave64 instruction on this chip, in cycles per SIMD: and / or / xor / add / sub / shift right /
// three-input bit operation 2; shift left, byte permute, sub-dword selects, three-operand integer forms, 24-bit and 32-bit
// multiplies (low and high half alike), 64-bit multiply-add, byte dot product 4.
DASH_HD uint32_t mul24(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul24(a, b);
#else
    return a * b;
#endif
}
// sum of byte products a.b0*b.b0 + .. + a.b3*b.b3
DASH_HD uint32_t dot4(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__) && __has_builtin(__builtin_amdgcn_udot4)
    return __builtin_amdgcn_udot4(a, b, 0u, false);
#else
    uint32_t s = 0;
    for (int i = 0; i < 4; i++) s += ((a >> (8 * i)) & 0xff) * ((b >> (8 * i)) & 0xff);
    return s;
#endif
}
// load through a pointer that is known to address device global memory (pointers that were themselves
// loaded from memory would otherwise be dereferenced with flat instructions, which also occupy the LDS queue)
DASH_HD uint32_t gload32(const uint32_t* p) {
#if defined(__HIP_DEVICE_COMPILE__)
    return *(const __attribute__((address_space(1))) uint32_t*)p;
#else
    return *p;
#endif
}
template <class MI> DASH_HD uint32_t div_m(uint32_t n, const MI& M) { return mulhi(n, M.mmagic); }           // n < 2^24
template <class MI> DASH_HD uint32_t mod_m(uint32_t n, const MI& M) { return n - mul24(div_m(n, M), M.m); }  // n < 2^24
DASH_HD uint32_t byte_of(uint32_t w, int b) { return (w >> (8 * b)) & 0xffu; }

// 0xff in every byte of x whose top bit is set, 0x00 elsewhere (shifts and subtractions only: a
// multiplication by 255 costs twice an addition)
DASH_HD uint32_t ge_mask(uint32_t x) {
    uint32_t hi = x & 0x80808080u;
    return (hi - (hi >> 7)) | hi;
}
// Moduli above 128 (the accumulation moduli k d_j of the 12-prime digit set): a sum of two digits does not fit a
// byte, so the digits go through 16-bit fields, two per word; "x >= m ? x - m : x" is min(x, x - m) on unsigned
// 16-bit fields (the difference wraps to a large number when x < m): packed 16-bit subtract and minimum.
DASH_HD uint32_t redmod2x16(uint32_t x, uint32_t m) {      // both fields below 2 m
#if defined(__HIP_DEVICE_COMPILE__)
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const u16x2 v = __builtin_bit_cast(u16x2, x), mm = __builtin_bit_cast(u16x2, m * 0x00010001u);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(v, (u16x2)(v - mm)));
#else
    uint32_t lo = x & 0xffffu, hi = x >> 16;
    lo = lo >= m ? lo - m : lo;
    hi = hi >= m ? hi - m : hi;
    return lo | (hi << 16);
#endif
}
// (a + b) mod m on 4 packed digits, a, b < m per byte.
template <class MI>
DASH_HD uint32_t addmod4(uint32_t a, uint32_t b, const MI& M) {
    if constexpr (cmod_m<MI>::value == 2) return a ^ b;          // digits are bits (one per byte)
    if (M.m <= 128) {
        uint32_t t = a + b;                                       // bytes <= 2m-2 <= 254
        return t - (ge_mask(t + M.c4) & M.m4);
    }
    const uint32_t ev = redmod2x16((a & 0x00ff00ffu) + (b & 0x00ff00ffu), M.m);
    const uint32_t od = redmod2x16(((a >> 8) & 0x00ff00ffu) + ((b >> 8) & 0x00ff00ffu), M.m);
    return ev | (od << 8);
}
// (a - b) mod m on 4 packed digits.
template <class MI>
DASH_HD uint32_t submod4(uint32_t a, uint32_t b, const MI& M) {
    if constexpr (cmod_m<MI>::value == 2) return a ^ b;
    if (M.m <= 128) {
        uint32_t t = a + (M.m4 - b);                              // bytes in [1, 2m-1] <= 255
        return t - (ge_mask(t + M.c4) & M.m4);
    }
    const uint32_t m2 = M.m * 0x00010001u;                        // fields a + m - b in [1, 2m-1]
    const uint32_t ev = redmod2x16((a & 0x00ff00ffu) + (m2 - (b & 0x00ff00ffu)), M.m);
    const uint32_t od = redmod2x16(((a >> 8) & 0x00ff00ffu) + (m2 - ((b >> 8) & 0x00ff00ffu)), M.m);
    return ev | (od << 8);
}
// (a + c * b) mod m on 4 packed digits, c < m.
template <class MI>
DASH_HD uint32_t axpymod4(uint32_t a, uint32_t c, uint32_t b, const MI& M) {
    if constexpr (cmod_m<MI>::value == 2) return a ^ (b & (0u - (c & 1u)));
    uint32_t r = 0;
    for (int b8 = 0; b8 < 4; b8++) r |= mod_m(byte_of(a, b8) + mul24(c, byte_of(b, b8)), M) << (8 * b8);
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

// acc = acc * mul + add (mod 2^128) for an accumulator known to fit W words: W multiplications
template <int W>
DASH_HD void muladd128_w(U128& a, uint32_t mul, uint32_t add) {
    uint64_t t = add;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        if (i < W) { t += (uint64_t)a.w[i] * mul; a.w[i] = (uint32_t)t; t >>= 32; }
        else if (i == W) a.w[i] = (uint32_t)t;
    }
}
// compile-time descriptions: super-digit T (counted from the top) and all below it.  Before it is folded in, the
// accumulator is below Qc^T, so only the words that can be non-zero are multiplied.
template <class MI, int T, class LoadDw>
DASH_HD void compress_from(U128& acc, LoadDw& dw, uint32_t& w0) {
    constexpr int NS = ((int)MI::ndw + (int)MI::gc - 1) / (int)MI::gc;
    if constexpr (T < NS) {
        constexpr int top = (int)MI::ndw - (NS - 1) * (int)MI::gc;        // dwords of the top super-digit (may be short)
        constexpr int cnt = T == 0 ? top : (int)MI::gc;
        constexpr int hi = T == 0 ? (int)MI::ndw - 1 : (int)MI::ndw - 1 - top - (T - 1) * (int)MI::gc;
        constexpr uint32_t wlo = 1u | (MI::m << 8), whi = (1u << 16) | (MI::m << 24), m2 = MI::m * MI::m, m4 = m2 * m2;
        uint32_t S = 0;
#pragma unroll
        for (int c = 0; c < cnt; c++) {
            const uint32_t w = dw(hi - c);
            if (hi - c == 0) w0 = w;
            const uint32_t v = dot4(w, wlo) + mul24(m2, dot4(w, whi));     // < m^4; both factors below 2^17
            S = c == 0 ? v : (MI::Qc < (1u << 24) ? mul24(S, m4) : S * m4) + v;
        }
        constexpr int wbits = T * (int)cm::bits_of((uint64_t)MI::Qc - 1);
        constexpr int W = T == 0 ? 0 : (wbits + 31) / 32 > 4 ? 4 : (wbits + 31) / 32;
        muladd128_w<W>(acc, MI::Qc, S);
        compress_from<MI, T + 1>(acc, dw, w0);
    }
}

// compress(l) = sum_j l[j] m^j mod 2^128 (Horner from the top digit).  dw(i) returns packed digits
// 4i..4i+3 of the label, digits past lam zero.  *colour receives digit 0.
// Four digits at a time: v = d0 + m d1 + m^2 d2 + m^3 d3 by two byte dot products; gc such values
// make one 32-bit super-digit; the 128-bit accumulator is multiplied once per super-digit.  The top
// dword may hold fewer than 4 digits: its missing digits are zero, which Horner ignores.
template <class MI, class LoadDw>
DASH_HD U128 compress(const MI& M, LoadDw dw, uint32_t* colour) {
    U128 acc = {{0, 0, 0, 0}};
    if constexpr (cmod_m<MI>::value == 2) {   // digits are bits: pack them (compile-time description only:
                                                        // with run-time trip counts the word index would be dynamic)
        uint32_t w0 = 0;
#pragma unroll
        for (int i = (int)M.ndw - 1; i >= 0; i--) {
            uint32_t w = dw(i);
            if (i == 0) w0 = w;
            acc.w[i >> 3] |= dot4(w, 0x08040201u) << (4 * (i & 7));
        }
        *colour = w0 & 0xffu;
        return acc;
    }
    if constexpr (cmod_m<MI>::value > 2) {
        uint32_t w0 = 0;
        compress_from<MI, 0>(acc, dw, w0);
        *colour = w0 & 0xffu;
        return acc;
    }
    const uint32_t wlo = 1u | (M.m << 8), whi = (1u << 16) | (M.m << 24), m2 = M.m * M.m, m4 = m2 * m2;
    uint32_t S = 0, w0 = 0;
    uint32_t left = M.ndw % M.gc;        // dwords still to take into the current super-digit;
    if (left == 0) left = M.gc;          // the first (top) group may be short: acc is still 0
#pragma unroll
    for (int i = (int)M.ndw - 1; i >= 0; i--) {
        uint32_t w = dw(i);
        if (i == 0) w0 = w;
        uint32_t v = dot4(w, wlo) + mul24(m2, dot4(w, whi));     // < m^4; both factors below 2^17
        S = (M.Qc < (1u << 24) ? mul24(S, m4) : S * m4) + v;     // S < Qc / m^4
        if (--left == 0) { muladd128(acc, M.Qc, S); S = 0; left = M.gc; }
    }
    *colour = w0 & 0xffu;
    return acc;
}

// ---------------------------------------------------------------------------------------------
// AES-128 encryption.  The state is four little-endian column words: word c holds bytes
// in[4c..4c+3], which are exactly the four 32-bit limbs of the 128-bit block read as a little-endian
// integer.  T[r][x] = column r of MixColumns times S[x]; T[r] = T[0] rotated left by 8r bits.
// rk: 44 round-key words in the same byte order.
// ---------------------------------------------------------------------------------------------
// three-input exclusive or (one v_bitop3_b32 on gfx950)
DASH_HD uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__) && __has_builtin(__builtin_amdgcn_bitop3_b32)
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
#else
    return a ^ b ^ c;
#endif
}

// Tab: the T-tables.  T.template at<R, B>(w) is entry (byte B of w) of table R; the accessor gets the whole
// word so that a table layout can build its address from the byte in place.  A layout with
// Tab::two_tables holds T0 and T1 only: T2 = rot16(T0), T3 = rot16(T1), and one rotation serves both.
template <class Tab, class = void> struct tab_two : std::false_type {};
template <class Tab> struct tab_two<Tab, std::enable_if_t<Tab::two_tables>> : std::true_type {};
DASH_HD uint32_t rot16(uint32_t v) { return (v << 16) | (v >> 16); }

template <class Tab>
DASH_HD void aes128_encrypt(uint32_t s[4], const uint32_t* rk, const Tab& T) {
    uint32_t a0 = s[0] ^ rk[0], a1 = s[1] ^ rk[1], a2 = s[2] ^ rk[2], a3 = s[3] ^ rk[3];
    if constexpr (tab_two<Tab>::value) {
#pragma unroll
        for (int r = 1; r < 10; r++) {
            uint32_t b0 = xor3(T.template at<0, 0>(a0), T.template at<1, 1>(a1), rk[4 * r + 0]) ^ rot16(T.template at<0, 2>(a2) ^ T.template at<1, 3>(a3));
            uint32_t b1 = xor3(T.template at<0, 0>(a1), T.template at<1, 1>(a2), rk[4 * r + 1]) ^ rot16(T.template at<0, 2>(a3) ^ T.template at<1, 3>(a0));
            uint32_t b2 = xor3(T.template at<0, 0>(a2), T.template at<1, 1>(a3), rk[4 * r + 2]) ^ rot16(T.template at<0, 2>(a0) ^ T.template at<1, 3>(a1));
            uint32_t b3 = xor3(T.template at<0, 0>(a3), T.template at<1, 1>(a0), rk[4 * r + 3]) ^ rot16(T.template at<0, 2>(a1) ^ T.template at<1, 3>(a2));
            a0 = b0; a1 = b1; a2 = b2; a3 = b3;
        }
        // last round: S[x] sits in bytes 1 and 2 of T0 and in bytes 2 and 3 of T1
        s[0] = (((T.template at<0, 0>(a0) >> 8) & 0xffu) | (T.template at<0, 1>(a1) & 0xff00u) | (T.template at<0, 2>(a2) & 0xff0000u) | (T.template at<1, 3>(a3) & 0xff000000u)) ^ rk[40];
        s[1] = (((T.template at<0, 0>(a1) >> 8) & 0xffu) | (T.template at<0, 1>(a2) & 0xff00u) | (T.template at<0, 2>(a3) & 0xff0000u) | (T.template at<1, 3>(a0) & 0xff000000u)) ^ rk[41];
        s[2] = (((T.template at<0, 0>(a2) >> 8) & 0xffu) | (T.template at<0, 1>(a3) & 0xff00u) | (T.template at<0, 2>(a0) & 0xff0000u) | (T.template at<1, 3>(a1) & 0xff000000u)) ^ rk[42];
        s[3] = (((T.template at<0, 0>(a3) >> 8) & 0xffu) | (T.template at<0, 1>(a0) & 0xff00u) | (T.template at<0, 2>(a1) & 0xff0000u) | (T.template at<1, 3>(a2) & 0xff000000u)) ^ rk[43];
    } else {
#pragma unroll
    for (int r = 1; r < 10; r++) {
        uint32_t b0 = xor3(xor3(T.template at<0, 0>(a0), T.template at<1, 1>(a1), T.template at<2, 2>(a2)), T.template at<3, 3>(a3), rk[4 * r + 0]);
        uint32_t b1 = xor3(xor3(T.template at<0, 0>(a1), T.template at<1, 1>(a2), T.template at<2, 2>(a3)), T.template at<3, 3>(a0), rk[4 * r + 1]);
        uint32_t b2 = xor3(xor3(T.template at<0, 0>(a2), T.template at<1, 1>(a3), T.template at<2, 2>(a0)), T.template at<3, 3>(a1), rk[4 * r + 2]);
        uint32_t b3 = xor3(xor3(T.template at<0, 0>(a3), T.template at<1, 1>(a0), T.template at<2, 2>(a1)), T.template at<3, 3>(a2), rk[4 * r + 3]);
        a0 = b0; a1 = b1; a2 = b2; a3 = b3;
    }
    // last round: SubBytes + ShiftRows only.  S[x] sits in byte 0 of T2, byte 1 of T3, byte 2 of T0, byte 3 of T1.
    s[0] = ((T.template at<2, 0>(a0) & 0xffu) | (T.template at<3, 1>(a1) & 0xff00u) | (T.template at<0, 2>(a2) & 0xff0000u) | (T.template at<1, 3>(a3) & 0xff000000u)) ^ rk[40];
    s[1] = ((T.template at<2, 0>(a1) & 0xffu) | (T.template at<3, 1>(a2) & 0xff00u) | (T.template at<0, 2>(a3) & 0xff0000u) | (T.template at<1, 3>(a0) & 0xff000000u)) ^ rk[41];
    s[2] = ((T.template at<2, 0>(a2) & 0xffu) | (T.template at<3, 1>(a3) & 0xff00u) | (T.template at<0, 2>(a0) & 0xff0000u) | (T.template at<1, 3>(a1) & 0xff000000u)) ^ rk[42];
    s[3] = ((T.template at<2, 0>(a3) & 0xffu) | (T.template at<3, 1>(a0) & 0xff00u) | (T.template at<0, 2>(a1) & 0xff0000u) | (T.template at<1, 3>(a2) & 0xff000000u)) ^ rk[43];
    }
}

// AES-128 by the FOUR lanes of a quad (lanes 4i .. 4i + 3 of a wave) together: all four call with the same s, all four
// return with the same result.  Lane c keeps column c of the state; a round takes the neighbours' columns with three
// quad permutes and does 4 look-ups instead of 16: a third of the instructions per lane, for kernels whose run time is
// the chain of one lane (few elements).  The four lanes must be active together.  (Host build: each caller encrypts
// on its own.)
template <class Tab>
DASH_HD void aes128_encrypt_quad(uint32_t s[4], const uint32_t* rk, const Tab& T) {
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t c = __lane_id() & 3u;
    auto pick = [&](uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3) { return c == 0 ? k0 : c == 1 ? k1 : c == 2 ? k2 : k3; };
    // value of the lane 1, 2, 3 places up in the quad (cyclic), and of lane i of the quad
    auto up1 = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x39, 0xf, 0xf, true); };    // quad_perm:[1,2,3,0]
    auto up2 = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true); };    // quad_perm:[2,3,0,1]
    auto up3 = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x93, 0xf, 0xf, true); };    // quad_perm:[3,0,1,2]
    uint32_t a = pick(s[0], s[1], s[2], s[3]) ^ pick(rk[0], rk[1], rk[2], rk[3]);
#pragma unroll
    for (int r = 1; r < 10; r++) {
        const uint32_t a1 = up1(a), a2 = up2(a), a3 = up3(a);
        a = xor3(xor3(T.template at<0, 0>(a), T.template at<1, 1>(a1), T.template at<2, 2>(a2)), T.template at<3, 3>(a3),
                 pick(rk[4 * r], rk[4 * r + 1], rk[4 * r + 2], rk[4 * r + 3]));
    }
    {
        const uint32_t a1 = up1(a), a2 = up2(a), a3 = up3(a);
        a = ((T.template at<2, 0>(a) & 0xffu) | (T.template at<3, 1>(a1) & 0xff00u) | (T.template at<0, 2>(a2) & 0xff0000u) |
             (T.template at<1, 3>(a3) & 0xff000000u)) ^ pick(rk[40], rk[41], rk[42], rk[43]);
    }
    s[0] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x00, 0xf, 0xf, true);      // quad_perm:[0,0,0,0]
    s[1] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x55, 0xf, 0xf, true);
    s[2] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0xAA, 0xf, 0xf, true);
    s[3] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0xFF, 0xf, 0xf, true);
#else
    aes128_encrypt(s, rk, T);
#endif
}

// value that lane I (0..3) of the caller's quad holds (all four lanes active)
template <int I> DASH_HD uint32_t quad_lane(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, I * 0x55, 0xf, 0xf, true);      // quad_perm:[I,I,I,I]
#else
    return v;
#endif
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
// the same by the four lanes of a quad together (aes128_encrypt_quad): same arguments and same result in all four
template <class Tab>
DASH_HD U128 hash_block_quad(const U128& K, uint64_t elem, uint32_t slot, uint32_t layer, const uint32_t* rk, const Tab& T) {
    uint32_t x[4] = {K.w[0] ^ (uint32_t)elem, K.w[1] ^ (uint32_t)(elem >> 32), K.w[2] ^ slot, K.w[3] ^ (layer & 0xffffu)};
    uint32_t s[4] = {x[0], x[1], x[2], x[3]};
    aes128_encrypt_quad(s, rk, T);
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
// for i = 0..ndw-1.  With m = 2^tw * mo, a super-digit of gd digits is taken off the 128-bit number by
// a shift (its low dsh bits) and a long division by Qd = mo^gd <= 2^15 over 16-bit half-words (every
// partial dividend r * 2^16 + half is below 2^31, where the magic division is exact):
//     h mod m^gd = ((h >> dsh) mod Qd) << dsh | (h & (2^dsh - 1)),   h div m^gd = (h >> dsh) div Qd.
// After each super-digit the number is shorter by Qdbits bits; half-words known to be zero are skipped.
// ---------------------------------------------------------------------------------------------
template <class MI>
DASH_HD uint32_t take_superdigit(U128& x, const MI& M, uint32_t bits) {
    uint32_t low = 0;
    if (M.dsh) {
        low = x.w[0] & ((1u << M.dsh) - 1u);
#pragma unroll
        for (int i = 0; i < 3; i++) x.w[i] = (x.w[i] >> M.dsh) | (x.w[i + 1] << (32 - M.dsh));
        x.w[3] >>= M.dsh;
        bits = bits > M.dsh ? bits - M.dsh : 0;
    }
    if (M.Qd == 1) return low;                       // power of two: nothing left to divide
    const uint32_t nh = (bits + 15) / 16;            // significant half-words
    uint32_t r = 0;
#pragma unroll
    for (int i = 3; i >= 0; i--) {
        if ((uint32_t)(2 * i) >= nh) continue;
        uint32_t w = x.w[i], q1 = 0;
        if ((uint32_t)(2 * i + 1) < nh) {
            uint32_t cur = (r << 16) | (w >> 16);
            q1 = mulhi(cur, M.Qdmagic) >> M.Qdshift;
            r = cur - mul24(q1, M.Qd);
        }
        uint32_t cur = (r << 16) | (w & 0xffffu);
        uint32_t q0 = mulhi(cur, M.Qdmagic) >> M.Qdshift;
        r = cur - mul24(q0, M.Qd);
        x.w[i] = (q1 << 16) | q0;
    }
    return (r << M.dsh) | low;
}

// Compile-time descriptions: the gd digits of a super-digit S < m^G are split by halving, S = hi * m^G1 + lo,
// so that all but the first division work on numbers below 2^15, where floor(n / D) = (n * M) >> s with a
// 24-bit multiplication (M = ceil(2^s / D), s = bits(n) + ceil(log2 D): n * (M D - 2^s) < 2^s, so the result is
// exact, and n * M < 2^32).  The halving also shortens the chain of dependent divisions from G to log2 G.
template <class MI, int G>
DASH_HD void split_digits(uint32_t S, uint32_t* d) {
    if constexpr (G == 1) {
        d[0] = S;
    } else {
        constexpr int G1 = G / 2, G2 = G - G1;
        constexpr uint64_t mG = cm::ipow(MI::m, G), mG1 = cm::ipow(MI::m, G1), D = cm::ipow(MI::mo, G1);
        constexpr uint32_t sh = MI::tw * G1;
        constexpr uint64_t nmax = (mG - 1) >> sh;                 // S >> sh <= nmax
        constexpr uint32_t a = cm::bits_of(nmax);
        const uint32_t n = S >> sh;                               // floor(S / m^G1) = floor(n / D)
        uint32_t hi;
        if constexpr (D == 1) {
            hi = n;
        } else if constexpr (a <= 15) {
            constexpr uint32_t sft = a + cm::ceil_log2(D);
            constexpr uint32_t Mg = (uint32_t)(((1ull << sft) + D - 1) / D);
            static_assert(nmax * Mg < (1ull << 32) && Mg < (1u << 24), "24-bit magic division out of range");
            hi = mul24(n, Mg) >> sft;
        } else {
            static_assert(a + cm::ceil_log2(D) <= 32 && D < (1ull << 32), "multiply-high division out of range");
            hi = mulhi(n, (uint32_t)(((1ull << 32) + D - 1) / D));
        }
        static_assert(mG1 < (1ull << 24) && (mG - 1) / mG1 < (1ull << 24), "24-bit multiply out of range");
        const uint32_t lo = S - mul24(hi, (uint32_t)mG1);
        split_digits<MI, G1>(lo, d);
        split_digits<MI, G2>(hi, d + G1);
    }
}
// super-digit SD and all after it (compile-time descriptions under the ceil rule: m^lam >= 2^128, so the last
// super-digit holds exactly the digits that are left)
template <class MI, int SD, class Emit>
DASH_HD void decompress_from(const MI& M, U128& x, uint32_t& w, Emit& emit) {
    constexpr int first = SD * (int)MI::gd;
    if constexpr (first < (int)MI::lam) {
        constexpr int G = (int)MI::lam - first < (int)MI::gd ? (int)MI::lam - first : (int)MI::gd;
        constexpr uint32_t bits = 128u > SD * MI::Qdbits ? 128u - SD * MI::Qdbits : 0u;
        const uint32_t S = take_superdigit(x, M, bits);
        uint32_t d[G];
        split_digits<MI, G>(S, d);
#pragma unroll
        for (int t = 0; t < G; t++) {
            const int j = first + t;
            w |= d[t] << (8 * (j & 3));
            if ((j & 3) == 3) { emit(j >> 2, w); w = 0; }
        }
        decompress_from<MI, SD + 1>(M, x, w, emit);
    }
}

template <class MI, class Emit>
DASH_HD void decompress(const MI& M, const U128& h, Emit emit) {
    if constexpr (cmod_m<MI>::value > 2) {
        U128 x = h;
        uint32_t w = 0;
        decompress_from<MI, 0>(M, x, w, emit);
        if (MI::lam & 3) emit((int)(MI::lam >> 2), w);
        return;
    }
    if constexpr (cmod_m<MI>::value == 2) {   // digits are bits: spread 4 bits into 4 bytes
#pragma unroll
        for (int i = 0; i < (int)M.ndw; i++) {
            uint32_t nib = (h.w[i >> 3] >> (4 * (i & 7))) & 0xfu;
            emit(i, mul24(nib, 0x00204081u) & 0x01010101u);
        }
        return;
    }
    U128 x = h;
    uint32_t S = 0, have = 0;     // digits left in the current super-digit
    uint32_t bits = 128;          // the number is below 2^bits
    uint32_t w = 0;
#pragma unroll
    for (uint32_t j = 0; j < M.lam; j++) {
        if (have == 0) {
            S = take_superdigit(x, M, bits);
            bits = bits > M.Qdbits ? bits - M.Qdbits : 0;
            have = M.gd;
        }
        uint32_t q = M.omagic ? mulhi(S >> M.tw, M.omagic) : (S >> M.tw);   // S div m = (S >> tw) div mo; omagic = 0: mo = 1
        uint32_t d = S - mul24(q, M.m);
        S = q; have--;
        w |= d << (8 * (j & 3));
        if ((j & 3) == 3) { emit((int)(j >> 2), w); w = 0; }
    }
    if (M.lam & 3) emit((int)(M.lam >> 2), w);
}

struct Limbs { uint32_t l[8]; };
DASH_HD Limbs to_limbs(const U128& h) {
    Limbs x;
#pragma unroll
    for (int i = 0; i < 4; i++) { x.l[2 * i] = h.w[i] & 0xffffu; x.l[2 * i + 1] = h.w[i] >> 16; }
    return x;
}

// digit 0 alone: h mod m
template <class MI>
DASH_HD uint32_t mod_u128(const U128& h, const MI& M) {
    Limbs x = to_limbs(h);
    uint32_t r = 0;
#pragma unroll
    for (int i = 7; i >= 0; i--) r = mod_m((r << 16) | x.l[i], M);    // r < 256, (r<<16)|limb < 2^24
    return r;
}

// The moduli with a compile-time description: the CRT primes up to 37 and the accumulation moduli of
// the default digit sets, with their label lengths under the ceil rule.
#define DASH_HOT_MODS(X) \
    X(2, 128) X(3, 81) X(5, 56) X(7, 46) X(11, 38) X(13, 35) X(17, 32) X(19, 31) X(23, 29) X(29, 27) X(31, 26) X(37, 25) \
    X(26, 28) X(96, 20) X(46, 24) X(204, 17) X(10, 39) X(91, 20) X(22, 29) X(90, 20)

// f(description of M): compile-time description for the hot moduli, run-time otherwise
template <class F>
DASH_HD void with_mod(const ModInfo& M, F&& f) {
#define DASH_MOD_CASE(MOD, LAM) case MOD: if (M.lam == LAM) { f(CMod<MOD, LAM>{M.dtab}); return; } break;
    switch (M.m) {
        DASH_HOT_MODS(DASH_MOD_CASE)
        default: break;
    }
#undef DASH_MOD_CASE
    f(M);
}

// description of type QD (ModInfo itself, or a CMod) built from the run-time record
template <class QD> struct make_mod { static DASH_HD QD from(const ModInfo& M) { return QD{M.dtab}; } };
template <> struct make_mod<ModInfo> { static DASH_HD ModInfo from(const ModInfo& M) { return M; } };

// index of the compile-time description that fits M (1..), 0 if none
DASH_HD int hot_mod_index(const ModInfo& M) {
    int idx = 0;
#define DASH_MOD_IDX(MOD, LAM) idx++; if (M.m == MOD && M.lam == LAM) return idx;
    DASH_HOT_MODS(DASH_MOD_IDX)
#undef DASH_MOD_IDX
    return 0;
}

// Digit sets (d_1; d, .., d) of the sign gadget whose kernels exist with compile-time moduli, as (m_c, lambda, m_1, lambda):
// m_1 = d_1 the accumulation modulus of digit 1, m_c = k d that of the others.  The default sets of the 8-, 12-, 7- and
// 9-prime bases (the bases of the paper's models), under the ceil rule.
#define DASH_DIGIT_SETS(X) X(96, 20, 26, 28) X(204, 17, 46, 24) X(91, 20, 10, 39) X(90, 20, 22, 29)
template <class MC_, class M1_> struct DigitSet { typedef MC_ MC; typedef M1_ M1; };
// index (1..) of the set with these two moduli, 0 if none
DASH_HD int digit_set_index(const ModInfo& Mc, const ModInfo& M1) {
    int idx = 0;
#define DASH_SET_IDX(MC, LC, M1_, L1) idx++; if (Mc.m == MC && Mc.lam == LC && M1.m == M1_ && M1.lam == L1) return idx;
    DASH_DIGIT_SETS(DASH_SET_IDX)
#undef DASH_SET_IDX
    return 0;
}
// f(DigitSet of compile-time descriptions) for index 1.., f(DigitSet<ModInfo, ModInfo>) for 0
template <class F>
void with_digit_set(int index, F&& f) {
    int idx = 0;
#define DASH_SET_CASE(MC, LC, M1_, L1) if (++idx == index) { f(DigitSet<CMod<MC, LC>, CMod<M1_, L1>>{}); return; }
    DASH_DIGIT_SETS(DASH_SET_CASE)
#undef DASH_SET_CASE
    f(DigitSet<ModInfo, ModInfo>{});
}

}  // namespace dash
