// Host build of the kernels' per-lane arithmetic (dash_core.h + dash_hostconst.h) so that the CPU test
// suite can compare it with the oracle before anything runs on a GPU.  Test code, not part of libdash.
#include <stdint.h>
#include <string.h>

#include "../paper_2302_06361_amd/csrc/dash_hostconst.h"

using namespace dash;
using namespace dash::hostconst;

namespace {
uint32_t TT[1024];
bool ready = false;
uint8_t SB[256];
struct HostTab {
    template <int R, int B> uint32_t at(uint32_t w) const { return TT[R * 256 + ((w >> (8 * B)) & 0xffu)]; }
};
struct HostTab2 {      // T0 and T1 only
    static constexpr bool two_tables = true;
    template <int R, int B> uint32_t at(uint32_t w) const { static_assert(R < 2, "two tables"); return TT[R * 256 + ((w >> (8 * B)) & 0xffu)]; }
};
void init() { if (!ready) { make_sbox(SB); make_ttab(SB, TT); ready = true; } }
uint32_t pack_dw(const uint8_t* lab, uint32_t lam, int i) {
    uint32_t w = 0;
    for (int b = 0; b < 4; b++) if ((uint32_t)(4 * i + b) < lam) w |= (uint32_t)lab[4 * i + b] << (8 * b);
    return w;
}
}  // namespace

extern "C" {
// AES-128 of one block with the four-table and with the two-table formulation
void cc_aes_both(const uint8_t key[16], const uint8_t in[16], uint8_t out4[16], uint8_t out2[16]) {
    init();
    uint32_t rk[44];
    expand_key(key, SB, rk);
    uint32_t s[4], t[4];
    memcpy(s, in, 16); memcpy(t, in, 16);
    aes128_encrypt(s, rk, HostTab{});
    aes128_encrypt(t, rk, HostTab2{});
    memcpy(out4, s, 16); memcpy(out2, t, 16);
}
int cc_lambda(int m, int rule) { return label_length(m, rule); }

// H_q(label, tweak) with the fixed key 00..0f
void cc_hash(const uint8_t* label, int p, int q, int rule, uint64_t elem, uint32_t slot, uint32_t layer, uint8_t* out, uint32_t* colour) {
    init();
    ModInfo Mp, Mq;
    fill_modinfo(Mp, p, rule);
    fill_modinfo(Mq, q, rule);
    uint8_t key[16];
    for (int i = 0; i < 16; i++) key[i] = (uint8_t)i;
    uint32_t rk[44];
    expand_key(key, SB, rk);
    U128 K = compress(Mp, [&](int i) { return pack_dw(label, Mp.lam, i); }, colour);
    U128 h = hash_block(K, elem, slot, layer, rk, HostTab());
    memset(out, 0, Mq.ndw * 4);
    decompress(Mq, h, [&](int i, uint32_t w) { memcpy(out + 4 * i, &w, 4); });
}
// the same through the compile-time modulus descriptions where one exists
void cc_hash_spec(const uint8_t* label, int p, int q, int rule, uint64_t elem, uint32_t slot, uint32_t layer, uint8_t* out, uint32_t* colour) {
    init();
    ModInfo Mp, Mq;
    fill_modinfo(Mp, p, rule);
    fill_modinfo(Mq, q, rule);
    uint8_t key[16];
    for (int i = 0; i < 16; i++) key[i] = (uint8_t)i;
    uint32_t rk[44];
    expand_key(key, SB, rk);
    U128 K;
    with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return pack_dw(label, P.lam, i); }, colour); });
    U128 h = hash_block(K, elem, slot, layer, rk, HostTab());
    memset(out, 0, Mq.ndw * 4);
    with_mod(Mq, [&](auto Q) { decompress(Q, h, [&](int i, uint32_t w) { memcpy(out + 4 * i, &w, 4); }); });
}
void cc_draw(const uint8_t seed[16], int domain, uint32_t layer, uint32_t slot, uint64_t elem, int m, int rule, uint8_t* out, uint32_t* digit0) {
    init();
    ModInfo M;
    fill_modinfo(M, m, rule);
    uint32_t rk[44];
    expand_key(seed, SB, rk);
    U128 h = prg_block(elem, slot, layer, domain, m, rk, HostTab());
    memset(out, 0, M.ndw * 4);
    decompress(M, h, [&](int i, uint32_t w) { memcpy(out + 4 * i, &w, 4); });
    *digit0 = mod_u128(h, M);
}
// packed-digit arithmetic on one dword
uint32_t cc_addmod4(uint32_t a, uint32_t b, int m) { ModInfo M; fill_modinfo(M, m, 0); return addmod4(a, b, M); }
uint32_t cc_submod4(uint32_t a, uint32_t b, int m) { ModInfo M; fill_modinfo(M, m, 0); return submod4(a, b, M); }
uint32_t cc_axpymod4(uint32_t a, uint32_t c, uint32_t b, int m) { ModInfo M; fill_modinfo(M, m, 0); return axpymod4(a, c, b, M); }
uint32_t cc_mod_m(uint32_t n, int m) { ModInfo M; fill_modinfo(M, m, 0); return mod_m(n, M); }
}
