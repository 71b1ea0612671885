// Host emulation of the fused carry-chain kernel of the evaluator: runs chain_eval_body /
// chain_eval_generic_body (the code the __global__ kernels call) lane by lane over exactly-sized host
// buffers under the sanitizers.  Test code, not part of libdash.
//
// usage: chain_emul <in.bin> <out.bin>
//   in : int32 n n_elem rule layer variant(0 generic, 1 <96,26>, 2 <204,46>) lam2(0: by the rule) pad pad; uint64 elem_base;
//        int32 m[n] (digit 1..n); int32 slot[n];
//        for j = 1..n: u8 sum_j[n_elem][lam(m_j)];
//        for j = 1..n: u8 table_j[n_elem][m_j][pitch(out modulus of gate j)]   (out modulus: m_{j-1}, or 2 for j = 1)
//   out: u8 bit[n_elem][lambda of modulus 2]
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../paper_2302_06361_amd/csrc/dash_bodies.h"
#include "../paper_2302_06361_amd/csrc/dash_hostconst.h"

using namespace dash;
using namespace dash::hostconst;

static uint32_t TT[1024];
struct HostTab {
    template <int R, int B> uint32_t at(uint32_t w) const { return TT[R * 256 + ((w >> (8 * B)) & 0xffu)]; }
};

static std::vector<uint8_t> to_chunked(const uint8_t* compact, uint32_t n, const ModInfo& M) {
    std::vector<uint8_t> v((size_t)M.nchunk * n * 16, 0);
    for (uint32_t e = 0; e < n; e++)
        for (uint32_t j = 0; j < M.lam; j++) v[((size_t)(j / 16) * n + e) * 16 + j % 16] = compact[(size_t)e * M.lam + j];
    return v;
}

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[8];
    uint64_t elem_base;
    if (fread(hd, 4, 8, f) != 8 || fread(&elem_base, 8, 1, f) != 1) return 2;
    const int n = hd[0], rule = hd[2], layer = hd[3], variant = hd[4];
    const uint32_t E = (uint32_t)hd[1];
    if (n < 2 || n > kMaxChain) return 2;
    std::vector<int32_t> m(n + 1), slot(n + 1);
    if (fread(m.data() + 1, 4, n, f) != (size_t)n || fread(slot.data() + 1, 4, n, f) != (size_t)n) return 2;
    std::vector<ModInfo> mods(256);
    for (int q = 2; q < 256; q++) fill_modinfo(mods[q], q, rule);
    if (hd[5]) { mods[2].lam = (uint32_t)hd[5]; mods[2].nchunk = (mods[2].lam + 15) / 16; mods[2].ndw = (mods[2].lam + 3) / 4; }
    const uint32_t lam2 = mods[2].lam;
    uint8_t S[256];
    make_sbox(S);
    make_ttab(S, TT);

    ChainLaunch L;
    memset(&L, 0, sizeof(L));
    const uint8_t key[16] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15};
    expand_key(key, S, L.key.rk);
    L.mods = mods.data(); L.elem_base = elem_base; L.layer = (uint32_t)layer; L.n_elem = E; L.n = (uint32_t)n;
    std::vector<std::vector<uint8_t>> sum(n + 1), carry(n + 1), table(n + 1);
    for (int j = 1; j <= n; j++) {
        const ModInfo& M = mods[m[j]];
        std::vector<uint8_t> c((size_t)E * M.lam);
        if (fread(c.data(), 1, c.size(), f) != c.size()) return 2;
        sum[j] = to_chunked(c.data(), E, M);
        carry[j].assign((size_t)M.nchunk * E * 16, 0xEE);
    }
    for (int j = 1; j <= n; j++) {
        const ModInfo& Mo = mods[j >= 2 ? m[j - 1] : 2];
        table[j].resize((size_t)E * m[j] * Mo.ndw * 4);
        if (fread(table[j].data(), 1, table[j].size(), f) != table[j].size()) return 2;
    }
    fclose(f);
    std::vector<uint8_t> bit((size_t)mods[2].nchunk * E * 16, 0xEE);
    for (int j = 1; j <= n; j++) {
        L.m[j] = (uint32_t)m[j]; L.slot[j] = (uint32_t)slot[j]; L.table[j] = table[j].data();
        L.sum[j] = LView{sum[j].data(), (int64_t)16 * E, 16u};
        if (j < n) L.carry[j] = LView{carry[j].data(), (int64_t)16 * E, 16u};
    }
    L.bit = LView{bit.data(), (int64_t)16 * E, 16u};
    HostTab T;
    const bool quad = hd[6] != 0;      // four lanes per element (on the host each of them hashes on its own)
    const uint32_t tiles = (E * (quad ? 4 : 1) + kThreads - 1) / kThreads;
    for (uint32_t bx = 0; bx < tiles; bx++)
        for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) {
            with_digit_set(variant, [&](auto ds) {
                typedef decltype(ds) DS;
                if constexpr (cmod_m<typename DS::MC>::value != 0) {
                    if (quad) chain_eval_body<typename DS::MC, typename DS::M1, true>(L, bx, tx, T);
                    else chain_eval_body<typename DS::MC, typename DS::M1>(L, bx, tx, T);
                } else chain_eval_generic_body(L, bx, tx, T);
            });
        }
    std::vector<uint8_t> out((size_t)E * lam2);
    for (uint32_t e = 0; e < E; e++)
        for (uint32_t d = 0; d < lam2; d++) out[(size_t)e * lam2 + d] = bit[((size_t)(d / 16) * E + e) * 16 + d % 16];
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(out.data(), 1, out.size(), f);
    fclose(f);
    return 0;
}
