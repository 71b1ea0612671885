// Host emulation of the fused digit-gate kernels: runs digits_eval_body / digits_garble_body (the code the
// __global__ kernels call) lane by lane over exactly-sized host buffers under the sanitizers.  Test code, not part
// of libdash.
//
// usage: digits_emul <in.bin> <out.bin>
//   in : int32 n n_elem rule layer variant(0 run-time constants, else the index of the digit set's compile-time kernels: 1 <96,26>, 2 <204,46>, 3 <91,10>, 4 <90,22>) nres slot0 mode(0 evaluate, 1 garble, 2 evaluate with a lane per digit gate, 3 garble with a lane per row, 4 evaluate with the sums over the residues formed in the same pass: out = for j: u8 S_j[n_elem][lam(m_j)]); uint64 elem_base;
//        int32 m[n] (digit 1..n); int32 p[nres];
//        for t < nres: u8 label_t[n_elem][lam(p_t)]            (active labels; garble: zero labels)
//      evaluate:
//        for t < nres, j = 1..n: u8 table_tj[n_elem][p_t][pitch(m_j)]
//      garble:
//        for t < nres: u8 delta_t[lam(p_t)];  for j: u8 delta_mj[lam(m_j)];
//        for t < nres, j: u8 out0_tj[n_elem][lam(m_j)];  for t < nres: u8 phi_t[n][p_t]
//   out: evaluate: for t < nres, j = 1..n: u8 out_tj[n_elem][lam(m_j)];  garble: for t, j: table_tj
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

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[8];
    uint64_t elem_base;
    if (fread(hd, 4, 8, f) != 8 || fread(&elem_base, 8, 1, f) != 1) return 2;
    const int n = hd[0], rule = hd[2], layer = hd[3], variant = hd[4], nres = hd[5], slot0 = hd[6], garble = hd[7] == 1 || hd[7] == 3;
    const bool wide_rows = hd[7] == 3;      // garble with one lane per ciphertext row
    const bool wide = hd[7] == 2;      // evaluate with one lane per digit gate
    const bool sums = hd[7] == 4;      // evaluate, the digit gates adding up their outputs (compile-time digit sets)
    const uint32_t E = (uint32_t)hd[1];
    if (n < 1 || n > kMaxChain || nres < 1 || nres > 16) return 2;
    std::vector<int32_t> m(n + 1), p(nres);
    if (fread(m.data() + 1, 4, n, f) != (size_t)n || fread(p.data(), 4, nres, f) != (size_t)nres) return 2;
    std::vector<ModInfo> mods(256);
    for (int q = 2; q < 256; q++) fill_modinfo(mods[q], q, rule);
    uint8_t S[256];
    make_sbox(S);
    make_ttab(S, TT);

    DigitsLaunch L;
    memset(&L, 0, sizeof(L));
    const uint8_t key[16] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15};
    expand_key(key, S, L.key.rk);
    L.mods = mods.data(); L.elem_base = elem_base; L.layer = (uint32_t)layer; L.n_elem = E; L.n = (uint32_t)n; L.nres = (uint32_t)nres;
    L.out_cs = (int64_t)16 * E;
    size_t out_bytes = 0;
    for (int j = 1; j <= n; j++) {
        L.m[j] = (uint32_t)m[j];
        L.row_prefix[j] = j == 1 ? 0 : L.row_prefix[j - 1] + mods[m[j - 1]].ndw * 4;
        L.out_prefix[j] = out_bytes;
        out_bytes += (size_t)mods[m[j]].nchunk * E * 16;
    }
    const uint32_t rows_pitch = L.row_prefix[n] + mods[m[n]].ndw * 4;
    std::vector<std::vector<uint8_t>> act(nres), table(nres), out(nres);
    for (int t = 0; t < nres; t++) {
        const ModInfo& Mp = mods[p[t]];
        std::vector<uint8_t> c((size_t)E * Mp.lam);
        if (fread(c.data(), 1, c.size(), f) != c.size()) return 2;
        act[t].assign((size_t)Mp.nchunk * E * 16, 0);
        for (uint32_t e = 0; e < E; e++)
            for (uint32_t d = 0; d < Mp.lam; d++) act[t][((size_t)(d / 16) * E + e) * 16 + d % 16] = c[(size_t)e * Mp.lam + d];
    }
    std::vector<std::vector<uint32_t>> dtab(256);
    std::vector<std::vector<uint8_t>> phi(nres);
    auto read_dtab = [&](int q) {
        ModInfo& M = mods[q];
        std::vector<uint8_t> delta(M.lam);
        if (fread(delta.data(), 1, delta.size(), f) != delta.size()) exit(2);
        dtab[q].assign((size_t)M.m * M.ndw, 0);
        for (uint32_t a = 0; a < M.m; a++)
            for (uint32_t d = 0; d < M.lam; d++) dtab[q][(size_t)a * M.ndw + d / 4] |= (uint32_t)((a * delta[d]) % M.m) << (8 * (d % 4));
        M.dtab = dtab[q].data();
    };
    if (garble) {
        for (int t = 0; t < nres; t++) read_dtab(p[t]);
        for (int j = 1; j <= n; j++) read_dtab(m[j]);
    }
    for (int t = 0; t < nres; t++) {
        table[t].resize((size_t)E * p[t] * rows_pitch);
        out[t].assign(out_bytes, garble ? 0 : 0xEE);
        if (!garble) {
            if (fread(table[t].data(), 1, table[t].size(), f) != table[t].size()) return 2;
        } else {
            memset(table[t].data(), 0xEE, table[t].size());
            for (int j = 1; j <= n; j++) {
                const ModInfo& M = mods[m[j]];
                std::vector<uint8_t> c((size_t)E * M.lam);
                if (fread(c.data(), 1, c.size(), f) != c.size()) return 2;
                uint8_t* base = out[t].data() + L.out_prefix[j];
                for (uint32_t e = 0; e < E; e++)
                    for (uint32_t d = 0; d < M.lam; d++) base[((size_t)(d / 16) * E + e) * 16 + d % 16] = c[(size_t)e * M.lam + d];
            }
        }
        DigitsRes& R = L.res[t];
        R.p = (uint32_t)p[t]; R.slot0 = (uint32_t)(slot0 + t * n);
        R.in = LView{act[t].data(), (int64_t)16 * E, 16u};
        R.table = table[t].data(); R.out = out[t].data();
    }
    if (garble)
        for (int t = 0; t < nres; t++) {
            phi[t].resize((size_t)n * p[t]);
            if (fread(phi[t].data(), 1, phi[t].size(), f) != phi[t].size()) return 2;
            L.res[t].phi = phi[t].data();
        }
    fclose(f);
    HostTab T;
    if (garble) {
        for (uint32_t by = 0; by < (uint32_t)nres; by++) {
            const uint32_t tiles = (uint32_t)(((uint64_t)E * p[by] + kThreads - 1) / kThreads);
            for (uint32_t bx = 0; bx < tiles; bx++)
                for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++)
                    for (uint32_t j0 = wide_rows ? 1 : 0; j0 <= (wide_rows ? (uint32_t)n : 0u); j0++) {
                        with_digit_set(variant, [&](auto ds) {
                            typedef decltype(ds) DS;
                            digits_garble_body<typename DS::MC, typename DS::M1>(L, bx, by, tx, T, j0);
                        });
                    }
        }
        f = fopen(argv[2], "wb");
        if (!f) return 2;
        for (int t = 0; t < nres; t++) fwrite(table[t].data(), 1, table[t].size(), f);      // [j][e][a][pitch_j] per residue
        fclose(f);
        return 0;
    }
    if (sums) {
        if (variant == 0) return 2;
        size_t sum_bytes = 0;
        for (int j = 1; j <= n; j++) { L.sum_prefix[j] = sum_bytes; sum_bytes += (size_t)mods[m[j]].nchunk * E * 16; }
        std::vector<uint8_t> S(sum_bytes, 0xEE);
        L.sum1 = S.data();
        const uint32_t blocks = (E + kSumElems - 1) / kSumElems;
        for (uint32_t bx = 0; bx < blocks; bx++)
            for (uint32_t j = 0; j <= (uint32_t)n + 1; j++) {       // (digit 0 and n + 1: lanes that must do nothing)
                std::vector<uint32_t> acc((size_t)kSumElems * kSumDw * 2, 0);
                with_digit_set(variant, [&](auto ds) {
                    typedef decltype(ds) DS;
                    if constexpr (cmod_m<typename DS::MC>::value != 0) {
                        for (uint32_t by = 0; by < (uint32_t)nres; by++)
                            for (uint32_t el = 0; el < (uint32_t)kSumElems; el++)
                                digits_sum_phase1<typename DS::MC, typename DS::M1>(NoCast{}, L, bx, by, j, el, T, acc.data());
                        for (uint32_t el = 0; el < (uint32_t)kSumElems; el++) digits_sum_phase2<typename DS::MC, typename DS::M1>(L, bx, j, el, acc.data());
                    }
                });
            }
        f = fopen(argv[2], "wb");
        if (!f) return 2;
        for (int j = 1; j <= n; j++) {
            const ModInfo& M = mods[m[j]];
            std::vector<uint8_t> c((size_t)E * M.lam);
            const uint8_t* base = S.data() + L.sum_prefix[j];
            for (uint32_t e = 0; e < E; e++)
                for (uint32_t d = 0; d < M.nchunk * 16; d++) {
                    const uint8_t v = base[((size_t)(d / 16) * E + e) * 16 + d % 16];
                    if (d < M.lam) c[(size_t)e * M.lam + d] = v;
                    else if (v != 0) return 3;      // digits past lambda must be zero
                }
            fwrite(c.data(), 1, c.size(), f);
        }
        fclose(f);
        return 0;
    }
    const uint32_t tiles = (E + kThreads - 1) / kThreads;
    for (uint32_t by = 0; by < (uint32_t)nres; by++)
        for (uint32_t bx = 0; bx < tiles; bx++)
            for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) {
                if (wide) {      // one lane per digit gate (digit 0 and n + 1: lanes that must do nothing)
                    for (uint32_t j = 0; j <= (uint32_t)n + 1; j++) {
                        with_digit_set(variant, [&](auto ds) {
                            typedef decltype(ds) DS;
                            digits_eval_wide_body<typename DS::MC, typename DS::M1>(L, bx, by, j, tx, T);
                        });
                    }
                    continue;
                }
                with_digit_set(variant, [&](auto ds) {
                    typedef decltype(ds) DS;
                    digits_eval_body<typename DS::MC, typename DS::M1>(L, bx, by, tx, T);
                });
            }
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    for (int t = 0; t < nres; t++)
        for (int j = 1; j <= n; j++) {
            const ModInfo& M = mods[m[j]];
            std::vector<uint8_t> c((size_t)E * M.lam);
            const uint8_t* base = out[t].data() + L.out_prefix[j];
            for (uint32_t e = 0; e < E; e++)
                for (uint32_t d = 0; d < M.lam; d++) c[(size_t)e * M.lam + d] = base[((size_t)(d / 16) * E + e) * 16 + d % 16];
            // digits past lambda must have been cleared
            for (uint32_t e = 0; e < E; e++)
                for (uint32_t d = M.lam; d < M.nchunk * 16; d++)
                    if (base[((size_t)(d / 16) * E + e) * 16 + d % 16] != 0) return 3;
            fwrite(c.data(), 1, c.size(), f);
        }
    fclose(f);
    return 0;
}
