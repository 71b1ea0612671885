// Host emulation of ONE evaluator launch (and, below, one garbler launch) that mixes output moduli: 16 jobs, one per modulus with a compile-time
// description, run through eval_body<ModInfo> (the instantiation that picks a description per job) lane by lane over
// exactly-sized host buffers under the address sanitizer: every table-row address and every label store must stay
// inside its job's buffers.  The results are compared with the single-modulus instantiations on the same inputs.
// Test code, not part of libdash.   usage: mixed_emul <n_elem> <seed> <which list of 16 moduli: 0 or 1>
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
static uint64_t rng_state;
static uint32_t rnd() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }

int main(int argc, char** argv) {
    if (argc != 4) return 2;
    const uint32_t n = (uint32_t)atoi(argv[1]);
    rng_state = (uint64_t)atoll(argv[2]);
    std::vector<ModInfo> mods(256);
    for (int m = 2; m < 256; m++) fill_modinfo(mods[m], m, 0);
    // the default digit sets (d_1; d, .., d) of the 8-, 12-, 7- and 9-prime bases must find their kernels with compile-time
    // moduli: accumulation moduli m_1 = d_1 and m_c = k d (Appendix, Approximated Garbled Sign)
    static const int sets[4][3] = {{8, 26, 12}, {12, 46, 17}, {7, 10, 13}, {9, 22, 10}};
    for (int i = 0; i < 4; i++)
        if (digit_set_index(mods[sets[i][0] * sets[i][2]], mods[sets[i][1]]) != i + 1) { fprintf(stderr, "digit set %d has no compile-time kernels\n", i); return 1; }
    uint8_t S[256], fixed[16];
    make_sbox(S);
    make_ttab(S, TT);
    for (int i = 0; i < 16; i++) fixed[i] = (uint8_t)i;
    // 20 moduli have compile-time descriptions, a launch takes 16 jobs: two lists
    static const int hot0[16] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 26, 96, 46, 204};
    static const int hot1[16] = {10, 91, 22, 90, 2, 3, 5, 7, 11, 13, 17, 19, 26, 96, 46, 204};
    const int* hot = atoi(argv[3]) ? hot1 : hot0;
    GateLaunch G;
    memset(&G, 0, sizeof(G));
    expand_key(fixed, S, G.key.rk);
    G.mods = mods.data(); G.layer = 11; G.njobs = 16;
    std::vector<std::vector<uint8_t>> in(16), table(16), out(16), out_typed(16);
    for (int j = 0; j < 16; j++) {
        const int q = hot[j], p = hot[(j * 7 + 3) % 16];            // every hot modulus once as output, inputs mixed
        const ModInfo &Mp = mods[p], &Mq = mods[q];
        in[j].assign((size_t)Mp.nchunk * n * 16, 0);
        for (uint32_t e = 0; e < n; e++)
            for (uint32_t d = 0; d < Mp.lam; d++) in[j][((size_t)(d / 16) * n + e) * 16 + d % 16] = (uint8_t)(rnd() % p);
        table[j].assign((size_t)n * p * Mq.ndw * 4, 0);
        for (size_t r = 0; r < (size_t)n * p; r++)
            for (uint32_t d = 0; d < Mq.lam; d++) table[j][r * Mq.ndw * 4 + d] = (uint8_t)(rnd() % q);
        out[j].assign((size_t)Mq.nchunk * n * 16, 0xEE);
        out_typed[j].assign((size_t)Mq.nchunk * n * 16, 0xDD);
        GateJob& J = G.jobs[j];
        J.p = p; J.q = q; J.slot = 100 + j; J.mode = PAY_PHI;
        J.elem_base = (1ull << 35) + 3 + 1000 * j; J.n_elem = n;
        J.in = LView{in[j].data(), (int64_t)16 * n, 16u};
        J.table = table[j].data();
        J.out = LView{out[j].data(), (int64_t)16 * n, 16u};
    }
    const uint32_t nb = (n + kThreads - 1) / kThreads;
    for (int j = 0; j < 16; j++)
        for (uint32_t bx = 0; bx < nb; bx++)
            for (uint32_t tx = 0; tx < kThreads; tx++) eval_body<ModInfo>(G, bx, j, tx, HostTab());
    for (int j = 0; j < 16; j++) {
        G.jobs[j].out = LView{out_typed[j].data(), (int64_t)16 * n, 16u};
        for (uint32_t bx = 0; bx < nb; bx++)
            for (uint32_t tx = 0; tx < kThreads; tx++)
                with_mod(mods[hot[j]], [&](auto Qd) {
                    if constexpr (cmod_m<decltype(Qd)>::value != 0) eval_body<decltype(Qd)>(G, bx, j, tx, HostTab());
                });
        if (out[j] != out_typed[j]) { fprintf(stderr, "job %d (q = %d): mixed launch differs\n", j, hot[j]); return 1; }
        for (uint8_t b : out[j]) if (b >= hot[j]) { fprintf(stderr, "job %d: digit out of range\n", j); return 1; }
    }
    // The garbler's launch for few rows (garble_body<PerJobMod>): the same 16 jobs garbled in one pass, every table byte equal to
    // the single-modulus instantiation's and to the run-time-constant one's.
    std::vector<std::vector<uint32_t>> dtab(256);
    for (int j = 0; j < 16; j++) {
        ModInfo& M = mods[hot[j]];
        dtab[hot[j]].assign((size_t)M.m * M.ndw, 0);
        std::vector<uint32_t> delta(M.lam);
        for (uint32_t d = 0; d < M.lam; d++) delta[d] = d == 0 ? 1u : rnd() % M.m;
        for (uint32_t a = 0; a < M.m; a++)
            for (uint32_t d = 0; d < M.lam; d++) dtab[hot[j]][(size_t)a * M.ndw + d / 4] |= ((a * delta[d]) % M.m) << (8 * (d % 4));
        M.dtab = dtab[hot[j]].data();
    }
    std::vector<std::vector<uint8_t>> phi(16), out0(16), tab_any(16), tab_typed(16), tab_run(16);
    for (int j = 0; j < 16; j++) {
        GateJob& J = G.jobs[j];
        const ModInfo& Mq = mods[J.q];
        phi[j].resize((size_t)n * J.p);
        for (auto& v : phi[j]) v = (uint8_t)(rnd() % J.q);
        out0[j].assign((size_t)Mq.nchunk * n * 16, 0);
        for (uint32_t e = 0; e < n; e++)
            for (uint32_t d = 0; d < Mq.lam; d++) out0[j][((size_t)(d / 16) * n + e) * 16 + d % 16] = (uint8_t)(rnd() % J.q);
        J.phi = phi[j].data(); J.phi_stride = J.p;
        J.out = LView{out0[j].data(), (int64_t)16 * n, 16u};
        tab_any[j].assign(table[j].size(), 0xEE);
        tab_typed[j].assign(table[j].size(), 0xDD);
        tab_run[j].assign(table[j].size(), 0xCC);
    }
    for (int j = 0; j < 16; j++) {
        const uint32_t gb = (uint32_t)(((uint64_t)n * G.jobs[j].p + kThreads - 1) / kThreads);
        for (uint32_t bx = 0; bx < gb; bx++)
            for (uint32_t tx = 0; tx < kThreads; tx++) {
                DirectSink sink;
                G.jobs[j].table = tab_any[j].data();
                garble_body<PerJobMod>(G, bx, j, tx, HostTab(), sink);
                G.jobs[j].table = tab_run[j].data();
                garble_body<ModInfo>(G, bx, j, tx, HostTab(), sink);
                G.jobs[j].table = tab_typed[j].data();
                with_mod(mods[hot[j]], [&](auto Qd) {
                    if constexpr (cmod_m<decltype(Qd)>::value != 0) garble_body<decltype(Qd)>(G, bx, j, tx, HostTab(), sink);
                });
            }
        if (tab_any[j] != tab_typed[j] || tab_any[j] != tab_run[j]) { fprintf(stderr, "job %d (q = %d): garbled tables differ\n", j, hot[j]); return 1; }
    }
    printf("ok\n");
    return 0;
}
