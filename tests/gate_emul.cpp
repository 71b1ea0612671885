// Host emulation of the gate kernels: runs draw_body / garble_body / eval_body (the very code the
// __global__ kernels call) lane by lane over exactly-sized host buffers, so that an address sanitizer
// sees every out-of-bounds access.  Test code, not part of libdash.
//
// usage: gate_emul <in.bin> <out.bin>
//   in : int32 p q rule n layer slot phi_stride pad; uint64 elem_base; u8 seed[16];
//        u8 delta_p[lam_p] delta_q[lam_q] in0[n][lam_p] act[n][lam_p] phi[phi_stride ? n*p : p]
//   out: u8 out0[n][lam_q] table[n][p][pitch_q] out[n][lam_q]
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

// chunk-major LabelTensor from compact labels, exactly nchunk*n*16 bytes
static std::vector<uint8_t> to_chunked(const uint8_t* compact, uint32_t n, const ModInfo& M) {
    std::vector<uint8_t> v((size_t)M.nchunk * n * 16, 0);
    for (uint32_t e = 0; e < n; e++)
        for (uint32_t j = 0; j < M.lam; j++) v[((size_t)(j / 16) * n + e) * 16 + j % 16] = compact[(size_t)e * M.lam + j];
    return v;
}
static void from_chunked(const std::vector<uint8_t>& v, uint32_t n, const ModInfo& M, uint8_t* compact) {
    for (uint32_t e = 0; e < n; e++)
        for (uint32_t j = 0; j < M.lam; j++) compact[(size_t)e * M.lam + j] = v[((size_t)(j / 16) * n + e) * 16 + j % 16];
}
static std::vector<uint32_t> make_dtab(const uint8_t* delta, const ModInfo& M) {
    std::vector<uint32_t> t((size_t)M.m * M.ndw, 0);
    for (uint32_t a = 0; a < M.m; a++)
        for (uint32_t j = 0; j < M.lam; j++) t[(size_t)a * M.ndw + j / 4] |= (uint32_t)((a * delta[j]) % M.m) << (8 * (j % 4));
    return t;
}

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[8];
    uint64_t elem_base;
    uint8_t seed[16];
    if (fread(hd, 4, 8, f) != 8 || fread(&elem_base, 8, 1, f) != 1 || fread(seed, 1, 16, f) != 16) return 2;
    const int p = hd[0], q = hd[1], rule = hd[2], layer = hd[4], slot = hd[5], phi_stride = hd[6];
    const uint32_t n = (uint32_t)hd[3];
    std::vector<ModInfo> mods(256);
    for (int m = 2; m < 256; m++) fill_modinfo(mods[m], m, rule);
    ModInfo &Mp = mods[p], &Mq = mods[q];
    std::vector<uint8_t> dp(Mp.lam), dq(Mq.lam), in0((size_t)n * Mp.lam), act((size_t)n * Mp.lam), phi(phi_stride ? (size_t)n * p : (size_t)p);
    if (fread(dp.data(), 1, dp.size(), f) != dp.size() || fread(dq.data(), 1, dq.size(), f) != dq.size() ||
        fread(in0.data(), 1, in0.size(), f) != in0.size() || fread(act.data(), 1, act.size(), f) != act.size() ||
        fread(phi.data(), 1, phi.size(), f) != phi.size()) return 2;
    fclose(f);
    std::vector<uint32_t> tp = make_dtab(dp.data(), Mp), tq = make_dtab(dq.data(), Mq);
    Mp.dtab = tp.data();
    if (p != q) Mq.dtab = tq.data();

    uint8_t S[256];
    make_sbox(S);
    make_ttab(S, TT);
    uint8_t fixed[16];
    for (int i = 0; i < 16; i++) fixed[i] = (uint8_t)i;

    std::vector<uint8_t> cin0 = to_chunked(in0.data(), n, Mp), cact = to_chunked(act.data(), n, Mp);
    std::vector<uint8_t> cout0((size_t)Mq.nchunk * n * 16, 0xEE), cout((size_t)Mq.nchunk * n * 16, 0xEE);
    std::vector<uint8_t> table((size_t)n * p * Mq.ndw * 4, 0xEE);
    const uint32_t nb_e = (n + kThreads - 1) / kThreads;

    DrawLaunch D;
    memset(&D, 0, sizeof(D));
    expand_key(seed, S, D.key.rk);
    D.mods = mods.data(); D.layer = layer;
    D.jobs[0] = DrawJob{(uint32_t)q, DOM_GATE, (uint32_t)slot, 0, LView{cout0.data(), (int64_t)16 * n, 16u}, elem_base, n, 0u};
    for (uint32_t bx = 0; bx < nb_e; bx++)
        for (uint32_t tx = 0; tx < kThreads; tx++) draw_body(D, bx, 0, tx, HostTab());

    GateLaunch G;
    memset(&G, 0, sizeof(G));
    expand_key(fixed, S, G.key.rk);
    G.mods = mods.data(); G.layer = layer;
    GateJob& J = G.jobs[0];
    J.elem_base = elem_base; J.n_elem = n;
    J.p = p; J.q = q; J.in = LView{cin0.data(), (int64_t)16 * n, 16u}; J.phi = phi.data(); J.phi_stride = phi_stride;
    J.slot = slot; J.mode = PAY_PHI; J.out = LView{cout0.data(), (int64_t)16 * n, 16u}; J.table = table.data();
    const uint64_t rows = (uint64_t)n * p;
    for (uint32_t bx = 0; bx < (rows + kThreads - 1) / kThreads; bx++)
        for (uint32_t tx = 0; tx < kThreads; tx++)
            with_mod(Mq, [&](auto Qd) { DirectSink sink; garble_body<decltype(Qd)>(G, bx, 0, tx, HostTab(), sink); });

    J.in = LView{cact.data(), (int64_t)16 * n, 16u};
    J.out = LView{cout.data(), (int64_t)16 * n, 16u};
    for (uint32_t bx = 0; bx < nb_e; bx++)
        for (uint32_t tx = 0; tx < kThreads; tx++)
            with_mod(Mq, [&](auto Qd) { eval_body<decltype(Qd)>(G, bx, 0, tx, HostTab()); });

    std::vector<uint8_t> o0((size_t)n * Mq.lam), o((size_t)n * Mq.lam);
    from_chunked(cout0, n, Mq, o0.data());
    from_chunked(cout, n, Mq, o.data());
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(o0.data(), 1, o0.size(), f);
    fwrite(table.data(), 1, table.size(), f);
    fwrite(o.data(), 1, o.size(), f);
    fclose(f);
    return 0;
}
