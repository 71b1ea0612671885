// Host emulation of two evaluator kernels that read a wire of modulus 2: cast_halve_body (scaling gadget) and
// hg_finish_body (half gate), lane by lane over exactly-sized host buffers under the sanitizers.  Test code, not
// part of libdash.
//
// usage: cast_emul <in.bin> <out.bin>
//   in : int32 p n_elem rule layer slot addc lam2(0: by the rule) lam_p(0: by the rule); uint64 elem_base;
//        u8 y[n][lam2] x[n][lam_p] one[lam_p] table[n][2][pitch_p]          (cast and halve)
//        u8 U[n][lam_p] V[n][lam_p] S[n][2][4]                              (half gate: z = V + beta x - U)
//   out: u8 b[n][lam_p] z[n][lam_p]
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
static void from_chunked(const std::vector<uint8_t>& v, uint32_t n, const ModInfo& M, uint8_t* compact) {
    for (uint32_t e = 0; e < n; e++)
        for (uint32_t j = 0; j < M.lam; j++) compact[(size_t)e * M.lam + j] = v[((size_t)(j / 16) * n + e) * 16 + j % 16];
}
static void set_lam(ModInfo& M, int lam) { M.lam = (uint32_t)lam; M.nchunk = (M.lam + 15) / 16; M.ndw = (M.lam + 3) / 4; }

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t hd[8];
    uint64_t elem_base;
    if (fread(hd, 4, 8, f) != 8 || fread(&elem_base, 8, 1, f) != 1) return 2;
    const int p = hd[0], rule = hd[2], layer = hd[3], slot = hd[4], addc = hd[5];
    const uint32_t n = (uint32_t)hd[1];
    std::vector<ModInfo> mods(256);
    for (int m = 2; m < 256; m++) fill_modinfo(mods[m], m, rule);
    if (hd[6]) set_lam(mods[2], hd[6]);
    if (hd[7]) set_lam(mods[p], hd[7]);
    const ModInfo &M2 = mods[2], &Mp = mods[p];
    auto rd = [&](size_t bytes) { std::vector<uint8_t> v(bytes); if (fread(v.data(), 1, bytes, f) != bytes) exit(2); return v; };
    std::vector<uint8_t> y = rd((size_t)n * M2.lam), x = rd((size_t)n * Mp.lam), one = rd(Mp.lam), table = rd((size_t)n * 2 * Mp.ndw * 4);
    std::vector<uint8_t> U = rd((size_t)n * Mp.lam), V = rd((size_t)n * Mp.lam), S = rd((size_t)n * 8);
    fclose(f);
    uint8_t Sb[256], fixed[16];
    make_sbox(Sb);
    make_ttab(Sb, TT);
    for (int i = 0; i < 16; i++) fixed[i] = (uint8_t)i;
    std::vector<uint8_t> cy = to_chunked(y.data(), n, M2), cx = to_chunked(x.data(), n, Mp), cone = to_chunked(one.data(), 1, Mp);
    std::vector<uint8_t> cU = to_chunked(U.data(), n, Mp), cV = to_chunked(V.data(), n, Mp);
    std::vector<uint8_t> cb((size_t)Mp.nchunk * n * 16, 0xEE), cz((size_t)Mp.nchunk * n * 16, 0xEE);
    const uint32_t tiles = (n + kThreads - 1) / kThreads;

    CastLaunch C;
    memset(&C, 0, sizeof(C));
    expand_key(fixed, Sb, C.key.rk);
    C.mods = mods.data(); C.elem_base = elem_base; C.layer = (uint32_t)layer; C.n_elem = n;
    C.y = LView{cy.data(), (int64_t)16 * n, 16u};
    CastJob& J = C.jobs[0];
    J.p = (uint32_t)p; J.slot = (uint32_t)slot; J.table = table.data(); J.addc = (uint32_t)addc;
    J.x = LView{cx.data(), (int64_t)16 * n, 16u};
    J.one = LView{cone.data(), 16, 0u};
    J.out = LView{cb.data(), (int64_t)16 * n, 16u};
    for (uint32_t bx = 0; bx < tiles; bx++)
        for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) cast_halve_body(C, bx, 0, tx, HostTab());

    HgLaunch H;
    memset(&H, 0, sizeof(H));
    expand_key(fixed, Sb, H.key.rk);
    H.mods = mods.data(); H.elem_base = elem_base; H.layer = (uint32_t)layer; H.n_elem = n;
    H.jobs[0] = HgJob{(uint32_t)p, (uint32_t)slot + 2, LView{cx.data(), (int64_t)16 * n, 16u}, LView{cy.data(), (int64_t)16 * n, 16u},
                      LView{cU.data(), (int64_t)16 * n, 16u}, LView{cV.data(), (int64_t)16 * n, 16u}, LView{cz.data(), (int64_t)16 * n, 16u}, S.data(), nullptr, nullptr};
    for (uint32_t bx = 0; bx < tiles; bx++)
        for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) hg_finish_body(H, bx, 0, tx, HostTab());

    // The lane-per-digit form of the cast step with the digit gates behind it (cast_digit_wide_body) against the two bodies
    // it combines (cast_halve_body above, digits_eval_wide_body on its output): same b, same digit wires.  Two digits with
    // moduli 26 and 96, tables filled by a small generator; exactly-sized buffers.  (Only primes with a compile-time
    // description take that form.)
    if (hot_mod_index(Mp)) {
        const uint32_t dm[3] = {0, 26, 96};
        DigitsLaunch D;
        memset(&D, 0, sizeof(D));
        expand_key(fixed, Sb, D.key.rk);
        D.mods = mods.data(); D.elem_base = elem_base; D.layer = (uint32_t)layer; D.n_elem = n; D.n = 2; D.nres = 1;
        D.out_cs = (int64_t)16 * n;
        size_t out_bytes = 0, tab_bytes = 0;
        for (int j = 1; j <= 2; j++) {
            D.m[j] = dm[j];
            D.row_prefix[j] = j == 1 ? 0 : D.row_prefix[j - 1] + mods[dm[j - 1]].ndw * 4;
            D.out_prefix[j] = out_bytes;
            out_bytes += (size_t)mods[dm[j]].nchunk * n * 16;
            tab_bytes += (size_t)n * p * mods[dm[j]].ndw * 4;
        }
        std::vector<uint8_t> dtab(tab_bytes);
        uint32_t lcg = 12345u + (uint32_t)p;
        size_t at = 0;
        for (int j = 1; j <= 2; j++)
            for (size_t r = 0; r < (size_t)n * p; r++)
                for (uint32_t d = 0; d < mods[dm[j]].ndw * 4; d++) {
                    lcg = lcg * 1664525u + 1013904223u;
                    dtab[at++] = d < mods[dm[j]].lam ? (uint8_t)((lcg >> 16) % dm[j]) : 0;
                }
        std::vector<uint8_t> o_ref(out_bytes, 0xEE), o_new(out_bytes, 0xEE), cb2((size_t)Mp.nchunk * n * 16, 0xEE);
        D.res[0].p = (uint32_t)p; D.res[0].slot0 = (uint32_t)slot + 7; D.res[0].table = dtab.data();
        D.res[0].in = LView{cb.data(), (int64_t)16 * n, 16u}; D.res[0].out = o_ref.data();
        for (uint32_t bx = 0; bx < tiles; bx++)
            for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++)
                for (uint32_t j = 0; j <= 3; j++) digits_eval_wide_body<ModInfo, ModInfo>(D, bx, 0, j, tx, HostTab());
        CastLaunch C2 = C;
        C2.jobs[0].out = LView{cb2.data(), (int64_t)16 * n, 16u};
        D.res[0].in = C2.jobs[0].out; D.res[0].out = o_new.data();
        for (uint32_t bx = 0; bx < tiles; bx++)
            for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++)
                for (uint32_t j = 0; j <= 3; j++) cast_digit_wide_body<ModInfo, ModInfo>(C2, D, bx, 0, j, tx, HostTab());
        if (cb2 != cb) { fprintf(stderr, "cast_digit_wide_body: b differs\n"); return 3; }
        if (o_new != o_ref) { fprintf(stderr, "cast_digit_wide_body: digit wires differ\n"); return 3; }
    }

    // The whole half gate in one pass (hg_eval_quad_body, four lanes per element) against the bodies it replaces: the two
    // projection gates through eval_body, whose outputs U' and V' go into hg_finish_body.  Tables from a small generator,
    // exactly-sized buffers; primes with a compile-time description only.
    if (hot_mod_index(Mp)) {
        const size_t pitch = (size_t)Mp.ndw * 4;
        std::vector<uint8_t> G((size_t)n * p * pitch), Eh((size_t)n * 2 * pitch);
        uint32_t lcg = 777u + (uint32_t)p;
        for (auto* t : {&G, &Eh})
            for (size_t r = 0; r < t->size() / pitch; r++)
                for (size_t d = 0; d < pitch; d++) {
                    lcg = lcg * 1664525u + 1013904223u;
                    (*t)[r * pitch + d] = d < Mp.lam ? (uint8_t)((lcg >> 16) % p) : 0;
                }
        std::vector<uint8_t> u2((size_t)Mp.nchunk * n * 16, 0xEE), v2((size_t)Mp.nchunk * n * 16, 0xEE);
        std::vector<uint8_t> z_ref((size_t)Mp.nchunk * n * 16, 0xEE), z_new((size_t)Mp.nchunk * n * 16, 0xDD);
        GateLaunch GL;
        memset(&GL, 0, sizeof(GL));
        expand_key(fixed, Sb, GL.key.rk);
        GL.mods = mods.data(); GL.layer = (uint32_t)layer; GL.njobs = 2;
        for (int j = 0; j < 2; j++) {
            GateJob& Q = GL.jobs[j];
            Q.p = j == 0 ? (uint32_t)p : 2u; Q.q = (uint32_t)p; Q.slot = (uint32_t)slot + j; Q.mode = PAY_PHI;
            Q.elem_base = elem_base; Q.n_elem = n;
            Q.in = j == 0 ? LView{cx.data(), (int64_t)16 * n, 16u} : LView{cy.data(), (int64_t)16 * n, 16u};
            Q.table = j == 0 ? G.data() : Eh.data();
            Q.out = LView{(j == 0 ? u2 : v2).data(), (int64_t)16 * n, 16u};
            for (uint32_t bx = 0; bx < tiles; bx++)
                for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) eval_body<ModInfo>(GL, bx, j, tx, HostTab());
        }
        HgLaunch H2 = H;
        H2.jobs[0].U = LView{u2.data(), (int64_t)16 * n, 16u};
        H2.jobs[0].V = LView{v2.data(), (int64_t)16 * n, 16u};
        H2.jobs[0].z = LView{z_ref.data(), (int64_t)16 * n, 16u};
        for (uint32_t bx = 0; bx < tiles; bx++)
            for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) hg_finish_body(H2, bx, 0, tx, HostTab());
        H2.jobs[0].U = LView{nullptr, 0, 0u};
        H2.jobs[0].V = LView{nullptr, 0, 0u};
        H2.jobs[0].z = LView{z_new.data(), (int64_t)16 * n, 16u};
        H2.jobs[0].G = G.data(); H2.jobs[0].Eh = Eh.data();
        const uint32_t qtiles = (n * 4 + kThreads - 1) / kThreads;
        for (uint32_t bx = 0; bx < qtiles; bx++)
            for (uint32_t tx = 0; tx < (uint32_t)kThreads; tx++) hg_eval_quad_body(H2, bx, 0, tx, HostTab());
        if (z_new != z_ref) { fprintf(stderr, "hg_eval_quad_body: z differs\n"); return 3; }
    }

    std::vector<uint8_t> ob((size_t)n * Mp.lam), oz((size_t)n * Mp.lam);
    from_chunked(cb, n, Mp, ob.data());
    from_chunked(cz, n, Mp, oz.data());
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(ob.data(), 1, ob.size(), f);
    fwrite(oz.data(), 1, oz.size(), f);
    fclose(f);
    return 0;
}
