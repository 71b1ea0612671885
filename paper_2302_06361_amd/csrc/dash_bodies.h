// dash_bodies.h -- the per-lane bodies of the gate kernels, as host+device templates over the AES
// table accessor.  The __global__ kernels in dash_gates.hip call them with (blockIdx, threadIdx) and
// the LDS copy of the tables; the CPU test suite runs the very same bodies lane by lane under a
// sanitizer, against host memory.
#pragma once
#include "dash_core.h"
#include "dash_launch.h"

namespace dash {

// dword i (digits 4i..4i+3) of element e of a label view
DASH_HD uint32_t ld_dw(const LView& v, uint32_t e, int i) {
    return *(const uint32_t*)(v.p + (int64_t)(i >> 2) * v.cs + (uint64_t)e * v.es + (i & 3) * 4);
}
DASH_HD void st_dw(const LView& v, uint32_t e, int i, uint32_t w) {
    *(uint32_t*)(v.p + (int64_t)(i >> 2) * v.cs + (uint64_t)e * v.es + (i & 3) * 4) = w;
}

// PRG labels: one lane per (job, element)
template <class Tab>
DASH_HD void draw_body(const DrawLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const DrawJob& J = L.jobs[by];
    uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    const ModInfo M = L.mods[J.m];
    U128 h = prg_block(L.elem_base + e, J.slot, L.layer, J.domain, J.m, L.key.rk, T);
    if (J.digit0_only) { J.out.p[e] = (uint8_t)mod_u128(h, M); return; }
    with_mod(M, [&](auto Q) {
        decompress(Q, h, [&](int i, uint32_t w) { st_dw(J.out, e, i, w); });
        for (int i = (int)Q.ndw; i < (int)Q.nchunk * 4; i++) st_dw(J.out, e, i, 0);
    });
}

// free gates: out = sum_t coef_t * term_t mod m
DASH_HD void affine_body(const AffineLaunch& L, uint32_t bx, uint32_t by, uint32_t tx) {
    const AffineJob& J = L.jobs[by];
    uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    const ModInfo M = L.mods[J.m];
    for (int i = 0; i < (int)M.nchunk * 4; i++) {
        uint32_t acc[4] = {0, 0, 0, 0};
        for (uint32_t t = 0; t < J.term_count; t++) {
            uint32_t w = ld_dw(L.terms[J.term_first + t].v, e, i), cf = L.terms[J.term_first + t].coef;
            for (int b = 0; b < 4; b++) acc[b] += mul24(cf, byte_of(w, b));      // <= 16 * 254 * 254 < 2^24
        }
        st_dw(J.out, e, i, mod_m(acc[0], M) | (mod_m(acc[1], M) << 8) | (mod_m(acc[2], M) << 16) | (mod_m(acc[3], M) << 24));
    }
}

// garble: one lane per ciphertext row r = gate * p + a.  QD: description type of the output modulus
// (every job of a launch has the same output modulus), fixed at compile time for the hot moduli.
template <class QD, class Tab>
DASH_HD void garble_body(const GateLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const GateJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    const QD Q = make_mod<QD>::from(Mq);
    // The block's first row is divided once (scalar unit); the lane's offset from it is small enough
    // for the 24-bit magic division.
    const uint64_t r0 = (uint64_t)bx * kThreads;
    if (r0 >= (uint64_t)L.n_elem * Mp.m) return;
    const uint32_t g0 = (uint32_t)(r0 / Mp.m);
    const uint32_t off = (uint32_t)(r0 - (uint64_t)g0 * Mp.m) + tx;
    const uint32_t dg = div_m(off, Mp);
    const uint32_t g = g0 + dg, a = off - dg * Mp.m;
    if (g >= L.n_elem) return;

    // label of value a on the input wire: zero label + a * R_p (row a of the table of offset multiples)
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) {
        const uint32_t* da = P.dtab + (size_t)a * P.ndw;
        K = compress(P, [&](int i) { return addmod4(ld_dw(J.in, g, i), da[i], P); }, &colour);
    });
    U128 h = hash_block(K, L.elem_base + g, J.slot, L.layer, L.key.rk, T);

    if (J.mode == PAY_SHORT) {
        uint32_t v = mod_m(a + J.r[g] + mod_u128(h, Q), Q);
        *(uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * 4) = v;
        return;
    }
    uint32_t* row = (uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * (Q.ndw * 4));
    if (J.mode == PAY_EHALF) {
        uint32_t cf = mod_m(a + J.r[g], Q);
        cf = cf ? Q.m - cf : 0;                          // minus (a + r) * x0
        decompress(Q, h, [&](int i, uint32_t hd) {
            uint32_t pay = axpymod4(ld_dw(J.out, g, i), cf, ld_dw(J.x0, g, i), Q);
            row[i] = addmod4(pay, hd, Q);
        });
        return;
    }
    uint32_t f;
    if (J.mode == PAY_MULR) f = mod_m(a * J.r[g], Q);
    else f = J.phi[(size_t)g * J.phi_stride + a];
    const uint32_t* df = Q.dtab + (size_t)f * Q.ndw;
    decompress(Q, h, [&](int i, uint32_t hd) {
        row[i] = addmod4(addmod4(ld_dw(J.out, g, i), df[i], Q), hd, Q);
    });
}

// eval: one lane per gate
template <class QD, class Tab>
DASH_HD void eval_body(const GateLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const GateJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    const QD Q = make_mod<QD>::from(Mq);
    uint32_t g = bx * kThreads + tx;
    if (g >= L.n_elem) return;
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return ld_dw(J.in, g, i); }, &colour); });
    U128 h = hash_block(K, L.elem_base + g, J.slot, L.layer, L.key.rk, T);
    const uint32_t* row = (const uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * (Q.ndw * 4));
    decompress(Q, h, [&](int i, uint32_t hd) { st_dw(J.out, g, i, submod4(row[i], hd, Q)); });
    for (int i = (int)Q.ndw; i < (int)Q.nchunk * 4; i++) st_dw(J.out, g, i, 0);
}

// evaluator side of the mixed-modulus half gate: z = V + beta * x - U
template <class Tab>
DASH_HD void hg_finish_body(const HgLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const HgJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p];
    uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    uint32_t colour = 0;
    U128 K = compress(CMod<2, 128>{nullptr}, [&](int i) { return ld_dw(J.y, e, i); }, &colour);
    U128 h = hash_block(K, L.elem_base + e, J.slot, L.layer, L.key.rk, T);
    uint32_t s = *(const uint32_t*)(J.S + ((size_t)e * 2 + colour) * 4);
    uint32_t beta = mod_m(s + Mp.m - mod_u128(h, Mp), Mp);
    for (int i = 0; i < (int)Mp.nchunk * 4; i++) {
        uint32_t v = axpymod4(ld_dw(J.V, e, i), beta, ld_dw(J.x, e, i), Mp);
        st_dw(J.z, e, i, submod4(v, ld_dw(J.U, e, i), Mp));
    }
}

}  // namespace dash
