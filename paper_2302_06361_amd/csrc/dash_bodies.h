// dash_bodies.h -- the per-lane bodies of the gate kernels, as host+device templates over the AES
// table accessor.  The __global__ kernels in dash_gates.hip call them with (blockIdx, threadIdx) and
// the LDS copy of the tables; the CPU test suite runs the very same bodies lane by lane under a
// sanitizer, against host memory.
#pragma once
#include "dash_core.h"
#include "dash_launch.h"

namespace dash {

// dword i (digits 4i..4i+3) of element e of a label view
// The chunk base is wave-uniform (scalar registers); the lane part is a 32-bit byte offset, so the
// access is "scalar base + 32-bit vector offset" (elements per view are limited to 2^28 for this).
DASH_HD uint32_t lane_off(const LView& v, uint32_t e) { return v.es ? e << 4 : 0u; }   // es is 16 or 0
DASH_HD uint32_t ld_dw(const LView& v, uint32_t e, int i) {
    const uint8_t* base = v.p + (int64_t)(i >> 2) * v.cs + (i & 3) * 4;
    return *(const uint32_t*)(base + lane_off(v, e));
}
DASH_HD void st_dw(const LView& v, uint32_t e, int i, uint32_t w) {
    uint8_t* base = v.p + (int64_t)(i >> 2) * v.cs + (i & 3) * 4;
    *(uint32_t*)(base + lane_off(v, e)) = w;
}

// a whole 16-digit chunk of element e at once (label tensors are 16-byte aligned): one 16-byte access
struct alignas(16) Dw4 { uint32_t w[4]; };
DASH_HD Dw4 ld_chunk(const LView& v, uint32_t e, int ch) { return *(const Dw4*)(v.p + (int64_t)ch * v.cs + lane_off(v, e)); }
DASH_HD void st_chunk(const LView& v, uint32_t e, int ch, const Dw4& d) { *(Dw4*)(v.p + (int64_t)ch * v.cs + lane_off(v, e)) = d; }

// compressed label and colour of a wire of modulus 2 (a sign bit or a mod-2 residue): the 128-digit description
// when that is the context's label length of modulus 2, the run-time record otherwise
template <class LoadDw>
DASH_HD U128 compress_mod2(const ModInfo* mods, LoadDw dw, uint32_t* colour) {
    if (mods[2].lam == 128) return compress(CMod<2, 128>{nullptr}, dw, colour);
    const ModInfo M2 = mods[2];
    return compress(M2, dw, colour);
}

// PRG labels: one lane per (job, element)
template <class Tab>
DASH_HD void draw_body(const DrawLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const DrawJob& J = L.jobs[by];
    uint32_t e = bx * kThreads + tx;
    if (e >= J.n_elem) return;
    const ModInfo M = L.mods[J.m];
    U128 h = prg_block(J.elem_base + e, J.slot, L.layer, J.domain, J.m, L.key.rk, T);
    if (J.digit0_only) { J.out.p[e] = (uint8_t)mod_u128(h, M); return; }
    with_mod(M, [&](auto Q) {
        decompress(Q, h, [&](int i, uint32_t w) { st_dw(J.out, e, i, w); });
        for (int i = (int)Q.ndw; i < (int)Q.nchunk * 4; i++) st_dw(J.out, e, i, 0);
    });
}

// free gates: out = sum_t coef_t * term_t mod m.  One lane per (element, 16-digit chunk): a 16-byte load
// per term.  Sums with unit coefficients (the mixed-radix additions of the sign gadget) accumulate two
// digits per 32-bit word in 16-bit fields; general coefficients go digit by digit.
DASH_HD void affine_body(const AffineLaunch& L, uint32_t bx, uint32_t by, uint32_t tx) {
    const AffineJob& J = L.jobs[by];
    const ModInfo M = L.mods[J.m];
    const uint64_t idx = (uint64_t)bx * kThreads + tx;
    if (idx >= (uint64_t)L.n_elem * M.nchunk) return;
    const uint32_t ch = (uint32_t)(idx / L.n_elem), e = (uint32_t)(idx - (uint64_t)ch * L.n_elem);
    const Term* T = L.terms + J.term_first;
    uint32_t out[4];
    if (J.unit) {
        uint32_t ev[4] = {0, 0, 0, 0}, od[4] = {0, 0, 0, 0};      // digits 0,2 / 1,3 of each dword, 16 bits each
        for (uint32_t t = 0; t < J.term_count; t++) {
            const uint32_t* src = (const uint32_t*)(T[t].v.p + (int64_t)ch * T[t].v.cs + lane_off(T[t].v, e));
            for (int q = 0; q < 4; q++) { uint32_t w = src[q]; ev[q] += w & 0x00ff00ffu; od[q] += (w >> 8) & 0x00ff00ffu; }
        }
        for (int q = 0; q < 4; q++)
            out[q] = mod_m(ev[q] & 0xffffu, M) | (mod_m(od[q] & 0xffffu, M) << 8) | (mod_m(ev[q] >> 16, M) << 16) | (mod_m(od[q] >> 16, M) << 24);
    } else {
        for (int q = 0; q < 4; q++) {
            uint32_t acc[4] = {0, 0, 0, 0};
            for (uint32_t t = 0; t < J.term_count; t++) {
                const uint32_t* src = (const uint32_t*)(T[t].v.p + (int64_t)ch * T[t].v.cs + lane_off(T[t].v, e));
                uint32_t w = src[q], cf = T[t].coef;
                for (int b = 0; b < 4; b++) acc[b] += mul24(cf, byte_of(w, b));      // <= 16 * 254 * 254 < 2^24
            }
            out[q] = mod_m(acc[0], M) | (mod_m(acc[1], M) << 8) | (mod_m(acc[2], M) << 16) | (mod_m(acc[3], M) << 24);
        }
    }
    uint32_t* dst = (uint32_t*)(J.out.p + (int64_t)ch * J.out.cs + lane_off(J.out, e));
    for (int q = 0; q < 4; q++) dst[q] = out[q];
}

// Where a finished ciphertext row goes.  DirectSink stores it dword by dword at its place in the table;
// the kernel for long rows stages rows in LDS instead and writes them out cooperatively.
struct DirectSink {
    uint32_t* row;
    DASH_HD void begin(uint8_t* table, uint64_t row_index, uint32_t pitch) { row = (uint32_t*)(table + row_index * pitch); }
    DASH_HD void put(int i, uint32_t w) { row[i] = w; }
};

// tag: the output modulus' compile-time description is chosen per job inside the kernel
struct PerJobMod {};

// garble: one lane per ciphertext row r = gate * p + a.  QD: description type of the output modulus
// (every job of a launch has the same output modulus), fixed at compile time for the hot moduli.
template <class QD, class Tab, class Sink>
DASH_HD void garble_body(const GateLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T, Sink& sink) {
    const GateJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    // The block's first row is divided once (scalar unit); the lane's offset from it is small enough
    // for the 24-bit magic division.
    const uint64_t r0 = (uint64_t)bx * kThreads;
    if (r0 >= (uint64_t)J.n_elem * Mp.m) return;
    const uint32_t g0 = (uint32_t)(r0 / Mp.m);
    const uint32_t off = (uint32_t)(r0 - (uint64_t)g0 * Mp.m) + tx;
    const uint32_t dg = div_m(off, Mp);
    const uint32_t g = g0 + dg, a = off - dg * Mp.m;
    if (g >= J.n_elem) return;

    // label of value a on the input wire: zero label + a * R_p (row a of the table of offset multiples)
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) {
        const uint32_t* da = P.dtab + a * P.ndw;
        K = compress(P, [&](int i) { return addmod4(ld_dw(J.in, g, i), gload32(da + i), P); }, &colour);
    });
    U128 h = hash_block(K, J.elem_base + g, J.slot, L.layer, L.key.rk, T);

    // the output modulus: the kernel's compile-time description, or the run-time record (the instantiation for any
    // modulus, which also serves launches that mix output moduli; choosing a compile-time description per job inside
    // it, as eval_body does, was measured much slower on large launches: the kernel then needs the registers of its
    // largest case), or, QD = PerJobMod, that choice per job: for launches of few rows, where a lane's run time and
    // not the number of waves in flight decides)
    auto finish = [&](const auto& Q) {
        typedef std::decay_t<decltype(Q)> QT;
        if (J.mode == PAY_SHORT) {
            uint32_t v = mod_m(a + J.r[g] + mod_u128(h, Q), Q);
            *(uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * 4) = v;
            return;
        }
        sink.begin(J.table, (uint64_t)g * Mp.m + colour, Q.ndw * 4);
        if (J.mode == PAY_EHALF) {
            uint32_t cf = mod_m(a + J.r[g], Q);
            cf = cf ? Q.m - cf : 0;                          // minus (a + r) * x0
            decompress(Q, h, [&](int i, uint32_t hd) {
                uint32_t pay = axpymod4(ld_dw(J.out, g, i), cf, ld_dw(J.x0, g, i), Q);
                sink.put(i, addmod4(pay, hd, Q));
            });
            return;
        }
        uint32_t f;
        if (J.mode == PAY_MULR) f = mod_m(a * J.r[g], Q);
        else f = J.phi[(size_t)g * J.phi_stride + a];
        const uint32_t* df = Q.dtab + f * Q.ndw;
        if constexpr (cmod_m<QT>::value != 0) {
            // payload first (its loads do not wait behind the row stores), then one pass over the hash digits
            uint32_t pay[QT::ndw];
#pragma unroll
            for (int i = 0; i < (int)QT::ndw; i++) pay[i] = addmod4(ld_dw(J.out, g, i), gload32(df + i), Q);
            decompress(Q, h, [&](int i, uint32_t hd) { sink.put(i, addmod4(pay[i], hd, Q)); });
        } else {
            decompress(Q, h, [&](int i, uint32_t hd) {
                sink.put(i, addmod4(addmod4(ld_dw(J.out, g, i), gload32(df + i), Q), hd, Q));
            });
        }
    };
    if constexpr (cmod_m<QD>::value != 0) finish(make_mod<QD>::from(Mq));
    else if constexpr (std::is_same<QD, PerJobMod>::value) with_mod(Mq, finish);
    else finish(Mq);
}

// eval: one lane per gate
template <class QD, class Tab>
DASH_HD void eval_body(const GateLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const GateJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p], Mq = L.mods[J.q];
    uint32_t g = bx * kThreads + tx;
    if (g >= J.n_elem) return;
    uint32_t colour = ld_dw(J.in, g, 0) & 0xffu;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return ld_dw(J.in, g, i); }, &colour); });
    // (the output modulus as in garble_body; the row is named by the colour, digit 0 of the label: its loads are issued
    // before the hash, not after)
    auto finish = [&](const auto& Q) {
        typedef std::decay_t<decltype(Q)> QT;
        const uint32_t* row = (const uint32_t*)(J.table + ((size_t)g * Mp.m + colour) * (Q.ndw * 4));
        uint32_t rw[cmod_ndw<QT>::value];
        if constexpr (cmod_m<QT>::value != 0) {
#pragma unroll
            for (int i = 0; i < (int)QT::ndw; i++) rw[i] = row[i];
        }
        U128 h = hash_block(K, J.elem_base + g, J.slot, L.layer, L.key.rk, T);
        if constexpr (cmod_m<QT>::value != 0) {
            decompress(Q, h, [&](int i, uint32_t hd) { st_dw(J.out, g, i, submod4(rw[i], hd, Q)); });
        } else {
            decompress(Q, h, [&](int i, uint32_t hd) { st_dw(J.out, g, i, submod4(row[i], hd, Q)); });
        }
        for (int i = (int)Q.ndw; i < (int)Q.nchunk * 4; i++) st_dw(J.out, g, i, 0);
    };
    if constexpr (cmod_m<QD>::value != 0) finish(make_mod<QD>::from(Mq));
    else with_mod(Mq, finish);
}

// ---- evaluator, carry chain of the sign gadget ------------------------------------------------
// One gate of the chain for element e: the input label comes dword by dword from in_dw, the output label
// goes dword by dword to out.
// QUAD: the four lanes of a quad work on the same element and share the AES (hash_block_quad).
template <bool QUAD = false, class MI, class MO, class Tab, class In, class Out>
DASH_HD void chain_gate(const ChainLaunch& L, const MI& Mi, const MO& Mo, uint32_t e, int j, In in_dw, Out out, const Tab& T) {
    uint32_t colour = in_dw(0) & 0xffu;       // the row's loads go out before the hash
    const uint32_t* row = (const uint32_t*)(L.table[j] + ((size_t)e * Mi.m + colour) * (Mo.ndw * 4));
    uint32_t rw[cmod_ndw<MO>::value];
    if constexpr (cmod_m<MO>::value != 0) {
#pragma unroll
        for (int i = 0; i < (int)MO::ndw; i++) rw[i] = row[i];
    }
    U128 K = compress(Mi, in_dw, &colour);
    U128 h = QUAD ? hash_block_quad(K, L.elem_base + e, L.slot[j], L.layer, L.key.rk, T)
                  : hash_block(K, L.elem_base + e, L.slot[j], L.layer, L.key.rk, T);
    if constexpr (cmod_m<MO>::value != 0) {
        decompress(Mo, h, [&](int i, uint32_t hd) { out(i, submod4(rw[i], hd, Mo)); });
    } else {
        decompress(Mo, h, [&](int i, uint32_t hd) { out(i, submod4(row[i], hd, Mo)); });
    }
}

// dword i of the final gate's output: the sign bit wire, and (scaling gadget) the same wire plus a constant
DASH_HD void chain_out(const ChainLaunch& L, uint32_t e, int i, uint32_t w) {
    st_dw(L.bit, e, i, w);
    if (L.up.p) st_dw(L.up, e, i, L.up_coef ? addmod4(w, ld_dw(L.up_one, e, i), CMod<2, 128>{nullptr}) : w);
}

// Digit sets whose digits 2..n share one accumulation modulus (description MC) and whose first digit has
// description M1, both fixed at compile time: the carry label stays in registers from gate to gate.  The output
// wire has modulus 2 and 128 digits (the launcher takes the generic body for any other label length of modulus 2).
// QUAD (layers of few elements, where the chain of one lane is the run time): four neighbouring lanes per element; they
// do everything alike except the AES, which they share, and the stores, which the first of them does.
template <class MC, class M1, bool QUAD = false, class Tab>
DASH_HD void chain_eval_body(const ChainLaunch& L, uint32_t bx, uint32_t tx, const Tab& T) {
    const uint32_t lane = bx * kThreads + tx;
    const uint32_t e = QUAD ? lane >> 2 : lane;
    const bool writer = !QUAD || (lane & 3u) == 0;
    if (e >= L.n_elem) return;
    const MC Mc{nullptr};
    const M1 Mf{nullptr};
    const CMod<2, 128> M2{nullptr};
    uint32_t cw[MC::ndw], c1[M1::ndw];
#pragma unroll
    for (int i = 0; i < (int)MC::ndw; i++) cw[i] = 0;
    const int n = (int)L.n;
    // The digit sums do not depend on the chain: the sum of the next digit is fetched before the hash of the current
    // gate, so that its latency passes under the hash (a lane has nothing else to overlap it with).
    uint32_t sm[MC::ndw], s1[M1::ndw];
#pragma unroll
    for (int i = 0; i < (int)MC::ndw; i++) sm[i] = ld_dw(L.sum[n], e, i);
    for (int j = n; j >= 3; j--) {                  // carry out of digit j into digit j-1, same modulus
        uint32_t in[MC::ndw];
#pragma unroll
        for (int i = 0; i < (int)MC::ndw; i++) in[i] = addmod4(sm[i], cw[i], Mc);   // cw = 0 at j = n
#pragma unroll
        for (int i = 0; i < (int)MC::ndw; i++) sm[i] = ld_dw(L.sum[j - 1], e, i);
        chain_gate<QUAD>(L, Mc, Mc, e, j, [&](int i) { return in[i]; }, [&](int i, uint32_t w) { cw[i] = w; }, T);
    }
    {                                               // digit 2 -> carry into digit 1 (modulus of the first digit)
        uint32_t in[MC::ndw];
#pragma unroll
        for (int i = 0; i < (int)MC::ndw; i++) in[i] = addmod4(sm[i], cw[i], Mc);
#pragma unroll
        for (int i = 0; i < (int)M1::ndw; i++) s1[i] = ld_dw(L.sum[1], e, i);
        chain_gate<QUAD>(L, Mc, Mf, e, 2, [&](int i) { return in[i]; }, [&](int i, uint32_t w) { c1[i] = w; }, T);
    }
    {                                               // final gate: digit 1 -> the sign bit
        uint32_t in[M1::ndw];
#pragma unroll
        for (int i = 0; i < (int)M1::ndw; i++) in[i] = addmod4(s1[i], c1[i], Mf);
        Dw4 bits[8];                                // the 128 digits of the output wire: stored 16 bytes at a time
        chain_gate<QUAD>(L, Mf, M2, e, 1, [&](int i) { return in[i]; }, [&](int i, uint32_t w) { bits[i >> 2].w[i & 3] = w; }, T);
        if (!writer) return;
#pragma unroll
        for (int ch = 0; ch < 8; ch++) st_chunk(L.bit, e, ch, bits[ch]);
        if (L.up.p) {
#pragma unroll
            for (int ch = 0; ch < 8; ch++) {
                if (L.up_coef) {
                    const Dw4 ow = ld_chunk(L.up_one, e, ch);
#pragma unroll
                    for (int q = 0; q < 4; q++) bits[ch].w[q] = addmod4(bits[ch].w[q], ow.w[q], M2);
                }
                st_chunk(L.up, e, ch, bits[ch]);
            }
        }
    }
}

// Any digit set, run-time constants: the carry label goes through its buffer in memory (written and read
// back by the same lane).
template <class Tab>
DASH_HD void chain_eval_generic_body(const ChainLaunch& L, uint32_t bx, uint32_t tx, const Tab& T) {
    const uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    const int n = (int)L.n;
    for (int j = n; j >= 1; j--) {
        const ModInfo Mi = L.mods[L.m[j]];
        const bool has_carry = j < n;
        auto in_dw = [&](int i) {
            uint32_t w = ld_dw(L.sum[j], e, i);
            return has_carry ? addmod4(w, ld_dw(L.carry[j], e, i), Mi) : w;
        };
        if (j >= 2) {
            const ModInfo Mo = L.mods[L.m[j - 1]];
            chain_gate(L, Mi, Mo, e, j, in_dw, [&](int i, uint32_t w) { st_dw(L.carry[j - 1], e, i, w); }, T);
            for (int i = (int)Mo.ndw; i < (int)Mo.nchunk * 4; i++) st_dw(L.carry[j - 1], e, i, 0);
        } else if (L.mods[2].lam == 128) {
            const CMod<2, 128> M2{nullptr};
            chain_gate(L, Mi, M2, e, 1, in_dw, [&](int i, uint32_t w) { chain_out(L, e, i, w); }, T);
        } else {                                // another label length of modulus 2: run-time constants
            const ModInfo M2 = L.mods[2];
            chain_gate(L, Mi, M2, e, 1, in_dw, [&](int i, uint32_t w) { chain_out(L, e, i, w); }, T);
            for (int i = (int)M2.ndw; i < (int)M2.nchunk * 4; i++) chain_out(L, e, i, 0);
        }
    }
}

// ---- evaluator, digit gates of the sign gadget -------------------------------------------------
// gate (residue, digit j) of element e with the compressed input label K and its colour already known
template <class MO, class Tab>
DASH_HD void digit_gate(const DigitsLaunch& L, const DigitsRes& R, const MO& Mo, const U128& K, uint32_t colour, uint32_t e, int j, const Tab& T) {
    const uint8_t* seg = R.table + (size_t)L.n_elem * R.p * L.row_prefix[j];
    const uint32_t* row = (const uint32_t*)(seg + ((size_t)e * R.p + colour) * (Mo.ndw * 4));
    uint32_t rw[cmod_ndw<MO>::value];
    if constexpr (cmod_m<MO>::value != 0) {
#pragma unroll
        for (int i = 0; i < (int)MO::ndw; i++) rw[i] = row[i];
    }
    const LView out{R.out + L.out_prefix[j], L.out_cs, 16u};
    U128 h = hash_block(K, L.elem_base + e, R.slot0 + (uint32_t)(j - 1), L.layer, L.key.rk, T);
    if constexpr (cmod_m<MO>::value != 0) {
        decompress(Mo, h, [&](int i, uint32_t hd) { st_dw(out, e, i, submod4(rw[i], hd, Mo)); });
    } else {
        decompress(Mo, h, [&](int i, uint32_t hd) { st_dw(out, e, i, submod4(row[i], hd, Mo)); });
    }
    for (int i = (int)Mo.ndw; i < (int)Mo.nchunk * 4; i++) st_dw(out, e, i, 0);
}
// the same gate with its output label handed to put(dword index, packed digits) instead of stored (compile-time moduli)
template <class MO, class Tab, class Put>
DASH_HD void digit_gate_to(const DigitsLaunch& L, const DigitsRes& R, const MO& Mo, const U128& K, uint32_t colour, uint32_t e, int j, const Tab& T,
                           Put put) {
    const uint8_t* seg = R.table + (size_t)L.n_elem * R.p * L.row_prefix[j];
    const uint32_t* row = (const uint32_t*)(seg + ((size_t)e * R.p + colour) * (MO::ndw * 4));
    uint32_t rw[MO::ndw];
#pragma unroll
    for (int i = 0; i < (int)MO::ndw; i++) rw[i] = row[i];
    U128 h = hash_block(K, L.elem_base + e, R.slot0 + (uint32_t)(j - 1), L.layer, L.key.rk, T);
    decompress(Mo, h, [&](int i, uint32_t hd) { put(i, submod4(rw[i], hd, Mo)); });
}

// MC, M1: descriptions of the accumulation moduli of digits 2..n and of digit 1 (compile time), or ModInfo for
// both (any digit set: then every digit's constants are read from the table of moduli)
template <class MC, class M1, class Tab>
DASH_HD void digits_eval_body(const DigitsLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const DigitsRes& R = L.res[by];
    const uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    const ModInfo Mp = L.mods[R.p];
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return ld_dw(R.in, e, i); }, &colour); });
    if constexpr (cmod_m<MC>::value != 0) {
        digit_gate(L, R, M1{nullptr}, K, colour, e, 1, T);
        const MC Mc{nullptr};
        for (int j = 2; j <= (int)L.n; j++) digit_gate(L, R, Mc, K, colour, e, j, T);
    } else {
        for (int j = 1; j <= (int)L.n; j++) {
            const ModInfo Mo = L.mods[L.m[j]];      // a copy in registers: through the reference every use is a load
            digit_gate(L, R, Mo, K, colour, e, j, T);
        }
    }
}

// The same gates with one lane per (element, residue, digit j): every lane compresses the label again, but a lane's
// chain is one hash instead of n.  For gadgets over few elements, whose time is the length of that chain.
template <class MC, class M1, class Tab>
DASH_HD void digits_eval_wide_body(const DigitsLaunch& L, uint32_t bx, uint32_t by, uint32_t j, uint32_t tx, const Tab& T) {
    const DigitsRes& R = L.res[by];
    const uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem || j < 1 || j > L.n) return;
    const ModInfo Mp = L.mods[R.p];
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return ld_dw(R.in, e, i); }, &colour); });
    if constexpr (cmod_m<MC>::value != 0) {
        if (j == 1) digit_gate(L, R, M1{nullptr}, K, colour, e, 1, T);
        else digit_gate(L, R, MC{nullptr}, K, colour, e, (int)j, T);
    } else {
        const ModInfo Mo = L.mods[L.m[j]];
        digit_gate(L, R, Mo, K, colour, e, (int)j, T);
    }
}

// ---- garbler, digit gates of the sign gadget ---------------------------------------------------
// One lane per (element g, value a) of a residue: the label of a is formed and compressed once, then one
// ciphertext row per digit: rows[colour] = out0 + phi_j(a) R_{m_j} + H_{m_j}(label, slot_j).
template <class MO, class Tab>
DASH_HD void digit_row(const DigitsLaunch& L, const DigitsRes& R, const MO& Mo, const U128& K, uint32_t colour, uint32_t g, uint32_t a, int j,
                       const Tab& T) {
    uint8_t* seg = R.table + (size_t)L.n_elem * R.p * L.row_prefix[j];
    uint32_t* row = (uint32_t*)(seg + ((size_t)g * R.p + colour) * (Mo.ndw * 4));
    const LView out0{R.out + L.out_prefix[j], L.out_cs, 16u};
    const uint32_t f = R.phi[(size_t)(j - 1) * R.p + a];
    const uint32_t* df = Mo.dtab + f * Mo.ndw;
    U128 h = hash_block(K, L.elem_base + g, R.slot0 + (uint32_t)(j - 1), L.layer, L.key.rk, T);
    if constexpr (cmod_m<MO>::value != 0) {
        uint32_t pay[MO::ndw];
#pragma unroll
        for (int i = 0; i < (int)MO::ndw; i++) pay[i] = addmod4(ld_dw(out0, g, i), gload32(df + i), Mo);
        decompress(Mo, h, [&](int i, uint32_t hd) { row[i] = addmod4(pay[i], hd, Mo); });
    } else {
        decompress(Mo, h, [&](int i, uint32_t hd) { row[i] = addmod4(addmod4(ld_dw(out0, g, i), gload32(df + i), Mo), hd, Mo); });
    }
}
// j0 = 0: all n digits of the lane's (element, value); j0 = 1..n: digit j0 only (gadgets over few elements: a lane per
// row, a chain of one hash)
template <class MC, class M1, class Tab>
DASH_HD void digits_garble_body(const DigitsLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T, uint32_t j0 = 0) {
    const DigitsRes& R = L.res[by];
    const ModInfo Mp = L.mods[R.p];
    const uint64_t r0 = (uint64_t)bx * kThreads;
    if (r0 >= (uint64_t)L.n_elem * Mp.m) return;
    const uint32_t g0 = (uint32_t)(r0 / Mp.m);
    const uint32_t off = (uint32_t)(r0 - (uint64_t)g0 * Mp.m) + tx;
    const uint32_t dg = div_m(off, Mp);
    const uint32_t g = g0 + dg, a = off - dg * Mp.m;
    if (g >= L.n_elem) return;
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    with_mod(Mp, [&](auto P) {
        const uint32_t* da = P.dtab + a * P.ndw;
        K = compress(P, [&](int i) { return addmod4(ld_dw(R.in, g, i), gload32(da + i), P); }, &colour);
    });
    const int jlo = j0 ? (int)j0 : 1, jhi = j0 ? (int)j0 : (int)L.n;
    if constexpr (cmod_m<MC>::value != 0) {
        if (jlo == 1) digit_row(L, R, M1{L.mods[L.m[1]].dtab}, K, colour, g, a, 1, T);
        if (jhi >= 2) {
            const MC Mc{L.mods[L.m[2]].dtab};
            for (int j = jlo < 2 ? 2 : jlo; j <= jhi; j++) digit_row(L, R, Mc, K, colour, g, a, j, T);
        }
    } else {
        for (int j = jlo; j <= jhi; j++) {
            const ModInfo Mo = L.mods[L.m[j]];      // a copy in registers: through the reference every use is a load
            digit_row(L, R, Mo, K, colour, g, a, j, T);
        }
    }
}

// evaluator, scaling gadget: cast = rows[colour(y)] - H_p(y) (two-row gate Z_2 -> Z_p, identity function), then
// b = (x + addc * one - cast) * 2^-1 mod p.  The cast label itself is not stored.
template <class P>
DASH_HD uint32_t halve4(uint32_t x, uint32_t cast, uint32_t inv2, const P& Pm) {
    if (Pm.m <= 127) {
        // four digits at once (p odd): t = (x - cast) mod p, then t / 2 for even t and (t + p) / 2 for odd t.  Bytes stay
        // below 2p <= 254, and the bit that the shift brings in from the byte above is masked off.
        const uint32_t t = submod4(x, cast, Pm);
        const uint32_t odd = t & 0x01010101u;
        return ((t + odd * Pm.m) >> 1) & 0x7f7f7f7fu;
    }
    uint32_t b = 0;
    // digits past lambda: x and cast are 0 there, and inv2 * p = 0 mod p
    for (int b8 = 0; b8 < 4; b8++) b |= mod_m(mul24(inv2, byte_of(x, b8) + Pm.m - byte_of(cast, b8)), Pm) << (8 * b8);
    return b;
}
// compile-time label length: b of element e in registers (xw: its chunks), 16-byte loads
template <class PD>
DASH_HD void cast_halve_regs(const CastJob& J, const PD& P, uint32_t e, uint32_t colour, const U128& h, Dw4* xw) {
    constexpr int ndw = (int)PD::ndw, nch = (int)PD::nchunk;
    const uint32_t inv2 = (J.p + 1) / 2;
    const uint32_t* row = (const uint32_t*)(J.table + ((size_t)e * 2 + colour) * (P.ndw * 4));
    uint32_t rw[ndw];
#pragma unroll
    for (int i = 0; i < ndw; i++) rw[i] = row[i];
#pragma unroll
    for (int ch = 0; ch < nch; ch++) xw[ch] = ld_chunk(J.x, e, ch);
    if (J.addc) {
#pragma unroll
        for (int ch = 0; ch < nch; ch++) {
            const Dw4 ow = ld_chunk(J.one, e, ch);
#pragma unroll
            for (int q = 0; q < 4; q++) xw[ch].w[q] = J.addc == 1 ? addmod4(xw[ch].w[q], ow.w[q], P) : axpymod4(xw[ch].w[q], J.addc, ow.w[q], P);
        }
    }
    decompress(P, h, [&](int i, uint32_t hd) { xw[i >> 2].w[i & 3] = halve4(xw[i >> 2].w[i & 3], submod4(rw[i], hd, P), inv2, P); });
#pragma unroll
    for (int i = ndw; i < nch * 4; i++) xw[i >> 2].w[i & 3] = 0;
}
template <class Tab>
DASH_HD void cast_halve_body(const CastLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const CastJob& J = L.jobs[by];
    const uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    const ModInfo Mp = L.mods[J.p];
    uint32_t colour = 0;
    U128 K = compress_mod2(L.mods, [&](int i) { return ld_dw(L.y, e, i); }, &colour);
    U128 h = hash_block(K, L.elem_base + e, J.slot, L.layer, L.key.rk, T);
    const uint32_t inv2 = (J.p + 1) / 2;
    with_mod(Mp, [&](auto P) {
        typedef decltype(P) PD;
        if constexpr (cmod_m<PD>::value != 0) {
            Dw4 xw[PD::nchunk];
            cast_halve_regs(J, P, e, colour, h, xw);
#pragma unroll
            for (int ch = 0; ch < (int)PD::nchunk; ch++) st_chunk(J.out, e, ch, xw[ch]);
        } else {
            const uint32_t* row = (const uint32_t*)(J.table + ((size_t)e * 2 + colour) * (P.ndw * 4));
            decompress(P, h, [&](int i, uint32_t hd) {
                const uint32_t cast = submod4(row[i], hd, P);
                uint32_t x = ld_dw(J.x, e, i);
                if (J.addc) x = J.addc == 1 ? addmod4(x, ld_dw(J.one, e, i), P) : axpymod4(x, J.addc, ld_dw(J.one, e, i), P);
                st_dw(J.out, e, i, halve4(x, cast, inv2, P));
            });
            for (int i = (int)P.ndw; i < (int)P.nchunk * 4; i++) st_dw(J.out, e, i, 0);
        }
    });
}

// The cast step and ONE digit gate per lane: lane (element, odd prime, digit j) forms b as above (the lanes of
// digit 1 store it), compresses it from its registers and evaluates digit gate j: a chain of two hashes, for
// gadgets over few elements.  Only for primes with a compile-time description (the launcher checks).
template <class MC, class M1, class Tab>
DASH_HD void cast_digit_wide_body(const CastLaunch& C, const DigitsLaunch& L, uint32_t bx, uint32_t by, uint32_t j, uint32_t tx, const Tab& T) {
    const CastJob& J = C.jobs[by];
    const DigitsRes& R = L.res[by];
    const uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem || j < 1 || j > L.n) return;
    const ModInfo Mp = C.mods[J.p];
    uint32_t colour = 0;
    U128 K2 = compress_mod2(C.mods, [&](int i) { return ld_dw(C.y, e, i); }, &colour);
    U128 h = hash_block(K2, C.elem_base + e, J.slot, C.layer, C.key.rk, T);
    with_mod(Mp, [&](auto P) {
        typedef decltype(P) PD;
        if constexpr (cmod_m<PD>::value != 0) {
            Dw4 xw[PD::nchunk];
            cast_halve_regs(J, P, e, colour, h, xw);
            if (j == 1) {
#pragma unroll
                for (int ch = 0; ch < (int)PD::nchunk; ch++) st_chunk(J.out, e, ch, xw[ch]);
            }
            uint32_t cb = 0;
            const U128 K = compress(P, [&](int i) { return xw[i >> 2].w[i & 3]; }, &cb);
            if constexpr (cmod_m<MC>::value != 0) {
                if (j == 1) digit_gate(L, R, M1{nullptr}, K, cb, e, 1, T);
                else digit_gate(L, R, MC{nullptr}, K, cb, e, (int)j, T);
            } else {
                const ModInfo Mo = L.mods[L.m[j]];
                digit_gate(L, R, Mo, K, cb, e, (int)j, T);
            }
        }
    });
}

// ---- evaluator, few elements: digit gates that add up their outputs --------------------------
// A block takes 64 elements and one digit j; wave w of it takes residue w.  Every lane evaluates its digit gate (the
// scaling gadget's lanes do the cast step first, as in cast_digit_wide_body) and adds the output label into the block's
// accumulator, two digits per 32-bit word in 16-bit fields (phase 1); after a barrier the first wave reduces the sums
// mod m_j and stores the wire S_j (phase 2).  The digit wires themselves are not stored, and the launch that added them
// up is not needed.  Digit sets with compile-time moduli only.
constexpr int kSumDw = 10;                  // dwords per label of the longest such modulus (39 digits)
constexpr int kSumElems = 64;
DASH_HD void sum_add(uint32_t* a, uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    atomicAdd(a, v);
#else
    *a += v;
#endif
}
struct NoCast {};       // in place of the CastLaunch: the digit gates of a plain sign gadget
template <class MC, class M1, class CastT, class Tab>
DASH_HD void digits_sum_phase1(const CastT& C, const DigitsLaunch& L, uint32_t bx, uint32_t by, uint32_t j, uint32_t el, const Tab& T,
                               uint32_t* acc) {
    static_assert(MC::ndw <= kSumDw && M1::ndw <= kSumDw, "accumulator rows");
    const DigitsRes& R = L.res[by];
    const uint32_t e = bx * kSumElems + el;
    if (e >= L.n_elem || j < 1 || j > L.n) return;
    const ModInfo Mp = L.mods[R.p];
    uint32_t colour = 0;
    U128 K = {{0, 0, 0, 0}};
    if constexpr (std::is_same<CastT, CastLaunch>::value) {        // scaling gadget: b of this residue first (stored by the lanes of digit 1)
        const CastJob& J = C.jobs[by];
        uint32_t c2 = 0;
        const U128 K2 = compress_mod2(C.mods, [&](int i) { return ld_dw(C.y, e, i); }, &c2);
        const U128 h = hash_block(K2, C.elem_base + e, J.slot, C.layer, C.key.rk, T);
        with_mod(Mp, [&](auto P) {
            typedef decltype(P) PD;
            if constexpr (cmod_m<PD>::value != 0) {
                Dw4 xw[PD::nchunk];
                cast_halve_regs(J, P, e, c2, h, xw);
                if (j == 1) {
#pragma unroll
                    for (int ch = 0; ch < (int)PD::nchunk; ch++) st_chunk(J.out, e, ch, xw[ch]);
                }
                K = compress(P, [&](int i) { return xw[i >> 2].w[i & 3]; }, &colour);
            }
        });
    } else {
        with_mod(Mp, [&](auto P) { K = compress(P, [&](int i) { return ld_dw(R.in, e, i); }, &colour); });
    }
    uint32_t* row = acc + (size_t)el * (kSumDw * 2);
    auto put = [&](int i, uint32_t w) {
        sum_add(row + 2 * i, w & 0x00ff00ffu);
        sum_add(row + 2 * i + 1, (w >> 8) & 0x00ff00ffu);
    };
    if (j == 1) digit_gate_to(L, R, M1{nullptr}, K, colour, e, 1, T, put);
    else digit_gate_to(L, R, MC{nullptr}, K, colour, e, (int)j, T, put);
}
template <class MO>
DASH_HD void digits_sum_store(const DigitsLaunch& L, const MO& Mo, uint32_t e, uint32_t j, const uint32_t* row) {
    const LView out{L.sum1 + L.sum_prefix[j], L.out_cs, 16u};
#pragma unroll
    for (int ch = 0; ch < (int)MO::nchunk; ch++) {
        Dw4 z;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int i = 4 * ch + q;
            uint32_t w = 0;
            if (i < (int)MO::ndw) {      // fields below 16 * 255 < 2^24
                const uint32_t ev = row[2 * i], od = row[2 * i + 1];
                w = mod_m(ev & 0xffffu, Mo) | (mod_m(ev >> 16, Mo) << 16) | (mod_m(od & 0xffffu, Mo) << 8) | (mod_m(od >> 16, Mo) << 24);
            }
            z.w[q] = w;
        }
        st_chunk(out, e, ch, z);
    }
}
template <class MC, class M1>
DASH_HD void digits_sum_phase2(const DigitsLaunch& L, uint32_t bx, uint32_t j, uint32_t el, const uint32_t* acc) {
    const uint32_t e = bx * kSumElems + el;
    if (e >= L.n_elem || j < 1 || j > L.n) return;
    const uint32_t* row = acc + (size_t)el * (kSumDw * 2);
    if (j == 1) digits_sum_store(L, M1{nullptr}, e, j, row);
    else digits_sum_store(L, MC{nullptr}, e, j, row);
}

// evaluator side of the mixed-modulus half gate: z = V + beta * x - U
template <class Tab>
DASH_HD void hg_finish_body(const HgLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const HgJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p];
    uint32_t e = bx * kThreads + tx;
    if (e >= L.n_elem) return;
    uint32_t colour = 0;
    U128 K = compress_mod2(L.mods, [&](int i) { return ld_dw(J.y, e, i); }, &colour);
    U128 h = hash_block(K, L.elem_base + e, J.slot, L.layer, L.key.rk, T);
    uint32_t s = *(const uint32_t*)(J.S + ((size_t)e * 2 + colour) * 4);
    uint32_t beta = mod_m(s + Mp.m - mod_u128(h, Mp), Mp);
    with_mod(Mp, [&](auto P) {
        typedef decltype(P) PD;
        if constexpr (cmod_m<PD>::value != 0) {
            // compile-time label length: all loads first, 16 bytes each, then the arithmetic in registers
            constexpr int nch = (int)PD::nchunk;
            Dw4 v[nch], x[nch], u[nch];
#pragma unroll
            for (int ch = 0; ch < nch; ch++) { v[ch] = ld_chunk(J.V, e, ch); x[ch] = ld_chunk(J.x, e, ch); u[ch] = ld_chunk(J.U, e, ch); }
#pragma unroll
            for (int ch = 0; ch < nch; ch++) {
#pragma unroll
                for (int q = 0; q < 4; q++) v[ch].w[q] = submod4(axpymod4(v[ch].w[q], beta, x[ch].w[q], P), u[ch].w[q], P);
                st_chunk(J.z, e, ch, v[ch]);
            }
        } else {
            for (int i = 0; i < (int)P.nchunk * 4; i++) {
                uint32_t v = axpymod4(ld_dw(J.V, e, i), beta, ld_dw(J.x, e, i), P);
                st_dw(J.z, e, i, submod4(v, ld_dw(J.U, e, i), P));
            }
        }
    });
}

// The whole evaluator side of the mixed-modulus half gate (Appendix) for layers of few elements, where three dependent
// launches cost more than their work: the four lanes of a quad take one (element, prime).  Lane 0 evaluates the garbler
// half (U, from the label of x), lane 1 the evaluator half (V, from the sign bit's label), lane 2 the row that carries
// beta: three hashes side by side; lane 0 then collects V and beta from its neighbours and stores z = V + beta x - U.
// Primes with compile-time descriptions only (the launcher checks).  On the host a caller with role 0 works through
// the three roles itself.
template <class Tab>
DASH_HD void hg_eval_quad_body(const HgLaunch& L, uint32_t bx, uint32_t by, uint32_t tx, const Tab& T) {
    const HgJob& J = L.jobs[by];
    const ModInfo Mp = L.mods[J.p];
    const uint32_t lane = bx * kThreads + tx, e = lane >> 2, c = lane & 3u;
    if (e >= L.n_elem) return;
    with_mod(Mp, [&](auto P) {
        typedef decltype(P) PD;
        if constexpr (cmod_m<PD>::value != 0) {
            constexpr int ndw = (int)PD::ndw, nch = (int)PD::nchunk;
            Dw4 x[nch];
            // one role: w = the gate's output label (roles 0 and 1), beta (role 2; role 3 repeats it and is not used)
            auto run_role = [&](uint32_t role, uint32_t* w, uint32_t& beta) {
                uint32_t colour = 0;
                U128 K;
                if (role == 0) {
#pragma unroll
                    for (int ch = 0; ch < nch; ch++) x[ch] = ld_chunk(J.x, e, ch);
                    K = compress(P, [&](int i) { return x[i >> 2].w[i & 3]; }, &colour);
                } else {
                    K = compress_mod2(L.mods, [&](int i) { return ld_dw(J.y, e, i); }, &colour);
                }
                const uint32_t rows = role == 0 ? Mp.m : 2u;
                const uint8_t* table = role == 0 ? J.G : J.Eh;
                uint32_t rw[ndw];
                uint32_t srow = 0;
                if (role < 2) {
                    const uint32_t* row = (const uint32_t*)(table + ((size_t)e * rows + colour) * (ndw * 4));
#pragma unroll
                    for (int i = 0; i < ndw; i++) rw[i] = row[i];
                } else {
                    srow = *(const uint32_t*)(J.S + ((size_t)e * 2 + colour) * 4);
                }
                const uint32_t slot = J.slot - 2 + (role < 2 ? role : 2u);
                const U128 h = hash_block(K, L.elem_base + e, slot, L.layer, L.key.rk, T);
                if (role < 2) decompress(P, h, [&](int i, uint32_t hd) { w[i] = submod4(rw[i], hd, P); });
                else beta = mod_m(srow + Mp.m - mod_u128(h, Mp), Mp);
            };
            uint32_t u[ndw], v[ndw], beta = 0;
#if defined(__HIP_DEVICE_COMPILE__)
            run_role(c, u, beta);
#pragma unroll
            for (int i = 0; i < ndw; i++) v[i] = quad_lane<1>(u[i]);
            beta = quad_lane<2>(beta);
            if (c != 0) return;
#else
            if (c != 0) return;
            uint32_t unused = 0;
            run_role(1, v, unused);
            run_role(2, u, beta);
            run_role(0, u, unused);
#endif
#pragma unroll
            for (int ch = 0; ch < nch; ch++) {
                Dw4 z;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int i = 4 * ch + q;
                    z.w[q] = i < ndw ? submod4(axpymod4(v[i], beta, x[ch].w[q], P), u[i], P) : 0u;
                }
                st_chunk(J.z, e, ch, z);
            }
        }
    });
}

}  // namespace dash
