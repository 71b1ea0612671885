// dash_layers.hip -- the gadget pipelines: approximated sign (Appendix, Approximated Garbled Sign and
// Garbled Mixed-Radix Addition), ReLU = a * sgn_{0,1}(a) with mixed-modulus half gates (Appendix),
// CRT scaling by 2 (Sec. The Scaling Operation), sign activation, raw projection-gate batches.
//
// Host code only: each pipeline is a fixed sequence of launches of the kernels in dash_gates.hip
// over all elements of the layer; gates at the same depth of the gadget share one launch.
#include <string.h>

#include <algorithm>
#include <functional>
#include <vector>

#include "dash_internal.h"

namespace dash {
namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline size_t pitch_of(const dash_ctx* c, int m) { return (size_t)c->mods[m].ndw * 4; }
inline size_t label_bytes(const dash_ctx* c, int m, int64_t E) { return align256((size_t)c->mods[m].nchunk * 16 * (size_t)E); }

// ---- slots of one sign gadget ---------------------------------------------------------------
inline int sign_nslots(const dash_ctx* c) { return c->k * c->n + c->n; }
inline int sign_slot_in(const dash_ctx* c, int s) {
    int k = c->k, n = c->n;
    if (s < k * n) return c->prime[s / n];
    if (s < k * n + n - 1) return c->mj[(s - k * n) + 2];
    return c->mj[1];
}
inline int sign_slot_out(const dash_ctx* c, int s) {
    int k = c->k, n = c->n;
    if (s < k * n) return c->mj[(s % n) + 1];
    if (s < k * n + n - 1) return c->mj[(s - k * n) + 1];
    return 2;
}
inline size_t sign_slot_bytes(const dash_ctx* c, int s, int first_res) {
    if (s < c->k * c->n && s / c->n < first_res) return 0;
    return (size_t)sign_slot_in(c, s) * pitch_of(c, sign_slot_out(c, s));
}
size_t sign_bytes(const dash_ctx* c, int first_res) {
    size_t b = 0;
    for (int s = 0; s < sign_nslots(c); s++) b += sign_slot_bytes(c, s, first_res);
    return b;
}
size_t relu_bytes(const dash_ctx* c) {
    size_t b = sign_bytes(c, 0);
    for (int i = 0; i < c->k; i++) b += (size_t)(c->prime[i] + 2) * pitch_of(c, c->prime[i]) + 8;
    return b;
}
size_t scale_bytes(const dash_ctx* c) {
    size_t b = sign_bytes(c, 1);
    for (int i = 1; i < c->k; i++) b += 2 * pitch_of(c, c->prime[i]);
    return b;
}
size_t signact_bytes(const dash_ctx* c) {
    size_t b = sign_bytes(c, 0);
    for (int i = 0; i < c->k; i++) b += 2 * pitch_of(c, c->prime[i]);
    return b;
}

// ---- scratch arena ---------------------------------------------------------------------------
struct Arena {
    uint8_t* base;
    size_t off;
    LView labels(const dash_ctx* c, int m, int64_t E) {
        LView v{base ? base + off : nullptr, (int64_t)16 * E, 16u};
        off += label_bytes(c, m, E);
        return v;
    }
    uint8_t* bytes(size_t n) { uint8_t* p = base ? base + off : nullptr; off += align256(n); return p; }
};

// wires of one sign gadget
struct SignWires {
    LView A[DASH_MAX_PRIMES][DASH_MAX_DIGITS + 1];
    LView C[DASH_MAX_DIGITS + 1];   // C[j]: carry into digit j (j = 1..n-1)
    LView S[DASH_MAX_DIGITS + 1];   // S[j]: free sum of the digit wires of digit j and the carry into it
    LView bit;
};
void plan_sign(const dash_ctx* c, Arena& ar, int64_t E, int first_res, SignWires& w) {
    for (int i = first_res; i < c->k; i++)
        for (int j = 1; j <= c->n; j++) w.A[i][j] = ar.labels(c, c->mj[j], E);
    for (int j = 1; j < c->n; j++) w.C[j] = ar.labels(c, c->mj[j], E);
    for (int j = 1; j <= c->n; j++) w.S[j] = ar.labels(c, c->mj[j], E);
    w.bit = ar.labels(c, 2, E);
}

// ---- launch batchers -------------------------------------------------------------------------
// Collects independent gate jobs and launches them grouped by output modulus (a launch runs one
// instantiation of the gate kernel, chosen by the output modulus), up to kMaxJobs per launch.
// mixed = true puts jobs of any output moduli into the same launch (the instantiation with run-time
// constants; garbling launches of few rows: the one that picks compile-time constants per job): for the
// many small batches whose output moduli all differ (one cast or half gate per prime), where a launch
// per modulus would cost more than the slower digit extraction, and for gadgets of few rows altogether.
struct GateBatcher {
    static constexpr int kSlots = 4;
    const dash_ctx* c; bool garble; hipStream_t s; bool mixed = false;
    uint32_t E; uint64_t elem_base;      // of the jobs that do not bring their own
    GateLaunch L[kSlots]; int nj[kSlots]; int status = DASH_OK;
    GateBatcher(const dash_ctx* c_, bool g, uint32_t E_, uint32_t layer, uint64_t elem_base_, hipStream_t s_, bool mixed_ = false)
        : c(c_), garble(g), s(s_), mixed(mixed_), E(E_), elem_base(elem_base_) {
        memset(L, 0, sizeof(L));
        for (int t = 0; t < kSlots; t++) { L[t].layer = layer; nj[t] = 0; }
    }
    void launch(int t) {
        if (nj[t] && status == DASH_OK) status = garble ? launch_garble(c, L[t], nj[t], s) : launch_eval(c, L[t], nj[t], s);
        nj[t] = 0;
    }
    void add(GateJob J, bool own_range = false) {      // own_range: J.n_elem and J.elem_base are set by the caller
        if (!own_range) { J.n_elem = E; J.elem_base = elem_base; }
        int t = -1, free_slot = -1;
        for (int u = 0; u < kSlots; u++) {
            if (nj[u] && (mixed || L[u].jobs[0].q == J.q)) t = u;
            if (!nj[u] && free_slot < 0) free_slot = u;
        }
        if (t < 0) {
            if (free_slot < 0) { launch(0); free_slot = 0; }
            t = free_slot;
        } else if (nj[t] == kMaxJobs) launch(t);
        L[t].jobs[nj[t]++] = J;
    }
    void flush() { for (int t = 0; t < kSlots; t++) launch(t); }
};
struct DrawBatcher {
    const dash_ctx* c; hipStream_t s; DrawLaunch L; int nj = 0, status = DASH_OK;
    uint32_t E; uint64_t elem_base;
    DrawBatcher(const dash_ctx* c_, uint32_t E_, uint32_t layer, uint64_t elem_base_, hipStream_t s_) : c(c_), s(s_), E(E_), elem_base(elem_base_) {
        memset(&L, 0, sizeof(L));
        L.layer = layer;
    }
    void add(int m, int domain, uint32_t slot, LView out, bool digit0 = false) { add_range(m, domain, slot, out, E, elem_base, digit0); }
    void add_range(int m, int domain, uint32_t slot, LView out, uint32_t n, uint64_t base, bool digit0 = false) {
        if (nj == kMaxDrawJobs) flush();
        L.jobs[nj++] = DrawJob{(uint32_t)m, (uint32_t)domain, slot, digit0 ? 1u : 0u, out, base, n, 0u};
    }
    void flush() { if (nj && status == DASH_OK) status = launch_draw(c, L, nj, s); nj = 0; }
};
struct AffineBatcher {
    const dash_ctx* c; hipStream_t s; AffineLaunch L; int nj = 0, nt = 0, status = DASH_OK;
    AffineBatcher(const dash_ctx* c_, uint32_t E, hipStream_t s_) : c(c_), s(s_) { memset(&L, 0, sizeof(L)); L.n_elem = E; }
    void add(int m, LView out, const Term* t, int n) {
        if (nj == kMaxJobs || nt + n > kMaxTerms) flush();
        L.jobs[nj++] = AffineJob{(uint32_t)m, (uint32_t)nt, (uint32_t)n, 0, out};
        for (int i = 0; i < n; i++) L.terms[nt++] = t[i];
    }
    void flush() { if (nj && status == DASH_OK) status = launch_affine(c, L, nj, s); nj = nt = 0; }
};

GateJob phi_job(int p, int q, LView in, const uint8_t* phi, uint32_t slot, LView out, uint8_t* table) {
    GateJob J;
    memset(&J, 0, sizeof(J));
    J.p = p; J.q = q; J.in = in; J.phi = phi; J.phi_stride = 0; J.slot = slot; J.mode = PAY_PHI; J.out = out; J.table = table;
    return J;
}

// One sign gadget over E elements.  x[i]: input residues (i >= first_res).  seg: start of the gadget's
// first segment inside the layer table (already offset for the element count), offsets per slot follow
// the slot order.  On return w.bit holds [X >= P/2] (negate = 0) or its complement.
// up (optional): a second output wire, bit + up_coef * up_one.
// garbler: fresh zero labels of every gate output of a sign gadget
void sign_draws(const dash_ctx* c, DrawBatcher& db, int first_res, uint32_t slot_base, const SignWires& w) {
    const int k = c->k, n = c->n;
    for (int i = first_res; i < k; i++)
        for (int j = 1; j <= n; j++) db.add(c->mj[j], DOM_GATE, slot_base + i * n + (j - 1), w.A[i][j]);
    for (int j = n; j >= 2; j--) db.add(c->mj[j - 1], DOM_GATE, slot_base + k * n + (j - 2), w.C[j - 1]);
    db.add(2, DOM_GATE, slot_base + k * n + n - 1, w.bit);
}

// Launches of few rows are bound by the time of one lane, not by the number of lanes: gates of different output moduli
// then share a launch (the instantiation that picks the modulus' compile-time description per job).
bool few_rows(const dash_ctx* c, uint64_t rows) { return rows <= c->few_rows_max; }

int sign_core(const dash_ctx* c, bool garble, uint32_t E, uint32_t layer, uint64_t elem_base, const LView* x, int first_res,
              int negate, uint32_t slot_base, uint8_t* seg, const SignWires& w, hipStream_t s, const LView* up = nullptr,
              const LView* up_one = nullptr, uint32_t up_coef = 0, CastLaunch* pre = nullptr, int pre_jobs = 0, bool drawn = false,
              const std::function<void(AffineBatcher&)>* pre_affine = nullptr, const std::vector<GateJob>* extra_gates = nullptr) {
    // pre (evaluator of the scaling gadget): the cast-and-halve step that produces x[first_res..]; it runs in the
    // launch of the digit gates when they are fused, else in a launch of its own before them
    // drawn (garbler): the caller has drawn the zero labels (sign_draws) in a launch of its own
    // pre_affine, extra_gates (garbler): free gates and projection gates of the caller that depend on drawn labels only; they
    // share the gadget's free-gate launch and, where the launches have few rows, its launch of the carry chain's gates
    const int k = c->k, n = c->n;
    size_t off[DASH_MAX_PRIMES * DASH_MAX_DIGITS + DASH_MAX_DIGITS], cum = 0;
    for (int sl = 0; sl < sign_nslots(c); sl++) { off[sl] = cum * E; cum += sign_slot_bytes(c, sl, first_res); }

    if (garble && !drawn) {
        DrawBatcher db(c, E, layer, elem_base, s);
        sign_draws(c, db, first_res, slot_base, w);
        db.flush();
        if (db.status) return db.status;
    }
    // mixed-radix addition, least significant digit first: carry out of digit j into digit j-1.  The garbler knows every
    // zero label up front (all are drawn), so it forms all digit sums first, in one free-gate launch, and garbles the n gates
    // of the chain in one launch at the end; the evaluator has to follow the chain.
    if (garble) {
        AffineBatcher ab(c, E, s);
        if (pre_affine) (*pre_affine)(ab);
        for (int j = n; j >= 1; j--) {
            Term t[kMaxTerms];
            int nt = 0;
            for (int i = first_res; i < k; i++) t[nt++] = Term{w.A[i][j], 1};
            if (j < n) t[nt++] = Term{w.C[j], 1};
            ab.add(c->mj[j], w.S[j], t, nt);
        }
        if (up) {       // the output wire's zero label is drawn, so its shifted copy can be formed here already
            Term tu[2] = {Term{w.bit, 1}, Term{*up_one, up_coef}};
            ab.add(2, *up, tu, 2);
        }
        ab.flush();
        if (ab.status) return ab.status;
    }
    GateBatcher gb(c, garble, E, layer, elem_base, s);
    bool sums_done = false;
    // digit gates: residue i -> digit j of its rounded CRT fraction.  The n gates of a residue share their input
    // label: one launch for all k n gates, whose lanes form and compress a label once for n rows (garbler) or n
    // gates (evaluator).  Small gadgets keep one gate per lane (n times the lanes, a chain n times shorter).
    if (E < c->fused_min_elems[garble ? 0 : 1]) {
        if (pre) {
            const int st = launch_cast_halve(c, *pre, pre_jobs, s);
            if (st) return st;
        }
        for (int i = first_res; i < k; i++)
            for (int j = 1; j <= n; j++) {
                int sl = i * n + (j - 1);
                gb.add(phi_job(c->prime[i], c->mj[j], x[i], c->phi_digit[i][j], slot_base + sl, w.A[i][j], seg + off[sl]));
            }
        gb.flush();
    } else {
        DigitsLaunch DL;
        memset(&DL, 0, sizeof(DL));
        DL.n_elem = E; DL.layer = layer; DL.elem_base = elem_base; DL.n = (uint32_t)n; DL.nres = (uint32_t)(k - first_res);
        DL.out_cs = w.A[first_res][1].cs;
        for (int j = 1; j <= n; j++) {
            DL.m[j] = (uint32_t)c->mj[j];
            DL.row_prefix[j] = j == 1 ? 0 : DL.row_prefix[j - 1] + (uint32_t)pitch_of(c, c->mj[j - 1]);
            DL.out_prefix[j] = (uint64_t)(w.A[first_res][j].p - w.A[first_res][1].p);
        }
        for (int i = first_res; i < k; i++) {
            DigitsRes& R = DL.res[i - first_res];
            R.p = (uint32_t)c->prime[i]; R.slot0 = slot_base + (uint32_t)(i * n); R.in = x[i];
            R.table = seg + off[i * n]; R.out = w.A[i][1].p; R.phi = c->phi_digit[i][1];
            for (int j = 1; j <= n; j++) {     // the kernels' address rules must be the layout planned above
                if (off[i * n + j - 1] != off[i * n] + (size_t)E * c->prime[i] * DL.row_prefix[j]) return DASH_EINVAL;
                if (w.A[i][j].p != R.out + DL.out_prefix[j] || w.A[i][j].cs != DL.out_cs || w.A[i][j].es != 16u) return DASH_EINVAL;
                if (c->phi_digit[i][j] != R.phi + (size_t)(j - 1) * c->prime[i]) return DASH_EINVAL;
            }
        }
        if (!garble && n >= 2) {      // where the launch may write the digit sums itself (it says so in sums_in_launch)
            bool regular = true;
            for (int j = 1; j <= n; j++) {
                DL.sum_prefix[j] = (uint64_t)(w.S[j].p - w.S[1].p);
                if (w.S[j].p < w.S[1].p || w.S[j].cs != DL.out_cs || w.S[j].es != 16u) regular = false;
            }
            if (regular) DL.sum1 = w.S[1].p;
        }
        const int st = garble ? launch_digits_garble(c, DL, s) : pre ? launch_cast_digits_eval(c, *pre, pre_jobs, DL, s) : launch_digits_eval(c, DL, s);
        if (st) return st;
        sums_done = DL.sums_in_launch != 0;
    }
    auto sum_digit = [&](AffineBatcher& ab, int j) {
        Term t[kMaxTerms];
        int nt = 0;
        for (int i = first_res; i < k; i++) t[nt++] = Term{w.A[i][j], 1};
        if (j < n) t[nt++] = Term{w.C[j], 1};
        ab.add(c->mj[j], w.S[j], t, nt);
    };
    auto chain_gate = [&](int j) {
        if (j >= 2) {
            int sl = k * n + (j - 2);
            gb.add(phi_job(c->mj[j], c->mj[j - 1], w.S[j], c->phi_carry[j], slot_base + sl, w.C[j - 1], seg + off[sl]));
        } else {
            int sl = k * n + n - 1;
            gb.add(phi_job(c->mj[1], 2, w.S[1], c->phi_final[negate], slot_base + sl, w.bit, seg + off[sl]));
        }
    };
    if (garble) {
        uint64_t rows = 0, extra_rows = 0;
        for (int j = 1; j <= n; j++) rows += (uint64_t)E * c->mj[j];
        if (extra_gates) for (const GateJob& J : *extra_gates) extra_rows += (uint64_t)E * J.p;
        gb.mixed = few_rows(c, rows + extra_rows);
        if (extra_gates) {
            if (gb.mixed) {
                for (const GateJob& J : *extra_gates) gb.add(J);
            } else {      // a launch of their own, mixed if they are few; else one per output modulus, its compile-time code
                GateBatcher ge(c, true, E, layer, elem_base, s, few_rows(c, extra_rows));
                for (const GateJob& J : *extra_gates) ge.add(J);
                ge.flush();
                if (ge.status) return ge.status;
                gb.mixed = few_rows(c, rows);
            }
        }
        for (int j = n; j >= 1; j--) chain_gate(j);
        gb.flush();
        return gb.status;
    }
    if (n >= 2) {
        // evaluator: all digit sums (without carries) in one free-gate launch, then the whole chain in one (adding the
        // digit wires inside the chain's lanes instead was measured slower: one lane per element, its loads in a row)
        if (!sums_done) {
            AffineBatcher ab(c, E, s);
            for (int j = n; j >= 1; j--) {
                Term t[kMaxTerms];
                int nt = 0;
                for (int i = first_res; i < k; i++) t[nt++] = Term{w.A[i][j], 1};
                ab.add(c->mj[j], w.S[j], t, nt);
            }
            ab.flush();
            if (ab.status) return ab.status;
        }
        ChainLaunch CL;
        memset(&CL, 0, sizeof(CL));
        CL.n_elem = E; CL.layer = layer; CL.elem_base = elem_base; CL.n = (uint32_t)n;
        for (int j = 1; j <= n; j++) {
            const int sl = j >= 2 ? k * n + (j - 2) : k * n + n - 1;
            CL.m[j] = (uint32_t)c->mj[j];
            CL.slot[j] = slot_base + (uint32_t)sl;
            CL.table[j] = seg + off[sl];
            CL.sum[j] = w.S[j];
            if (j < n) CL.carry[j] = w.C[j];
        }
        CL.bit = w.bit;
        if (up) { CL.up = *up; CL.up_one = *up_one; CL.up_coef = up_coef; }
        return launch_chain_eval(c, CL, s);
    }
    for (int j = n; j >= 1; j--) {
        AffineBatcher ab(c, E, s);
        sum_digit(ab, j);
        ab.flush();
        if (ab.status) return ab.status;
        chain_gate(j);
        gb.flush();
    }
    if (up && gb.status == DASH_OK) {      // single-digit sets: no fused chain, a free-gate launch instead
        AffineBatcher ab(c, E, s);
        Term t[2] = {Term{w.bit, 1}, Term{*up_one, up_coef}};
        ab.add(2, *up, t, 2);
        ab.flush();
        return ab.status;
    }
    return gb.status;
}

int check_bundle(const dash_ctx* c, const dash_labels* t, int64_t n) {
    if (!t || t->n_elem < n) return DASH_EINVAL;
    for (int i = 0; i < c->k; i++)
        if (!t->data[i] || ((uintptr_t)t->data[i] & 15) || (t->chunk_stride[i] & 15) || t->chunk_stride[i] < 16 * n) return DASH_EINVAL;
    return DASH_OK;
}

// ---- ReLU ------------------------------------------------------------------------------------
struct ReluPlan { SignWires w; LView U[DASH_MAX_PRIMES], V[DASH_MAX_PRIMES]; uint8_t* r[DASH_MAX_PRIMES]; };
void plan_relu(const dash_ctx* c, Arena& ar, int64_t E, ReluPlan& p) {
    plan_sign(c, ar, E, 0, p.w);
    for (int i = 0; i < c->k; i++) {
        p.U[i] = ar.labels(c, c->prime[i], E);
        p.V[i] = ar.labels(c, c->prime[i], E);
        p.r[i] = ar.bytes((size_t)E);
    }
}

int relu_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables,
               uint8_t* scratch, hipStream_t s) {
    const int k = c->k, ns = sign_nslots(c);
    const uint32_t E = (uint32_t)L->n_elem, layer = (uint32_t)L->layer_id;
    const uint64_t eb = (uint64_t)L->elem_base;
    Arena ar{scratch, 0};
    ReluPlan pl;
    plan_relu(c, ar, E, pl);
    LView x[DASH_MAX_PRIMES];
    for (int i = 0; i < k; i++) x[i] = view_of(in, i);
    size_t cum = sign_bytes(c, 0);
    uint8_t *G[DASH_MAX_PRIMES], *Eh[DASH_MAX_PRIMES], *S[DASH_MAX_PRIMES];
    for (int i = 0; i < k; i++) {
        size_t pit = pitch_of(c, c->prime[i]);
        G[i] = tables + cum * E; cum += c->prime[i] * pit;
        Eh[i] = tables + cum * E; cum += 2 * pit;
        S[i] = tables + cum * E; cum += 8;
    }
    // pos = [X < P/2] by the sign gadget, then the half gates
    if (garble) {
        // every zero label and mask is drawn first; the half gates and the zero label of the product depend on drawn labels
        // only, so they go into the sign gadget's launches (sign_core: pre_affine, extra_gates)
        DrawBatcher db(c, E, layer, eb, s);
        sign_draws(c, db, 0, 0, pl.w);
        for (int i = 0; i < k; i++) {
            db.add(c->prime[i], DOM_GATE, ns + 3 * i, pl.U[i]);
            db.add(c->prime[i], DOM_GATE, ns + 3 * i + 1, pl.V[i]);
            db.add(c->prime[i], DOM_MASK, ns + 3 * i, LView{pl.r[i], 0, 1}, true);
        }
        db.flush();
        if (db.status) return db.status;
        std::vector<GateJob> halves;
        for (int i = 0; i < k; i++) {
            int p = c->prime[i];
            GateJob J = phi_job(p, p, x[i], nullptr, ns + 3 * i, pl.U[i], G[i]);          // garbler half: a -> a*r
            J.mode = PAY_MULR; J.r = pl.r[i];
            halves.push_back(J);
            J = phi_job(2, p, pl.w.bit, nullptr, ns + 3 * i + 1, pl.V[i], Eh[i]);         // evaluator half: -(b+r)*x0
            J.mode = PAY_EHALF; J.r = pl.r[i]; J.x0 = x[i];
            halves.push_back(J);
            J = phi_job(2, p, pl.w.bit, nullptr, ns + 3 * i + 2, pl.V[i], S[i]);          // b + r for the evaluator
            J.mode = PAY_SHORT; J.r = pl.r[i];
            halves.push_back(J);
        }
        const std::function<void(AffineBatcher&)> product = [&](AffineBatcher& ab) {         // zero label of the product: V0 - U0
            for (int i = 0; i < k; i++) {
                Term t[2] = {Term{pl.V[i], 1}, Term{pl.U[i], (uint32_t)c->prime[i] - 1}};
                ab.add(c->prime[i], view_of(out, i), t, 2);
            }
        };
        // (a caller that garbles in place, out over in, gets the product's label written after the last read of in)
        bool in_place = false;
        for (int i = 0; i < k; i++) {
            const uint8_t *a = (const uint8_t*)in->data[i], *b = (const uint8_t*)out->data[i];
            const int64_t la = in->chunk_stride[i] * c->mods[c->prime[i]].nchunk, lb = out->chunk_stride[i] * c->mods[c->prime[i]].nchunk;
            if (a < b + lb && b < a + la) in_place = true;
        }
        const int st = sign_core(c, true, E, layer, eb, x, 0, 1, 0, tables, pl.w, s, nullptr, nullptr, 0, nullptr, 0, true,
                                 in_place ? nullptr : &product, &halves);
        if (st || !in_place) return st;
        AffineBatcher ab(c, E, s);
        product(ab);
        ab.flush();
        return ab.status;
    }
    int st = sign_core(c, false, E, layer, eb, x, 0, 1, 0, tables, pl.w, s);
    if (st) return st;
    HgLaunch H;
    memset(&H, 0, sizeof(H));
    H.n_elem = E; H.layer = layer; H.elem_base = eb;
    int nj = 0;
    for (int i = 0; i < k; i++) {
        H.jobs[nj++] = HgJob{(uint32_t)c->prime[i], (uint32_t)(ns + 3 * i + 2), x[i], pl.w.bit, pl.U[i], pl.V[i], view_of(out, i), S[i], G[i], Eh[i]};
    }
    if (hg_eval_quad_wanted(c, E)) return launch_hg_eval_quad(c, H, nj, s);      // few elements: the whole half gate in one launch
    GateBatcher gb(c, false, E, layer, eb, s, true);
    for (int i = 0; i < k; i++) {
        int p = c->prime[i];
        gb.add(phi_job(p, p, x[i], nullptr, ns + 3 * i, pl.U[i], G[i]));
        gb.add(phi_job(2, p, pl.w.bit, nullptr, ns + 3 * i + 1, pl.V[i], Eh[i]));
    }
    gb.flush();
    if (gb.status) return gb.status;
    return launch_hg_finish(c, H, nj, s);
}

// ---- sign activation -------------------------------------------------------------------------
int signact_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables,
                  uint8_t* scratch, hipStream_t s) {
    const int k = c->k, ns = sign_nslots(c);
    const uint32_t E = (uint32_t)L->n_elem, layer = (uint32_t)L->layer_id;
    const uint64_t eb = (uint64_t)L->elem_base;
    Arena ar{scratch, 0};
    SignWires w;
    plan_sign(c, ar, E, 0, w);
    LView x[DASH_MAX_PRIMES];
    for (int i = 0; i < k; i++) x[i] = view_of(in, i);
    int st = sign_core(c, garble, E, layer, eb, x, 0, 0, 0, tables, w, s);
    if (st) return st;
    if (garble) {
        DrawBatcher db(c, E, layer, eb, s);
        for (int i = 0; i < k; i++) db.add(c->prime[i], DOM_GATE, ns + i, view_of(out, i));
        db.flush();
        if (db.status) return db.status;
    }
    size_t cum = sign_bytes(c, 0);
    GateBatcher gb(c, garble, E, layer, eb, s, true);
    for (int i = 0; i < k; i++) {
        gb.add(phi_job(2, c->prime[i], w.bit, c->phi_pm1[i], ns + i, view_of(out, i), tables + cum * E));
        cum += 2 * pitch_of(c, c->prime[i]);
    }
    gb.flush();
    return gb.status;
}

// ---- scaling by 2, `repeat` times ------------------------------------------------------------
struct ScalePlan { LView buf[2][DASH_MAX_PRIMES]; LView up, cast[DASH_MAX_PRIMES], b[DASH_MAX_PRIMES]; SignWires w; };
void plan_scale(const dash_ctx* c, Arena& ar, int64_t E, ScalePlan& p) {
    for (int t = 0; t < 2; t++)
        for (int i = 0; i < c->k; i++) p.buf[t][i] = ar.labels(c, c->prime[i], E);
    p.up = ar.labels(c, 2, E);
    for (int i = 1; i < c->k; i++) { p.cast[i] = ar.labels(c, c->prime[i], E); p.b[i] = ar.labels(c, c->prime[i], E); }
    plan_sign(c, ar, E, 1, p.w);
}

int scale_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables,
                uint8_t* scratch, hipStream_t s) {
    const int k = c->k, ns = sign_nslots(c);
    if (c->prime[0] != 2 || k < 2) return DASH_EUNSUPPORTED;
    if (L->repeat < 1) return DASH_EINVAL;
    const uint32_t E = (uint32_t)L->n_elem, layer = (uint32_t)L->layer_id;
    const uint64_t eb = (uint64_t)L->elem_base;
    Arena ar{scratch, 0};
    ScalePlan pl;
    plan_scale(c, ar, E, pl);
    const size_t bpe = scale_bytes(c);
    const uint32_t slots_per_rep = (uint32_t)(k - 1 + ns);
    // constant-one wires: zero labels for the garbler, active labels for the evaluator
    LView one[DASH_MAX_PRIMES];
    for (int i = 0; i < k; i++) one[i] = LView{garble ? c->d_one0[i] : c->d_one[i], 16, 0u};
    const uint64_t quarter = c->P / 4;

    // Per repetition: the casts of the mod-2 wire into the odd primes and b_i = (x_i - cast_i) / 2 (evaluator: one
    // cast-and-halve launch; garbler: the cast gates, then the halving of the zero labels as a free-gate launch), then the
    // sign gadget, whose free-gate (garbler) or chain (evaluator) launch also writes the next repetition's shifted mod-2
    // wire.  The ShiftDown of the odd residues is a constant that the next repetition's halving adds first; only the
    // last repetition writes it out.
    LView x[DASH_MAX_PRIMES];
    for (int i = 0; i < k; i++) x[i] = view_of(in, i);
    const uint32_t c0 = (uint32_t)((2 - quarter % 2) % 2);
    // ShiftUp: + P/2, i.e. +1 on the mod-2 residue only (the garbler forms it in its first free-gate launch)
    auto shift_up = [&](AffineBatcher& ab) {
        Term t[2] = {Term{x[0], 1}, Term{one[0], 1}};
        ab.add(2, pl.up, t, 2);
    };
    if (!garble) {
        AffineBatcher ab(c, E, s);
        shift_up(ab);
        ab.flush();
        if (ab.status) return ab.status;
    }
    for (int rep = 0; rep < L->repeat; rep++) {
        uint8_t* tb = tables + (size_t)rep * bpe * E;
        const uint32_t sb = rep * slots_per_rep;
        const bool last = rep == L->repeat - 1;
        // b of this repetition alternates between two buffer sets (the halving reads the one before)
        LView* bnew = rep & 1 ? pl.buf[0] : pl.b;
        const LView* bold = rep & 1 ? pl.b : pl.buf[0];
        // the shifted mod-2 wire likewise: this repetition reads one buffer (its cast gates: the garbler's run in the gadget's
        // last launch) while the sign gadget writes the next repetition's into the other
        const LView up_cur = rep & 1 ? pl.buf[1][0] : pl.up, up_next = rep & 1 ? pl.up : pl.buf[1][0];
        auto addc_of = [&](uint32_t p) { return rep == 0 ? 0u : (uint32_t)((p - quarter % p) % p); };
        size_t cum = 0;
        if (garble) {
            DrawBatcher db(c, E, layer, eb, s);      // with the zero labels of this repetition's sign gadget
            for (int i = 1; i < k; i++) db.add(c->prime[i], DOM_GATE, sb + (i - 1), pl.cast[i]);
            sign_draws(c, db, 1, sb + (k - 1), pl.w);
            db.flush();
            if (db.status) return db.status;
            // the cast gates and the halving of the zero labels depend on drawn labels only: they go into the sign gadget's
            // launches (its free-gate launch; its carry-chain launch where the rows are few)
            std::vector<GateJob> casts;
            for (int i = 1; i < k; i++) {
                casts.push_back(phi_job(2, c->prime[i], up_cur, c->phi_ident, sb + (i - 1), pl.cast[i], tb + cum * E));
                cum += 2 * pitch_of(c, c->prime[i]);
            }
            const std::function<void(AffineBatcher&)> halving = [&](AffineBatcher& ab) {
                if (rep == 0) shift_up(ab);
                for (int i = 1; i < k; i++) {
                    const uint32_t p = c->prime[i], inv2 = (p + 1) / 2, addc = addc_of(p);
                    Term t[3] = {Term{rep == 0 ? x[i] : bold[i], inv2}, Term{pl.cast[i], p - inv2}, Term{one[i], (inv2 * addc) % p}};
                    ab.add(p, bnew[i], t, addc ? 3 : 2);
                }
            };
            const uint32_t upc = (c0 + 1) % 2;
            const int st = sign_core(c, true, E, layer, eb, bnew, 1, 0, sb + (k - 1), tb + cum * E, pl.w, s, last ? nullptr : &up_next,
                                     last ? nullptr : &one[0], upc, nullptr, 0, true, &halving, &casts);
            if (st) return st;
        } else {
            CastLaunch CL;
            memset(&CL, 0, sizeof(CL));
            CL.n_elem = E; CL.layer = layer; CL.elem_base = eb; CL.y = up_cur;
            int nj = 0;
            for (int i = 1; i < k; i++) {
                const uint32_t p = c->prime[i];
                CastJob& J = CL.jobs[nj++];
                J.p = p; J.slot = sb + (i - 1); J.table = tb + cum * E;
                J.x = rep == 0 ? x[i] : bold[i];
                // the constant comes as a label of its own (the context holds addc * one): coefficient 1, a packed addition
                J.one = LView{c->d_shift[i], 16, 0u};
                J.addc = addc_of(p) ? 1u : 0u;
                J.out = bnew[i];
                cum += 2 * pitch_of(c, p);
            }
            // (k - 1 <= kMaxJobs: one launch, which sign_core merges with the digit gates' when those are fused)
            const uint32_t upc = (c0 + 1) % 2;
            const int st = sign_core(c, false, E, layer, eb, bnew, 1, 0, sb + (k - 1), tb + cum * E, pl.w, s, last ? nullptr : &up_next,
                                     last ? nullptr : &one[0], upc, &CL, nj);
            if (st) return st;
        }
        if (last) {
            AffineBatcher ab(c, E, s);
            Term t0[2] = {Term{pl.w.bit, 1}, Term{one[0], c0}};
            ab.add(2, view_of(out, 0), t0, 2);
            for (int i = 1; i < k; i++) {
                uint32_t p = c->prime[i];
                Term t[2] = {Term{bnew[i], 1}, Term{one[i], (uint32_t)((p - quarter % p) % p)}};
                ab.add(p, view_of(out, i), t, 2);
            }
            ab.flush();
            if (ab.status) return ab.status;
        }
    }
    return DASH_OK;
}

}  // namespace

int layer_sizes(const dash_ctx* c, const dash_layer* L, int64_t* out_elems, size_t* table_bytes, size_t* scratch_bytes) {
    int64_t oe = 0;
    size_t tb = 0, sb = 0;
    const int64_t E = L->n_elem;
    if (E < 0) return DASH_EINVAL;
    Arena ar{nullptr, 0};
    switch (L->kind) {
        case DASH_DENSE:
            if (L->in_c < 1 || L->out_c < 1) return DASH_EINVAL;
            oe = L->out_c; break;
        case DASH_CONV2D: {
            if (L->in_c < 1 || L->out_c < 1 || L->kh < 1 || L->kw < 1 || L->stride < 1 || L->pad < 0) return DASH_EINVAL;
            int oh = (L->in_h + 2 * L->pad - L->kh) / L->stride + 1, ow = (L->in_w + 2 * L->pad - L->kw) / L->stride + 1;
            if (oh < 1 || ow < 1) return DASH_EINVAL;
            oe = (int64_t)oh * ow * L->out_c; break;
        }
        case DASH_SUMPOOL:
            if (L->in_h < 2 || L->in_w < 2 || L->in_c < 1) return DASH_EINVAL;
            oe = (int64_t)(L->in_h / 2) * (L->in_w / 2) * L->in_c; break;
        case DASH_RELU: { ReluPlan p; plan_relu(c, ar, E, p); oe = E; tb = relu_bytes(c) * (size_t)E; sb = ar.off; break; }
        case DASH_SIGN: { SignWires w; plan_sign(c, ar, E, 0, w); oe = E; tb = signact_bytes(c) * (size_t)E; sb = ar.off; break; }
        case DASH_SCALE: {
            if (L->repeat < 1) return DASH_EINVAL;
            ScalePlan p; plan_scale(c, ar, E, p); oe = E; tb = scale_bytes(c) * (size_t)E * (size_t)L->repeat; sb = ar.off; break;
        }
        case DASH_PROJ: {
            if (L->p_index < 0 || L->p_index >= c->k || L->q_index < 0 || L->q_index >= c->k) return DASH_EINVAL;
            oe = E; tb = (size_t)E * c->prime[L->p_index] * pitch_of(c, c->prime[L->q_index]); break;
        }
        default: return DASH_EINVAL;
    }
    if (out_elems) *out_elems = oe;
    if (table_bytes) *table_bytes = tb;
    if (scratch_bytes) *scratch_bytes = sb;
    return DASH_OK;
}

// ---- packed storage format of the tables ------------------------------------------------------
// Segments of a layer's table buffer in order: (rows per gate, modulus of the rows; 0 = one-digit rows of 4 bytes)
struct SegDesc { uint32_t rows, q; };
static int table_segments(const dash_ctx* c, const dash_layer* L, std::vector<SegDesc>& out) {
    const int k = c->k, ns = sign_nslots(c);
    auto sign = [&](int first_res) {
        for (int s = 0; s < ns; s++)
            if (sign_slot_bytes(c, s, first_res)) out.push_back(SegDesc{(uint32_t)sign_slot_in(c, s), (uint32_t)sign_slot_out(c, s)});
    };
    switch (L->kind) {
        case DASH_RELU:
            sign(0);
            for (int i = 0; i < k; i++) {
                out.push_back(SegDesc{(uint32_t)c->prime[i], (uint32_t)c->prime[i]});
                out.push_back(SegDesc{2u, (uint32_t)c->prime[i]});
                out.push_back(SegDesc{2u, 0u});
            }
            return DASH_OK;
        case DASH_SIGN:
            sign(0);
            for (int i = 0; i < k; i++) out.push_back(SegDesc{2u, (uint32_t)c->prime[i]});
            return DASH_OK;
        case DASH_SCALE:
            if (L->repeat < 1) return DASH_EINVAL;
            for (int r = 0; r < L->repeat; r++) {
                for (int i = 1; i < k; i++) out.push_back(SegDesc{2u, (uint32_t)c->prime[i]});
                sign(1);
            }
            return DASH_OK;
        case DASH_PROJ:
            if (L->p_index < 0 || L->p_index >= k || L->q_index < 0 || L->q_index >= k) return DASH_EINVAL;
            out.push_back(SegDesc{(uint32_t)c->prime[L->p_index], (uint32_t)c->prime[L->q_index]});
            return DASH_OK;
        case DASH_DENSE: case DASH_CONV2D: case DASH_SUMPOOL: return DASH_OK;       // free gates: no tables
    }
    return DASH_EINVAL;
}
// every row must be below 2^128 as a base-q number
static bool rows_fit_128_bits(const dash_ctx* c, const std::vector<SegDesc>& segs) {
    for (const SegDesc& sd : segs)
        if (sd.q && !fits_128_bits(sd.q, c->mods[sd.q].lam)) return false;
    return true;
}
static inline size_t packed_seg_bytes(const SegDesc& sd, size_t E) { return sd.q ? E * sd.rows * 16 : (E * sd.rows + 15) & ~(size_t)15; }

int tables_packed_bytes(const dash_ctx* c, const dash_layer* L, size_t* bytes) {
    if (L->n_elem < 0) return DASH_EINVAL;
    std::vector<SegDesc> segs;
    const int st = table_segments(c, L, segs);
    if (st) return st;
    if (!rows_fit_128_bits(c, segs)) return DASH_EUNSUPPORTED;
    size_t b = 0;
    for (const SegDesc& sd : segs) b += packed_seg_bytes(sd, (size_t)L->n_elem);
    *bytes = b;
    return DASH_OK;
}

int tables_repack(dash_ctx* c, const dash_layer* L, bool pack, uint8_t* tables, uint8_t* packed, hipStream_t s) {
    if (L->n_elem < 0) return DASH_EINVAL;
    if (L->n_elem > 0x7fffffff) return DASH_ESIZE;
    std::vector<SegDesc> segs;
    int st = table_segments(c, L, segs);
    if (st) return st;
    if (!rows_fit_128_bits(c, segs)) return DASH_EUNSUPPORTED;
    if (L->n_elem == 0 || segs.empty()) return DASH_OK;
    if (!tables || !packed || ((uintptr_t)tables & 3) || ((uintptr_t)packed & 15)) return DASH_EINVAL;
    const size_t E = (size_t)L->n_elem;
    PackLaunch PL;
    memset(&PL, 0, sizeof(PL));
    PL.n_elem = (uint32_t)E;
    size_t toff = 0, poff = 0;
    for (const SegDesc& sd : segs) {
        if (PL.nseg == (uint32_t)kMaxPackSegs) {
            st = launch_pack(c, PL, pack, s);
            if (st) return st;
            PL.nseg = 0;
        }
        PL.seg[PL.nseg++] = PackSeg{tables + toff, packed + poff, sd.q, sd.rows};
        toff += E * sd.rows * (sd.q ? pitch_of(c, (int)sd.q) : 4);
        poff += packed_seg_bytes(sd, E);
    }
    return launch_pack(c, PL, pack, s);
}

int activation_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables,
                     uint8_t* scratch, hipStream_t s) {
    if (L->n_elem > 0x7fffffff) return DASH_ESIZE;
    if (L->n_elem == 0) return DASH_OK;
    if (c->k > 15) return DASH_EUNSUPPORTED;     // a carry gate sums k digit wires and a carry in one launch
    int st = check_bundle(c, in, L->n_elem);
    if (!st) st = check_bundle(c, out, L->n_elem);
    if (st) return st;
    if (!tables || !scratch || ((uintptr_t)tables & 3) || ((uintptr_t)scratch & 255)) return DASH_EINVAL;
    switch (L->kind) {
        case DASH_RELU: return relu_layer(c, L, garble, in, out, tables, scratch, s);
        case DASH_SIGN: return signact_layer(c, L, garble, in, out, tables, scratch, s);
        case DASH_SCALE: return scale_layer(c, L, garble, in, out, tables, scratch, s);
    }
    return DASH_EINVAL;
}

// n independent gates Z_p -> Z_q with per-gate function tables (the projection-gate microbenchmark)
static int check_proj(const dash_ctx* c, const dash_layer* L, const dash_labels* in, const dash_labels* out, const uint8_t* tables) {
    if (!L || !in || !out || L->kind != DASH_PROJ) return DASH_EINVAL;
    if (L->layer_id < 0 || L->layer_id > 65535 || L->elem_base < 0 || L->n_elem < 0) return DASH_EINVAL;
    if (L->n_elem > 0x7fffffff) return DASH_ESIZE;
    if (L->n_elem == 0) return DASH_OK;
    if (L->p_index < 0 || L->p_index >= c->k || L->q_index < 0 || L->q_index >= c->k) return DASH_EINVAL;
    if (!L->phi || !tables || ((uintptr_t)tables & 3)) return DASH_EINVAL;
    const int pi = L->p_index, qi = L->q_index, p = c->prime[pi];
    if (L->phi_stride != 0 && L->phi_stride != p) return DASH_EINVAL;
    if (!in->data[pi] || !out->data[qi] || in->n_elem < L->n_elem || out->n_elem < L->n_elem) return DASH_EINVAL;
    if (((uintptr_t)in->data[pi] & 15) || ((uintptr_t)out->data[qi] & 15) || (in->chunk_stride[pi] & 15) || (out->chunk_stride[qi] & 15) ||
        in->chunk_stride[pi] < 16 * L->n_elem || out->chunk_stride[qi] < 16 * L->n_elem) return DASH_EINVAL;
    return DASH_OK;
}

// Several independent PROJ calls at once: calls with the same layer id and output modulus share gate launches (up to
// kMaxJobs per launch, each job with its own gate count and element base), and all fresh zero labels of a layer id
// are drawn in shared launches.
int proj_layers(dash_ctx* c, bool garble, int n, const dash_layer* Ls, const dash_labels* ins, dash_labels* outs, uint8_t* const* tables,
                hipStream_t s) {
    for (int i = 0; i < n; i++) {
        const int st = check_proj(c, Ls + i, ins + i, outs + i, tables ? tables[i] : nullptr);
        if (st) return st;
    }
    std::vector<int> order;
    for (int i = 0; i < n; i++) if (Ls[i].n_elem > 0) order.push_back(i);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        if (Ls[a].layer_id != Ls[b].layer_id) return Ls[a].layer_id < Ls[b].layer_id;
        return Ls[a].q_index < Ls[b].q_index;
    });
    for (size_t r0 = 0; r0 < order.size();) {
        size_t r1 = r0;
        while (r1 < order.size() && Ls[order[r1]].layer_id == Ls[order[r0]].layer_id) r1++;
        const uint32_t layer = (uint32_t)Ls[order[r0]].layer_id;
        if (garble) {
            DrawBatcher db(c, 0, layer, 0, s);
            for (size_t r = r0; r < r1; r++) {
                const dash_layer& L = Ls[order[r]];
                db.add_range(c->prime[L.q_index], DOM_GATE, 0, view_of(outs + order[r], L.q_index), (uint32_t)L.n_elem, (uint64_t)L.elem_base);
            }
            db.flush();
            if (db.status) return db.status;
        }
        GateBatcher gb(c, garble, 0, layer, 0, s);
        for (size_t r = r0; r < r1; r++) {
            const dash_layer& L = Ls[order[r]];
            GateJob J = phi_job(c->prime[L.p_index], c->prime[L.q_index], view_of(ins + order[r], L.p_index), L.phi, 0,
                                view_of(outs + order[r], L.q_index), tables[order[r]]);
            J.phi_stride = (uint32_t)L.phi_stride;
            J.n_elem = (uint32_t)L.n_elem; J.elem_base = (uint64_t)L.elem_base;
            gb.add(J, true);
        }
        gb.flush();
        if (gb.status) return gb.status;
        r0 = r1;
    }
    return DASH_OK;
}

int proj_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables, hipStream_t s) {
    uint8_t* const tb[1] = {tables};
    return proj_layers(c, garble, 1, L, in, out, tb, s);
}

}  // namespace dash
