// dash_launch.h -- argument blocks of the gate kernels (plain C++: shared by the HIP translation units
// and by the host build of the kernel bodies that the CPU test suite runs).
#pragma once
#include <stdint.h>

#include "dash_core.h"

namespace dash {

constexpr int kMaxJobs = 16;    // gate batches per launch (blockIdx.y)
constexpr int kMaxDrawJobs = 64;   // label draws per launch: all fresh zero labels of a base-8 sign gadget (their jobs are small)
constexpr int kMaxTerms = 96;   // label terms per launch, shared by its jobs
constexpr int kThreads = 256;
constexpr int kMaxChain = 16;   // mixed-radix digits of the sign gadget

// PRG domains (byte 14 of the counter block)
enum { DOM_DELTA = 0, DOM_INPUT = 1, DOM_GATE = 2, DOM_MASK = 3, DOM_ONE = 4 };

// A view of a LabelTensor of one modulus: digit j of element e at p + (j/16)*cs + e*es + j%16.
struct LView {
    uint8_t* p;
    int64_t cs;    // chunk stride in bytes
    uint32_t es;   // element stride in bytes: 16, or 0 for a single label broadcast to all elements
};
struct Term {
    LView v;
    uint32_t coef;   // in [0, m)
};

// Payload modes of the garble kernel
enum { PAY_PHI = 0,     // out0 + phi(a) * R_q
       PAY_MULR = 1,    // out0 + (a * r mod q) * R_q            (garbler half gate)
       PAY_EHALF = 2,   // out0 - ((a + r) mod q) * x0           (evaluator half gate)
       PAY_SHORT = 3 }; // one digit: (a + r) mod q, 4-byte rows  (evaluator's known input)

struct GateJob {
    uint32_t p, q;            // input / output modulus
    LView in;                 // labels of the input wires (zero labels for garble, active for eval)
    const uint8_t* phi;       // PAY_PHI
    uint32_t phi_stride;
    uint32_t slot;
    uint32_t mode;
    uint32_t pad_;
    LView out;                // garble: zero labels of the output wires (read); eval: output labels (written)
    uint8_t* table;           // segment base
    const uint8_t* r;         // PAY_MULR / EHALF / SHORT: mask per element
    LView x0;                 // PAY_EHALF: zero labels of the x wire
    uint64_t elem_base;       // index of the job's gate 0 inside its layer (hash tweaks)
    uint32_t n_elem;          // gates of this job (the jobs of one launch may differ in size)
    uint32_t pad2_;
};

struct AesKey { uint32_t rk[44]; };

struct GateLaunch {
    AesKey key;
    const uint32_t* ttab;       // device [4][256]
    const ModInfo* mods;        // device [256]
    uint32_t layer;
    uint32_t njobs;             // set by the launcher
    GateJob jobs[kMaxJobs];
};

struct DrawJob {
    uint32_t m, domain, slot, digit0_only;
    LView out;       // digit0_only: out.p is a byte array [n_elem]
    uint64_t elem_base;   // PRG counter of the job's element 0
    uint32_t n_elem;      // labels of this job (the jobs of one launch may differ in size)
    uint32_t pad_;
};
struct DrawLaunch {
    AesKey key;
    const uint32_t* ttab;
    const ModInfo* mods;
    uint32_t layer;
    uint32_t pad_;
    DrawJob jobs[kMaxDrawJobs];
};

struct AffineJob {
    uint32_t m, term_first, term_count;
    uint32_t unit;       // 1 if every coefficient is 1
    LView out;
};
struct AffineLaunch {
    const ModInfo* mods;
    uint32_t n_elem;
    Term terms[kMaxTerms];
    AffineJob jobs[kMaxJobs];
};

// half-gate evaluation: z = V + beta * x - U, beta = S[colour(y)] - H_p(y, slot)[0]
struct HgJob {
    uint32_t p, slot;
    LView x, y, U, V, z;
    const uint8_t* S;     // [elem][2][4]
    // the two projection gates in front (the whole half gate in one launch, hg_eval_quad_body): garbler half [elem][p] rows
    // with slot - 2, evaluator half [elem][2] rows with slot - 1; U and V are not stored then
    const uint8_t *G, *Eh;
};
struct HgLaunch {
    AesKey key;
    const uint32_t* ttab;
    const ModInfo* mods;
    uint64_t elem_base;
    uint32_t layer;
    uint32_t n_elem;
    HgJob jobs[kMaxJobs];
};

// evaluator side of the mixed-radix addition of one sign gadget (Appendix, Garbled Mixed-Radix Addition):
// digits n..1 in turn, one lane per element
struct ChainLaunch {
    AesKey key;
    const uint32_t* ttab;
    const ModInfo* mods;
    uint64_t elem_base;
    uint32_t layer;
    uint32_t n_elem;
    uint32_t n;                          // digits
    uint32_t m[kMaxChain + 1];           // accumulation modulus of digit j (1-based)
    uint32_t slot[kMaxChain + 1];        // slot of the gate that digit j feeds (carry gate for j >= 2, final gate for j = 1)
    uint8_t* table[kMaxChain + 1];       // its segment
    LView sum[kMaxChain + 1];            // free sum of the digit wires of digit j, WITHOUT the carry
    LView carry[kMaxChain + 1];          // carry into digit j (j < n): written by gate j+1, read back by the same lane
    LView bit;                           // output wire (Z_2)
    // optional second output: up = bit + up_coef * up_one (the shifts of the scaling gadget on the mod-2 residue)
    LView up, up_one;
    uint32_t up_coef, pad_;
};

// evaluator, scaling gadget (Sec. The Scaling Operation): cast of the mod-2 wire y into Z_p (a two-row
// gate) and the halving that uses it, b = (x + addc * one - cast) / 2 mod p, one lane per (element, odd prime)
struct CastJob {
    uint32_t p, slot;
    uint8_t* table;          // [elem][2][pitch_p]
    LView x, one, out;       // residue of the value, constant-one wire of the prime, b
    uint32_t addc, pad_;     // constant added to x first (the ShiftDown of the repetition before), in [0, p)
};
struct CastLaunch {
    AesKey key;
    const uint32_t* ttab;
    const ModInfo* mods;
    uint64_t elem_base;
    uint32_t layer;
    uint32_t n_elem;
    LView y;
    CastJob jobs[kMaxJobs];
};

// packed storage format of ciphertext tables: every row of a segment, a vector in Z_q^lambda, as the 128-bit integer
// sum_j row[j] q^j (Sec. Implementation, compress), 16 bytes per row; the one-digit rows of a half gate as one byte
struct PackSeg {
    const uint8_t* rows;     // the segment in the working format: [gate][row][pitch_q]  (pack: read; unpack: written)
    uint8_t* packed;         // the segment in the packed format: [gate][row][16]        (pack: written; unpack: read)
    uint32_t q;              // modulus of the rows; 0 = one-digit rows (4 bytes <-> 1 byte)
    uint32_t rows_per_gate;
};
constexpr int kMaxPackSegs = 96;
struct PackLaunch {
    const ModInfo* mods;
    uint32_t n_elem, nseg;
    PackSeg seg[kMaxPackSegs];
};

// the digit gates of one sign gadget (Appendix, approximated sign: residue i -> digit j of its
// rounded CRT fraction): the n gates of a residue share their input label, so one lane takes (element, residue),
// compresses the label once and evaluates its n gates (the garbler: one lane per (element, value a, residue)).  Output wire (i, j) and table segment (i, j) are at fixed
// offsets from those of (i, 1).
struct DigitsRes {
    uint32_t p, slot0;       // input modulus; slot of the gate to digit 1 (digit j: slot0 + j - 1)
    LView in;                // label of the residue: active (evaluator) or zero label (garbler)
    uint8_t* table;          // segment of gate (i, 1)
    uint8_t* out;            // label tensor of wire (i, 1)
    const uint8_t* phi;      // garbler: function tables [n][p] of the residue's gates
};
struct DigitsLaunch {
    AesKey key;
    const uint32_t* ttab;
    const ModInfo* mods;
    uint64_t elem_base;
    uint32_t layer;
    uint32_t n_elem;
    uint32_t n, nres;
    uint32_t m[kMaxChain + 1];            // accumulation modulus of digit j (1-based)
    uint32_t row_prefix[kMaxChain + 1];   // sum of the row pitches of digits 1 .. j-1: segment (i, j) starts
                                          // n_elem * p_i * row_prefix[j] bytes after segment (i, 1)
    uint64_t out_prefix[kMaxChain + 1];   // wire (i, j) starts this many bytes after wire (i, 1)
    int64_t out_cs;                       // chunk stride of the output wires
    // evaluator, optional: the wires S_j = sum over the residues of the digit wires (i, j) mod m_j, which the launch
    // writes as well when it takes the form that adds them up itself (then it sets sums_in_launch and stores no digit wire)
    uint8_t* sum1;                        // label tensor of S_1 (chunk stride out_cs), or null
    uint64_t sum_prefix[kMaxChain + 1];   // S_j starts this many bytes after S_1
    uint32_t sums_in_launch;
    DigitsRes res[16];
};

}  // namespace dash

