// dash_internal.h -- host-side structures shared by the translation units of libdash.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/dash.h"
#include "../../include/dash_profile.h"
#include "dash_core.h"
#include "dash_launch.h"

namespace dash {
// benchmark instrumentation: event pairs around the launches of one kernel class
struct ProfRec { hipEvent_t a, b; double units, bytes; };
struct ProfState {
    bool on = false;
    std::vector<ProfRec> rec[DASH_PROF_KINDS];
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
};
struct ProfScope {      // records the first event at construction, the second at destruction
    ProfState* p; int kind; hipStream_t s; ProfRec r;
    ProfScope(ProfState* p_, int kind_, hipStream_t s_, double units, double bytes) : p(p_ && p_->on ? p_ : nullptr), kind(kind_), s(s_) {
        if (!p) return;
        r.a = p->get(); r.b = p->get(); r.units = units; r.bytes = bytes;
        (void)hipEventRecord(r.a, s);
    }
    ~ProfScope() { if (p) { (void)hipEventRecord(r.b, s); p->rec[kind].push_back(r); } }
};
}  // namespace dash

struct dash_ctx {
    int device;
    dash::ProfState* prof;
    int k;
    int prime[DASH_MAX_PRIMES];
    int rule;
    int n;                           // mixed-radix digits
    int d[DASH_MAX_DIGITS + 1];      // 1-based
    int mj[DASH_MAX_DIGITS + 1];
    uint64_t P;
    dash::ModInfo mods[256];         // host copy (dtab = device pointers)
    dash::AesKey fixed, seed;
    // device memory owned by the context
    dash::ModInfo* d_mods;
    uint32_t* d_ttab;
    uint8_t* d_pool;                 // offset labels, delta tables, constant wires, function tables
    size_t pool_bytes;
    uint8_t* d_delta[256];           // chunked label of R_m (nchunk*16 bytes)
    uint8_t* d_one0[DASH_MAX_PRIMES];
    uint8_t* d_one[DASH_MAX_PRIMES];
    uint8_t* d_shift[DASH_MAX_PRIMES];   // (-floor(P / 4) mod p) times the active one-label: the ShiftDown constant of the scaling gadget, evaluator's side
    // function tables (device)
    const uint8_t* phi_digit[DASH_MAX_PRIMES][DASH_MAX_DIGITS + 1];  // [i][j] -> [p_i]
    const uint8_t* phi_carry[DASH_MAX_DIGITS + 1];                   // [j] -> [m_j], j = 2..n
    const uint8_t* phi_final[2];                                     // [negate] -> [m_1]
    const uint8_t* phi_ident;                                        // {0, 1}
    const uint8_t* d_zero;                                           // 256 zero bytes
    uint64_t banked_min_lanes;       // launches of this many lanes or more use the bank-replicated AES tables
    uint64_t fused_min_elems[2];     // [garble, eval]: sign gadgets over this many elements or more run their digit gates in
                                     // the fused kernels (a lane walks the n gates of a residue); smaller ones one gate per lane
    uint64_t wide_max_lanes;         // evaluator: sign gadgets of at most this many digit gates run them one per lane
    int sum_in_launch;               // evaluator: digit gates of few elements add up their outputs in their own launch (1) or leave
                                     // it to a free-gate launch (0)
    uint64_t quad_max_lanes;         // evaluator: carry chains of at most this many lanes (4 per element) run four lanes per element
    uint64_t few_rows_max;           // garbler: launches of at most this many rows take the forms for few rows (a lane per row of the
                                     // digit gates; gates of different output moduli in one launch)
    uint64_t digits_banked_min_lanes;   // the banked-table threshold of the fused garbling kernel (n hashes per lane)
    const uint8_t* phi_pm1[DASH_MAX_PRIMES];                         // {1, p-1}
    int gemm_tile;                   // tile shape of the MFMA contraction: 0 by layer shape, 1 big, 2 wide (tuning and test hook)
};

namespace dash {

#define DASH_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return DASH_EHIP; } while (0)

// launch helpers (dash_gates.hip).  Each checks its own limits and returns a dash status.
int launch_draw(const dash_ctx* c, DrawLaunch& L, int njobs, hipStream_t s);
int launch_affine(const dash_ctx* c, AffineLaunch& L, int njobs, hipStream_t s);
int launch_garble(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s);
int launch_eval(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s);
int launch_chain_eval(const dash_ctx* c, ChainLaunch& L, hipStream_t s);
int launch_digits_eval(const dash_ctx* c, DigitsLaunch& L, hipStream_t s);
int launch_digits_garble(const dash_ctx* c, DigitsLaunch& L, hipStream_t s);
int launch_cast_halve(const dash_ctx* c, CastLaunch& L, int njobs, hipStream_t s);
int launch_cast_digits_eval(const dash_ctx* c, CastLaunch& C, int njobs, DigitsLaunch& L, hipStream_t s);
int launch_hg_finish(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s);
bool digits_sum_wanted(const DigitsLaunch& L, int typed);
bool hg_eval_quad_wanted(const dash_ctx* c, uint32_t n_elem);
int launch_hg_eval_quad(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s);

// layer pipelines (dash_layers.hip)
int layer_sizes(const dash_ctx* c, const dash_layer* L, int64_t* out_elems, size_t* table_bytes, size_t* scratch_bytes);
int activation_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out,
                     uint8_t* tables, uint8_t* scratch, hipStream_t s);
int proj_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out,
               uint8_t* tables, hipStream_t s);
int proj_layers(dash_ctx* c, bool garble, int n, const dash_layer* Ls, const dash_labels* ins, dash_labels* outs, uint8_t* const* tables,
                hipStream_t s);

// packed table format (dash_layers.hip)
int tables_packed_bytes(const dash_ctx* c, const dash_layer* L, size_t* bytes);
int tables_repack(dash_ctx* c, const dash_layer* L, bool pack, uint8_t* tables, uint8_t* packed, hipStream_t s);
int launch_pack(const dash_ctx* c, PackLaunch& L, bool pack, hipStream_t s);

// linear layers (dash_linear.hip)
int linear_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, hipStream_t s);
// dense layers on the matrix cores (dash_gemm.hip)
bool dense_mfma_wanted(const dash_layer* L, int64_t batch);
int dense_mfma(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, hipStream_t s);

// true if every vector of lam digits below m is below 2^128 as a base-m number (m^lam <= 2^128)
inline bool fits_128_bits(uint32_t m, uint32_t lam) {
    if ((m & (m - 1)) == 0) { uint32_t t = 0; while ((1u << t) < m) t++; return t * lam <= 128; }
    unsigned __int128 r = 1;
    for (uint32_t j = 0; j < lam; j++) {
        if (r > ~(unsigned __int128)0 / m) return false;
        r *= m;
    }
    return true;
}

inline LView view_of(const dash_labels* t, int i) { return LView{(uint8_t*)t->data[i], t->chunk_stride[i], 16u}; }

}  // namespace dash
