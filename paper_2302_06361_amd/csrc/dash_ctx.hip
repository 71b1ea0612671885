// dash_ctx.hip -- context (CRT base, label lengths, offset labels, function tables of the sign
// gadget), En / De kernels and the C ABI entry points of include/dash.h.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "dash_bodies.h"
#include "dash_hostconst.h"
#include "dash_internal.h"

using namespace dash;
using namespace dash::hostconst;

// ------------------------------------------------------------------------------------------------
// Host-side constants
// ------------------------------------------------------------------------------------------------
namespace {

int inv_mod(int a, int p) { for (int t = 1; t < p; t++) if ((a * t) % p == 1) return t; return 0; }

// Smallest-table mixed-radix digits with d_1 even, k*d_j <= 255, prod >= k*P (equal lower digits).
bool search_digits(int k, uint64_t P, const int* primes, int rule, int* n_out, int* d_out) {
    u128 need = (u128)k * P;
    int dmax = 255 / k;
    if (dmax < 2) return false;
    double best = 1e300;
    int sp = 0;
    for (int i = 0; i < k; i++) sp += primes[i];
    for (int n = 1; n <= DASH_MAX_DIGITS; n++)
        for (int d = 2; d <= dmax; d++) {
            u128 low = 1;
            for (int j = 1; j < n; j++) low *= (u128)d;
            u128 d1 = (need + low - 1) / low;
            if (d1 < 2) d1 = 2;
            if (d1 & 1) d1++;
            if (d1 > 254) continue;
            int pit_lo = 4 * ((label_length(k * d, rule) + 3) / 4), pit_1 = 4 * ((label_length((int)d1, rule) + 3) / 4);
            double cost = (double)sp * (pit_1 + (n - 1) * pit_lo) + (double)(n > 1 ? (n - 2) * k * d * pit_lo + k * d * pit_1 : 0) +
                          (double)d1 * 128;
            if (cost < best) { best = cost; *n_out = n; d_out[0] = (int)d1; for (int j = 1; j < n; j++) d_out[j] = d; }
            if (n == 1) break;
        }
    return best < 1e300;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// small kernels: offset-multiple tables, En, De
// ------------------------------------------------------------------------------------------------
namespace dash {

// R_m: force the colour digit to 1, then dtab[a][i] = packed digits of a * R_m mod m
__global__ void k_delta_tab(ModInfo M, uint8_t* delta, uint32_t* dtab) {
    uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= M.m) return;
    for (uint32_t i = 0; i < M.ndw; i++) {
        uint32_t w = *(const uint32_t*)(delta + (i >> 2) * 16 + (i & 3) * 4);
        if (i == 0) w = (w & ~0xffu) | 1u;
        dtab[a * M.ndw + i] = axpymod4(0, a, w, M);
    }
}
__global__ void k_fix_colour(uint8_t* delta) { delta[0] = 1; }

struct EncodeArgs {
    const ModInfo* mods;
    uint32_t n;
    uint32_t prime[DASH_MAX_PRIMES];      // 0: residue absent from the bundles
    LView zero[DASH_MAX_PRIMES], out[DASH_MAX_PRIMES];
    const int64_t* values;
};

// En: one lane per (value, 16-digit chunk) of one residue (blockIdx.y): active = zero + (value mod p) R_p
__global__ __launch_bounds__(kThreads) void k_encode(const EncodeArgs A) {
    const uint32_t m = A.prime[blockIdx.y];
    if (m == 0) return;
    const ModInfo M = A.mods[m];
    const uint64_t t = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint32_t ch = (uint32_t)(t / A.n), e = (uint32_t)(t - (uint64_t)ch * A.n);      // a wave's lanes: consecutive values of one chunk
    if (ch >= M.nchunk) return;
    int64_t v = A.values[e] % (int64_t)m;
    if (v < 0) v += m;
    const uint32_t* dv = M.dtab + (size_t)v * M.ndw;
    const Dw4 z = ld_chunk(A.zero[blockIdx.y], e, (int)ch);
    Dw4 w;
#pragma unroll
    for (uint32_t q = 0; q < 4; q++) w.w[q] = ch * 4 + q < M.ndw ? addmod4(z.w[q], dv[ch * 4 + q], M) : 0;
    st_chunk(A.out[blockIdx.y], e, (int)ch, w);
}

struct DecodeArgs {
    const ModInfo* mods;
    uint32_t k, n;
    uint32_t prime[DASH_MAX_PRIMES];
    uint64_t crt_part[DASH_MAX_PRIMES];   // P / p_i
    uint32_t crt_inv[DASH_MAX_PRIMES];    // (P / p_i)^-1 mod p_i
    uint64_t P;
    LView act[DASH_MAX_PRIMES], zero[DASH_MAX_PRIMES];
    int64_t* values;
    uint8_t* valid;
};

// De: 16 lanes per value, one per residue: lane (value, i) recovers the residue a_i from the colours, checks the whole
// label of residue i and forms its CRT term ((a_i * (P/p_i)^-1) mod p_i) * (P/p_i), which is below P; the value's first
// lane then adds up the terms.  (A lane per value that walked over the residues
// spent the latency of k dependent label comparisons: 37 us for the ten outputs of one inference.)
__global__ __launch_bounds__(kThreads) void k_decode(const DecodeArgs A) {
    static_assert(DASH_MAX_PRIMES == 16 && kThreads % 16 == 0, "lane roles");
    __shared__ uint32_t res[kThreads];                   // residue, or 0xffffffff for a label that is not valid
    __shared__ uint64_t term[kThreads];                  // CRT term of the residue
    const uint32_t e = blockIdx.x * (kThreads / 16) + threadIdx.x / 16, i = threadIdx.x % 16;
    uint32_t r = 0;
    if (e < A.n && i < A.k) {
        const ModInfo M = A.mods[A.prime[i]];
        const LView &a = A.act[i], &z = A.zero[i];
        uint32_t a0 = *(const uint32_t*)(a.p + (uint64_t)e * 16), z0 = *(const uint32_t*)(z.p + (uint64_t)e * 16);
        uint32_t v = mod_m((a0 & 0xff) + M.m - (z0 & 0xff), M);      // colour difference; R's colour is 1
        const uint32_t* dv = M.dtab + (size_t)v * M.ndw;
        // whole label: active = zero + v R, a 16-digit chunk (16 bytes of each label) at a time
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        uint32_t bad = 0;
        for (uint32_t ch = 0; ch < M.nchunk; ch++) {
            const u32x4 aw = *(const u32x4*)(a.p + (int64_t)ch * a.cs + (uint64_t)e * 16);
            const u32x4 zw = *(const u32x4*)(z.p + (int64_t)ch * z.cs + (uint64_t)e * 16);
#pragma unroll
            for (uint32_t q = 0; q < 4; q++) {
                const uint32_t j = 4 * ch + q;
                if (j < M.ndw) bad |= aw[q] ^ addmod4(zw[q], dv[j], M);
            }
        }
        r = bad ? 0xffffffffu : v;
        term[threadIdx.x] = (uint64_t)mod_m(v * A.crt_inv[i], M) * A.crt_part[i];
    }
    res[threadIdx.x] = r;
    __syncthreads();
    if (e >= A.n || i != 0) return;
    bool ok = true;
    uint64_t X = 0;                     // running CRT sum, kept below P
    for (uint32_t t = 0; t < A.k; t++) {
        const uint32_t v = res[threadIdx.x + t];
        if (v == 0xffffffffu) { ok = false; continue; }
        X += term[threadIdx.x + t];       // both below P < 2^62
        if (X >= A.P) X -= A.P;
    }
    int64_t s = (2 * X >= A.P) ? (int64_t)X - (int64_t)A.P : (int64_t)X;
    A.values[e] = ok ? s : 0;
    A.valid[e] = ok ? 1 : 0;
}

// 128-bit wire format (Sec. Evaluation, online communication: labels travel compressed to 128 bits;
// Sec. Implementation: compress by Horner's method): one lane per label.
__global__ __launch_bounds__(kThreads) void k_pack(const ModInfo* mods, uint32_t m, uint32_t n, LView lab, uint8_t* packed) {
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= n) return;
    const ModInfo M = mods[m];
    uint32_t colour;
    const U128 x = compress(M, [&](int i) { return *(const uint32_t*)(lab.p + (int64_t)(i >> 2) * lab.cs + (uint64_t)e * 16 + (i & 3) * 4); },
                            &colour);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    *(u32x4*)(packed + (uint64_t)e * 16) = u32x4{x.w[0], x.w[1], x.w[2], x.w[3]};
}
__global__ __launch_bounds__(kThreads) void k_unpack(const ModInfo* mods, uint32_t m, uint32_t n, const uint8_t* packed, LView lab) {
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= n) return;
    const ModInfo M = mods[m];
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = *(const u32x4*)(packed + (uint64_t)e * 16);
    const U128 x = {{v.x, v.y, v.z, v.w}};
    auto put = [&](int i, uint32_t w) { *(uint32_t*)(lab.p + (int64_t)(i >> 2) * lab.cs + (uint64_t)e * 16 + (i & 3) * 4) = w; };
    decompress(M, x, put);
    for (uint32_t i = M.ndw; i < M.nchunk * 4; i++) put((int)i, 0u);      // digits past lambda are zero in a LabelTensor
}

}  // namespace dash

// ------------------------------------------------------------------------------------------------
// Scratch memory of dash_eval_layer_noalloc: a fixed device array inside the library's code object (every GPU
// that loads the library holds its own copy until the process ends).  In host code the array's name is only a
// handle for hipGetSymbolAddress; the device address is resolved once per device, at context creation with that
// device current, and only that pointer is ever handed to kernels.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) uint8_t scratch[DASH_NOALLOC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static uint8_t* g_scratch_ptr[kMaxDevices];      // per device; written under g_scratch_lock
static std::mutex g_scratch_lock;

// the calling thread's current device must be `device`
static int resolve_scratch(int device) {
    if (device < 0 || device >= kMaxDevices) return DASH_ESIZE;
    std::lock_guard<std::mutex> lock(g_scratch_lock);
    if (g_scratch_ptr[device]) return DASH_OK;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DASH_EHIP;
    g_scratch_ptr[device] = (uint8_t*)ptr;
    return DASH_OK;
}

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" {

const char* dash_strerror(int status) {
    switch (status) {
        case DASH_OK: return "ok";
        case DASH_EINVAL: return "invalid argument";
        case DASH_ESIZE: return "size not supported";
        case DASH_EHIP: return "HIP runtime error";
        case DASH_EUNSUPPORTED: return "not implemented";
    }
    return "unknown status";
}

int dash_ctx_create(dash_ctx** out, const uint16_t* primes, int k, int lambda_rule, const uint16_t* lambda,
                    const uint8_t seed[16], const uint16_t* sign_digits, int n_digits, int hip_device) {
    if (!out || !primes || !seed || k < 1 || k > DASH_MAX_PRIMES) return DASH_EINVAL;
    if (lambda_rule != DASH_LAMBDA_CEIL && lambda_rule != DASH_LAMBDA_FLOOR) return DASH_EINVAL;
    uint64_t prod = 1;
    for (int i = 0; i < k; i++) {
        if (primes[i] < 2 || primes[i] > 127) return DASH_EINVAL;
        for (int j = 0; j < i; j++) if (primes[j] == primes[i]) return DASH_EINVAL;
        for (int t = 2; t * t <= primes[i]; t++) if (primes[i] % t == 0) return DASH_EINVAL;
        if (lambda && (lambda[i] < 1 || lambda[i] > 128)) return DASH_EINVAL;
        // P, 2 P (decode), k P (digit search) and the CRT coefficients are 64-bit numbers in this library
        if (prod > (1ull << 62) / primes[i]) return DASH_ESIZE;
        prod *= primes[i];
    }
    dash_ctx* c = new (std::nothrow) dash_ctx();
    if (!c) return DASH_EINVAL;
    memset(c, 0, sizeof(*c));
    c->device = hip_device; c->k = k; c->rule = lambda_rule;
    c->banked_min_lanes = 1u << 20;
    if (const char* e = getenv("DASH_BANKED_MIN_LANES")) c->banked_min_lanes = strtoull(e, nullptr, 10);   // tuning and test hook
    c->fused_min_elems[0] = 0; c->fused_min_elems[1] = 0;
    c->wide_max_lanes = 1u << 18;
    if (const char* e = getenv("DASH_WIDE_MAX_LANES")) c->wide_max_lanes = strtoull(e, nullptr, 10);                 // tuning and test hook
    c->sum_in_launch = 1;
    if (const char* e = getenv("DASH_SUM_IN_LAUNCH")) c->sum_in_launch = atoi(e) != 0;                               // tuning and test hook
    c->quad_max_lanes = 1u << 18;
    if (const char* e = getenv("DASH_QUAD_MAX_LANES")) c->quad_max_lanes = strtoull(e, nullptr, 10);                 // tuning and test hook
    c->few_rows_max = 1u << 20;
    if (const char* e = getenv("DASH_GARBLE_FEW_ROWS")) c->few_rows_max = strtoull(e, nullptr, 10);                 // tuning and test hook
    c->digits_banked_min_lanes = 1u << 20;
    if (const char* e = getenv("DASH_FUSED_MIN_ELEMS_GARBLE")) c->fused_min_elems[0] = strtoull(e, nullptr, 10);
    if (const char* e = getenv("DASH_FUSED_MIN_ELEMS_EVAL")) c->fused_min_elems[1] = strtoull(e, nullptr, 10);
    if (const char* e = getenv("DASH_DIGITS_BANKED_MIN_LANES")) c->digits_banked_min_lanes = strtoull(e, nullptr, 10);
    if (const char* e = getenv("DASH_GEMM_TILE")) c->gemm_tile = e[0] == 'w' ? 2 : e[0] == 'b' ? 1 : 0;      // "wide" / "big"
    c->prof = new (std::nothrow) ProfState();
    c->P = 1;
    for (int i = 0; i < k; i++) { c->prime[i] = primes[i]; c->P *= primes[i]; }

    if (sign_digits) {
        if (n_digits < 1 || n_digits > DASH_MAX_DIGITS) { delete c; return DASH_EINVAL; }
        c->n = n_digits;
        for (int j = 1; j <= n_digits; j++) c->d[j] = sign_digits[j - 1];
    } else {
        static const int fixed8[] = {26, 12, 12, 12, 12, 12, 12};
        static const int fixed12[] = {46, 17, 17, 17, 17, 17, 17, 17, 17, 17, 17};
        int dd[DASH_MAX_DIGITS];
        bool first_primes = true;
        static const int fp[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
        for (int i = 0; i < k && i < 12; i++) if (c->prime[i] != fp[i]) first_primes = false;
        if (first_primes && k == 8) { c->n = 7; memcpy(dd, fixed8, sizeof(fixed8)); }
        else if (first_primes && k == 12) { c->n = 11; memcpy(dd, fixed12, sizeof(fixed12)); }
        else if (!search_digits(k, c->P, c->prime, lambda_rule, &c->n, dd)) { delete c; return DASH_EUNSUPPORTED; }
        for (int j = 1; j <= c->n; j++) c->d[j] = dd[j - 1];
    }
    if (c->d[1] < 2 || (c->d[1] & 1) || c->d[1] > 254) { delete c; return DASH_EINVAL; }
    c->mj[1] = c->d[1];
    for (int j = 2; j <= c->n; j++) {
        if (c->d[j] < 2 || k * c->d[j] > 255) { delete c; return DASH_EINVAL; }
        c->mj[j] = k * c->d[j];
    }

    uint8_t S[256];
    uint32_t T[1024];
    make_sbox(S);
    make_ttab(S, T);
    uint8_t fixed_key[16];
    for (int i = 0; i < 16; i++) fixed_key[i] = (uint8_t)i;
    expand_key(fixed_key, S, c->fixed.rk);
    expand_key(seed, S, c->seed.rk);

    // moduli in use: 2, the primes, the accumulation moduli
    bool used[256] = {false};
    used[2] = true;
    for (int i = 0; i < k; i++) used[c->prime[i]] = true;
    for (int j = 1; j <= c->n; j++) used[c->mj[j]] = true;
    for (int m = 2; m < 256; m++) fill_modinfo(c->mods[m], m, lambda_rule);
    if (lambda)     // explicit label lengths of the CRT primes
        for (int i = 0; i < k; i++) {
            ModInfo& Mi = c->mods[c->prime[i]];
            Mi.lam = lambda[i]; Mi.nchunk = (Mi.lam + 15) / 16; Mi.ndw = (Mi.lam + 3) / 4;
        }

    // function tables of the sign gadget (Appendix, Approximated Garbled Sign)
    std::vector<uint8_t> phi;
    std::vector<size_t> off_digit((size_t)k * (c->n + 1)), off_carry(c->n + 1), off_final(2), off_pm1(k);
    u128 Mrad = 1;
    for (int j = 1; j <= c->n; j++) Mrad *= (u128)c->d[j];
    for (int i = 0; i < k; i++) {
        int p = c->prime[i];
        int inv = inv_mod((int)((c->P / p) % p), p);
        for (int j = 1; j <= c->n; j++) {
            off_digit[(size_t)i * (c->n + 1) + j] = phi.size();
            u128 w = 1;
            for (int t = c->n; t > j; t--) w *= (u128)c->d[t];
            for (int x = 0; x < p; x++) {
                int u = (x * inv) % p;
                u128 N = (Mrad * (u128)u + (u128)(p - 1)) / (u128)p;    // fraction rounded up to 1/M
                phi.push_back((uint8_t)((N / w) % (u128)c->d[j]));
            }
        }
    }
    for (int j = 2; j <= c->n; j++) {
        off_carry[j] = phi.size();
        for (int s = 0; s < c->mj[j]; s++) phi.push_back((uint8_t)((s / c->d[j]) % c->mj[j - 1]));
    }
    for (int neg = 0; neg < 2; neg++) {
        off_final[neg] = phi.size();
        for (int s = 0; s < c->mj[1]; s++) { int up = (2 * s >= c->d[1]); phi.push_back((uint8_t)(neg ? 1 - up : up)); }
    }
    size_t off_ident = phi.size();
    phi.push_back(0); phi.push_back(1);
    for (int i = 0; i < k; i++) { off_pm1[i] = phi.size(); phi.push_back(1); phi.push_back((uint8_t)(c->prime[i] == 2 ? 1 : c->prime[i] - 1)); }
    while (phi.size() % 256) phi.push_back(0);

    // device pool layout
    size_t bytes = phi.size();
    size_t off_delta[256], off_dtab[256], off_one0[DASH_MAX_PRIMES], off_one[DASH_MAX_PRIMES], off_shift[DASH_MAX_PRIMES];
    auto take = [&](size_t n) { size_t o = bytes; bytes += (n + 255) & ~(size_t)255; return o; };
    for (int m = 2; m < 256; m++) if (used[m]) {
        off_delta[m] = take(c->mods[m].nchunk * 16);
        off_dtab[m] = take((size_t)m * c->mods[m].ndw * 4);
    }
    for (int i = 0; i < k; i++) {
        off_one0[i] = take(c->mods[c->prime[i]].nchunk * 16); off_one[i] = take(c->mods[c->prime[i]].nchunk * 16);
        off_shift[i] = take(c->mods[c->prime[i]].nchunk * 16);
    }
    const size_t off_zero = take(256);
    c->pool_bytes = bytes;

    int status = DASH_EHIP;
    do {
        if (hipSetDevice(hip_device) != hipSuccess) break;
        if ((status = resolve_scratch(hip_device)) != DASH_OK) break;
        status = DASH_EHIP;
        if (hipMalloc((void**)&c->d_pool, bytes) != hipSuccess) break;
        if (hipMalloc((void**)&c->d_mods, sizeof(ModInfo) * 256) != hipSuccess) break;
        if (hipMalloc((void**)&c->d_ttab, sizeof(T)) != hipSuccess) break;
        if (hipMemset(c->d_pool, 0, bytes) != hipSuccess) break;
        if (hipMemcpy(c->d_pool, phi.data(), phi.size(), hipMemcpyHostToDevice) != hipSuccess) break;
        if (hipMemcpy(c->d_ttab, T, sizeof(T), hipMemcpyHostToDevice) != hipSuccess) break;
        for (int m = 2; m < 256; m++) if (used[m]) {
            c->d_delta[m] = c->d_pool + off_delta[m];
            c->mods[m].dtab = (const uint32_t*)(c->d_pool + off_dtab[m]);
        }
        if (hipMemcpy(c->d_mods, c->mods, sizeof(ModInfo) * 256, hipMemcpyHostToDevice) != hipSuccess) break;
        for (int i = 0; i < k; i++) {
            c->d_one0[i] = c->d_pool + off_one0[i];
            c->d_one[i] = c->d_pool + off_one[i];
            c->d_shift[i] = c->d_pool + off_shift[i];
            for (int j = 1; j <= c->n; j++) c->phi_digit[i][j] = c->d_pool + off_digit[(size_t)i * (c->n + 1) + j];
            c->phi_pm1[i] = c->d_pool + off_pm1[i];
        }
        for (int j = 2; j <= c->n; j++) c->phi_carry[j] = c->d_pool + off_carry[j];
        c->phi_final[0] = c->d_pool + off_final[0];
        c->phi_final[1] = c->d_pool + off_final[1];
        c->phi_ident = c->d_pool + off_ident;
        c->d_zero = c->d_pool + off_zero;

        // offset labels R_m and their multiples
        bool fail = false;
        for (int m = 2; m < 256 && !fail; m++) if (used[m]) {
            DrawLaunch L;
            memset(&L, 0, sizeof(L));
            L.layer = 0;
            L.jobs[0] = DrawJob{(uint32_t)m, DOM_DELTA, 0, 0, LView{c->d_delta[m], 16, 16}, 0, 1u, 0u};
            if (launch_draw(c, L, 1, 0) != DASH_OK) { fail = true; break; }
            hipLaunchKernelGGL(k_delta_tab, dim3((m + 63) / 64), dim3(64), 0, 0, c->mods[m], c->d_delta[m],
                               (uint32_t*)(c->d_pool + off_dtab[m]));
            hipLaunchKernelGGL(k_fix_colour, dim3(1), dim3(1), 0, 0, c->d_delta[m]);
        }
        if (fail) break;
        // constant-one wires: zero label from the PRG, active = zero + R_p
        for (int i = 0; i < k && !fail; i++) {
            int p = c->prime[i];
            DrawLaunch L;
            memset(&L, 0, sizeof(L));
            L.jobs[0] = DrawJob{(uint32_t)p, DOM_ONE, 0, 0, LView{c->d_one0[i], 16, 16}, 0, 1u, 0u};
            if (launch_draw(c, L, 1, 0) != DASH_OK) { fail = true; break; }
            AffineLaunch A;
            memset(&A, 0, sizeof(A));
            A.n_elem = 1;
            A.terms[0] = Term{LView{c->d_one0[i], 16, 16}, 1};
            A.terms[1] = Term{LView{c->d_delta[p], 16, 16}, 1};
            A.jobs[0] = AffineJob{(uint32_t)p, 0, 2, 0, LView{c->d_one[i], 16, 16}};
            if (launch_affine(c, A, 1, 0) != DASH_OK) { fail = true; break; }
            // the constant that the scaling gadget's halving adds from its second repetition on (Sec. The Scaling Operation,
            // ShiftDown by floor(P / 4)), as a label: (-floor(P / 4) mod p) * one
            memset(&A, 0, sizeof(A));
            A.n_elem = 1;
            A.terms[0] = Term{LView{c->d_one[i], 16, 16}, (uint32_t)(((uint64_t)p - (c->P / 4) % (uint64_t)p) % (uint64_t)p)};
            A.jobs[0] = AffineJob{(uint32_t)p, 0, 1, 0, LView{c->d_shift[i], 16, 16}};
            if (launch_affine(c, A, 1, 0) != DASH_OK) { fail = true; break; }
        }
        if (fail) break;
        if (hipDeviceSynchronize() != hipSuccess) break;
        status = DASH_OK;
    } while (0);
    if (status != DASH_OK) { dash_ctx_destroy(c); return status; }
    *out = c;
    return DASH_OK;
}

void dash_ctx_destroy(dash_ctx* c) {
    if (!c) return;
    if (c->d_pool) (void)hipFree(c->d_pool);
    if (c->d_mods) (void)hipFree(c->d_mods);
    if (c->d_ttab) (void)hipFree(c->d_ttab);
    if (c->prof) {
        for (int kd = 0; kd < DASH_PROF_KINDS; kd++)
            for (auto& r : c->prof->rec[kd]) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (auto e : c->prof->pool) (void)hipEventDestroy(e);
        delete c->prof;
    }
    delete c;
}

int dash_profile_enable(dash_ctx* c, int on) {
    if (!c || !c->prof) return DASH_EINVAL;
    c->prof->on = on != 0;
    return DASH_OK;
}
int dash_profile_read(dash_ctx* c, int kind, double* ms, int64_t* launches, double* units, double* alg_bytes) {
    if (!c || !c->prof || kind < 0 || kind >= DASH_PROF_KINDS) return DASH_EINVAL;
    double t = 0, u = 0, b = 0;
    auto& v = c->prof->rec[kind];
    for (auto& r : v) {
        DASH_HIP(hipEventSynchronize(r.b));
        float dt = 0;
        DASH_HIP(hipEventElapsedTime(&dt, r.a, r.b));
        t += dt; u += r.units; b += r.bytes;
        c->prof->pool.push_back(r.a); c->prof->pool.push_back(r.b);
    }
    if (ms) *ms = t;
    if (launches) *launches = (int64_t)v.size();
    if (units) *units = u;
    if (alg_bytes) *alg_bytes = b;
    v.clear();
    return DASH_OK;
}

int dash_lambda(const dash_ctx* c, int m) { return (c && m >= 2 && m <= 255) ? (int)c->mods[m].lam : 0; }

static int copy_label_to_host(const dash_ctx* c, const uint8_t* dev, int m, uint8_t* host) {
    uint8_t buf[128];
    DASH_HIP(hipMemcpy(buf, dev, c->mods[m].nchunk * 16, hipMemcpyDeviceToHost));
    memcpy(host, buf, c->mods[m].lam);
    return DASH_OK;
}
int dash_ctx_offset(const dash_ctx* c, int m, uint8_t* host_out) {
    if (!c || !host_out || m < 2 || m > 255 || !c->d_delta[m]) return DASH_EINVAL;
    return copy_label_to_host(c, c->d_delta[m], m, host_out);
}
int dash_ctx_one(const dash_ctx* c, int i, int which, uint8_t* host_out) {
    if (!c || !host_out || i < 0 || i >= c->k || which < 0 || which > 1) return DASH_EINVAL;
    return copy_label_to_host(c, which ? c->d_one[i] : c->d_one0[i], c->prime[i], host_out);
}
int dash_ctx_digits(const dash_ctx* c, uint16_t* host_digits) {
    if (!c || !host_digits) return DASH_EINVAL;
    for (int j = 1; j <= c->n; j++) host_digits[j - 1] = (uint16_t)c->d[j];
    return c->n;
}

static int check_labels(const dash_ctx* c, const dash_labels* t, int64_t n, int only = -1) {
    if (!t || t->n_elem < n) return DASH_EINVAL;
    for (int i = 0; i < c->k; i++) {
        if (only >= 0 && i != only) continue;
        if (n > 0 && !t->data[i]) return DASH_EINVAL;
        if (((uintptr_t)t->data[i] & 15) || (t->chunk_stride[i] & 15) || t->chunk_stride[i] < 16 * n) return DASH_EINVAL;
    }
    return DASH_OK;
}

int dash_input_labels(dash_ctx* c, int64_t first_wire, int64_t n, dash_labels* zero, void* stream) {
    if (!c || !zero || first_wire < 0 || n < 0 || n > zero->n_elem) return DASH_EINVAL;
    if (n > 0x7fffffff) return DASH_ESIZE;
    int st = check_labels(c, zero, n);
    if (st) return st;
    DrawLaunch L;
    memset(&L, 0, sizeof(L));
    L.layer = 0;
    for (int i = 0; i < c->k; i++) L.jobs[i] = DrawJob{(uint32_t)c->prime[i], DOM_INPUT, 0, 0, view_of(zero, i), (uint64_t)first_wire, (uint32_t)n, 0u};
    return launch_draw(c, L, c->k, (hipStream_t)stream);
}

int dash_encode(dash_ctx* c, const int64_t* values, int64_t n, const dash_labels* zero, dash_labels* out, void* stream) {
    if (!c || !zero || !out || (!values && n > 0) || n < 0) return DASH_EINVAL;
    if (n > 0x7fffffff) return DASH_ESIZE;
    if (zero->n_elem < n || out->n_elem < n) return DASH_EINVAL;
    for (int i = 0; i < c->k; i++) {
        if (!zero->data[i] && !out->data[i]) continue;      // residue not present in either bundle: skipped
        int st = check_labels(c, zero, n, i);
        if (!st) st = check_labels(c, out, n, i);
        if (st) return st;
    }
    if (n == 0) return DASH_OK;
    EncodeArgs A;
    memset(&A, 0, sizeof(A));
    A.mods = c->d_mods; A.n = (uint32_t)n; A.values = values;
    uint32_t nchunk = 0;
    for (int i = 0; i < c->k; i++) {
        if (!zero->data[i] && !out->data[i]) continue;
        A.prime[i] = (uint32_t)c->prime[i]; A.zero[i] = view_of(zero, i); A.out[i] = view_of(out, i);
        nchunk = std::max(nchunk, c->mods[c->prime[i]].nchunk);
    }
    if (nchunk == 0) return DASH_OK;
    hipLaunchKernelGGL(k_encode, dim3((uint32_t)(((uint64_t)n * nchunk + kThreads - 1) / kThreads), (uint32_t)c->k), dim3(kThreads), 0,
                       (hipStream_t)stream, A);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

int dash_decode(dash_ctx* c, const dash_labels* act, const dash_labels* zero, int64_t n, int64_t* values, uint8_t* valid,
                void* stream) {
    if (!c || n < 0 || (n > 0 && (!values || !valid))) return DASH_EINVAL;
    if (n > 0x7fffffff) return DASH_ESIZE;
    int st = check_labels(c, act, n);
    if (!st) st = check_labels(c, zero, n);
    if (st) return st;
    if (n == 0) return DASH_OK;
    DecodeArgs A;
    memset(&A, 0, sizeof(A));
    A.mods = c->d_mods; A.k = c->k; A.n = (uint32_t)n; A.P = c->P; A.values = values; A.valid = valid;
    for (int i = 0; i < c->k; i++) {
        int p = c->prime[i];
        uint64_t Ai = c->P / p;
        A.prime[i] = p;
        A.crt_part[i] = Ai;
        A.crt_inv[i] = (uint32_t)inv_mod((int)(Ai % p), p);
        A.act[i] = view_of(act, i);
        A.zero[i] = view_of(zero, i);
    }
    hipLaunchKernelGGL(k_decode, dim3((uint32_t)((n + kThreads / 16 - 1) / (kThreads / 16))), dim3(kThreads), 0, (hipStream_t)stream, A);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

static int pack_args(const dash_ctx* c, const dash_labels* labels, const void* packed, int64_t n) {
    if (!c || n < 0 || (n > 0 && !packed)) return DASH_EINVAL;
    if (n > 0x7fffffff) return DASH_ESIZE;
    if ((uintptr_t)packed & 15) return DASH_EINVAL;
    const int st = check_labels(c, labels, n);
    if (st) return st;
    for (int i = 0; i < c->k; i++) {
        const ModInfo& M = c->mods[c->prime[i]];
        if (labels->data[i] && !dash::fits_128_bits(M.m, M.lam)) return DASH_EUNSUPPORTED;
    }
    return DASH_OK;
}

int dash_labels_pack(dash_ctx* c, const dash_labels* labels, int64_t n, void* packed, void* stream) {
    const int st = pack_args(c, labels, packed, n);
    if (st || n == 0) return st;
    for (int i = 0; i < c->k; i++) {
        if (!labels->data[i]) continue;
        hipLaunchKernelGGL(k_pack, dim3((uint32_t)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, (hipStream_t)stream, c->d_mods,
                           (uint32_t)c->prime[i], (uint32_t)n, view_of(labels, i), (uint8_t*)packed + (size_t)i * (size_t)n * 16);
    }
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

int dash_labels_unpack(dash_ctx* c, const void* packed, int64_t n, dash_labels* labels, void* stream) {
    const int st = pack_args(c, labels, packed, n);
    if (st || n == 0) return st;
    for (int i = 0; i < c->k; i++) {
        if (!labels->data[i]) continue;
        hipLaunchKernelGGL(k_unpack, dim3((uint32_t)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, (hipStream_t)stream, c->d_mods,
                           (uint32_t)c->prime[i], (uint32_t)n, (const uint8_t*)packed + (size_t)i * (size_t)n * 16, view_of(labels, i));
    }
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

int dash_layer_sizes(const dash_ctx* c, const dash_layer* L, int64_t* out_elems, size_t* table_bytes, size_t* scratch_bytes) {
    if (!c || !L) return DASH_EINVAL;
    return layer_sizes(c, L, out_elems, table_bytes, scratch_bytes);
}

static int run_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, uint8_t* tables,
                     uint8_t* scratch, hipStream_t s) {
    if (!c || !L || !in || !out) return DASH_EINVAL;
    if (L->layer_id < 0 || L->layer_id > 65535 || L->elem_base < 0 || L->n_elem < 0) return DASH_EINVAL;
    switch (L->kind) {
        case DASH_DENSE: case DASH_CONV2D: case DASH_SUMPOOL: return linear_layer(c, L, garble, in, out, s);
        case DASH_RELU: case DASH_SCALE: case DASH_SIGN: return activation_layer(c, L, garble, in, out, tables, scratch, s);
        case DASH_PROJ: return proj_layer(c, L, garble, in, out, tables, s);
    }
    return DASH_EINVAL;
}

int dash_garble_layer(dash_ctx* c, const dash_layer* L, const dash_labels* in_zero, dash_labels* out_zero, void* tables,
                      void* scratch, void* stream) {
    return run_layer(c, L, true, in_zero, out_zero, (uint8_t*)tables, (uint8_t*)scratch, (hipStream_t)stream);
}
int dash_eval_layer(dash_ctx* c, const dash_layer* L, const dash_labels* in_act, const void* tables, dash_labels* out_act,
                    void* scratch, void* stream) {
    return run_layer(c, L, false, in_act, out_act, (uint8_t*)tables, (uint8_t*)scratch, (hipStream_t)stream);
}


size_t dash_tables_packed_bytes(const dash_ctx* c, const dash_layer* L) {
    size_t b = 0;
    if (!c || !L || tables_packed_bytes(c, L, &b) != DASH_OK) return 0;
    return b;
}
int dash_tables_pack(dash_ctx* c, const dash_layer* L, const void* tables, void* packed, void* stream) {
    if (!c || !L) return DASH_EINVAL;
    return tables_repack(c, L, true, (uint8_t*)tables, (uint8_t*)packed, (hipStream_t)stream);
}
int dash_tables_unpack(dash_ctx* c, const dash_layer* L, const void* packed, void* tables, void* stream) {
    if (!c || !L) return DASH_EINVAL;
    return tables_repack(c, L, false, (uint8_t*)tables, (uint8_t*)packed, (hipStream_t)stream);
}

// n independent layer calls: lists of PROJ calls go to the launcher that merges them, anything else is run in turn
static int run_layers(dash_ctx* c, bool garble, int n, const dash_layer* Ls, const dash_labels* ins, dash_labels* outs, void* const* tables,
                      void* const* scratch, hipStream_t s) {
    if (!c || n < 0 || (n > 0 && (!Ls || !ins || !outs))) return DASH_EINVAL;
    bool all_proj = n > 0;
    for (int i = 0; i < n; i++) if (Ls[i].kind != DASH_PROJ) all_proj = false;
    if (all_proj) return proj_layers(c, garble, n, Ls, ins, outs, (uint8_t* const*)tables, s);
    for (int i = 0; i < n; i++) {
        const int st = run_layer(c, Ls + i, garble, ins + i, outs + i, tables ? (uint8_t*)tables[i] : nullptr,
                                 scratch ? (uint8_t*)scratch[i] : nullptr, s);
        if (st) return st;
    }
    return DASH_OK;
}
int dash_garble_layers(dash_ctx* c, int n, const dash_layer* layers, const dash_labels* in_zero, dash_labels* out_zero, void* const* tables,
                       void* const* scratch, void* stream) {
    return run_layers(c, true, n, layers, in_zero, out_zero, tables, scratch, (hipStream_t)stream);
}
int dash_eval_layers(dash_ctx* c, int n, const dash_layer* layers, const dash_labels* in_act, const void* const* tables, dash_labels* out_act,
                     void* const* scratch, void* stream) {
    return run_layers(c, false, n, layers, in_act, out_act, (void* const*)tables, scratch, (hipStream_t)stream);
}

int dash_eval_layer_noalloc(dash_ctx* c, const dash_layer* L, const dash_labels* in_act, const void* tables, dash_labels* out_act,
                            void* stream) {
    if (!c || !L) return DASH_EINVAL;
    size_t need = 0;
    const int st = layer_sizes(c, L, nullptr, nullptr, &need);
    if (st) return st;
    if (need > (size_t)DASH_NOALLOC_SCRATCH_BYTES) return DASH_ESIZE;
    if (c->device < 0 || c->device >= kMaxDevices) return DASH_ESIZE;
    uint8_t* ptr = g_scratch_ptr[c->device];       // resolved by dash_ctx_create on this device
    if (!ptr) return DASH_EHIP;
    return run_layer(c, L, false, in_act, out_act, (uint8_t*)tables, ptr, (hipStream_t)stream);
}

}  // extern "C"
