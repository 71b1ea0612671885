// dash_linear.hip -- the "free" linear layers on LabelTensors (Sec. Arithmetic Garbled Circuits: free
// addition and multiplication by a public constant; Sec. System-level Architecture: Dense and Conv2D;
// the Conv2D figure of Sec. LabelTensors): per CRT prime p
//     out[b][oy][ox][co][digit] = sum_{ky,kx,ci} (W[co][ky][kx][ci] mod p) * in[b][iy][ix][ci][digit]
//                                 (+ (bias[co] mod p) * one[digit])        mod p
// The garbler applies it to zero labels, the evaluator to active labels; the arithmetic is the same.
//
//   k_weights_prepare : int32 weights -> per-prime int8 residues in [0, p), rows padded to 64
//   k_linear_direct   : any shape; one lane per (output value, 16-digit chunk)
//   (dense layers that fill MFMA tiles go to k_dense_mfma in dash_gemm.hip)
//   k_sumpool         : 2x2 sum, stride 2
#include <string.h>

#include "dash_internal.h"

namespace dash {

constexpr int kKpad = 64;   // weight rows are padded to a multiple of 64 entries

__host__ __device__ inline int64_t kpad_of(int K) { return ((int64_t)K + kKpad - 1) / kKpad * kKpad; }
__host__ __device__ inline int64_t mpad_of(int M) { return ((int64_t)M + 31) / 32 * 32; }

struct PrepArgs {
    const int32_t* w;
    int8_t* out;
    int M, K, k;
    uint32_t prime[DASH_MAX_PRIMES];
};

__global__ __launch_bounds__(kThreads) void k_weights_prepare(const PrepArgs A) {
    const int64_t Kp = kpad_of(A.K), Mp = mpad_of(A.M);
    int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= Mp * Kp) return;
    int64_t row = idx / Kp, col = idx - row * Kp;
    int32_t w = (row < A.M && col < A.K) ? A.w[row * A.K + col] : 0;
    for (int i = 0; i < A.k; i++) {
        int32_t p = (int32_t)A.prime[i];
        int32_t r = w % p;
        if (r < 0) r += p;
        A.out[(int64_t)i * Mp * Kp + idx] = (int8_t)r;
    }
}

struct LinPrime {
    uint32_t p;
    const int8_t* w;        // [Mpad][Kpad] residues of this prime
    const uint8_t* one;     // chunked label of the constant-one wire (zero or active), or NULL
    LView in, out;
};
struct LinArgs {
    const ModInfo* mods;
    const int32_t* bias;    // [out_c] or NULL
    int64_t kpad;
    int batch, in_h, in_w, in_c, out_c, kh, kw, stride, pad, out_h, out_w;
    LinPrime pr[DASH_MAX_PRIMES];
};

// S lanes per (output value, chunk): 16 accumulators, one 16-byte label word per tap; blockIdx.y = prime.  S = 1 for
// layers with enough outputs to fill the chip; S = 16 for layers with few (the last dense layers of a network at
// batch 1): the reduction index is dealt out in groups of four to 16 neighbouring lanes, whose partial sums are
// added up with lane shuffles, so that a lane's loop is 16 times shorter.
template <int S>
__global__ __launch_bounds__(kThreads) void k_linear_direct(const LinArgs AA) {
    struct { uint32_t p; const int8_t* w; const int32_t* bias; const uint8_t* one; LView in, out; int64_t kpad;
             int batch, in_h, in_w, in_c, out_c, kh, kw, stride, pad, out_h, out_w; } A;
    {
        const LinPrime& P = AA.pr[blockIdx.y];
        A.p = P.p; A.w = P.w; A.bias = AA.bias; A.one = P.one; A.in = P.in; A.out = P.out; A.kpad = AA.kpad;
        A.batch = AA.batch; A.in_h = AA.in_h; A.in_w = AA.in_w; A.in_c = AA.in_c; A.out_c = AA.out_c; A.kh = AA.kh; A.kw = AA.kw;
        A.stride = AA.stride; A.pad = AA.pad; A.out_h = AA.out_h; A.out_w = AA.out_w;
    }
    const ModInfo M = AA.mods[A.p];
    const int64_t n_out = (int64_t)A.batch * A.out_h * A.out_w * A.out_c;
    const int64_t gl = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t idx = gl / S;
    const int sl = (int)(gl % S);                       // this lane's share of the reduction index
    if (idx >= n_out * M.nchunk) return;                // (the S lanes of an output leave together)
    const uint32_t ch = (uint32_t)(idx / n_out);
    const int64_t o = idx - (int64_t)ch * n_out;
    int co = (int)(o % A.out_c);
    int64_t t = o / A.out_c;
    int ox = (int)(t % A.out_w); t /= A.out_w;
    int oy = (int)(t % A.out_h);
    int b = (int)(t / A.out_h);
    uint32_t acc[16];
    for (int d = 0; d < 16; d++) acc[d] = 0;
    const int8_t* wrow = A.w + (int64_t)co * A.kpad;
    const uint8_t* inc = A.in.p + (int64_t)ch * A.in.cs;
    // The reduction index k = (ky * kw + kx) * in_c + ci runs in groups of four (the weight rows are padded with zeros to a
    // multiple of 64): four 16-byte label words, their 4 x 4 byte blocks turned around with byte permutes so that a dword
    // holds one digit of the four taps, then one byte dot product with the four weights per digit (48 instructions per
    // four taps instead of 128 with a multiply-add per byte).
    const int K = A.kh * A.kw * A.in_c;
    int ky = 0, kx = 0, ci = 0;
    for (int k0 = 4 * sl; k0 < K; k0 += 4 * S) {
        if constexpr (S > 1) {                          // not consecutive groups: the tap of k0 by division
            const int tap = k0 / A.in_c;
            ci = k0 - tap * A.in_c; ky = tap / A.kw; kx = tap - ky * A.kw;
        }
        const uint32_t w4 = *(const uint32_t*)(wrow + k0);
        uint4 v[4];
#pragma unroll
        for (int t = 0; t < 4; t++) {
            const int iy = oy * A.stride + ky - A.pad, ix = ox * A.stride + kx - A.pad;
            const bool ok = k0 + t < K && iy >= 0 && iy < A.in_h && ix >= 0 && ix < A.in_w;
            v[t] = make_uint4(0, 0, 0, 0);
            if (ok) v[t] = *(const uint4*)(inc + ((((int64_t)b * A.in_h + iy) * A.in_w + ix) * A.in_c + ci) * 16);
            if (++ci == A.in_c) { ci = 0; if (++kx == A.kw) { kx = 0; ky++; } }
        }
        const uint32_t vq[4][4] = {{v[0].x, v[1].x, v[2].x, v[3].x}, {v[0].y, v[1].y, v[2].y, v[3].y},
                                   {v[0].z, v[1].z, v[2].z, v[3].z}, {v[0].w, v[1].w, v[2].w, v[3].w}};
#pragma unroll
        for (int q = 0; q < 4; q++) {
            // v_perm_b32(hi, lo, sel): byte i of the result = byte sel.i of the 8 bytes {hi:lo}
            const uint32_t ab02 = __builtin_amdgcn_perm(vq[q][1], vq[q][0], 0x06020400u), ab13 = __builtin_amdgcn_perm(vq[q][1], vq[q][0], 0x07030501u);
            const uint32_t cd02 = __builtin_amdgcn_perm(vq[q][3], vq[q][2], 0x06020400u), cd13 = __builtin_amdgcn_perm(vq[q][3], vq[q][2], 0x07030501u);
            const uint32_t d0 = __builtin_amdgcn_perm(cd02, ab02, 0x05040100u), d1 = __builtin_amdgcn_perm(cd13, ab13, 0x05040100u);
            const uint32_t d2 = __builtin_amdgcn_perm(cd02, ab02, 0x07060302u), d3 = __builtin_amdgcn_perm(cd13, ab13, 0x07060302u);
            acc[4 * q + 0] = __builtin_amdgcn_udot4(d0, w4, acc[4 * q + 0], false);
            acc[4 * q + 1] = __builtin_amdgcn_udot4(d1, w4, acc[4 * q + 1], false);
            acc[4 * q + 2] = __builtin_amdgcn_udot4(d2, w4, acc[4 * q + 2], false);
            acc[4 * q + 3] = __builtin_amdgcn_udot4(d3, w4, acc[4 * q + 3], false);
        }
    }
    if constexpr (S > 1) {
        // the S partial sums of every accumulator (S consecutive lanes of one wave, all of them here): butterfly
#pragma unroll
        for (int off = S / 2; off >= 1; off >>= 1)
#pragma unroll
            for (int d = 0; d < 16; d++) acc[d] += (uint32_t)__shfl_xor((int)acc[d], off, 64);
        if (sl != 0) return;
    }
    // (p-1)^2 * K < 2^31 is checked on the host; reduce in two steps so the magic division applies (n < 2^24)
    uint32_t bm = 0;
    if (A.bias) { int32_t r = A.bias[co] % (int32_t)M.m; bm = (uint32_t)(r < 0 ? r + (int32_t)M.m : r); }
    uint32_t outw[4];
    for (int q = 0; q < 4; q++) {
        uint32_t w = 0;
        for (int bb = 0; bb < 4; bb++) {
            uint32_t a = acc[4 * q + bb];
            uint32_t r = mod_m(mod_m(a >> 12, M) * (4096u % M.m) + (a & 4095u), M);   // a = hi*4096 + lo
            if (bm) r = mod_m(r + bm * A.one[ch * 16 + 4 * q + bb], M);
            w |= r << (8 * bb);
        }
        outw[q] = w;
    }
    *(uint4*)(A.out.p + (int64_t)ch * A.out.cs + o * 16) = make_uint4(outw[0], outw[1], outw[2], outw[3]);
}

struct PoolPrime { uint32_t p; LView in, out; };
struct PoolArgs {
    const ModInfo* mods;
    int batch, in_h, in_w, ch;
    PoolPrime pr[DASH_MAX_PRIMES];
};
// blockIdx.y = prime
__global__ __launch_bounds__(kThreads) void k_sumpool(const PoolArgs AA) {
    struct { uint32_t p; LView in, out; int batch, in_h, in_w, ch; } A;
    A.p = AA.pr[blockIdx.y].p; A.in = AA.pr[blockIdx.y].in; A.out = AA.pr[blockIdx.y].out;
    A.batch = AA.batch; A.in_h = AA.in_h; A.in_w = AA.in_w; A.ch = AA.ch;
    const ModInfo M = AA.mods[A.p];
    const int oh = A.in_h / 2, ow = A.in_w / 2;
    const int64_t n_out = (int64_t)A.batch * oh * ow * A.ch;
    int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= n_out * M.nchunk) return;
    const uint32_t chunk = (uint32_t)(idx / n_out);
    const int64_t o = idx - (int64_t)chunk * n_out;
    int c = (int)(o % A.ch);
    int64_t t = o / A.ch;
    int ox = (int)(t % ow); t /= ow;
    int oy = (int)(t % oh);
    int b = (int)(t / oh);
    uint32_t w[4] = {0, 0, 0, 0};
    for (int dy = 0; dy < 2; dy++)
        for (int dx = 0; dx < 2; dx++) {
            int64_t e = (((int64_t)b * A.in_h + 2 * oy + dy) * A.in_w + 2 * ox + dx) * A.ch + c;
            uint4 v = *(const uint4*)(A.in.p + (int64_t)chunk * A.in.cs + e * 16);
            w[0] = addmod4(w[0], v.x, M); w[1] = addmod4(w[1], v.y, M);
            w[2] = addmod4(w[2], v.z, M); w[3] = addmod4(w[3], v.w, M);
        }
    *(uint4*)(A.out.p + (int64_t)chunk * A.out.cs + o * 16) = make_uint4(w[0], w[1], w[2], w[3]);
}

int linear_layer(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, hipStream_t s) {
    int64_t per_out = 0;
    int st = layer_sizes(c, L, &per_out, nullptr, nullptr);
    if (st) return st;
    const int64_t batch = L->n_elem;
    if (batch == 0) return DASH_OK;
    int in_h = L->in_h, in_w = L->in_w, kh = L->kh, kw = L->kw, stride = L->stride, pad = L->pad, out_c = L->out_c;
    if (L->kind == DASH_DENSE) { in_h = in_w = kh = kw = stride = 1; pad = 0; }
    if (L->kind == DASH_SUMPOOL) out_c = L->in_c;
    const int64_t n_in = (int64_t)batch * in_h * in_w * L->in_c, n_out = batch * per_out;
    if (n_in > 0x7fffffff || n_out > 0x7fffffff) return DASH_ESIZE;
    if (!in || !out || in->n_elem < n_in || out->n_elem < n_out) return DASH_EINVAL;
    for (int i = 0; i < c->k; i++) {
        if (!in->data[i] || !out->data[i] || ((uintptr_t)in->data[i] & 15) || ((uintptr_t)out->data[i] & 15)) return DASH_EINVAL;
        if ((in->chunk_stride[i] & 15) || (out->chunk_stride[i] & 15) || in->chunk_stride[i] < 16 * n_in || out->chunk_stride[i] < 16 * n_out)
            return DASH_EINVAL;
    }
    if (L->kind == DASH_SUMPOOL) {
        PoolArgs A;
        memset(&A, 0, sizeof(A));
        A.mods = c->d_mods; A.batch = (int)batch; A.in_h = in_h; A.in_w = in_w; A.ch = L->in_c;
        int64_t lanes = 0;          // of the prime with the most chunks; the others' surplus blocks exit
        for (int i = 0; i < c->k; i++) {
            A.pr[i] = PoolPrime{(uint32_t)c->prime[i], view_of(in, i), view_of(out, i)};
            const int64_t l = n_out * c->mods[c->prime[i]].nchunk;
            lanes = l > lanes ? l : lanes;
        }
        hipLaunchKernelGGL(k_sumpool, dim3((uint32_t)((lanes + kThreads - 1) / kThreads), c->k), dim3(kThreads), 0, s, A);
        DASH_HIP(hipGetLastError());
        return DASH_OK;
    }
    if (!L->weights) return DASH_EINVAL;
    const int K = kh * kw * L->in_c;
    const int64_t Kp = kpad_of(K), Mp = mpad_of(out_c);
    for (int i = 0; i < c->k; i++) {
        uint64_t p1 = (uint64_t)(c->prime[i] - 1);
        if (p1 * p1 * (uint64_t)K >= (1ull << 31)) return DASH_ESIZE;      // int32 accumulators must not overflow
    }
    if (dense_mfma_wanted(L, batch)) return dense_mfma(c, L, garble, in, out, s);
    const int out_h = (in_h + 2 * pad - kh) / stride + 1, out_w = (in_w + 2 * pad - kw) / stride + 1;
    LinArgs A;
    memset(&A, 0, sizeof(A));
    A.mods = c->d_mods; A.bias = L->bias; A.kpad = Kp;
    A.batch = (int)batch; A.in_h = in_h; A.in_w = in_w; A.in_c = L->in_c; A.out_c = out_c;
    A.kh = kh; A.kw = kw; A.stride = stride; A.pad = pad; A.out_h = out_h; A.out_w = out_w;
    int64_t lanes = 0;              // of the prime with the most chunks; the others' surplus blocks exit
    double macs = 0, bytes = 0;
    for (int i = 0; i < c->k; i++) {
        LinPrime& P = A.pr[i];
        P.p = c->prime[i];
        P.w = (const int8_t*)L->weights + (int64_t)i * Mp * Kp;
        P.one = L->bias ? (garble ? c->d_one0[i] : c->d_one[i]) : nullptr;
        P.in = view_of(in, i); P.out = view_of(out, i);
        const int64_t l = n_out * c->mods[c->prime[i]].nchunk;
        lanes = l > lanes ? l : lanes;
        const double lam = c->mods[c->prime[i]].lam;
        macs += (double)n_out * K * lam;
        bytes += ((double)n_in + n_out) * lam + (double)out_c * K;
    }
    {
        ProfScope ps(c->prof, DASH_PROF_LINEAR, s, macs, bytes);
        // few outputs and a long reduction: 16 lanes per output
        if (lanes <= 16384 && K >= 64)
            hipLaunchKernelGGL(k_linear_direct<16>, dim3((uint32_t)((lanes * 16 + kThreads - 1) / kThreads), c->k), dim3(kThreads), 0, s, A);
        else
            hipLaunchKernelGGL(k_linear_direct<1>, dim3((uint32_t)((lanes + kThreads - 1) / kThreads), c->k), dim3(kThreads), 0, s, A);
    }
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash

extern "C" {

size_t dash_weights_bytes(const dash_ctx* c, int out_c, int K) {
    if (!c || out_c < 1 || K < 1) return 0;
    return (size_t)c->k * (size_t)dash::mpad_of(out_c) * (size_t)dash::kpad_of(K);
}

int dash_weights_prepare(dash_ctx* c, const int32_t* w, int out_c, int K, void* prepared, void* stream) {
    if (!c || !w || !prepared || out_c < 1 || K < 1) return DASH_EINVAL;
    dash::PrepArgs A;
    memset(&A, 0, sizeof(A));
    A.w = w; A.out = (int8_t*)prepared; A.M = out_c; A.K = K; A.k = c->k;
    for (int i = 0; i < c->k; i++) A.prime[i] = c->prime[i];
    int64_t n = dash::mpad_of(out_c) * dash::kpad_of(K);
    if ((n + dash::kThreads - 1) / dash::kThreads > 0x7fffffff) return DASH_ESIZE;
    hipLaunchKernelGGL(dash::k_weights_prepare, dim3((uint32_t)((n + dash::kThreads - 1) / dash::kThreads)), dim3(dash::kThreads), 0,
                       (hipStream_t)stream, A);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // extern "C"
