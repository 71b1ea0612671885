// dash_gemm.hip -- the dense linear layer on LabelTensors as an int8 MFMA contraction (Sec. Arithmetic
// Garbled Circuits: free addition and multiplication by a public constant; Sec. System-level
// Architecture: Dense): per CRT prime p
//     out[b][j][digit] = sum_i (W[j][i] mod p) * in[b][i][digit]  (+ (bias[j] mod p) * one[digit])   mod p.
// Residues and reduced weights are below p <= 127, so both operands are int8; the int32 accumulators are
// exact because (p-1)^2 * K < 2^31 (checked by the caller) and a single reduction mod p follows.
//
// Shape.  A "group" is the 16 digits of one chunk of one batch element: in memory a K x 16 byte matrix
// X_G (rows = input features, consecutive rows 16 bytes apart).  The layer is  Out_G (M x 16) = W (M x K)
// * X_G  for every group, i.e. one GEMM  M x K x (16 * groups)  per prime whose B operand is
// N-contiguous.  The MFMA wants K-contiguous bytes in registers for both operands, so the loader turns
// every 4 (k) x 4 (digit) byte block of X around with byte permutes before it goes to LDS; this costs
// 32 v_perm per thread and K-step of 64 and is shared by the four waves of the block.
//
// Tiling.  Block = 256 threads = 2 x 2 waves, block tile 256 (M) x 16 groups (256 columns), K-step 64,
// LDS double buffered (2 x (20 KB A + 20 KB B), rows padded from 64 to 80 bytes so that the 16-byte
// fragment reads of 8 consecutive lanes fall into different banks).  Wave tile 128 x 128 columns =
// 4 x 4 MFMA 32x32x32 per 32 of K, accumulators 256 registers per lane.  MFMA s (0..3) of a wave
// covers digit 4g+s of the 32 (group, g) pairs that its lanes stand for, so that after the last K-step a
// lane holds, for its pair, the four digits of one output dword for 64 output features.
#include <string.h>

#include "dash_internal.h"

namespace dash {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBM = 256;        // output features per block
constexpr int kBG = 16;         // groups per block (256 columns)
constexpr int kKT = 64;         // K per stage
constexpr int kRow = 80;        // bytes per LDS row (64 + 16 pad)

struct GemmPrime {
    uint32_t p, nchunk;
    uint32_t mmagic;            // ceil(2^32 / p)
    uint32_t pow12;             // 4096 mod p
    const int8_t* w;            // [Mpad][Kpad] residues of this prime
    const uint8_t* one;         // chunked label of the constant-one wire, or NULL
    LView in, out;
};
struct GemmArgs {
    int M, K, batch, nprimes;
    int64_t kpad, mpad;
    const int32_t* bias;
    uint32_t small_acc;         // 1 if (p-1)^2 K < 2^24 for every prime: one-step reduction
    GemmPrime pr[DASH_MAX_PRIMES];
};

// bytes (a.bS, b.bS, c.bS, d.bS) for S = 0..3: transposes a 4x4 byte block held in 4 dwords
__device__ __forceinline__ void transpose4x4(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t out[4]) {
    // v_perm_b32(hi, lo, sel): byte k of the result = byte sel.k of the 8 bytes {hi:lo} (lo = bytes 0..3)
    uint32_t ab02 = __builtin_amdgcn_perm(b, a, 0x06020400u);   // a0 b0 a2 b2
    uint32_t ab13 = __builtin_amdgcn_perm(b, a, 0x07030501u);   // a1 b1 a3 b3
    uint32_t cd02 = __builtin_amdgcn_perm(d, c, 0x06020400u);
    uint32_t cd13 = __builtin_amdgcn_perm(d, c, 0x07030501u);
    out[0] = __builtin_amdgcn_perm(cd02, ab02, 0x05040100u);    // a0 b0 c0 d0
    out[2] = __builtin_amdgcn_perm(cd02, ab02, 0x07060302u);    // a2 b2 c2 d2
    out[1] = __builtin_amdgcn_perm(cd13, ab13, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(cd13, ab13, 0x07060302u);
}

__global__ __launch_bounds__(256) void k_dense_mfma(const GemmArgs A) {
    const GemmPrime& P = A.pr[blockIdx.z];
    const int ngroups = (int)P.nchunk * A.batch;
    const int gblocks = (ngroups + kBG - 1) / kBG;
    if ((int)blockIdx.x >= gblocks) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const int row0 = blockIdx.y * kBM, grp0 = blockIdx.x * kBG;

    __shared__ __attribute__((aligned(16))) uint8_t As[2][kBM * kRow];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[2][4 * kBG * 4 * kRow];

    // ---- loader roles ----
    // A: 1024 16-byte pieces per stage, 4 per thread: piece id -> (row = id / 4, part = id % 4)
    // B: thread -> (group G = tid / 16, k quad kq = tid % 16): rows k = 4kq..4kq+3 of X_G, 16 bytes each
    const int bG = tid >> 4, bkq = tid & 15;
    const int gglob = grp0 + bG;
    const bool gvalid = gglob < ngroups;
    const int gch = gvalid ? gglob / A.batch : 0, gb = gvalid ? gglob - gch * A.batch : 0;
    const uint8_t* xg = P.in.p + (int64_t)gch * P.in.cs + ((int64_t)gb * A.K) * 16;

    uint4 ra[4], rb[4];
    auto load_stage = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int id = tid + 256 * i, row = row0 + (id >> 2), part = id & 3;
            ra[i] = row < A.mpad ? *(const uint4*)(P.w + (int64_t)row * A.kpad + k0 + part * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const int k = k0 + 4 * bkq + kk;
            rb[kk] = (gvalid && k < A.K) ? *(const uint4*)(xg + (int64_t)k * 16) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int id = tid + 256 * i;
            *(uint4*)(As[buf] + (id >> 2) * kRow + (id & 3) * 16) = ra[i];
        }
        const uint32_t r[4][4] = {{rb[0].x, rb[0].y, rb[0].z, rb[0].w}, {rb[1].x, rb[1].y, rb[1].z, rb[1].w},
                                  {rb[2].x, rb[2].y, rb[2].z, rb[2].w}, {rb[3].x, rb[3].y, rb[3].z, rb[3].w}};
#pragma unroll
        for (int g = 0; g < 4; g++) {
            uint32_t t[4];
            transpose4x4(r[0][g], r[1][g], r[2][g], r[3][g], t);     // t[s] = digit 4g+s at k = 4kq..4kq+3
#pragma unroll
            for (int s = 0; s < 4; s++) *(uint32_t*)(Bs[buf] + (((s * kBG + bG) * 4 + g) * kRow) + 4 * bkq) = t[s];
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int s = 0; s < 4; s++) acc[i][s] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    const int nk = (int)(A.kpad / kKT);
    load_stage(0);
    store_stage(0);
    __syncthreads();
    const int n = lane & 31, kh = lane >> 5;
    const int fa = (wm * 128 + n) * kRow + kh * 16;                              // + rb*32*kRow + ks*32
    const int fb = (((wn * 8 + (n >> 2)) * 4) + (n & 3)) * kRow + kh * 16;       // + s*kBG*4*kRow + ks*32
    for (int kt = 0; kt < nk; kt++) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_stage((kt + 1) * kKT);
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            v4i a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = *(const v4i*)(As[cur] + fa + i * 32 * kRow + ks * 32);
#pragma unroll
            for (int s = 0; s < 4; s++) b[s] = *(const v4i*)(Bs[cur] + fb + s * kBG * 4 * kRow + ks * 32);
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int s = 0; s < 4; s++) acc[i][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[s], acc[i][s], 0, 0, 0);
        }
        if (kt + 1 < nk) store_stage(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: reduce mod p, pack the four digits of a dword, store ----
    const int G = grp0 + wn * 8 + (n >> 2), g = n & 3;
    if (G >= ngroups) return;
    const int och = G / A.batch, ob = G - och * A.batch;
    uint8_t* og = P.out.p + (int64_t)och * P.out.cs + ((int64_t)ob * A.M) * 16 + 4 * g;
    uint32_t one4 = 0;
    if (A.bias) one4 = *(const uint32_t*)(P.one + och * 16 + 4 * g);
    auto red = [&](uint32_t v) -> uint32_t {
        if (!A.small_acc) {                                   // v = hi * 4096 + lo
            uint32_t hi = v >> 12;
            hi -= mul24(mulhi(hi, P.mmagic), P.p);
            v = mul24(hi, P.pow12) + (v & 4095u);
        }
        return v - mul24(mulhi(v, P.mmagic), P.p);
    };
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int j = row0 + wm * 128 + i * 32 + (r >> 2) * 8 + kh * 4 + (r & 3);
            if (j >= A.M) continue;
            uint32_t d[4];
#pragma unroll
            for (int s = 0; s < 4; s++) d[s] = red((uint32_t)acc[i][s][r]);
            if (A.bias) {
                int32_t bj = A.bias[j] % (int32_t)P.p;
                uint32_t bm = (uint32_t)(bj < 0 ? bj + (int32_t)P.p : bj);
#pragma unroll
                for (int s = 0; s < 4; s++) d[s] = red(d[s] + mul24(bm, (one4 >> (8 * s)) & 0xffu));
            }
            *(uint32_t*)(og + (int64_t)j * 16) = d[0] | (d[1] << 8) | (d[2] << 16) | (d[3] << 24);
        }
}

// true if the MFMA path should take this dense layer (large enough to fill tiles)
bool dense_mfma_wanted(const dash_layer* L, int64_t batch) {
    return L->kind == DASH_DENSE && (int64_t)L->in_c * L->out_c >= 64 * 64 && (int64_t)L->out_c * batch >= 64;
}

int dense_mfma(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, hipStream_t s) {
    const int M = L->out_c, K = L->in_c;
    const int64_t batch = L->n_elem;
    GemmArgs A;
    memset(&A, 0, sizeof(A));
    A.M = M; A.K = K; A.batch = (int)batch; A.nprimes = c->k;
    A.kpad = ((int64_t)K + 63) / 64 * 64; A.mpad = ((int64_t)M + 31) / 32 * 32;
    A.bias = L->bias;
    A.small_acc = 1;
    uint32_t max_nchunk = 1;
    double macs = 0, bytes = 0;
    for (int i = 0; i < c->k; i++) {
        GemmPrime& P = A.pr[i];
        const ModInfo& Mi = c->mods[c->prime[i]];
        P.p = c->prime[i]; P.nchunk = Mi.nchunk; P.mmagic = Mi.mmagic; P.pow12 = 4096u % P.p;
        P.w = (const int8_t*)L->weights + (int64_t)i * A.mpad * A.kpad;
        P.one = L->bias ? (garble ? c->d_one0[i] : c->d_one[i]) : nullptr;
        P.in = view_of(in, i); P.out = view_of(out, i);
        if ((uint64_t)(P.p - 1) * (P.p - 1) * (uint64_t)K >= (1ull << 24)) A.small_acc = 0;
        max_nchunk = Mi.nchunk > max_nchunk ? Mi.nchunk : max_nchunk;
        macs += (double)batch * M * K * Mi.lam;
        bytes += (double)batch * (M + K) * Mi.lam + (double)M * K;
    }
    const int64_t gblocks = ((int64_t)max_nchunk * batch + kBG - 1) / kBG;
    if (gblocks > 0x7fffffff) return DASH_ESIZE;
    dim3 grid((uint32_t)gblocks, (uint32_t)((M + kBM - 1) / kBM), c->k);
    ProfScope ps(c->prof, DASH_PROF_LINEAR, s, macs, bytes);
    hipLaunchKernelGGL(k_dense_mfma, grid, dim3(256), 0, s, A);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
