// dash_aesprof.hip -- AES-128 alone, in each form the library has: table look-ups in LDS (the two table layouts of
// the gate kernels) and bit planes without tables (dash_aes_sliced.h).  Measurement and checking only
// (include/dash_profile.h): the gate kernels hash with the tables.
#include <hip/hip_runtime.h>

#include "dash_aes_sliced.h"
#include "dash_hostconst.h"
#include "dash_tabs.h"

namespace dash {


// All four tables once per bank, 128 KB (one block of 1024 lanes per CU): no rotation.  T2 and T3 lie 64 KB above T0
// and T1; the permute takes that bit from byte 2 of the lane's constant.  Measured here only: the gate kernels are
// slower with it (half the waves per SIMD).
constexpr int kBankTab4Words = 32768;
struct BankTab4 {
    const uint8_t* t;
    uint32_t lane;       // byte 0: 4 * bank, byte 2: 1
    template <int R, int B> __device__ __forceinline__ uint32_t at(uint32_t w) const {
        constexpr uint32_t sel = (R >= 2 ? 0x0c020000u : 0x0c0c0000u) | ((4u + B) << 8);
        const uint32_t a = __builtin_amdgcn_perm(w, lane, sel);
        return *(const uint32_t*)(t + a + (R & 1) * 128);
    }
};
__device__ __forceinline__ BankTab4 load_banktab4(uint32_t* lds, const uint32_t* g) {
    for (int e = threadIdx.x; e < 1024; e += blockDim.x) {
        const uint32_t v = g[e];
        const int R = e >> 8, x = e & 255;
        uint4* dst = (uint4*)(lds + (R >> 1) * 16384 + x * 64 + (R & 1) * 32);
        const uint4 v4 = make_uint4(v, v, v, v);
#pragma unroll
        for (int i = 0; i < 8; i++) dst[i] = v4;
    }
    __syncthreads();
    return BankTab4{(const uint8_t*)lds, ((threadIdx.x & 31u) << 2) | 0x10000u};
}

// key masks of the bit-plane form (rounds 1..9), one copy per GPU, rewritten by every call
static __device__ uint32_t g_sliced_masks[9 * 128];

// one block per lane and pass; out = AES^repeat(in)
template <bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_aes_tab(AesKey K, const uint32_t* ttab, const uint4* in, uint4* out, uint64_t n, int repeat) {
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, ttab);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint4 v = in[i];
        uint32_t s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll 1
        for (int r = 0; r < repeat; r++) aes128_encrypt(s, K.rk, T);
        out[i] = make_uint4(s[0], s[1], s[2], s[3]);
    }
}

__global__ __launch_bounds__(kBigThreads) void k_aes_tab4(AesKey K, const uint32_t* ttab, const uint4* in, uint4* out, uint64_t n, int repeat) {
    __shared__ uint32_t tt[kBankTab4Words];
    const BankTab4 T = load_banktab4(tt, ttab);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint4 v = in[i];
        uint32_t s[4] = {v.x, v.y, v.z, v.w};
#pragma unroll 1
        for (int r = 0; r < repeat; r++) aes128_encrypt(s, K.rk, T);
        out[i] = make_uint4(s[0], s[1], s[2], s[3]);
    }
}

// 32 blocks per lane: a wave takes 2048 consecutive blocks, lane l the blocks l, l + 64, ... of them
__global__ __launch_bounds__(256) void k_aes_sliced(AesKey K, const uint32_t* km, const uint4* in, uint4* out, uint64_t n, int repeat) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t nwaves = n / 2048;
    for (uint64_t w = (uint64_t)blockIdx.x * 4 + wave; w < nwaves; w += (uint64_t)gridDim.x * 4) {
        const uint4* src = in + w * 2048 + lane;
        uint4* dst = out + w * 2048 + lane;
        uint32_t X[128];
#pragma unroll
        for (int j = 0; j < 32; j++) {
            const uint4 v = src[j * 64];
            X[j] = v.x; X[32 + j] = v.y; X[64 + j] = v.z; X[96 + j] = v.w;
        }
#pragma unroll 1
        for (int r = 0; r < repeat; r++) aes128_encrypt_sliced(X, K.rk, km);
#pragma unroll
        for (int j = 0; j < 32; j++) dst[j * 64] = make_uint4(X[j], X[32 + j], X[64 + j], X[96 + j]);
    }
}

}  // namespace dash

using namespace dash;

extern "C" int dash_profile_aes(dash_ctx* c, int variant, const uint8_t* key, const void* in, void* out, uint64_t n_blocks,
                                int repeat, void* stream) {
    if (!c || !key || (n_blocks && (!in || !out)) || repeat < 1) return DASH_EINVAL;
    if (variant < 0 || variant > 3) return DASH_EINVAL;
    if (n_blocks >= (1ull << 40)) return DASH_ESIZE;
    if (variant == 2 && n_blocks % 2048) return DASH_ESIZE;
    if (n_blocks == 0) return DASH_OK;
    if (hipSetDevice(c->device) != hipSuccess) return DASH_EHIP;
    uint8_t S[256];
    hostconst::make_sbox(S);
    AesKey K;
    hostconst::expand_key(key, S, K.rk);
    hipStream_t st = (hipStream_t)stream;
    if (variant == 2) {
        uint32_t km[9 * 128];
        sliced_key_masks(K.rk, km);
        uint32_t* d_km = nullptr;
        if (hipGetSymbolAddress((void**)&d_km, HIP_SYMBOL(g_sliced_masks)) != hipSuccess) return DASH_EHIP;
        // synchronous on purpose: the source is on this stack frame, and earlier calls' kernels must be done with the masks
        if (hipStreamSynchronize(st) != hipSuccess) return DASH_EHIP;
        if (hipMemcpy(d_km, km, sizeof(km), hipMemcpyHostToDevice) != hipSuccess) return DASH_EHIP;
        const uint64_t nwaves = n_blocks / 2048;
        uint64_t blocks = (nwaves + 3) / 4;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_aes_sliced, dim3((uint32_t)blocks), dim3(256), 0, st, K, d_km, (const uint4*)in, (uint4*)out, n_blocks, repeat);
    } else if (variant == 3) {
        uint64_t blocks = (n_blocks + kBigThreads - 1) / kBigThreads;
        if (blocks > 512) blocks = 512;
        hipLaunchKernelGGL(k_aes_tab4, dim3((uint32_t)blocks), dim3(kBigThreads), 0, st, K, c->d_ttab, (const uint4*)in, (uint4*)out, n_blocks, repeat);
    } else if (variant == 1) {
        uint64_t blocks = (n_blocks + kBigThreads - 1) / kBigThreads;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(k_aes_tab<true>, dim3((uint32_t)blocks), dim3(kBigThreads), 0, st, K, c->d_ttab, (const uint4*)in, (uint4*)out, n_blocks, repeat);
    } else {
        uint64_t blocks = (n_blocks + kThreads - 1) / kThreads;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_aes_tab<false>, dim3((uint32_t)blocks), dim3(kThreads), 0, st, K, c->d_ttab, (const uint4*)in, (uint4*)out, n_blocks, repeat);
    }
    return hipGetLastError() == hipSuccess ? DASH_OK : DASH_EHIP;
}
