// dash_gemm.hip -- the dense linear layer on LabelTensors as an int8 MFMA contraction (Sec. Arithmetic
// Garbled Circuits: free addition and multiplication by a public constant; Sec. System-level
// Architecture: Dense): per CRT prime p
//     out[b][j][digit] = sum_i (W[j][i] mod p) * in[b][i][digit]  (+ (bias[j] mod p) * one[digit])   mod p.
// Residues and reduced weights are below p <= 127, so both operands are int8; the int32 accumulators are
// exact because (p-1)^2 * K < 2^31 (checked by the caller) and a single reduction mod p follows.
//
// Convolutions run through the same kernel as an implicit GEMM (Sec. LabelTensors, the Conv2D figure): the
// "batch element" of a group is then an output pixel and row k = (ky, kx, ci) of its K x 16 matrix is the
// 16-byte word of input pixel (oy * stride - pad + ky, ox * stride - pad + kx), channel ci, or zeros
// outside the image; with the channel count a multiple of 4, the four rows a loader thread fetches are
// consecutive channels of one tap, i.e. 64 contiguous bytes.
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
// 4 x 4 MFMA 32x32x32 per 32 of K, accumulators 256 registers per lane (so one wave per SIMD).  MFMA s
// (0..3) of a wave covers digit 4g+s of the 32 (group, g) pairs that its lanes stand for, so that after the
// last K-step a lane holds, for its pair, the four digits of one output dword for 64 output features.
// (A second shape, 128 x 512 with 8 waves of 64 x 128 and two waves per SIMD, serves layers with few outputs.)
//
// Pipeline.  With one wave per SIMD nothing but the wave's own instruction order hides latency: global
// data is fetched a stage and a half ahead into one of two register sets, transposed and written to LDS
// during the first K half of the stage before, and ONE barrier in the middle of a stage separates these
// writes from the fragment reads of the next stage, which run under the MFMAs of the second half
// (sched_group_barrier interleaving; the global loads are spread over the whole stage).  Measured on the
// 4096 x 4096, batch 128, 12-prime case (per block tile, from time stamps inside the kernel): 3.1 us until
// the first MFMA, 64 stages of 0.86 us (a loop of nothing but the 32 MFMAs of a stage runs at 0.55 us per
// stage in the same launch shape: the matrix clock under load is about 2.1 GHz), 4.7 us of epilogue;
// 1.24 ms in all, 38 % of the 5.0 POP/s int8 peak.  Taking parts out of the loop: without the global loads
// 0.64 us per stage, without the fragment reads no change, without the byte transposes 0.83; the L2 answers
// in 380 cycles on average (counter TCP_TCC_READ_REQ_LATENCY), far less than the prefetch distance, three
// register sets (two and a half stages ahead) were slower, and so were two blocks of half the size per CU.
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "dash_internal.h"

namespace dash {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// A block is NWM x NWN waves, a wave tile (32 IFR) rows x 8 groups (128 columns).
template <int NWM_, int NWN_, int IFR_>
struct Tile {
    static constexpr int NWM = NWM_, NWN = NWN_, IFR = IFR_;
    static constexpr int BM = NWM * 32 * IFR;      // output features per block
    static constexpr int BG = NWN * 8;             // groups per block (16 columns each)
    static constexpr int T = 64 * NWM * NWN;       // lanes per block
    static constexpr int AP = BM * 4 / T;          // 16-byte pieces of the weight tile per lane and stage
    static_assert(BG * 16 == T && AP >= 1 && AP <= 4, "loader roles");
};
typedef Tile<2, 2, 4> TileBig;      // 256 x 256 block tile, 4 waves of 128 x 128: one wave per SIMD
typedef Tile<2, 4, 2> TileWide;     // 128 x 512 block tile, 8 waves of 64 x 128: two waves per SIMD
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
    // convolution geometry (conv = 0: dense, batch elements are the groups' columns)
    int conv, in_h, in_w, in_c, kw, stride, pad, out_h, out_w;
    uint32_t c_magic, kw_magic; // ceil(2^32 / in_c), ceil(2^32 / kw)
    const uint8_t* zero;        // 64 zero bytes on the device
    int sty;                    // block rows per super-tile: 4, 2 or 1 (kStBlocks / sty block columns)
    int gy4;                    // super-tile rows: ceil(ceil(M / kBM) / sty)
    int st_total;               // super-tiles of all primes
    int st_first[DASH_MAX_PRIMES + 1];   // first super-tile of every prime
    GemmPrime pr[DASH_MAX_PRIMES];
};

// Block -> tile.  Work-groups go to the 8 XCDs round-robin by their linear id, and each XCD has its own
// L2.  The 32 blocks that are resident on one XCD at a time are therefore ids xcd + 8 * (32 s .. 32 s + 31):
// they are given one "super-tile" of 4 (M) x 8 (groups) block tiles, so that together they read 4 row
// panels of the weights and 8 column panels of the labels (12 panel streams for 32 blocks) instead of
// 1 + 32 with a row-major order.  Super-tiles are numbered over all primes; tiles past the edge of a
// prime's grid exit.
// (Layers with fewer than 4 row blocks use 2 x 16 or 1 x 32.)
constexpr int kStBlocks = 32, kXcds = 8;

// Plain: no bias and every accumulator below 2^24, the common case: its epilogue has no branches at all
template <class TL, bool Conv, bool Plain>
__global__ __launch_bounds__(TL::T) void k_dense_mfma(const GemmArgs A) {
    constexpr int kBM = TL::BM, kBG = TL::BG, IFR = TL::IFR, AP = TL::AP, T = TL::T;
    const int xcd = blockIdx.x % kXcds, seq = blockIdx.x / kXcds;
    const int st = (seq / kStBlocks) * kXcds + xcd, within = seq % kStBlocks;
    if (st >= A.st_total) return;
    int pi = 0;
    while (st >= A.st_first[pi + 1]) pi++;
    const GemmPrime& P = A.pr[pi];
    const int ngroups = (int)P.nchunk * A.batch;
    const int gblocks = (ngroups + kBG - 1) / kBG;
    const int stl = st - A.st_first[pi];                    // super-tile inside the prime: row-major over (x super, y super)
    const int sty = A.sty, stx = kStBlocks / sty;
    const int by = (stl % A.gy4) * sty + within % sty, bx = (stl / A.gy4) * stx + within / sty;
    const int M = A.M, K = A.K;
    if (bx >= gblocks || by * kBM >= M) return;
    // everything the loops need, in registers: fields read through the argument block inside a loop are
    // fetched again (a scalar load and a wait) every time they are used
    const int8_t* const wbase = P.w;
    const int64_t kpad = A.kpad, mpad = A.mpad;
    const uint32_t prime = P.p, mmagic = P.mmagic, pow12 = P.pow12;
    const bool small_acc = A.small_acc != 0;
    const int32_t* const bias = A.bias;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave / TL::NWN, wn = wave % TL::NWN;
    const int row0 = by * kBM, grp0 = bx * kBG;

    // one LDS block: two stages of the A tile, two of the B tile; the epilogue reuses it for the output tile
    constexpr int kAbytes = kBM * kRow, kBbytes = 4 * kBG * 4 * kRow;
    constexpr int kOutStride = kBM * 16 + 16;                      // bytes per group of the staged output tile (padded)
    static_assert(kBG * kOutStride <= 2 * (kAbytes + kBbytes), "output tile fits the operand buffers");
    __shared__ __attribute__((aligned(16))) uint8_t smem[2 * (kAbytes + kBbytes)];
    auto As = [&](int b) __attribute__((always_inline)) { return smem + b * kAbytes; };
    auto Bs = [&](int b) __attribute__((always_inline)) { return smem + 2 * kAbytes + b * kBbytes; };

    // ---- loader roles ----
    // A: 4 kBM 16-byte pieces per stage, AP per thread: piece id -> (row = id / 4, part = id % 4)
    // B: thread -> (group G = tid / 16, k quad kq = tid % 16): rows k = 4kq..4kq+3 of X_G, 16 bytes each
    const int bG = tid >> 4, bkq = tid & 15;
    const int gglob = grp0 + bG;
    const bool gvalid = gglob < ngroups;
    // a group past the end reads group 0 (its results are never stored): loads need no predicate
    const int gch = gvalid ? gglob / A.batch : 0, gb = gvalid ? gglob - gch * A.batch : 0;
    const uint8_t* xg = P.in.p + (int64_t)gch * P.in.cs + (Conv ? (int64_t)0 : ((int64_t)gb * K) * 16);
    // convolution: gb = (image, oy, ox)
    const int in_h = A.in_h, in_w = A.in_w, in_c = A.in_c, kw = A.kw;
    const uint32_t c_magic = A.c_magic, kw_magic = A.kw_magic;
    const uint8_t* const zero = A.zero;
    int img = 0, iy0 = 0, ix0 = 0;
    if constexpr (Conv) {
        const int per = A.out_h * A.out_w;
        img = gb / per;
        const int r = gb - img * per, oy = r / A.out_w, ox = r - oy * A.out_w;
        iy0 = oy * A.stride - A.pad; ix0 = ox * A.stride - A.pad;
    }

    // Global data is fetched two stages ahead into one of two register sets (a stage of MFMAs is shorter
    // than a miss in the L2), transposed and written to LDS one stage ahead.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));     // (a plain vector: HIP's uint4 is a struct and was left in scratch memory)
    struct Regs { u32x4 a0, a1, a2, a3, b0, b1, b2, b3; };
    Regs Rx, Ry;
    const int arow = tid >> 2, apart = tid & 3;         // A piece i of this thread: row arow + (T / 4) i, 16-byte part apart
    auto a_src = [&](int i, int k0) __attribute__((always_inline)) {
        const int row = row0 + arow + (T / 4) * i;
        return (const u32x4*)(wbase + (int64_t)(row < mpad ? row : mpad - 1) * kpad + k0 + apart * 16);   // rows past M are never stored
    };
    auto b_src = [&](int kk, int k0) __attribute__((always_inline)) {
        const int k = k0 + 4 * bkq + kk;
        return (const u32x4*)(xg + (int64_t)(k < K ? k : K - 1) * 16);                                   // the weights are zero for k >= K
    };
    // convolution: rows k..k+3 (k a multiple of 4, in_c a multiple of 4) are channels ci..ci+3 of one tap
    auto conv_src = [&](int k0) __attribute__((always_inline)) {
        const uint32_t k = (uint32_t)(k0 + 4 * bkq);
        const uint32_t tap = mulhi(k, c_magic), ci = k - tap * (uint32_t)in_c;          // k < 2^24
        const uint32_t ky = kw > 1 ? mulhi(tap, kw_magic) : tap, kx = tap - ky * (uint32_t)kw;
        const int iy = iy0 + (int)ky, ix = ix0 + (int)kx;
        const bool ok = (int)k < K && iy >= 0 && iy < in_h && ix >= 0 && ix < in_w;
        const uint8_t* src = xg + ((((int64_t)img * in_h + iy) * in_w + ix) * in_c + ci) * 16;
        return (const u32x4*)(ok ? src : zero);
    };
    auto load_a = [&](int k0, Regs& R) __attribute__((always_inline)) {
        R.a0 = *a_src(0, k0);
        if constexpr (AP > 1) R.a1 = *a_src(1, k0);
        if constexpr (AP > 2) { R.a2 = *a_src(2, k0); R.a3 = *a_src(3, k0); }
    };
    auto load_b = [&](int k0, Regs& R, int half) __attribute__((always_inline)) {      // half 0: rows 0, 1; 1: rows 2, 3
        if constexpr (Conv) {
            const u32x4* src = conv_src(k0);
            if (half == 0) { R.b0 = src[0]; R.b1 = src[1]; } else { R.b2 = src[2]; R.b3 = src[3]; }
        } else {
            if (half == 0) { R.b0 = *b_src(0, k0); R.b1 = *b_src(1, k0); } else { R.b2 = *b_src(2, k0); R.b3 = *b_src(3, k0); }
        }
    };
    auto load_stage = [&](int k0, Regs& R) __attribute__((always_inline)) { load_a(k0, R); load_b(k0, R, 0); load_b(k0, R, 1); };
    auto store_stage = [&](int buf, const Regs& R) __attribute__((always_inline)) {
        uint8_t* ad = As(buf) + arow * kRow + apart * 16;
        *(u32x4*)(ad) = R.a0;
        if constexpr (AP > 1) *(u32x4*)(ad + (T / 4) * kRow) = R.a1;
        if constexpr (AP > 2) { *(u32x4*)(ad + 2 * (T / 4) * kRow) = R.a2; *(u32x4*)(ad + 3 * (T / 4) * kRow) = R.a3; }
        auto put = [&](int g, uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3) __attribute__((always_inline)) {      // dword g of rows k..k+3
            // v_perm_b32(hi, lo, sel): byte k of the result = byte sel.k of the 8 bytes {hi:lo} (lo = bytes 0..3)
            const uint32_t ab02 = __builtin_amdgcn_perm(w1, w0, 0x06020400u), ab13 = __builtin_amdgcn_perm(w1, w0, 0x07030501u);
            const uint32_t cd02 = __builtin_amdgcn_perm(w3, w2, 0x06020400u), cd13 = __builtin_amdgcn_perm(w3, w2, 0x07030501u);
            uint8_t* dst = Bs(buf) + ((bG * 4 + g) * kRow) + 4 * bkq;                    // + s * kBG * 4 * kRow: digit 4g+s
            *(uint32_t*)(dst + 0 * kBG * 4 * kRow) = __builtin_amdgcn_perm(cd02, ab02, 0x05040100u);
            *(uint32_t*)(dst + 1 * kBG * 4 * kRow) = __builtin_amdgcn_perm(cd13, ab13, 0x05040100u);
            *(uint32_t*)(dst + 2 * kBG * 4 * kRow) = __builtin_amdgcn_perm(cd02, ab02, 0x07060302u);
            *(uint32_t*)(dst + 3 * kBG * 4 * kRow) = __builtin_amdgcn_perm(cd13, ab13, 0x07060302u);
        };
        put(0, R.b0.x, R.b1.x, R.b2.x, R.b3.x);
        put(1, R.b0.y, R.b1.y, R.b2.y, R.b3.y);
        put(2, R.b0.z, R.b1.z, R.b2.z, R.b3.z);
        put(3, R.b0.w, R.b1.w, R.b2.w, R.b3.w);
    };

    v16i acc[IFR][4];
#pragma unroll
    for (int i = 0; i < IFR; i++)
#pragma unroll
        for (int s = 0; s < 4; s++) acc[i][s] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

    const int nk = (int)(kpad / kKT);
    const int n = lane & 31, kh = lane >> 5;
    const int fa = (wm * 32 * IFR + n) * kRow + kh * 16;                         // + i*32*kRow + ks*32
    const int fb = (((wn * 8 + (n >> 2)) * 4) + (n & 3)) * kRow + kh * 16;       // + s*kBG*4*kRow + ks*32
    // Software pipeline inside the wave (one wave per SIMD: nothing else hides latency).  Stage kt works on
    // LDS buffer kt & 1 and holds ALL its fragments in registers when it starts; its two halves of K are
    //   MFMAs of the first half   | byte transposes and LDS writes of stage kt + 1 (other buffer)
    //   barrier
    //   MFMAs of the second half  | fragment reads of stage kt + 1 (both halves), global loads of stage kt + 3
    // so the barrier is followed by MFMAs whose operands are already there, and no LDS latency is exposed.
    // Why one barrier is enough: a wave in the first half of stage kt has passed the barrier of stage kt - 1,
    // before which every wave finished its reads of buffer (kt + 1) & 1 (they belong to the second half of
    // stage kt - 2); and the reads after the barrier of stage kt see all writes before it.
    // Registers: first-half fragments (a0, b0) are free again after the first half; second-half fragments
    // alternate between two sets by the parity of the stage; global data of stage j lives in set j & 1.
    // sched_group_barrier(mask, n, id): 0x8 MFMA, 0x100 LDS read, 0x200 LDS write, 0x2 vector ALU, 0x20 global load.
    v4i a0[IFR], b0[4], a1[IFR], b1[4], a2[IFR], b2[4];
    auto read_frags = [&](int buf, int ks, v4i (&a)[IFR], v4i (&b)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < IFR; i++) a[i] = *(const v4i*)(As(buf) + fa + i * 32 * kRow + ks * 32);
#pragma unroll
        for (int q = 0; q < 4; q++) b[q] = *(const v4i*)(Bs(buf) + fb + q * kBG * 4 * kRow + ks * 32);
    };
    auto mfma_rows = [&](int i0, int i1, const v4i (&a)[IFR], const v4i (&b)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = i0; i < i1; i++)
#pragma unroll
            for (int q = 0; q < 4; q++) acc[i][q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[q], acc[i][q], 0, 0, 0);
    };
    auto mfma16 = [&](const v4i (&a)[IFR], const v4i (&b)[4]) __attribute__((always_inline)) { mfma_rows(0, IFR, a, b); };
    // one stage that has a successor: Rn holds stage kt + 1 and receives stage kt + 3; (as, bs) are this
    // stage's second-half fragments, (an, bn) receive the next stage's
    auto stage = [&](int kt, Regs& Rn, const v4i (&as)[IFR], const v4i (&bs)[4], v4i (&an)[IFR], v4i (&bn)[4]) __attribute__((always_inline)) {
        const int cur = kt & 1;
        const int knext = (kt + 3 < nk ? kt + 3 : nk - 1) * kKT;    // past the end: the last stage again, unused (no branch, so no
                                                                    // wait on these loads is forced before they are needed)
        // The global loads are spread over the whole stage, one per four MFMAs: the four waves of a block run in step,
        // and eight loads per wave in a row fill the queue to the texture unit, which then holds up the MFMAs behind them.
        store_stage(cur ^ 1, Rn);
        load_a(knext, Rn);                       // (after the LDS writes of the weight pieces have read these registers)
        mfma16(a0, b0);
#pragma unroll
        for (int t = 0; t < 4 * IFR; t++) {      // 32 byte permutes, 8 + AP LDS writes and AP global loads among 4 IFR MFMAs
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, IFR == 4 ? 3 : 5, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, IFR == 4 ? 1 : 2, 0);
            if (t >= AP && (t - AP) % 3 == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        load_b(knext, Rn, 0);
        // the fragments the next stage needs first are read first: two scheduling regions
        read_frags(cur ^ 1, 0, a0, b0);
        mfma_rows(0, IFR / 2, as, bs);
#pragma unroll
        for (int t = 0; t < 2 * IFR; t++) {      // IFR + 4 fragment reads, AP + 4 global loads and their addresses among 2 IFR MFMAs
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, IFR == 4 ? 1 : 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, Conv ? 6 : 2, 0);
            if (t % (IFR == 4 ? 4 : 2) == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_b(knext, Rn, 1);
        read_frags(cur ^ 1, 1, an, bn);
        mfma_rows(IFR / 2, IFR, as, bs);
#pragma unroll
        for (int t = 0; t < 2 * IFR; t++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, IFR == 4 ? 1 : 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, Conv ? 6 : 2, 0);
            if (t % (IFR == 4 ? 4 : 2) == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    load_stage(0, Rx);
    if (nk > 1) load_stage(kKT, Ry);
    store_stage(0, Rx);
    __syncthreads();
    load_stage((2 < nk ? 2 : nk - 1) * kKT, Rx);
    read_frags(0, 0, a0, b0);
    read_frags(0, 1, a1, b1);
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) { stage(kt, Ry, a1, b1, a2, b2); stage(kt + 1, Rx, a2, b2, a1, b1); }
    if (kt + 1 < nk) {      // nk even: one more stage with a successor, which leaves the last fragments in the second set
        stage(kt, Ry, a1, b1, a2, b2);
#pragma unroll
        for (int i = 0; i < IFR; i++) a1[i] = a2[i];
#pragma unroll
        for (int q = 0; q < 4; q++) b1[q] = b2[q];
    }
    mfma16(a0, b0);         // last stage: nothing left to fetch
    mfma16(a1, b1);

    // ---- epilogue: reduce mod p, pack the four digits of a dword, stage the output tile in LDS as
    // [group][row][16 digits] and store it 16 bytes per lane, consecutive lanes consecutive rows (rows of one
    // group are consecutive 16-byte words in memory) ----
    __syncthreads();                                    // every wave is done with the operand buffers
    const int Gl = wn * 8 + (n >> 2), g = n & 3;
    uint32_t one4 = 0;
    if (bias) {
        const int G = grp0 + Gl;
        if (G < ngroups) one4 = *(const uint32_t*)(P.one + (G / A.batch) * 16 + 4 * g);
    }
    auto red1 = [&](uint32_t v) -> uint32_t { return v - mul24(mulhi(v, mmagic), prime); };      // v < 2^24
    // 16 accumulators (four output dwords) at a time: enough independent work to fill the latencies (one wave per SIMD:
    // nothing else does), the two rare steps under one uniform branch per 16 instead of one per element, and the
    // scheduler cannot pull all 256 accumulator reads to the front.
#pragma unroll
    for (int i = 0; i < IFR; i++)
#pragma unroll
        for (int rq = 0; rq < 4; rq++) {
            uint32_t v[4][4];
#pragma unroll
            for (int rr = 0; rr < 4; rr++)
#pragma unroll
                for (int s = 0; s < 4; s++) v[rr][s] = (uint32_t)acc[i][s][rq * 4 + rr];
            const int jl0 = wm * 32 * IFR + i * 32 + rq * 8 + kh * 4;           // + rr
            if (!Plain && !small_acc) {       // large accumulators: below 2^24 first (v = hi * 4096 + lo)
#pragma unroll
                for (int rr = 0; rr < 4; rr++)
#pragma unroll
                    for (int s = 0; s < 4; s++) v[rr][s] = mul24(red1(v[rr][s] >> 12), pow12) + (v[rr][s] & 4095u);
            }
            if (!Plain && bias) {
#pragma unroll
                for (int rr = 0; rr < 4; rr++) {
                    const int j = row0 + jl0 + rr;
                    const int32_t bj = j < M ? bias[j] % (int32_t)prime : 0;
                    const uint32_t bm = (uint32_t)(bj < 0 ? bj + (int32_t)prime : bj);
#pragma unroll
                    for (int s = 0; s < 4; s++) v[rr][s] = red1(v[rr][s]) + mul24(bm, (one4 >> (8 * s)) & 0xffu);
                }
            }
#pragma unroll
            for (int rr = 0; rr < 4; rr++) {
                const uint32_t d0 = red1(v[rr][0]), d1 = red1(v[rr][1]), d2 = red1(v[rr][2]), d3 = red1(v[rr][3]);
                *(uint32_t*)(smem + Gl * kOutStride + (jl0 + rr) * 16 + 4 * g) = d0 | (d1 << 8) | (d2 << 16) | (d3 << 24);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    __syncthreads();
    // group gl of the tile is stored by all lanes together, lane -> row (kBM a multiple of T, or T of kBM)
    {
        constexpr int kPerGroup = kBM >= T ? kBM / T : 1;          // pieces per lane and group
        constexpr int kGroupsPerPass = kBM >= T ? 1 : T / kBM;     // groups stored side by side
        const int gsub = kBM >= T ? 0 : tid / kBM, jbase = kBM >= T ? tid : tid % kBM;
        int G = grp0 + gsub;
        int och = G / A.batch, ob = G - och * A.batch;             // one division; the rest is counted up
        const int batch = A.batch;
        const int64_t ocs = P.out.cs;
        uint8_t* const obase = P.out.p;
#pragma unroll 4
        for (int gl = gsub; gl < kBG; gl += kGroupsPerPass) {
            if (G < ngroups) {
#pragma unroll
                for (int t = 0; t < kPerGroup; t++) {
                    const int jl = jbase + t * T, j = row0 + jl;
                    if (j < M) *(u32x4*)(obase + (int64_t)och * ocs + ((int64_t)ob * M + j) * 16) = *(const u32x4*)(smem + gl * kOutStride + jl * 16);
                }
            }
            G += kGroupsPerPass; ob += kGroupsPerPass;
            while (ob >= batch) { ob -= batch; och++; }
        }
    }
}

// true if the MFMA path should take this dense or convolution layer (large enough to fill tiles; for a
// convolution the channel count must be a multiple of 4, see above)
bool dense_mfma_wanted(const dash_layer* L, int64_t batch) {
    if (L->kind == DASH_DENSE) return (int64_t)L->in_c * L->out_c >= 64 * 64 && (int64_t)L->out_c * batch >= 64;
    if (L->kind != DASH_CONV2D || L->in_c % 4 != 0 || L->stride < 1) return false;
    const int64_t K = (int64_t)L->kh * L->kw * L->in_c;
    const int64_t oh = (L->in_h + 2 * L->pad - L->kh) / L->stride + 1, ow = (L->in_w + 2 * L->pad - L->kw) / L->stride + 1;
    // (K * in_c < 2^31: the multiply-high divisions by in_c and kw are exact)
    return K * L->out_c >= 64 * 64 && K * L->in_c < (1ll << 31) && batch * oh * ow >= 16 && batch * oh * ow < (1ll << 31);
}

int dense_mfma(dash_ctx* c, const dash_layer* L, bool garble, const dash_labels* in, dash_labels* out, hipStream_t s) {
    const bool conv = L->kind == DASH_CONV2D;
    const int out_h = conv ? (L->in_h + 2 * L->pad - L->kh) / L->stride + 1 : 1, out_w = conv ? (L->in_w + 2 * L->pad - L->kw) / L->stride + 1 : 1;
    const int M = L->out_c, K = conv ? L->kh * L->kw * L->in_c : L->in_c;
    const int64_t batch = conv ? L->n_elem * out_h * out_w : L->n_elem;      // columns: batch elements, or output pixels
    GemmArgs A;
    memset(&A, 0, sizeof(A));
    A.M = M; A.K = K; A.batch = (int)batch; A.nprimes = c->k;
    if (conv) {
        A.conv = 1; A.in_h = L->in_h; A.in_w = L->in_w; A.in_c = L->in_c; A.kw = L->kw; A.stride = L->stride; A.pad = L->pad;
        A.out_h = out_h; A.out_w = out_w;
        A.c_magic = (uint32_t)(((1ull << 32) + L->in_c - 1) / L->in_c);
        A.kw_magic = L->kw > 1 ? (uint32_t)(((1ull << 32) + L->kw - 1) / L->kw) : 0;
        A.zero = c->d_zero;
    }
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
    if ((int64_t)max_nchunk * batch >= (1ll << 31) - 64) return DASH_ESIZE;      // group indices are 32-bit in the kernel
    // tile shape.  Measured on 4096 x 4096, batch 128, 12 primes: 256 x 256 (one wave per SIMD) 1.30 ms, 128 x 512
    // (two waves per SIMD) 1.41 ms; the latter wastes half as many rows when there are at most 128 outputs.
    const bool wide = c->gemm_tile ? c->gemm_tile == 2 : M <= 128;
    auto launch = [&](auto tl) -> int {
        typedef decltype(tl) TL;
        const int gy = (M + TL::BM - 1) / TL::BM;
        A.sty = gy >= 4 ? 4 : gy >= 2 ? 2 : 1;
        const int kStX = kStBlocks / A.sty;
        A.gy4 = (gy + A.sty - 1) / A.sty;
        int64_t st_total = 0;
        for (int i = 0; i < c->k; i++) {
            A.st_first[i] = (int)st_total;
            const int64_t gb = ((int64_t)A.pr[i].nchunk * batch + TL::BG - 1) / TL::BG;
            st_total += (gb + kStX - 1) / kStX * A.gy4;
            if (st_total > (1 << 24)) return DASH_ESIZE;
        }
        A.st_first[c->k] = (int)st_total;
        A.st_total = (int)st_total;
        dim3 grid((uint32_t)((st_total + kXcds - 1) / kXcds * kXcds * kStBlocks));
        ProfScope ps(c->prof, DASH_PROF_LINEAR, s, macs, bytes);
        const bool plain = A.small_acc && !A.bias;
        auto kernel = conv ? (plain ? k_dense_mfma<TL, true, true> : k_dense_mfma<TL, true, false>)
                           : (plain ? k_dense_mfma<TL, false, true> : k_dense_mfma<TL, false, false>);
        hipLaunchKernelGGL(kernel, grid, dim3(TL::T), 0, s, A);
        return DASH_OK;
    };
    const int st = wide ? launch(TileWide{}) : launch(TileBig{});
    if (st) return st;
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
