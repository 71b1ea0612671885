// dash_gates.hip -- gate-level kernels over LabelTensors.
//
//   k_draw        : PRG labels (fresh zero labels of gate outputs, input wires, masks)
//   k_affine      : free gates: out = sum_t coef_t * term_t mod m   (Sec. Arithmetic Garbled Circuits)
//   k_proj_garble : one lane per ciphertext row: hash the label of value a, add the payload, store
//                   the row at the position its colour names            (projection gates, point-and-permute)
//   (the fused digit gates of the sign gadget: dash_gates_digits.hip; the evaluator's kernels: dash_gates_eval.hip,
//   dash_gates_digits_eval.hip, dash_gates_cast.hip)
//
// A launch carries up to 16 homogeneous gate batches ("jobs", blockIdx.y); every lane of a block
// works on the same pair of moduli, so all modulus-dependent control flow is wave-uniform.  The
// moduli that carry nearly all of the work (the CRT primes and the accumulation moduli of the
// default digit sets, under the ceil label-length rule) run through compile-time descriptions; any
// other modulus takes the same code with run-time constants.
#include "dash_tabs.h"

namespace dash {

// ------------------------------------------------------------------------------------------ draw
template <bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_draw(const DrawLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.jobs[blockIdx.y].n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) draw_body(L, tile, blockIdx.y, tx, T);
}

int launch_draw(const dash_ctx* c, DrawLaunch& L, int njobs, hipStream_t s) {
    static_assert(sizeof(DrawLaunch) <= 4096, "kernel argument block");
    if (njobs < 1 || njobs > kMaxDrawJobs) return DASH_EINVAL;
    uint64_t lanes = 0;
    uint32_t nmax = 0;
    for (int j = 0; j < njobs; j++) {
        if (L.jobs[j].n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
        lanes += L.jobs[j].n_elem;
        nmax = L.jobs[j].n_elem > nmax ? L.jobs[j].n_elem : nmax;
    }
    if (nmax == 0) return DASH_OK;
    L.key = c->seed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    const bool banked = lanes >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((nmax + kThreads - 1) / kThreads, njobs, banked), njobs);
    if (banked) hipLaunchKernelGGL(k_draw<true>, grid, dim3(kBigThreads), 0, s, L);
    else hipLaunchKernelGGL(k_draw<false>, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ---------------------------------------------------------------------------------------- affine
__global__ __launch_bounds__(kThreads) void k_affine(const AffineLaunch L) {
    affine_body(L, blockIdx.x, blockIdx.y, threadIdx.x);
}

int launch_affine(const dash_ctx* c, AffineLaunch& L, int njobs, hipStream_t s) {
    static_assert(sizeof(AffineLaunch) <= 4096, "kernel argument block");
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.mods = c->d_mods;
    uint32_t nchunk = 1;
    for (int j = 0; j < njobs; j++) {
        AffineJob& J = L.jobs[j];
        if (J.m < 2 || J.m > 255 || J.term_count == 0 || J.term_first + J.term_count > (uint32_t)kMaxTerms) return DASH_EINVAL;
        J.unit = 1;
        for (uint32_t t = 0; t < J.term_count; t++) if (L.terms[J.term_first + t].coef != 1) J.unit = 0;
        nchunk = c->mods[J.m].nchunk > nchunk ? c->mods[J.m].nchunk : nchunk;
    }
    dim3 grid((uint32_t)(((uint64_t)L.n_elem * nchunk + kThreads - 1) / kThreads), njobs);
    hipLaunchKernelGGL(k_affine, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------------------- packed table rows
// one lane per row: working format [pitch_q bytes, one digit each] <-> 16-byte integer sum_j row[j] q^j
template <bool Pack>
__global__ __launch_bounds__(kThreads) void k_rows_repack(const PackLaunch L) {
    const PackSeg& S = L.seg[blockIdx.y];
    const uint64_t rows = (uint64_t)L.n_elem * S.rows_per_gate;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    if (S.q == 0) {                     // one-digit rows; the packed segment is padded with zeros to a multiple of 16 bytes
        const uint64_t padded = (rows + 15) & ~(uint64_t)15;
        for (uint64_t r = (uint64_t)blockIdx.x * kThreads + threadIdx.x; r < padded; r += (uint64_t)gridDim.x * kThreads) {
            if (Pack) S.packed[r] = r < rows ? S.rows[r * 4] : 0;
            else if (r < rows) *(uint32_t*)(const_cast<uint8_t*>(S.rows) + r * 4) = S.packed[r];
        }
        return;
    }
    for (uint64_t r = (uint64_t)blockIdx.x * kThreads + threadIdx.x; r < rows; r += (uint64_t)gridDim.x * kThreads) {
        const ModInfo M = L.mods[S.q];
        uint32_t* row = (uint32_t*)(const_cast<uint8_t*>(S.rows) + r * (M.ndw * 4));
        if (Pack) {
            uint32_t colour;
            const U128 x = compress(M, [&](int i) { return row[i]; }, &colour);
            *(u32x4*)(S.packed + r * 16) = u32x4{x.w[0], x.w[1], x.w[2], x.w[3]};
        } else {
            const u32x4 v = *(const u32x4*)(S.packed + r * 16);
            const U128 x = {{v.x, v.y, v.z, v.w}};
            decompress(M, x, [&](int i, uint32_t w) { row[i] = w; });
        }
    }
}

int launch_pack(const dash_ctx* c, PackLaunch& L, bool pack, hipStream_t s) {
    static_assert(sizeof(PackLaunch) <= 4096, "kernel argument block");
    if (L.nseg < 1 || L.nseg > (uint32_t)kMaxPackSegs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    L.mods = c->d_mods;
    uint64_t rows = 0;
    for (uint32_t i = 0; i < L.nseg; i++) {
        const uint64_t r = (uint64_t)L.n_elem * L.seg[i].rows_per_gate + 15;      // (+ the padding of a one-digit segment)
        rows = r > rows ? r : rows;
    }
    const uint64_t tiles = (rows + kThreads - 1) / kThreads;
    dim3 grid(grid_x_for(tiles, (int)L.nseg), L.nseg);
    if (pack) hipLaunchKernelGGL(k_rows_repack<true>, grid, dim3(kThreads), 0, s, L);
    else hipLaunchKernelGGL(k_rows_repack<false>, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ---------------------------------------------------------------------------------------- garble
// One instantiation per output-modulus description: QD = ModInfo (any modulus, run-time constants) or
// CMod<m, lam> for the hot moduli.  The input modulus is dispatched inside (its code is small).
// Rows of 64 bytes or more (pitch a multiple of 16): a lane that stored its own row dword by dword would
// touch 64 different cache lines with every store instruction.  Such rows are staged in LDS (row stride
// one word more than the pitch, so the column accesses spread over the banks) and written by the whole
// block, each lane 16 consecutive bytes, consecutive lanes consecutive pieces of a row.
template <class QD> struct stage_rows { static constexpr bool value = false; static constexpr int ndw = 1; };
template <uint32_t MOD, uint32_t LAM> struct stage_rows<CMod<MOD, LAM>> {
    static constexpr int ndw = (LAM + 3) / 4;
    static constexpr bool value = ndw >= 16 && ndw % 4 == 0;
};
struct StagedSink {
    uint32_t* st;        // this lane's row in LDS
    uint32_t* slot;      // where the row index goes
    __device__ __forceinline__ void begin(uint8_t*, uint64_t row_index, uint32_t) { *slot = (uint32_t)row_index; }
    __device__ __forceinline__ void put(int i, uint32_t w) { st[i] = w; }
};

// a row kept in the lane's registers, with the address it goes to (0: the lane has no row to stage)
template <int NDW> struct RegSink {
    uint32_t w[NDW];
    uint64_t addr = 0;
    __device__ __forceinline__ void begin(uint8_t* table, uint64_t row_index, uint32_t pitch) { addr = (uint64_t)(table + row_index * pitch); }
    __device__ __forceinline__ void put(int i, uint32_t v) { w[i] = v; }
};

template <class QD, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads, Banked ? 8 : 1) void k_proj_garble(const GateLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    const uint64_t rows = (uint64_t)L.jobs[blockIdx.y].n_elem * L.jobs[blockIdx.y].p;      // (unused by the one-dimensional banked forms)
    const uint32_t tiles = (uint32_t)((rows + kThreads - 1) / kThreads);
    if constexpr (stage_rows<QD>::value && Banked) {
        // Long rows with the bank-replicated tables: 64 KB of tables leave room to stage 16 dwords per lane, so a lane keeps
        // its row in registers and its wave writes the rows out in ndw / 16 passes of 64 bytes per row, 16 bytes per lane,
        // consecutive lanes consecutive pieces.  One-dimensional grid over the tiles of all jobs.
        constexpr int ndw = stage_rows<QD>::ndw, kPass = 16, stride = kPass + 1, pieces = kPass / 4;
        static_assert(ndw % kPass == 0, "whole passes");
        __shared__ uint32_t tt[kBankTabWords];
        __shared__ uint32_t stage[kBigThreads * stride];
        __shared__ uint64_t sdst[kBigThreads];
        const BankTab T = load_banktab(tt, L.ttab);
        const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
        const int lane = threadIdx.x & 63, w0 = threadIdx.x & ~63;       // this wave's rows: w0 .. w0 + 63
        auto tiles_of = [&](uint32_t j) { return (uint32_t)(((uint64_t)L.jobs[j].n_elem * L.jobs[j].p + kThreads - 1) / kThreads); };
        uint32_t total = 0;
        for (uint32_t j = 0; j < L.njobs; j++) total += tiles_of(j);
        uint32_t job = 0, base = 0, next = tiles_of(0);
        // (every wave stages and writes out its own 64 rows: no barrier between waves)
        const uint32_t rounds = (total + gridDim.x * kGateTiles - 1) / (gridDim.x * kGateTiles);
        for (uint32_t r = 0; r < rounds; r++) {
            const uint32_t t = (r * gridDim.x + blockIdx.x) * kGateTiles + sub;
            RegSink<ndw> sink;
            if (t < total) {
                while (t >= next) { job++; base = next; next += tiles_of(job); }
                garble_body<QD>(L, t - base, __builtin_amdgcn_readfirstlane(job), tx, T, sink);
            }
            sdst[threadIdx.x] = sink.addr;
#pragma unroll
            for (int pass = 0; pass < ndw / kPass; pass++) {
                if (sink.addr) {
#pragma unroll
                    for (int i = 0; i < kPass; i++) stage[threadIdx.x * stride + i] = sink.w[pass * kPass + i];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                for (int id = lane; id < 64 * pieces; id += 64) {
                    const int k = w0 + id / pieces, part = id % pieces;
                    const uint64_t d = sdst[k];
                    if (d) {
                        const uint32_t* src = stage + k * stride + part * 4;
                        uint32_t* dst = (uint32_t*)(d + (uint64_t)pass * (kPass * 4) + part * 16);
                        uint32_t v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];
                        dst[0] = v0; dst[1] = v1; dst[2] = v2; dst[3] = v3;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    } else if constexpr (stage_rows<QD>::value) {
        // Long rows, shared tables: every WAVE stages its 64 rows in its own part of LDS and writes them out itself, 16 bytes
        // per lane, eight consecutive lanes one row: no barrier between waves (a wave's LDS accesses complete in order).
        __shared__ uint32_t tt[kTabWords];
        const LdsTab T = load_ttab(tt, L.ttab);
        constexpr int ndw = stage_rows<QD>::ndw, stride = ndw + 1, pieces = ndw / 4;
        __shared__ uint32_t stage[kThreads * stride];
        __shared__ uint32_t srow[kThreads];
        uint8_t* table = L.jobs[blockIdx.y].table;
        const int lane = threadIdx.x & 63, w0 = threadIdx.x & ~63;       // this wave's rows: w0 .. w0 + 63
        for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
            srow[threadIdx.x] = 0xffffffffu;
            StagedSink sink{stage + threadIdx.x * stride, srow + threadIdx.x};
            garble_body<QD>(L, tile, blockIdx.y, threadIdx.x, T, sink);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int id = lane; id < 64 * pieces; id += 64) {
                const int k = w0 + id / pieces, part = id % pieces;
                const uint32_t r = srow[k];
                if (r != 0xffffffffu) {
                    const uint32_t* src = stage + k * stride + part * 4;
                    uint32_t* dst = (uint32_t*)(table + (uint64_t)r * (ndw * 4) + part * 16);
                    uint32_t v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];
                    dst[0] = v0; dst[1] = v1; dst[2] = v2; dst[3] = v3;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        __shared__ uint32_t tt[gate_tab<Banked>::words];
        const auto T = gate_tab<Banked>::load(tt, L.ttab);
        const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
        if constexpr (Banked) {
            // one-dimensional grid: the jobs differ in length (n_elem * p rows), so the blocks share the
            // concatenation of all jobs' tiles evenly.  job, base and next are the same in all lanes of a wave.
            auto tiles_of = [&](uint32_t j) { return (uint32_t)(((uint64_t)L.jobs[j].n_elem * L.jobs[j].p + kThreads - 1) / kThreads); };
            uint32_t total = 0;
            for (uint32_t j = 0; j < L.njobs; j++) total += tiles_of(j);
            uint32_t job = 0, base = 0, next = tiles_of(0);
            for (uint32_t t = blockIdx.x * kGateTiles + sub; t < total; t += gridDim.x * kGateTiles) {
                while (t >= next) { job++; base = next; next += tiles_of(job); }
                DirectSink sink;
                garble_body<QD>(L, t - base, __builtin_amdgcn_readfirstlane(job), tx, T, sink);
            }
        } else {
            for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) {
                DirectSink sink;
                garble_body<QD>(L, tile, blockIdx.y, tx, T, sink);
            }
        }
    }
}

#define DASH_GARBLE_K(MOD, LAM) k_proj_garble<CMod<MOD, LAM>, false>,
static const GateKernel kGarbleKernels[] = {k_proj_garble<ModInfo, false>, DASH_HOT_MODS(DASH_GARBLE_K)};
#undef DASH_GARBLE_K
// with BankTab
#define DASH_GARBLE_KB(MOD, LAM) k_proj_garble<CMod<MOD, LAM>, true>,
static const GateKernel kGarbleKernelsBanked[] = {k_proj_garble<ModInfo, true>, DASH_HOT_MODS(DASH_GARBLE_KB)};
#undef DASH_GARBLE_KB
#define DASH_GARBLE_S(MOD, LAM) stage_rows<CMod<MOD, LAM>>::value,
static const bool kGarbleStaged[] = {false, DASH_HOT_MODS(DASH_GARBLE_S)};
#undef DASH_GARBLE_S


int launch_garble(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    uint64_t rows = 0, tiles_sum = 0;      // rows of the largest job; tiles of all jobs
    double units = 0, bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
        if (J.n_elem == 0) continue;
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table) return DASH_EINVAL;
        const uint64_t r = (uint64_t)J.n_elem * J.p;
        rows = r > rows ? r : rows;
        tiles_sum += (r + kThreads - 1) / kThreads;
        const double lp = c->mods[J.p].lam, lq = J.mode == PAY_SHORT ? 1 : c->mods[J.q].lam;
        units += (double)r;
        bytes += (double)J.n_elem * (lp + (J.phi_stride ? J.p : 0) + lq + J.p * lq + (J.mode == PAY_EHALF ? lq : 0));
    }
    if (rows == 0) return DASH_OK;
    const uint64_t blocks = (rows + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffull || tiles_sum > 0x7fffffffull) return DASH_ESIZE;
    // jobs with one output modulus run its instantiation; a mix of output moduli (many small batches
    // in one launch) runs the instantiation with run-time constants
    const uint32_t q = common_q(L, njobs);
    if (rows >= (1ull << 32)) return DASH_ESIZE;      // staged rows carry a 32-bit row index
    const int ki = q ? hot_mod_index(c->mods[q]) : 0;
    const bool staged = kGarbleStaged[ki];
    const bool banked = (uint64_t)units >= c->banked_min_lanes;
    L.njobs = (uint32_t)njobs;
    dim3 grid(gate_grid_x_for(blocks, njobs, banked), njobs);
    if (banked) {       // one-dimensional: all jobs' tiles, 1024 lanes (4 tiles) per block at a time, two blocks per CU
        const uint64_t nb = (tiles_sum + 3) / 4;
        const uint64_t cap = staged ? 256 : 512;      // (long rows also stage in LDS: one block per CU)
        grid = dim3((uint32_t)(nb < cap ? nb : cap));
    }
    ProfScope ps(c->prof, DASH_PROF_GARBLE, s, units, bytes);
    GateKernel k = banked ? kGarbleKernelsBanked[ki] : kGarbleKernels[ki];
    if (ki == 0 && !banked && (uint64_t)units <= c->few_rows_max) k = k_proj_garble<PerJobMod, false>;      // few rows: see garble_body
    hipLaunchKernelGGL(k, grid, dim3(banked ? kBigThreads : kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
