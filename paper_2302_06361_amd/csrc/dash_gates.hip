// dash_gates.hip -- gate-level kernels over LabelTensors.
//
//   k_draw        : PRG labels (fresh zero labels of gate outputs, input wires, masks)
//   k_affine      : free gates: out = sum_t coef_t * term_t mod m   (Sec. Arithmetic Garbled Circuits)
//   k_proj_garble : one lane per ciphertext row: hash the label of value a, add the payload, store
//                   the row at the position its colour names            (projection gates, point-and-permute)
//   k_proj_eval   : one lane per gate: hash the active label, fetch the row its colour names, subtract
//   k_hg_finish   : evaluator side of the mixed-modulus half gate       (Appendix)
//
// A launch carries up to 16 homogeneous gate batches ("jobs", blockIdx.y); every lane of a block
// works on the same pair of moduli, so all modulus-dependent control flow is wave-uniform.  The
// moduli that carry nearly all of the work (the CRT primes and the accumulation moduli of the
// default digit sets, under the ceil label-length rule) run through compile-time descriptions; any
// other modulus takes the same code with run-time constants.
#include "dash_bodies.h"
#include "dash_internal.h"

namespace dash {

// AES tables in LDS, two layouts.
//
// LdsTab: T0..T3 once, 4 KB, shared by the block.  A wave's 64 look-ups fall on the 32 banks at random
// (bank = index mod 32): two thirds of the LDS cycles are bank collisions (SQ_LDS_BANK_CONFLICT /
// SQ_LDS_IDX_ACTIVE = 0.68), and AES alone runs at 3.8e10 blocks/s on the chip, exactly what 160 look-ups of
// 6.4 LDS cycles each allow.
//
// BankTab: every entry of T0 and T1 once per bank, 64 KB, for blocks of 1024 lanes (two blocks per CU, eight
// waves per SIMD); T2 and T3 are T0 and T1 rotated by 16 bits, one rotation per column for both.  Byte address
// of entry x of table R (0 or 1) for a lane that owns bank b:  x * 256 + R * 128 + b * 4,  so a look-up never
// collides, and the address still costs ONE instruction, a byte permute: byte 0 <- 4b (from the lane's
// constant), byte 1 <- the state byte; R * 128 goes into the instruction's offset.
//
// Measured on the LeNet batch-16 step: BankTab garbles 3.4e10 rows/s against 2.9e10, but launches that do not
// fill the chip get slower (64 KB to fill per block, fewer and larger blocks), so each kernel exists in both
// forms and the launcher takes BankTab from kBankedMinLanes lanes up.
constexpr int kTabWords = 1024;
constexpr int kBankTabWords = 16384;
constexpr int kBigThreads = 1024;                               // lanes per block with BankTab


struct LdsTab {
    const uint32_t* t;
    template <int R, int B> __device__ __forceinline__ uint32_t at(uint32_t w) const { return t[R * 256 + ((w >> (8 * B)) & 0xffu)]; }
};

__device__ __forceinline__ LdsTab load_ttab(uint32_t* lds, const uint32_t* g) {
    for (int i = threadIdx.x; i < kTabWords; i += blockDim.x) lds[i] = g[i];
    __syncthreads();
    return LdsTab{lds};
}

struct BankTab {
    static constexpr bool two_tables = true;
    const uint8_t* t;
    uint32_t lane;       // byte 0: 4 * bank
    template <int R, int B> __device__ __forceinline__ uint32_t at(uint32_t w) const {
        static_assert(R < 2, "T0 and T1 only");
        // v_perm_b32(hi = w, lo = lane): selector 0..3 bytes of lane, 4..7 bytes of w, 0x0c zero
        constexpr uint32_t sel = 0x0c0c0000u | ((4u + B) << 8);
        const uint32_t a = __builtin_amdgcn_perm(w, lane, sel);
        return *(const uint32_t*)(t + a + R * 128);
    }
};

__device__ __forceinline__ BankTab load_banktab(uint32_t* lds, const uint32_t* g) {
    // one global load per lane (entry x of table R), then its 32 copies as 8 16-byte LDS writes
    for (int e = threadIdx.x; e < 512; e += blockDim.x) {
        const uint32_t v = g[e];
        const int R = e >> 8, x = e & 255;
        uint4* dst = (uint4*)(lds + x * 64 + R * 32);
        const uint4 v4 = make_uint4(v, v, v, v);
#pragma unroll
        for (int i = 0; i < 8; i++) dst[i] = v4;
    }
    __syncthreads();
    return BankTab{(const uint8_t*)lds, (threadIdx.x & 31u) << 2};
}

template <bool Banked> struct gate_tab {
    typedef LdsTab type;
    static constexpr int threads = kThreads, words = kTabWords;
    static __device__ __forceinline__ type load(uint32_t* lds, const uint32_t* g) { return load_ttab(lds, g); }
};
template <> struct gate_tab<true> {
    typedef BankTab type;
    static constexpr int threads = kBigThreads, words = kBankTabWords;
    static __device__ __forceinline__ type load(uint32_t* lds, const uint32_t* g) { return load_banktab(lds, g); }
};

// Blocks walk over tiles of kThreads lanes with a grid stride, so that the table copy in LDS is paid
// once per block and not once per tile.
__host__ inline uint32_t grid_x_for(uint64_t tiles, int njobs) {
    uint64_t cap = 2560 / (uint64_t)njobs;           // about two resident rounds of blocks on 256 CUs
    if (cap < 1) cap = 1;
    return (uint32_t)(tiles < cap ? tiles : cap);
}
// the same for blocks of kBigThreads lanes (kBigThreads / kThreads tiles at a time)
__host__ inline uint32_t gate_grid_x_for(uint64_t tiles, int njobs, bool banked) {
    if (!banked) return grid_x_for(tiles, njobs);
    constexpr int kGateTiles = kBigThreads / kThreads;
    uint64_t blocks = (tiles + kGateTiles - 1) / kGateTiles;
    uint64_t cap = 1024 / (uint64_t)njobs;           // two blocks per CU, two rounds
    if (cap < 1) cap = 1;
    return (uint32_t)(blocks < cap ? blocks : cap);
}

// ------------------------------------------------------------------------------------------ draw
template <bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_draw(const DrawLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) draw_body(L, tile, blockIdx.y, tx, T);
}

int launch_draw(const dash_ctx* c, DrawLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->seed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    const bool banked = (uint64_t)L.n_elem * njobs >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((L.n_elem + kThreads - 1) / kThreads, njobs, banked), njobs);
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

template <class QD, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_proj_garble(const GateLaunch L) {
    static_assert(!(stage_rows<QD>::value && Banked), "staged rows use the shared tables");
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    const uint64_t rows = (uint64_t)L.n_elem * L.jobs[blockIdx.y].p;
    const uint32_t tiles = (uint32_t)((rows + kThreads - 1) / kThreads);
    if constexpr (stage_rows<QD>::value) {
        __shared__ uint32_t tt[kTabWords];
        const LdsTab T = load_ttab(tt, L.ttab);
        constexpr int ndw = stage_rows<QD>::ndw, stride = ndw + 1, pieces = ndw / 4;
        __shared__ uint32_t stage[kThreads * stride];
        __shared__ uint32_t srow[kThreads];
        uint8_t* table = L.jobs[blockIdx.y].table;
        for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
            srow[threadIdx.x] = 0xffffffffu;
            StagedSink sink{stage + threadIdx.x * stride, srow + threadIdx.x};
            garble_body<QD>(L, tile, blockIdx.y, threadIdx.x, T, sink);
            __syncthreads();
            for (int id = threadIdx.x; id < kThreads * pieces; id += kThreads) {
                const int k = id / pieces, part = id - k * pieces;
                const uint32_t r = srow[k];
                if (r != 0xffffffffu) {
                    const uint32_t* src = stage + k * stride + part * 4;
                    uint32_t* dst = (uint32_t*)(table + (uint64_t)r * (ndw * 4) + part * 16);
                    uint32_t v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];
                    dst[0] = v0; dst[1] = v1; dst[2] = v2; dst[3] = v3;
                }
            }
            __syncthreads();
        }
    } else {
        __shared__ uint32_t tt[gate_tab<Banked>::words];
        const auto T = gate_tab<Banked>::load(tt, L.ttab);
        const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
        if constexpr (Banked) {
            // one-dimensional grid: the jobs differ in length (n_elem * p rows), so the blocks share the
            // concatenation of all jobs' tiles evenly.  job, base and next are the same in all lanes of a wave.
            auto tiles_of = [&](uint32_t j) { return (uint32_t)(((uint64_t)L.n_elem * L.jobs[j].p + kThreads - 1) / kThreads); };
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

typedef void (*GateKernel)(const GateLaunch);
#define DASH_GARBLE_K(MOD, LAM) k_proj_garble<CMod<MOD, LAM>, false>,
static const GateKernel kGarbleKernels[] = {k_proj_garble<ModInfo, false>, DASH_HOT_MODS(DASH_GARBLE_K)};
#undef DASH_GARBLE_K
// with BankTab (the kernel for staged rows stays with the shared tables)
template <class QD, bool Staged = stage_rows<QD>::value> struct banked_garble { static constexpr GateKernel k = k_proj_garble<QD, true>; };
template <class QD> struct banked_garble<QD, true> { static constexpr GateKernel k = k_proj_garble<QD, false>; };
#define DASH_GARBLE_KB(MOD, LAM) banked_garble<CMod<MOD, LAM>>::k,
static const GateKernel kGarbleKernelsBanked[] = {k_proj_garble<ModInfo, true>, DASH_HOT_MODS(DASH_GARBLE_KB)};
#undef DASH_GARBLE_KB
#define DASH_GARBLE_S(MOD, LAM) stage_rows<CMod<MOD, LAM>>::value,
static const bool kGarbleStaged[] = {false, DASH_HOT_MODS(DASH_GARBLE_S)};
#undef DASH_GARBLE_S

// every job of a gate launch must have the same output modulus; returns it (0 if they differ)
static uint32_t common_q(const GateLaunch& L, int njobs) {
    for (int j = 1; j < njobs; j++) if (L.jobs[j].q != L.jobs[0].q) return 0;
    return L.jobs[0].q;
}

int launch_garble(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    uint32_t pmax = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table) return DASH_EINVAL;
        pmax = J.p > pmax ? J.p : pmax;
    }
    uint64_t rows = (uint64_t)L.n_elem * pmax;
    uint64_t blocks = (rows + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffull) return DASH_ESIZE;
    double units = 0, bytes = 0;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        double lp = c->mods[J.p].lam, lq = J.mode == PAY_SHORT ? 1 : c->mods[J.q].lam;
        units += (double)L.n_elem * J.p;
        bytes += (double)L.n_elem * (lp + (J.phi_stride ? J.p : 0) + lq + J.p * lq + (J.mode == PAY_EHALF ? lq : 0));
    }
    // jobs with one output modulus run its instantiation; a mix of output moduli (many small batches
    // in one launch) runs the instantiation with run-time constants
    const uint32_t q = common_q(L, njobs);
    if (rows >= (1ull << 32)) return DASH_ESIZE;      // staged rows carry a 32-bit row index
    const int ki = q ? hot_mod_index(c->mods[q]) : 0;
    const bool staged = kGarbleStaged[ki];
    const bool banked = !staged && (uint64_t)units >= c->banked_min_lanes;
    L.njobs = (uint32_t)njobs;
    dim3 grid(gate_grid_x_for(blocks, njobs, banked), njobs);
    if (banked) {       // one-dimensional: all jobs' tiles, 1024 lanes (4 tiles) per block at a time, two blocks per CU
        uint64_t tiles = 0;
        for (int j = 0; j < njobs; j++) tiles += ((uint64_t)L.n_elem * L.jobs[j].p + kThreads - 1) / kThreads;
        const uint64_t nb = (tiles + 3) / 4;
        grid = dim3((uint32_t)(nb < 512 ? nb : 512));
    }
    ProfScope ps(c->prof, DASH_PROF_GARBLE, s, units, bytes);
    hipLaunchKernelGGL(banked ? kGarbleKernelsBanked[ki] : kGarbleKernels[ki], grid, dim3(banked ? kBigThreads : kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------------------------------ eval
template <class QD, bool Banked>
__global__ __launch_bounds__(gate_tab<Banked>::threads) void k_proj_eval(const GateLaunch L) {
    constexpr int kGateTiles = gate_tab<Banked>::threads / kThreads;
    __shared__ uint32_t tt[gate_tab<Banked>::words];
    const auto T = gate_tab<Banked>::load(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    const uint32_t sub = threadIdx.x / kThreads, tx = threadIdx.x % kThreads;
    for (uint32_t tile = blockIdx.x * kGateTiles + sub; tile < tiles; tile += gridDim.x * kGateTiles) eval_body<QD>(L, tile, blockIdx.y, tx, T);
}
#define DASH_EVAL_K(MOD, LAM) k_proj_eval<CMod<MOD, LAM>, false>,
static const GateKernel kEvalKernels[] = {k_proj_eval<ModInfo, false>, DASH_HOT_MODS(DASH_EVAL_K)};
#undef DASH_EVAL_K
#define DASH_EVAL_KB(MOD, LAM) k_proj_eval<CMod<MOD, LAM>, true>,
static const GateKernel kEvalKernelsBanked[] = {k_proj_eval<ModInfo, true>, DASH_HOT_MODS(DASH_EVAL_KB)};
#undef DASH_EVAL_KB

int launch_eval(const dash_ctx* c, GateLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    for (int j = 0; j < njobs; j++) {
        const GateJob& J = L.jobs[j];
        if (J.p < 2 || J.p > 255 || J.q < 2 || J.q > 255 || !c->mods[J.p].dtab || !c->mods[J.q].dtab) return DASH_EINVAL;
        if (!J.in.p || !J.table || !J.out.p) return DASH_EINVAL;
    }
    const bool banked = (uint64_t)L.n_elem * njobs >= c->banked_min_lanes;
    dim3 grid(gate_grid_x_for((L.n_elem + kThreads - 1) / kThreads, njobs, banked), njobs);
    double bytes = 0;
    for (int j = 0; j < njobs; j++) bytes += (double)L.n_elem * (c->mods[L.jobs[j].p].lam + 2.0 * c->mods[L.jobs[j].q].lam);
    const uint32_t q = common_q(L, njobs);
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * njobs, bytes);
    const int ki = q ? hot_mod_index(c->mods[q]) : 0;
    hipLaunchKernelGGL(banked ? kEvalKernelsBanked[ki] : kEvalKernels[ki], grid, dim3(banked ? kBigThreads : kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ------------------------------------------------------------------- carry chain of the sign gadget, evaluator
// One launch for the n dependent gates of the mixed-radix addition (a launch per digit costs about 10 us each,
// whatever the layer size, and they cannot overlap).  Instantiations for the two default digit sets; any
// other set takes the body with run-time constants.
template <class MC, class M1>
__global__ __launch_bounds__(kThreads) void k_chain_eval(const ChainLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) chain_eval_body<MC, M1>(L, tile, threadIdx.x, T);
}
__global__ __launch_bounds__(kThreads) void k_chain_eval_generic(const ChainLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) chain_eval_generic_body(L, tile, threadIdx.x, T);
}

int launch_chain_eval(const dash_ctx* c, ChainLaunch& L, hipStream_t s) {
    if (L.n < 2 || L.n > (uint32_t)kMaxChain) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    bool uniform = true;
    double bytes = 0;
    for (uint32_t j = 1; j <= L.n; j++) {
        if (L.m[j] < 2 || L.m[j] > 255 || !L.table[j] || !L.sum[j].p || (j < L.n && !L.carry[j].p)) return DASH_EINVAL;
        if (j >= 3 && L.m[j] != L.m[2]) uniform = false;
        bytes += (double)L.n_elem * (c->mods[L.m[j]].lam + (j >= 2 ? c->mods[L.m[j - 1]].lam : 128));
    }
    if ((uint64_t)L.n_elem * 255 >= (1ull << 32)) return DASH_ESIZE;
    const ModInfo &Mc = c->mods[L.m[2]], &M1 = c->mods[L.m[1]];
    auto is = [](const ModInfo& M, uint32_t m, uint32_t lam) { return M.m == m && M.lam == lam; };
    dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, 1));
    ProfScope ps(c->prof, DASH_PROF_EVAL, s, (double)L.n_elem * L.n, bytes);
    if (uniform && is(Mc, 96, 20) && is(M1, 26, 28))
        hipLaunchKernelGGL((k_chain_eval<CMod<96, 20>, CMod<26, 28>>), grid, dim3(kThreads), 0, s, L);
    else if (uniform && is(Mc, 204, 17) && is(M1, 46, 24))
        hipLaunchKernelGGL((k_chain_eval<CMod<204, 17>, CMod<46, 24>>), grid, dim3(kThreads), 0, s, L);
    else
        hipLaunchKernelGGL(k_chain_eval_generic, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

// ----------------------------------------------------------------------------- half gate, evaluator
__global__ __launch_bounds__(kThreads) void k_hg_finish(const HgLaunch L) {
    __shared__ uint32_t tt[kTabWords];
    const LdsTab T = load_ttab(tt, L.ttab);
    const uint32_t tiles = (L.n_elem + kThreads - 1) / kThreads;
    for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) hg_finish_body(L, tile, blockIdx.y, threadIdx.x, T);
}

int launch_hg_finish(const dash_ctx* c, HgLaunch& L, int njobs, hipStream_t s) {
    if (njobs < 1 || njobs > kMaxJobs) return DASH_EINVAL;
    if (L.n_elem == 0) return DASH_OK;
    if (L.n_elem > (1u << 28)) return DASH_ESIZE;      // lane offsets into a chunk are 32-bit byte offsets
    L.key = c->fixed; L.ttab = c->d_ttab; L.mods = c->d_mods;
    dim3 grid(grid_x_for((L.n_elem + kThreads - 1) / kThreads, njobs), njobs);
    hipLaunchKernelGGL(k_hg_finish, grid, dim3(kThreads), 0, s, L);
    DASH_HIP(hipGetLastError());
    return DASH_OK;
}

}  // namespace dash
