// Token GEMM for gfx950: y[M, N] = x[M, K] . W[N, K]^T + bias for M <= 64 rows (the decode token's
// q/k/v projection of Eq. 1 / Eq. 5, the output projection of Eq. 3, the FFN of Eq. 4).
//
// With so few rows the operation reads every weight once and is bound by HBM, so the kernel is a
// weight streamer built around v_mfma_f32_16x16x32_f16 (W rows feed the row operand, x rows the
// column operand):
//   - a workgroup owns TPW tiles of 16 output features and all M rows of x; TPW is chosen so that the
//     grid is about one workgroup per CU.  Its 8 waves split K in interleaved slabs of 128 columns,
//     so the workgroup as a whole walks contiguous memory;
//   - lanes read W straight from global memory into MFMA operand registers with 16-byte loads.  In
//     the instruction's own operand layout (lane = row r, k-chunk c) one load instruction covers 16
//     rows x one whole 64-byte segment, so every fetched segment is fully used (a lane-contiguous k
//     permutation was 4x worse: each instruction then touched 64 segments for 16 bytes each).  The
//     loads are ordinary ones although each weight is used once: two consecutive instructions share
//     every 128-byte line, and with non-temporal loads the second one often missed again (measured
//     3-5 % slower at K = 4096, 13-15 % at K = 7168);
//   - x is tiny (M*K halfs) and comes from L2; one x fragment is reused for the TPW weight tiles, so
//     the L2->CU traffic for x stays below the HBM traffic for W (with one tile per workgroup it was
//     twice the weight bytes and capped the kernel at 2.2 TB/s);
//   - all 4*TPW weight loads of a slab are issued before the MFMAs of the previous slab (register double
//     buffering), so a wave always has one slab in flight; per-wave partial tiles are summed through LDS;
//   - the epilogue adds the bias, optionally applies ReLU and writes float32 for the first
//     `out_f32_cols` features (q) and float16 for the rest (k|v row of the cache, o, FFN).
//
// Second kernel for wide weight matrices (token_gemm_wide): once N is large enough for 128 (or 64) output features
// per workgroup to give well over a hundred workgroups, a workgroup of 4 waves owns RB = 128 / 64 output features over
// the whole of K.  Per 128 columns of K it brings in RB rows x 256 bytes of W and the M rows x 256 bytes of x by direct
// global->LDS DMA (a wave instruction covers 4 rows x 256 contiguous bytes; x then costs M / RB of the weight bytes
// instead of 2 / TPW), two stages in LDS, fragments read back in the MFMA operand layout (16-byte chunks of a row
// XOR-swizzled by the row number on the global-address side so that the 16 rows of a fragment read hit 16 different
// bank groups).  A wave owns RB / 4 output features for the workgroup's whole K range: no cross-wave reduction.
// Outputs with too few features to give every compute unit a block (N = hidden: the output projection of Eq. 3 and the
// second FFN matrix of Eq. 4) are cut along K instead: gridDim.y workgroups share a block of features, each takes a run
// of K stages, the float32 partial tiles meet in a workspace and the workgroup that arrives last adds them in slice order
// and writes the outputs.
#include "kvpr_internal.h"
#include <mutex>

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int SLAB = 128;   // K columns per wave step: 4 MFMA k-steps of 32
constexpr int TG_WAVES = 8;

template <int MT, int TPW>
__global__ __launch_bounds__(TG_WAVES * 64) void token_gemm(const _Float16* __restrict__ x,
                                                            const _Float16* __restrict__ W,
                                                            const _Float16* __restrict__ bias,
                                                            float* __restrict__ y32, _Float16* __restrict__ y16,
                                                            int M, int N, int K, int out_f32_cols, int64_t ld16,
                                                            int relu) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int n0 = blockIdx.x * (16 * TPW);
    const _Float16* wp[TPW];
#pragma unroll
    for (int p = 0; p < TPW; ++p) wp[p] = W + (int64_t)min(n0 + p * 16 + r, N - 1) * K + c * 8;
    const _Float16* xp[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) xp[t] = x + (int64_t)min(t * 16 + r, M - 1) * K + c * 8;

    floatx4 acc[TPW][MT];
#pragma unroll
    for (int p = 0; p < TPW; ++p)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[p][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Register double buffering: the loads of this wave's next slab are issued before the MFMAs of the current
    // one, so each wave always has a whole slab (TPW * 4 KiB of weights) in flight.
    const int slabs = K / SLAB;
    half8 wf0[TPW][4], xf0[MT][4], wf1[TPW][4], xf1[MT][4];
    // workgroups start at different slabs (the sum over k has no order): with every workgroup at the same k all
    // concurrent reads would share their low address bits (rows are K*2 bytes apart) and crowd a few HBM channels
    const int rot = (int)((blockIdx.x * 5u) % (unsigned)slabs);
    auto load = [&](half8 (&wf)[TPW][4], half8 (&xf)[MT][4], int s) {
        int sr = s + rot;
        if (sr >= slabs) sr -= slabs;
        const int k0 = sr * SLAB;
#pragma unroll
        for (int p = 0; p < TPW; ++p)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                wf[p][j] = *reinterpret_cast<const half8*>(wp[p] + k0 + j * 32);
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) xf[t][j] = *reinterpret_cast<const half8*>(xp[t] + k0 + j * 32);
    };
    auto mac = [&](const half8 (&wf)[TPW][4], const half8 (&xf)[MT][4]) {
#pragma unroll
        for (int p = 0; p < TPW; ++p)
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[p][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[p][j], xf[t][j], acc[p][t], 0, 0, 0);
    };
    // two buffers need (TPW + MT) * 32 registers on top of the accumulators: the widest shapes keep a single buffer
    constexpr bool kDoubleBuffer = (TPW + MT) * 32 + TPW * MT * 4 <= 200;
    int s = wave;
    if constexpr (kDoubleBuffer) {
        if (s < slabs) load(wf0, xf0, s);
        while (s < slabs) {
            if (s + TG_WAVES < slabs) load(wf1, xf1, s + TG_WAVES);
            mac(wf0, xf0);
            s += TG_WAVES;
            if (s >= slabs) break;
            if (s + TG_WAVES < slabs) load(wf0, xf0, s + TG_WAVES);
            mac(wf1, xf1);
            s += TG_WAVES;
        }
    } else {
        for (; s < slabs; s += TG_WAVES) {
            load(wf0, xf0, s);
            mac(wf0, xf0);
        }
    }

    // ---- sum the waves' partial tiles: element i of (tile p, m-tile t) in lane L is
    //      n = n0 + 16*p + 4*(L/16) + i,  m = 16*t + L%16
    __shared__ float red[TG_WAVES][TPW * MT * 4][64];
#pragma unroll
    for (int p = 0; p < TPW; ++p)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][(p * MT + t) * 4 + i][lane] = acc[p][t][i];
    __syncthreads();
    for (int e = threadIdx.x; e < TPW * MT * 4 * 64; e += TG_WAVES * 64) {
        const int row = e >> 6, ln = e & 63;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < TG_WAVES; ++w) v += red[w][row][ln];
        const int p = row / (MT * 4), t = (row / 4) % MT, i = row & 3;
        const int n = n0 + 16 * p + 4 * (ln >> 4) + i;
        const int m = 16 * t + (ln & 15);
        if (n >= N || m >= M) continue;
        if (bias) v += (float)bias[n];
        if (relu) v = fmaxf(v, 0.f);
        if (n < out_f32_cols)
            y32[(int64_t)m * out_f32_cols + n] = v;
        else
            y16[(int64_t)m * ld16 + (n - out_f32_cols)] = (_Float16)v;
    }
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

constexpr int WIDE_KB = 128;                    // K columns per stage
constexpr size_t TOKEN_WS_TICKET_BYTES = 4096;  // head of the workspace: one arrival counter per block of output features
constexpr int WIDE_ROW_BYTES = WIDE_KB * 2;     // one LDS row of a stage

template <int RB, int MT>
__global__ __launch_bounds__(256) void token_gemm_wide(const _Float16* __restrict__ x, const _Float16* __restrict__ W,
                                                       const _Float16* __restrict__ bias, float* __restrict__ y32,
                                                       _Float16* __restrict__ y16, int M, int N, int K, int out_f32_cols,
                                                       int64_t ld16, int relu, float* part, unsigned* ticket) {
    constexpr int RT = RB / 64;                             // 16-row tiles of W per wave
    constexpr int WI = RB / 16;                             // W DMA instructions per wave and stage (4 rows each, 4 waves)
    constexpr int WBYTES = RB * WIDE_ROW_BYTES, XBYTES = MT * 16 * WIDE_ROW_BYTES, STAGE = WBYTES + XBYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n0 = blockIdx.x * RB;

    // DMA sources.  Instruction q covers stage rows [4q, 4q+4); lane L lands at row 4q + L/16, physical 16-byte chunk L%16,
    // and therefore fetches logical chunk (L%16) ^ (row%16).
    const _Float16* srcw[WI];
#pragma unroll
    for (int i = 0; i < WI; ++i) {
        const int row = (wave + 4 * i) * 4 + (lane >> 4);
        srcw[i] = W + (int64_t)min(n0 + row, N - 1) * K + (((lane & 15) ^ (row & 15)) << 3);
    }
    const _Float16* srcx[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int row = (wave + 4 * i) * 4 + (lane >> 4);
        srcx[i] = x + (int64_t)min(row, M - 1) * K + (((lane & 15) ^ (row & 15)) << 3);
    }
    auto issue = [&](int k0, int buf) {
        unsigned char* base = lds + buf * STAGE + wave * 1024;
#pragma unroll
        for (int i = 0; i < WI; ++i)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(srcw[i] + k0), (lds_ptr_t)(base + i * 4096), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < MT; ++i)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(srcx[i] + k0), (lds_ptr_t)(base + WBYTES + i * 4096), 16, 0, 0);
    };

    // fragment addresses: lane (r, c) of MFMA k-step j reads logical chunk 4j + c of row r of its tile
    const int r = lane & 15, c = lane >> 4;
    int foff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) foff[j] = r * WIDE_ROW_BYTES + (((4 * j + c) ^ r) << 4);   // every tile starts at a multiple of 16 rows

    floatx4 acc[RT][MT];
#pragma unroll
    for (int p = 0; p < RT; ++p)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[p][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // gridDim.y workgroups share a block of output features: each takes a contiguous run of the K stages
    const int ks = gridDim.y, kz = blockIdx.y;
    const int all_stages = K / WIDE_KB;
    const int first = (int)((int64_t)all_stages * kz / ks);
    const int stages = (int)((int64_t)all_stages * (kz + 1) / ks) - first;
#pragma unroll
    for (int i = 0; i < WI; ++i) srcw[i] += (int64_t)first * WIDE_KB;
#pragma unroll
    for (int i = 0; i < MT; ++i) srcx[i] += (int64_t)first * WIDE_KB;
    // workgroups walk their stages from different starting points (the sum over k has no order): with every workgroup
    // at the same k all concurrent reads would share their low address bits (rows are K*2 bytes apart) and crowd a few
    // HBM channels
    int next = stages > 0 ? (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)stages) : 0;
    auto issue_next = [&](int buf) {
        issue(next * WIDE_KB, buf);
        if (++next == stages) next = 0;
    };
    if (stages > 0) issue_next(0);
    if (stages > 1) issue_next(1);
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        // this wave's share of stage s has landed (stage s + 1 may still be in flight), then everybody's
        if (s + 1 < stages) __builtin_amdgcn_s_waitcnt(0x0F70 | ((WI + MT) & 15) | (((WI + MT) >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_s_barrier();
        const unsigned char* wb = lds + buf * STAGE + (wave * RT) * 16 * WIDE_ROW_BYTES;
        const unsigned char* xb = lds + buf * STAGE + WBYTES;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8 wf[RT], xf[MT];
#pragma unroll
            for (int p = 0; p < RT; ++p) wf[p] = *reinterpret_cast<const half8*>(wb + p * 16 * WIDE_ROW_BYTES + foff[j]);
#pragma unroll
            for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const half8*>(xb + t * 16 * WIDE_ROW_BYTES + foff[j]);
#pragma unroll
            for (int p = 0; p < RT; ++p)
#pragma unroll
                for (int t = 0; t < MT; ++t) acc[p][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[p], xf[t], acc[p][t], 0, 0, 0);
        }
        if (s + 2 < stages) {
            __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): this wave has read what it needs of the buffer
            __builtin_amdgcn_s_barrier();                // ... and so has everybody else: refill it
            issue_next(buf);
        }
    }

    if (ks > 1) {
        // Partial tiles go to the workspace in register layout; the workgroup that arrives last at the block's ticket
        // adds the ks slices in slice order (so the sum does not depend on which one that is) and writes the outputs.
        // Device-wide fences would write back and invalidate a whole L2 per workgroup (measured: 4 times slower than
        // no split at all); instead every partial is stored and loaded as a relaxed device-scope atomic, which goes
        // through to the level all L2s share, and the ticket is taken only after this wave's stores have been
        // acknowledged (vmcnt(0)) and, by the barrier, everybody else's in the workgroup.
        const size_t per_slice = (size_t)gridDim.x * (4 * RT * MT * 4 * 64);
        float* mine = part + (size_t)blockIdx.x * (4 * RT * MT * 4 * 64) + (size_t)wave * (RT * MT * 4 * 64) + lane;
#pragma unroll
        for (int p = 0; p < RT; ++p)
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    __hip_atomic_store(mine + (size_t)kz * per_slice + ((p * MT + t) * 4 + i) * 64, acc[p][t][i],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the stores have been acknowledged
        __shared__ unsigned arrived;
        __syncthreads();
        if (threadIdx.x == 0) arrived = __hip_atomic_fetch_add(ticket + blockIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrived != (unsigned)(ks - 1)) return;       // uniform over the workgroup
#pragma unroll
        for (int p = 0; p < RT; ++p)
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                // all loads of a tile first (a slice beyond ks re-reads the last one and counts as zero), then the sums
                float v[8][4];
#pragma unroll
                for (int z = 0; z < 8; ++z)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        v[z][i] = __hip_atomic_load(mine + (size_t)min(z, ks - 1) * per_slice + ((p * MT + t) * 4 + i) * 64,
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float sum = v[0][i];
#pragma unroll
                    for (int z = 1; z < 8; ++z) sum += z < ks ? v[z][i] : 0.f;
                    acc[p][t][i] = sum;
                }
            }
        if (threadIdx.x == 0) ticket[blockIdx.x] = 0;    // ready for the next launch on this stream
    }

    // element i of (tile p, m-tile t) in lane L is  n = n0 + 16*(wave*RT + p) + 4*(L/16) + i,  m = 16*t + L%16
#pragma unroll
    for (int p = 0; p < RT; ++p)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int n = n0 + 16 * (wave * RT + p) + 4 * c + i;
                const int m = 16 * t + r;
                if (n >= N || m >= M) continue;
                float v = acc[p][t][i];
                if (bias) v += (float)bias[n];
                if (relu) v = fmaxf(v, 0.f);
                if (n < out_f32_cols)
                    y32[(int64_t)m * out_f32_cols + n] = v;
                else
                    y16[(int64_t)m * ld16 + (n - out_f32_cols)] = (_Float16)v;
            }
}

template <int RB, int MT>
int launch_wide(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                int out_f32_cols, int64_t ld16, int relu, int ks, void* ws, hipStream_t st) {
    auto kern = token_gemm_wide<RB, MT>;
    constexpr int lds_bytes = 2 * (RB + MT * 16) * WIDE_ROW_BYTES;
    static std::once_flag configured;
    static hipError_t configure_status = hipSuccess;
    std::call_once(configured, [&] {
        configure_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    KVPR_HIP(configure_status);
    const unsigned grid = (unsigned)((N + RB - 1) / RB);
    hipLaunchKernelGGL(kern, dim3(grid, (unsigned)ks), dim3(256), lds_bytes, st, (const _Float16*)x, (const _Float16*)w,
                       (const _Float16*)bias, (float*)y32, (_Float16*)y16, M, N, K, out_f32_cols, ld16, relu,
                       (float*)((unsigned char*)ws + TOKEN_WS_TICKET_BYTES), (unsigned*)ws);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int g_token_tpw = 0;   // 0 = choose from N; tests and sweeps can force 1..8
int g_token_wide = -1; // -1 = choose from N; 0 = never, 64 / 128 = force that many features per workgroup (tests, sweeps)
int g_token_ks = 0;    // 0 = choose; 1..8 = force that many K slices (needs a workspace; tests, sweeps)

// workspace bytes of a launch with `ks` K slices: the tickets, then ks partial tiles of float32 per block of RB features
size_t wide_ws_bytes(int rb, int mt, int N, int ks) {
    return TOKEN_WS_TICKET_BYTES + (size_t)ks * ((N + rb - 1) / rb) * rb * mt * 16 * sizeof(float);
}

template <int MT, int TPW>
int launch_t(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
             int out_f32_cols, int64_t ld16, int relu, hipStream_t st) {
    const unsigned grid = (unsigned)((N + 16 * TPW - 1) / (16 * TPW));
    hipLaunchKernelGGL((token_gemm<MT, TPW>), dim3(grid), dim3(TG_WAVES * 64), 0, st, (const _Float16*)x,
                       (const _Float16*)w, (const _Float16*)bias, (float*)y32, (_Float16*)y16, M, N, K, out_f32_cols,
                       ld16, relu);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

// Tiles per workgroup.  A launch runs in rounds of one workgroup per compute unit, and a round costs about its tiles
// per workgroup plus a fixed part of one and a half tiles (first-load latency, x fragments, the reduction): the choice
// minimises rounds x (tiles + 1.5) (ties: the wider workgroup), bounded by the LDS reduction buffer (TPW * MT <= 8 keeps it
// at 64 KiB) and by the accumulator registers.  The model orders all 32 measured (shape, tiles per workgroup) pairs of
// hidden 4096 / 7168, batch 32 correctly; e.g. q|k|v at hidden 7168 (1344 tiles): 3 per workgroup 85 us, 2: 95 us, 4: 110 us.
int compute_units() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
        else n = 256;
    }
    return n;
}

template <int MT>
int launch_mt(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
              int out_f32_cols, int64_t ld16, int relu, void* ws, size_t ws_bytes, hipStream_t st) {
    // wide kernel: 128 (or 64) features per workgroup once that gives about 150 workgroups, over all of K; with a
    // workspace also for narrower outputs, K cut into slices until there are about two workgroups per compute unit
    if (K % WIDE_KB == 0 && g_token_tpw <= 0) {
        const int stages = K / WIDE_KB;
        int rb, ks = 1;
        if (g_token_wide >= 0) {                         // forced by a test or a sweep
            rb = g_token_wide;
            if (g_token_ks > 0) ks = g_token_ks;
        } else {
            rb = (N + 127) / 128 >= 144 ? 128 : (N + 63) / 64 >= 144 ? 64 : 0;
            if (rb == 0 && ws) {
                // the fewest slices that give about one workgroup per compute unit, doubled when a slice would still be
                // longer than 64 stages, and never shorter than 4 stages: over hidden 4096 / 5120 / 7168 and K = h / 4h
                // this picks the best or second-best measured count (4, 3, 2 for K = h; 4, 3, 4 for K = 4h)
                rb = 64;
                const int nb = (N + 63) / 64, cus = compute_units();
                ks = 8;
                for (int c : {1, 2, 3, 4, 6, 8})
                    if (nb * c * 100 >= 85 * cus) { ks = c; break; }
                if (stages / ks > 64 && ks <= 4) ks *= 2;
                while (ks > 1 && stages / ks < 4) --ks;
            }
        }
        if (rb) {
            if (ks > stages) ks = stages;
            if (!ws || (size_t)((N + rb - 1) / rb) * sizeof(unsigned) > TOKEN_WS_TICKET_BYTES) ks = 1;
            while (ks > 1 && wide_ws_bytes(rb, MT, N, ks) > ws_bytes) --ks;
            if (ks == 1 && g_token_wide < 0 && (N + rb - 1) / rb < 144) rb = 0;   // nothing to split after all: the narrow kernel
        }
        if (rb == 128) return launch_wide<128, MT>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ks, ws, st);
        if (rb == 64) return launch_wide<64, MT>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ks, ws, st);
    }
    const int tiles = (N + 15) / 16;
    const int cap = 8 / MT;
    int tpw = g_token_tpw;
    if (tpw <= 0) {
        const int cus = compute_units();
        long best = -1;
        for (int t : {1, 2, 3, 4, 8}) {
            if (t > cap) break;
            const int grid = (tiles + t - 1) / t;
            const long cost = (long)((grid + cus - 1) / cus) * (2 * t + 3);
            if (best < 0 || cost <= best) { best = cost; tpw = t; }
        }
    }
    if (tpw > cap) tpw = cap;
    if (tpw >= 8) return launch_t<MT, (8 / MT >= 8 ? 8 : 1)>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    if (tpw >= 4) return launch_t<MT, (8 / MT >= 4 ? 4 : 1)>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    if (tpw == 3) return launch_t<MT, (8 / MT >= 3 ? 3 : 1)>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    if (tpw == 2) return launch_t<MT, (8 / MT >= 2 ? 2 : 1)>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    return launch_t<MT, 1>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
}

}  // namespace

// flags bit 0: ReLU.  ws (optional, device): workspace that lets a narrow output split K over several workgroups; its
// first 4096 bytes must be zero before the first launch that uses it and are zero again when a launch ends; launches
// that share a workspace must not overlap.
int launch_token_gemm_flags(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                            int out_f32_cols, int64_t ld16, int flags, hipStream_t st, void* ws, size_t ws_bytes) {
    const int relu = flags & 1;
    if (ws_bytes <= TOKEN_WS_TICKET_BYTES) ws = nullptr;
    if (M <= 16) return launch_mt<1>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ws, ws_bytes, st);
    if (M <= 32) return launch_mt<2>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ws, ws_bytes, st);
    if (M <= 48) return launch_mt<3>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ws, ws_bytes, st);
    return launch_mt<4>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, ws, ws_bytes, st);
}

// enough for 8 K slices of an output of `N` features and `M` rows
size_t token_gemm_workspace_bytes(int M, int N) {
    return wide_ws_bytes(128, (M + 15) / 16, N, 8);
}

}  // namespace kvpr

// v = -1: all automatic.  v in 0..8: tiles per workgroup of the narrow kernel (0 = automatic).
// v >= 0x100: bits 0..7 = features per workgroup of the wide kernel (0 = narrow kernel only, 64, 128),
// bits 12..15 = K slices (0 = one, or as many as the automatic choice takes when bits 0..7 are 0).
extern "C" int kvpr_debug_set_token_gemm_cfg(int v) {
    kvpr::g_token_tpw = 0; kvpr::g_token_wide = -1; kvpr::g_token_ks = 0;
    if (v < 0) return KVPR_OK;
    if (v >= 0x100) { kvpr::g_token_wide = v & 0xFF; kvpr::g_token_ks = (v >> 12) & 15; return KVPR_OK; }
    kvpr::g_token_tpw = v;
    return KVPR_OK;
}
