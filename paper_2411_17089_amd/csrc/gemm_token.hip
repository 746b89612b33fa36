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
#include "kvpr_internal.h"

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

int g_token_tpw = 0;   // 0 = choose from N; tests and sweeps can force 1..8

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
              int out_f32_cols, int64_t ld16, int relu, hipStream_t st) {
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

// flags bit 0: ReLU
int launch_token_gemm_flags(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                            int out_f32_cols, int64_t ld16, int flags, hipStream_t st) {
    const int relu = flags & 1;
    if (M <= 16) return launch_mt<1>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    if (M <= 32) return launch_mt<2>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    if (M <= 48) return launch_mt<3>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    return launch_mt<4>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
}

}  // namespace kvpr

extern "C" int kvpr_debug_set_token_gemm_cfg(int v) {
    kvpr::g_token_tpw = v;
    return KVPR_OK;
}
