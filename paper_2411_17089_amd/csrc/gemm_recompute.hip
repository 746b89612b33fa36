// Recompute GEMM for gfx950 (Eq. 7 with fused bias):
//     C[M, N] = A[M, K] . W[N, K]^T + bias[N]        float16 in / float32 accumulate / float16 out
// A = X[0:l] flattened to [l*batch, hidden], W = [Wk^T ; Wv^T] ([2h, h], K contiguous), C = rows
// [0, l) of the device KV buffer (row stride ldc = 2h), so the result needs no copy or merge pass.
//
// Design (MI355X): one workgroup owns a BM x BN tile of C and walks K in steps of 64.  Both operand
// tiles are K-contiguous, staged through LDS as 128-byte rows whose 16-byte chunks are XOR-swizzled
// by the row index so that the ds_read_b128 of 32 consecutive rows is bank-conflict free.  Waves
// hold (BM/WM) x (BN/WN) sub-tiles as 32x32 accumulators of v_mfma_f32_32x32x16_f16.  The MFMA is
// issued "transposed" (W rows feed the instruction's row operand, X rows its column operand) so
// that each lane ends up with 4 consecutive output columns per accumulator quad and writes 8-byte
// pieces of a C row.  LDS is double-buffered: global loads for step k+1 are in flight while the
// MFMAs of step k run, one barrier per step.  Workgroup ids are remapped so that the workgroups an
// XCD runs concurrently (ids equal mod 8) form a compact block of tiles sharing A/W panels in that
// XCD's L2.
#include "kvpr_internal.h"

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;          // halfs per K step = one 128-byte LDS row
constexpr int ROW_BYTES = 128;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, int WM, int WN, int GROUP_M>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bias_f16(
    const _Float16* __restrict__ A, const _Float16* __restrict__ W, const _Float16* __restrict__ bias,
    _Float16* __restrict__ C, int64_t M, int N, int K, int64_t ldc, int tiles_m, int tiles_n, int tiles_per_xcd) {
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wave
    constexpr int A_CHUNKS = BM * 8 / NT, W_CHUNKS = BN * 8 / NT;
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");
    constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- which tile: XCD-aware, grouped raster ----
    const int pid = blockIdx.x;
    const int logical = (pid & 7) * tiles_per_xcd + (pid >> 3);
    if (logical >= tiles_m * tiles_n) return;
    const int group_sz = GROUP_M * tiles_n;
    const int group = logical / group_sz;
    const int first_m = group * GROUP_M;
    const int gm = min(tiles_m - first_m, GROUP_M);
    const int in_group = logical - group * group_sz;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global -> register staging: chunk q covers row q/8, 16-byte chunk q%8 of a tile ----
    const _Float16* a_src[A_CHUNKS];
    const _Float16* w_src[W_CHUNKS];
    int a_dst[A_CHUNKS], w_dst[W_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
        const int q = tid + i * NT, row = q >> 3, c = q & 7;
        int64_t gr = m0 + row;
        if (gr > M - 1) gr = M - 1;                                  // clamp: tail rows re-read the last row
        a_src[i] = A + gr * K + c * 8;
        a_dst[i] = row * ROW_BYTES + swz(row, c) * 16;
    }
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
        const int q = tid + i * NT, row = q >> 3, c = q & 7;
        int gr = n0 + row;
        if (gr > N - 1) gr = N - 1;
        w_src[i] = W + (int64_t)gr * K + c * 8;
        w_dst[i] = BM * ROW_BYTES + row * ROW_BYTES + swz(row, c) * 16;
    }

    half8 a_reg[A_CHUNKS], w_reg[W_CHUNKS];
    auto load_global = [&](int kt) {
        const int koff = kt * BK;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) a_reg[i] = *reinterpret_cast<const half8*>(a_src[i] + koff);
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) w_reg[i] = *reinterpret_cast<const half8*>(w_src[i] + koff);
    };
    auto store_lds = [&](int buf) {
        unsigned char* base = lds + buf * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<half8*>(base + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) *reinterpret_cast<half8*>(base + w_dst[i]) = w_reg[i];
    };

    // ---- per-lane LDS read offsets of the MFMA fragments ----
    // lane supplies row (lane % 32) of a 32-row fragment and the 8 halfs of k-chunk (2*kk + lane/32)
    const int frow = lane & 31, fhalf = lane >> 5;
    int a_row[TM], w_row[TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) a_row[t] = wm * WTM + t * 32 + frow;
#pragma unroll
    for (int t = 0; t < TN; ++t) w_row[t] = wn * WTN + t * 32 + frow;

    floatx16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_global(kt + 1);
        const unsigned char* sa = lds + (kt & 1) * STAGE_BYTES;
        const unsigned char* sw = sa + BM * ROW_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            half8 af[TM], wf[TN];
            const int c = kk * 2 + fhalf;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                af[t] = *reinterpret_cast<const half8*>(sa + a_row[t] * ROW_BYTES + swz(a_row[t], c) * 16);
#pragma unroll
            for (int t = 0; t < TN; ++t)
                wf[t] = *reinterpret_cast<const half8*>(sw + w_row[t] * ROW_BYTES + swz(w_row[t], c) * 16);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], af[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register r of tile (i, j) holds
    //      n = n0 + wn*WTN + i*32 + 8*(r/4) + 4*(lane/32) + r%4,   m = m0 + wm*WTM + j*32 + lane%32
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n0 + wn * WTN + i * 32 + 8 * g + 4 * fhalf;
            if (n >= N) continue;                    // N % 4 == 0 is required, so a quad is all in or all out
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (bias) {
                const half4 b4 = *reinterpret_cast<const half4*>(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[e] = (float)b4[e];
            }
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int64_t m = m0 + wm * WTM + j * 32 + frow;
                if (m >= M) continue;
                half4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (_Float16)(acc[i][j][g * 4 + e] + bv[e]);
                *reinterpret_cast<half4*>(C + m * ldc + n) = o;
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int GROUP_M>
int launch_variant(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                   hipStream_t st) {
    auto kern = gemm_bias_f16<BM, BN, WM, WN, GROUP_M>;
    constexpr int lds_bytes = 2 * (BM + BN) * ROW_BYTES;
    static bool configured = false;   // per process; attribute is per function, device 0 only is used
    if (!configured) {
        KVPR_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     lds_bytes));
        configured = true;
    }
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
    const int64_t total = (int64_t)tiles_m * tiles_n;
    const int tiles_per_xcd = (int)((total + 7) / 8);
    const unsigned grid = (unsigned)(tiles_per_xcd * 8);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds_bytes, st, (const _Float16*)a, (const _Float16*)w,
                       (const _Float16*)bias, (_Float16*)c, M, N, K, ldc, tiles_m, tiles_n, tiles_per_xcd);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int g_gemm_variant = 0;

}  // namespace

int launch_gemm(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                hipStream_t st) {
    if (M == 0) return KVPR_OK;
    switch (g_gemm_variant) {
        case 1: return launch_variant<256, 256, 2, 4, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 2: return launch_variant<128, 128, 2, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
        case 3: return launch_variant<256, 128, 2, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
        default: return launch_variant<256, 256, 2, 2, 8>(a, w, bias, c, M, N, K, ldc, st);
    }
}

}  // namespace kvpr

extern "C" int kvpr_debug_set_gemm_variant(int v) {
    kvpr::g_gemm_variant = v;
    return KVPR_OK;
}
