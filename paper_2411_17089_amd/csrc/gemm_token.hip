// Token GEMM for gfx950: y[M, N] = x[M, K] . W[N, K]^T + bias for M <= 64 rows (the decode token's
// q/k/v projection of Eq. 1 / Eq. 5, the output projection of Eq. 3, the FFN of Eq. 4).
//
// With so few rows the operation reads every weight once and is bound by HBM, so the kernel is a
// weight streamer: a workgroup owns 32 output features, its waves split K, and every lane reads
// whole 128-byte lines of its weight row straight from global memory into MFMA operand registers
// (no LDS staging).  The k-index assignment inside a 128-column slab is permuted identically for W
// and x, which leaves the dot products unchanged and lets lane (row r, half c) own the contiguous
// 64 columns [64c, 64c+64) of row r.  x is tiny and comes from L2.  Per-wave partial 32x32 tiles are
// summed through LDS; the epilogue adds the bias, optionally applies ReLU and writes float32 for
// the first `out_f32_cols` features (q) and float16 for the rest (k|v rows, o, FFN).
#include "kvpr_internal.h"

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int SLAB = 128;   // K columns one wave consumes per outer step (8 MFMA k-steps of 16)

template <int WAVES, int MT>
__global__ __launch_bounds__(WAVES * 64) void token_gemm(const _Float16* __restrict__ x,
                                                         const _Float16* __restrict__ W,
                                                         const _Float16* __restrict__ bias, float* __restrict__ y32,
                                                         _Float16* __restrict__ y16, int M, int N, int K,
                                                         int out_f32_cols, int64_t ld16, int relu) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, c = lane >> 5;
    const int n0 = blockIdx.x * 32;
    const int nrow = min(n0 + r, N - 1);
    const _Float16* wp = W + (int64_t)nrow * K + c * 64;
    const _Float16* xp[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) xp[t] = x + (int64_t)min(t * 32 + r, M - 1) * K + c * 64;

    floatx16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    const int slabs = K / SLAB;
    for (int s = wave; s < slabs; s += WAVES) {
        const int k0 = s * SLAB;
        half8 wf[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) wf[j] = *reinterpret_cast<const half8*>(wp + k0 + j * 8);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            half8 xf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) xf[j] = *reinterpret_cast<const half8*>(xp[t] + k0 + j * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[j], xf[j], acc[t], 0, 0, 0);
        }
    }

    // ---- sum the waves' partial tiles: element (i, lane) of tile t is
    //      n = n0 + 8*(i/4) + 4*(lane/32) + i%4,  m = 32*t + lane%32
    __shared__ float red[WAVES][MT * 16][64];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave][t * 16 + i][lane] = acc[t][i];
    __syncthreads();
    for (int e = threadIdx.x; e < MT * 16 * 64; e += WAVES * 64) {
        const int ti = e >> 6, ln = e & 63;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += red[w][ti][ln];
        const int t = ti >> 4, i = ti & 15;
        const int n = n0 + 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
        const int m = 32 * t + (ln & 31);
        if (n >= N || m >= M) continue;
        if (bias) v += (float)bias[n];
        if (relu) v = fmaxf(v, 0.f);
        if (n < out_f32_cols)
            y32[(int64_t)m * out_f32_cols + n] = v;
        else
            y16[(int64_t)m * ld16 + (n - out_f32_cols)] = (_Float16)v;
    }
}

template <int WAVES, int MT>
int launch_t(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
             int out_f32_cols, int64_t ld16, int relu, hipStream_t st) {
    const unsigned grid = (unsigned)((N + 31) / 32);
    hipLaunchKernelGGL((token_gemm<WAVES, MT>), dim3(grid), dim3(WAVES * 64), 0, st, (const _Float16*)x,
                       (const _Float16*)w, (const _Float16*)bias, (float*)y32, (_Float16*)y16, M, N, K, out_f32_cols,
                       ld16, relu);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

}  // namespace

size_t token_gemm_workspace_bytes(int, int, int) { return 0; }

// flags bit 0: ReLU
int launch_token_gemm_flags(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                            int out_f32_cols, int64_t ld16, int flags, hipStream_t st) {
    const int relu = flags & 1;
    if (M <= 32) {
        if (N / 32 >= 512) return launch_t<8, 1>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
        return launch_t<16, 1>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
    }
    return launch_t<8, 2>(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, relu, st);
}

int launch_token_gemm(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                      int out_f32_cols, int64_t ld16, void*, hipStream_t st) {
    return launch_token_gemm_flags(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, 0, st);
}

}  // namespace kvpr
