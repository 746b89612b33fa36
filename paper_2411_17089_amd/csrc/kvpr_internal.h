// Internal declarations shared by the translation units of libkvpr (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "kvpr.h"

namespace kvpr {

// error plumbing: records text for kvpr_last_error() and returns `code`
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
#define KVPR_HIP(call)                                                                    \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return ::kvpr::fail(KVPR_E_HIP, "%s failed: %s (%s:%d)", #call,               \
                                hipGetErrorString(e_), __FILE__, __LINE__);               \
    } while (0)

// kernels (each validates nothing: callers check shapes first)
int launch_gemm(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K,
                int64_t ldc, hipStream_t st);
int launch_attention(const void* q, const void* kv, void* z, void* ws, int S, int batch, int hidden,
                     int n_heads, hipStream_t st);
size_t attention_workspace_bytes(int batch, int hidden, int n_heads, int S);
int launch_attention_mixed(const void* q, const void* kv16, const void* kvq, void* z, void* ws, int S, int split, int batch,
                           int hidden, int n_heads, int phase, hipStream_t st);
int launch_token_gemm_flags(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N,
                            int K, int out_f32_cols, int64_t ld16, int flags /*bit0: ReLU*/, hipStream_t st,
                            void* ws = nullptr, size_t ws_bytes = 0);
size_t token_gemm_workspace_bytes(int M, int N);
int launch_fill_u16(void* p, size_t n_halfs, uint16_t pattern, hipStream_t st);
int launch_fill_random(void* p, size_t n_halfs, float scale, uint32_t seed, hipStream_t st);
int launch_layernorm(const void* x, const void* g, const void* b, void* y, int rows, int h, hipStream_t st);
int launch_argmax_rows(const float* logits, int M, int N, int32_t* out, hipStream_t st);
int launch_gather_rows(const void* table, const int32_t* idx, void* out, int M, int h, hipStream_t st);
int launch_gemm_rope(const void* a, const void* w, const void* bias, void* c, int64_t M, int N, int K, int64_t ldc,
                     const void* table, int rope_cols, int head_dim, int batch, int pos0, hipStream_t st);
int launch_rmsnorm(const void* x, const void* g, void* y, int rows, int h, hipStream_t st);
int launch_silu_mul(const void* gu, void* y, int rows, int f, hipStream_t st);
int launch_rope_token(const void* qk32, const void* table, int pos, int batch, int h, int head_dim, void* q32, void* k16,
                      int64_t ldk, hipStream_t st);
size_t int4_row_bytes(int cols);
int launch_quant_int4(const void* src, void* dst, int64_t rows, int cols, hipStream_t st);
int launch_dequant_int4(const void* src, void* dst, int64_t rows, int cols, hipStream_t st);
int launch_add(const void* a, const void* b, void* y, size_t n, hipStream_t st);
int launch_copy_bytes(const void* src, void* dst, size_t bytes, hipStream_t st);
int launch_keep_warm(const void* w, size_t n_w, double seconds, double wall_clock_hz, void* sink, hipStream_t st);

}  // namespace kvpr
