// C entry points of the individual kernels: argument validation, then the launcher.
#include "kvpr_internal.h"

#include <cmath>

using kvpr::fail;

extern "C" int kvpr_recompute_gemm(const void* a, const void* w, const void* bias, void* cdev, int64_t M, int N, int K,
                                   int64_t ldc, void* stream) {
    if (M < 0 || N < 1 || K < 1) return fail(KVPR_E_RANGE, "M=%lld N=%d K=%d out of range", (long long)M, N, K);
    if (K % 64 || N % 8 || ldc < N || ldc % 8) return fail(KVPR_E_INVAL, "need K %% 64 == 0, N %% 8 == 0, ldc >= N, ldc %% 8 == 0 (16-byte row pieces)");
    if (M == 0) return KVPR_OK;
    if (!a || !w || !cdev) return fail(KVPR_E_INVAL, "a / w / c is null");
    return kvpr::launch_gemm(a, w, bias, cdev, M, N, K, ldc, (hipStream_t)stream);
}

extern "C" size_t kvpr_attention_workspace_bytes(int batch, int hidden, int n_heads, int S) {
    if (batch < 1 || hidden < 1 || S < 1) return 0;
    return kvpr::attention_workspace_bytes(batch, hidden, n_heads, S);
}

extern "C" int kvpr_decode_attention(const void* q, const void* kv, void* z, void* ws, int S, int batch, int hidden,
                                     int n_heads, void* stream) {
    if (S < 1 || batch < 1 || n_heads < 1) return fail(KVPR_E_RANGE, "S=%d batch=%d n_heads=%d out of range", S, batch, n_heads);
    if (hidden % n_heads || (hidden / n_heads != 64 && hidden / n_heads != 128))
        return fail(KVPR_E_INVAL, "head_dim must be 64 or 128");
    if (!q || !kv || !z || !ws) return fail(KVPR_E_INVAL, "q / kv / z / ws is null");
    return kvpr::launch_attention(q, kv, z, ws, S, batch, hidden, n_heads, (hipStream_t)stream);
}

extern "C" int kvpr_decode_attention_mixed(const void* q, const void* kv16, const void* kvq, void* z, void* ws, int S, int split,
                                           int batch, int hidden, int n_heads, void* stream) {
    if (S < 1 || batch < 1 || n_heads < 1 || split < 0 || split > S - 1)
        return fail(KVPR_E_RANGE, "S=%d split=%d batch=%d n_heads=%d out of range", S, split, batch, n_heads);
    if (hidden % n_heads || (hidden / n_heads != 64 && hidden / n_heads != 128) || hidden % 128)
        return fail(KVPR_E_INVAL, "head_dim must be 64 or 128 and hidden a multiple of 128");
    if (!q || !kv16 || !z || !ws) return fail(KVPR_E_INVAL, "q / kv16 / z / ws is null");
    if (int rc = kvpr::launch_attention_mixed(q, kv16, kvq, z, ws, S, split, batch, hidden, n_heads, 0, (hipStream_t)stream)) return rc;
    return kvpr::launch_attention_mixed(q, kv16, kvq, z, ws, S, split, batch, hidden, n_heads, 1, (hipStream_t)stream);
}

extern "C" int kvpr_token_gemm(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                               int out_f32_cols, int64_t ld16, void* stream) {
    if (M < 1 || M > 64 || N < 1 || K < 1) return fail(KVPR_E_RANGE, "M=%d (1..64) N=%d K=%d out of range", M, N, K);
    if (K % 128) return fail(KVPR_E_INVAL, "K must be a multiple of 128");
    if (out_f32_cols < 0 || out_f32_cols > N) return fail(KVPR_E_RANGE, "out_f32_cols outside [0, N]");
    if (!x || !w || (out_f32_cols > 0 && !y32) || (out_f32_cols < N && !y16)) return fail(KVPR_E_INVAL, "null pointer");
    if (out_f32_cols < N && ld16 < N - out_f32_cols) return fail(KVPR_E_INVAL, "ld16 too small");
    return kvpr::launch_token_gemm_flags(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, 0, (hipStream_t)stream);
}

extern "C" size_t kvpr_token_gemm_workspace_bytes(int M, int N) {
    if (M < 1 || M > 64 || N < 1) return 0;
    return kvpr::token_gemm_workspace_bytes(M, N);
}

extern "C" int kvpr_token_gemm_ws(const void* x, const void* w, const void* bias, void* y32, void* y16, int M, int N, int K,
                                  int out_f32_cols, int64_t ld16, void* ws, size_t ws_bytes, void* stream) {
    if (M < 1 || M > 64 || N < 1 || K < 1) return fail(KVPR_E_RANGE, "M=%d (1..64) N=%d K=%d out of range", M, N, K);
    if (K % 128) return fail(KVPR_E_INVAL, "K must be a multiple of 128");
    if (out_f32_cols < 0 || out_f32_cols > N) return fail(KVPR_E_RANGE, "out_f32_cols outside [0, N]");
    if (!x || !w || (out_f32_cols > 0 && !y32) || (out_f32_cols < N && !y16)) return fail(KVPR_E_INVAL, "null pointer");
    if (out_f32_cols < N && ld16 < N - out_f32_cols) return fail(KVPR_E_INVAL, "ld16 too small");
    if (ws && ((uintptr_t)ws & 15)) return fail(KVPR_E_INVAL, "workspace must be 16-byte aligned");
    return kvpr::launch_token_gemm_flags(x, w, bias, y32, y16, M, N, K, out_f32_cols, ld16, 0, (hipStream_t)stream, ws, ws ? ws_bytes : 0);
}

// ---- rotary models ----
extern "C" int kvpr_rope_table(float* out_host, int n_pos, int head_dim, double base) {
    if (!out_host) return fail(KVPR_E_INVAL, "out_host is null");
    if (n_pos < 1 || (head_dim != 64 && head_dim != 128)) return fail(KVPR_E_RANGE, "n_pos=%d head_dim=%d: need n_pos >= 1, head_dim 64 or 128", n_pos, head_dim);
    if (!(base > 0.0) || !std::isfinite(base)) return fail(KVPR_E_INVAL, "base must be finite and > 0");
    const int half_d = head_dim / 2;
    for (int i = 0; i < half_d; ++i) {
        const double theta = std::pow(base, -2.0 * i / head_dim);
        for (int p = 0; p < n_pos; ++p) {
            out_host[((size_t)p * half_d + i) * 2] = (float)std::cos(p * theta);
            out_host[((size_t)p * half_d + i) * 2 + 1] = (float)std::sin(p * theta);
        }
    }
    return KVPR_OK;
}

extern "C" int kvpr_recompute_gemm_rope(const void* a, const void* w, const void* bias, void* cdev, int64_t M, int N, int K,
                                        int64_t ldc, const void* table_dev, int n_pos, int rope_cols, int head_dim, int batch,
                                        int pos0, void* stream) {
    if (M < 0 || M >= ((int64_t)1 << 31) || N < 1 || K < 1) return fail(KVPR_E_RANGE, "M=%lld N=%d K=%d out of range", (long long)M, N, K);
    if (K % 64 || N % 8 || ldc < N || ldc % 8) return fail(KVPR_E_INVAL, "need K %% 64 == 0, N %% 8 == 0, ldc >= N, ldc %% 8 == 0 (16-byte row pieces)");
    if (head_dim != 64 && head_dim != 128) return fail(KVPR_E_INVAL, "head_dim must be 64 or 128");
    if (rope_cols < 0 || rope_cols > N || rope_cols % 128) return fail(KVPR_E_INVAL, "rope_cols must be a multiple of 128 in [0, N]");
    if (batch < 1 || pos0 < 0 || n_pos < 1) return fail(KVPR_E_RANGE, "batch=%d pos0=%d n_pos=%d out of range", batch, pos0, n_pos);
    if (M == 0) return KVPR_OK;
    if (pos0 + (M - 1) / batch >= n_pos) return fail(KVPR_E_RANGE, "rows reach position %lld, the table has %d", (long long)(pos0 + (M - 1) / batch), n_pos);
    if (!a || !w || !cdev || !table_dev) return fail(KVPR_E_INVAL, "a / w / c / table is null");
    return kvpr::launch_gemm_rope(a, w, bias, cdev, M, N, K, ldc, table_dev, rope_cols, head_dim, batch, pos0, (hipStream_t)stream);
}

extern "C" int kvpr_rope_token(const void* qk32, const void* table_dev, int n_pos, int pos, int batch, int hidden, int head_dim,
                               void* q32, void* k16, int64_t ldk, void* stream) {
    if (batch < 1 || hidden < 1 || pos < 0 || pos >= n_pos) return fail(KVPR_E_RANGE, "batch=%d hidden=%d pos=%d n_pos=%d out of range", batch, hidden, pos, n_pos);
    if ((head_dim != 64 && head_dim != 128) || hidden % head_dim) return fail(KVPR_E_INVAL, "head_dim must be 64 or 128 and divide hidden");
    if (ldk < hidden) return fail(KVPR_E_INVAL, "ldk too small");
    if (!qk32 || !table_dev || !q32 || !k16) return fail(KVPR_E_INVAL, "null pointer");
    return kvpr::launch_rope_token(qk32, table_dev, pos, batch, hidden, head_dim, q32, k16, ldk, (hipStream_t)stream);
}

extern "C" size_t kvpr_int4_row_bytes(int cols) {
    if (cols < 64 || cols % 64) return 0;
    return kvpr::int4_row_bytes(cols);
}

static int check_codec_args(const void* src, const void* dst, int64_t rows, int cols) {
    if (rows < 0 || cols < 64 || cols % 64) return fail(KVPR_E_RANGE, "rows=%lld cols=%d: need rows >= 0 and cols a positive multiple of 64", (long long)rows, cols);
    if (rows * (int64_t)(cols / 8) > ((int64_t)1 << 38)) return fail(KVPR_E_RANGE, "rows * cols too large");
    if (rows > 0 && (!src || !dst)) return fail(KVPR_E_INVAL, "src / dst is null");
    return KVPR_OK;
}

extern "C" int kvpr_quant_int4(const void* src, void* dst, int64_t rows, int cols, void* stream) {
    if (int rc = check_codec_args(src, dst, rows, cols)) return rc;
    return kvpr::launch_quant_int4(src, dst, rows, cols, (hipStream_t)stream);
}

extern "C" int kvpr_dequant_int4(const void* src, void* dst, int64_t rows, int cols, void* stream) {
    if (int rc = check_codec_args(src, dst, rows, cols)) return rc;
    return kvpr::launch_dequant_int4(src, dst, rows, cols, (hipStream_t)stream);
}
