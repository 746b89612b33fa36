// Group-wise 4-bit codec for the host store (Sec. 4.4 "KV Cache Compression").
//
// The paper names the scheme without fixing a format; this library's format is:
//   - a group is 64 consecutive columns of one row (a [K|V] row of one sequence, or an activation row);
//   - mn = min(group), mx = max(group) (float16 values, exact), scale = float16((mx - mn) / 15);
//     code = clamp(rint((x - mn) / scale), 0, 15), all in float32 with IEEE division and
//     round-half-to-even; a group with scale == 0 has all codes 0;
//   - dequantised value = float16(code * scale + mn) (code * scale is exact in float32);
//   - a packed row of C columns is C/2 code bytes (element 2k in the low nibble of byte k, 2k+1 in
//     the high nibble) followed by C/64 pairs (scale, mn) of float16: 9C/16 bytes.
//
// Both kernels are plain streaming kernels: 8 lanes own one group, every lane moves 16 bytes of
// float16 and 4 bytes of codes, so global accesses of a wave are contiguous on both sides.
#include "kvpr_internal.h"

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void quant_int4_kernel(const _Float16* __restrict__ src, uint8_t* __restrict__ dst,
                                                         int64_t n_vec, int vec_per_row, int packed_row_bytes) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = t < n_vec;                       // n_vec is a multiple of 8: the 8 lanes of a group live together
    const int64_t tt = live ? t : 0;
    const half8 v = *reinterpret_cast<const half8*>(src + tt * 8);
    float x[8];
    float mn = (float)v[0], mx = (float)v[0];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x[i] = (float)v[i];
        mn = fminf(mn, x[i]);
        mx = fmaxf(mx, x[i]);
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    const _Float16 scale16 = (_Float16)__fdiv_rn(mx - mn, 15.0f);
    const float scale = (float)scale16;
    uint32_t word = 0;
    if (scale > 0.f) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float q = rintf(__fdiv_rn(x[i] - mn, scale));
            q = fminf(fmaxf(q, 0.f), 15.f);
            word |= (uint32_t)q << (4 * i);
        }
    }
    if (!live) return;
    const int64_t row = t / vec_per_row;
    const int j = (int)(t - row * vec_per_row);
    uint8_t* out = dst + row * packed_row_bytes;
    *reinterpret_cast<uint32_t*>(out + (int64_t)j * 4) = word;
    if ((j & 7) == 0) {
        union { _Float16 h[2]; uint32_t u; } meta;
        meta.h[0] = scale16;
        meta.h[1] = (_Float16)mn;
        *reinterpret_cast<uint32_t*>(out + (int64_t)vec_per_row * 4 + (j >> 3) * 4) = meta.u;
    }
}

__global__ __launch_bounds__(256) void dequant_int4_kernel(const uint8_t* __restrict__ src, _Float16* __restrict__ dst,
                                                           int64_t n_vec, int vec_per_row, int packed_row_bytes) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_vec) return;
    const int64_t row = t / vec_per_row;
    const int j = (int)(t - row * vec_per_row);
    const uint8_t* in = src + row * packed_row_bytes;
    const uint32_t word = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(in + (int64_t)j * 4));
    union { _Float16 h[2]; uint32_t u; } meta;
    meta.u = *reinterpret_cast<const uint32_t*>(in + (int64_t)vec_per_row * 4 + (j >> 3) * 4);
    const float scale = (float)meta.h[0], mn = (float)meta.h[1];
    half8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (_Float16)((float)((word >> (4 * i)) & 15u) * scale + mn);
    *reinterpret_cast<half8*>(dst + t * 8) = v;
}

}  // namespace

size_t int4_row_bytes(int cols) { return (size_t)cols / 2 + (size_t)cols / 16; }

int launch_quant_int4(const void* src, void* dst, int64_t rows, int cols, hipStream_t st) {
    const int64_t n_vec = rows * (cols / 8);
    if (n_vec == 0) return KVPR_OK;
    hipLaunchKernelGGL(quant_int4_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, st, (const _Float16*)src,
                       (uint8_t*)dst, n_vec, cols / 8, (int)int4_row_bytes(cols));
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int launch_dequant_int4(const void* src, void* dst, int64_t rows, int cols, hipStream_t st) {
    const int64_t n_vec = rows * (cols / 8);
    if (n_vec == 0) return KVPR_OK;
    hipLaunchKernelGGL(dequant_int4_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, st, (const uint8_t*)src,
                       (_Float16*)dst, n_vec, cols / 8, (int)int4_row_bytes(cols));
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

}  // namespace kvpr
