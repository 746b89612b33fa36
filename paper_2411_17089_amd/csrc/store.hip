// Host store (Sec. 3.3 "pinned memory"): writing rows, borrowing the pinned arrays, and the prefill stand-in.
#include "context.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

using kvpr::fail;
using kvpr::check_weights;

extern "C" int kvpr_store_write(kvpr_ctx* c, int layer, int t0, int t1, const void* x_host, const void* kv_host) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (layer < 0 || layer >= c->slots()) return fail(KVPR_E_RANGE, "layer %d outside [0, %d)", layer, c->slots());
    if (t0 < 0 || t1 < t0 || t1 > c->d.max_seq) return fail(KVPR_E_RANGE, "rows [%d, %d) outside [0, %d]", t0, t1, c->d.max_seq);
    // the copy/store streams may still be touching the store
    KVPR_HIP(hipStreamSynchronize(c->copy));
    KVPR_HIP(hipStreamSynchronize(c->store));
    const size_t xr = c->x_row_halfs(), kr = c->kv_row_halfs();
    const size_t xsb = c->x_store_bytes(), ksb = c->kv_store_bytes();
    const size_t n = (size_t)(t1 - t0);
    // an array kept compressed is packed on the GPU (one codec implementation): float16 rows up, packed rows down
    auto write_packed = [&](const void* src, half* dev, char* stage, char* dst, size_t row_halfs, size_t row_store_bytes,
                            int cols) -> int {
        KVPR_HIP(hipDeviceSynchronize());
        KVPR_HIP(hipMemcpy(dev, src, n * row_halfs * sizeof(half), hipMemcpyHostToDevice));
        if (int rc = kvpr::launch_quant_int4(dev, stage, (int64_t)n * c->d.batch, cols, c->compute)) return rc;
        KVPR_HIP(hipMemcpyAsync(dst, stage, n * row_store_bytes, hipMemcpyDeviceToHost, c->compute));
        KVPR_HIP(hipStreamSynchronize(c->compute));
        return KVPR_OK;
    };
    if (x_host && n > 0) {
        if (c->qx) {
            if (int rc = write_packed(x_host, c->dx[0], c->dxq[0], c->hx[layer] + (size_t)t0 * xsb, xr, xsb, c->d.hidden)) return rc;
        } else {
            memcpy(c->hx[layer] + (size_t)t0 * xsb, x_host, n * xsb);
        }
    }
    if (x_host && t0 <= c->x_rows[layer]) c->x_rows[layer] = std::max(c->x_rows[layer], t1);
    if (kv_host && n > 0) {
        if (c->qkv) {
            if (int rc = write_packed(kv_host, c->dkv[0], c->dkvq[0], c->hkv[layer] + (size_t)t0 * ksb, kr, ksb, 2 * c->d.hidden)) return rc;
        } else {
            memcpy(c->hkv[layer] + (size_t)t0 * ksb, kv_host, n * ksb);
        }
    }
    if (kv_host && t0 <= c->kv_rows[layer]) c->kv_rows[layer] = std::max(c->kv_rows[layer], t1);
    return KVPR_OK;
}

extern "C" int kvpr_store_ptrs(kvpr_ctx* c, int layer, void** x_host, void** kv_host) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (layer < 0 || layer >= c->slots()) return fail(KVPR_E_RANGE, "layer %d outside [0, %d)", layer, c->slots());
    if (x_host) *x_host = c->hx[layer];
    if (kv_host) *kv_host = c->hkv[layer];
    // the caller may now write any row directly: treat all rows as holding data
    c->x_rows[layer] = c->d.max_seq;
    c->kv_rows[layer] = c->d.max_seq;
    return KVPR_OK;
}

extern "C" int kvpr_store_prefill_kv(kvpr_ctx* c, int layer, int seq, const kvpr_layer_weights* w) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (layer < 0 || layer >= c->slots()) return fail(KVPR_E_RANGE, "layer %d outside [0, %d)", layer, c->slots());
    if (seq < 0 || seq > c->d.max_seq) return fail(KVPR_E_RANGE, "seq %d outside [0, %d]", seq, c->d.max_seq);
    if (int rc = check_weights(c, w, false)) return rc;
    if (c->x_rows[layer] < seq) return fail(KVPR_E_STATE, "layer %d: only %d activation rows written", layer, c->x_rows[layer]);
    if (seq == 0) return KVPR_OK;
    const int h = c->d.hidden;
    const size_t xsb = c->x_store_bytes(), ksb = c->kv_store_bytes();
    KVPR_HIP(hipDeviceSynchronize());
    // the activations as the store returns them (dequantised if it keeps them packed)
    KVPR_HIP(hipMemcpyAsync(c->qx ? (void*)c->dxq[0] : (void*)c->dx[0], c->hx[layer], (size_t)seq * xsb, hipMemcpyHostToDevice, c->compute));
    if (c->qx)
        if (int rc = kvpr::launch_dequant_int4(c->dxq[0], c->dx[0], (int64_t)seq * c->d.batch, h, c->compute)) return rc;
    const half* wkv = (const half*)w->wqkv + (size_t)h * h;
    const half* bkv = w->bqkv ? (const half*)w->bqkv + h : nullptr;
    if (int rc = c->llama ? kvpr::launch_gemm_rope(c->dx[0], wkv, bkv, c->dkv[0], (int64_t)seq * c->d.batch, 2 * h, h, 2 * (int64_t)h,
                                                   c->rope_tab, h, c->d.head_dim, c->d.batch, 0, c->compute)
                          : kvpr::launch_gemm(c->dx[0], wkv, bkv, c->dkv[0], (int64_t)seq * c->d.batch, 2 * h, h, 2 * (int64_t)h, c->compute))
        return rc;
    if (c->qkv)
        if (int rc = kvpr::launch_quant_int4(c->dkv[0], c->dkvq[0], (int64_t)seq * c->d.batch, 2 * h, c->compute)) return rc;
    KVPR_HIP(hipMemcpyAsync(c->hkv[layer], c->qkv ? (const void*)c->dkvq[0] : (const void*)c->dkv[0], (size_t)seq * ksb,
                            hipMemcpyDeviceToHost, c->compute));
    KVPR_HIP(hipStreamSynchronize(c->compute));
    c->kv_rows[layer] = std::max(c->kv_rows[layer], seq);
    return KVPR_OK;
}
