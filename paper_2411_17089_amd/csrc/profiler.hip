// Profiler module (Sec. 3.1): measures, on this machine and for this context's shape, the constants the
// scheduler needs (pinned H2D rate, recompute GEMM rate) and a few rates that are only reported.
#include "context.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

using kvpr::fail;
using kvpr::check_weights;

// ---- profiler (Sec. 3.1) ----
namespace {

template <class F>
int time_median(hipStream_t st, int reps, F fn, double* seconds) {
    hipEvent_t e0, e1;
    KVPR_HIP(hipEventCreate(&e0));
    KVPR_HIP(hipEventCreate(&e1));
    int rc = fn();                                   // warm-up
    if (rc == KVPR_OK && hipStreamSynchronize(st) != hipSuccess) rc = fail(KVPR_E_HIP, "profiler warm-up failed");
    std::vector<float> ms(reps);
    for (int r = 0; r < reps && rc == KVPR_OK; ++r) {
        if (hipEventRecord(e0, st) != hipSuccess) { rc = fail(KVPR_E_HIP, "event record failed"); break; }
        rc = fn();
        if (rc != KVPR_OK) break;
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms[r], e0, e1) != hipSuccess)
            rc = fail(KVPR_E_HIP, "profiler timing failed");
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != KVPR_OK) return rc;
    std::sort(ms.begin(), ms.end());
    *seconds = (double)ms[reps / 2] * 1e-3;
    return KVPR_OK;
}

}  // namespace

extern "C" int kvpr_profile(kvpr_ctx* c, int batch, int seq, kvpr_profile_t* out) {
    if (!c || !out) return fail(KVPR_E_INVAL, "ctx / out is null");
    if (batch < 1 || seq < 1) return fail(KVPR_E_RANGE, "batch and seq must be >= 1");
    const int64_t rows = (int64_t)batch * seq;
    if (rows > (int64_t)c->d.batch * (c->d.max_seq - 1))
        return fail(KVPR_E_RANGE, "batch*seq = %lld exceeds the context's batch*(max_seq-1)", (long long)rows);
    const int h = c->d.hidden;
    // the link is measured on what a full cache copy of [seq, batch] moves: packed rows if the store keeps them packed
    const size_t kv_bytes = c->qkv ? (size_t)rows * kvpr::int4_row_bytes(2 * h) : (size_t)rows * 2 * h * sizeof(half);
    const size_t cap_bytes = (size_t)c->d.max_seq * c->kv_store_bytes();
    KVPR_HIP(hipDeviceSynchronize());
    kvpr_profile_t p{};
    double t = 0;
    char* hkv = c->hkv[0];
    half* dkv = c->dkv[0];
    char* kv_stage = c->qkv ? c->dkvq[0] : (char*)dkv;

    // v_com: one pinned copy of the size of the whole cache of [seq, batch]
    if (int rc = time_median(c->copy, 5, [&]() -> int {
            KVPR_HIP(hipMemcpyAsync(kv_stage, hkv, kv_bytes, hipMemcpyHostToDevice, c->copy));
            return KVPR_OK; }, &t)) return rc;
    p.h2d_bytes_per_s = (double)kv_bytes / t;
    // d2h: the same bytes back to where they came from (the store keeps its contents)
    if (int rc = time_median(c->store, 3, [&]() -> int {
            KVPR_HIP(hipMemcpyAsync(hkv, kv_stage, kv_bytes, hipMemcpyDeviceToHost, c->store));
            return KVPR_OK; }, &t)) return rc;
    p.d2h_bytes_per_s = (double)kv_bytes / t;
    // best H2D rate over a size sweep
    p.h2d_peak_bytes_per_s = p.h2d_bytes_per_s;
    for (size_t sz = (size_t)64 << 10; sz <= std::min(cap_bytes, (size_t)1 << 30); sz *= 4) {
        if (int rc = time_median(c->copy, 5, [&]() -> int {
                KVPR_HIP(hipMemcpyAsync(kv_stage, hkv, sz, hipMemcpyHostToDevice, c->copy));
                return KVPR_OK; }, &t)) return rc;
        p.h2d_peak_bytes_per_s = std::max(p.h2d_peak_bytes_per_s, (double)sz / t);
    }
    KVPR_HIP(hipDeviceSynchronize());

    // v_gpu: the recompute GEMM at M = batch*seq on random operands
    half* wtmp = nullptr;
    // big enough for the widest matrix of the layer: [Wq;Wk;Wv], or one FFN matrix ([gate;up] for the gated FFN)
    const size_t ffn_rows = (size_t)c->d.ffn_dim * (c->llama ? 2 : 1);
    const size_t wtmp_halfs = std::max((size_t)3 * h, ffn_rows) * h;
    if (hipMalloc((void**)&wtmp, wtmp_halfs * sizeof(half)) != hipSuccess)
        return fail(KVPR_E_NOMEM, "profiler weight buffer");
    int rc = kvpr::launch_fill_random(wtmp, wtmp_halfs, 0.035f, 1u, c->compute);
    if (!rc) rc = kvpr::launch_fill_random(c->dx[0], (size_t)rows * h, 1.7f, 2u, c->compute);
    if (!rc) rc = time_median(c->compute, 5, [&]() -> int {
            // rotary models: positions as if the context's batch held these rows (the rotation costs the same anywhere)
            return c->llama ? kvpr::launch_gemm_rope(c->dx[0], wtmp, nullptr, dkv, rows, 2 * h, h, 2 * (int64_t)h, c->rope_tab, h,
                                                     c->d.head_dim, c->d.batch, 0, c->compute)
                            : kvpr::launch_gemm(c->dx[0], wtmp, nullptr, dkv, rows, 2 * h, h, 2 * (int64_t)h, c->compute); }, &t);
    const double gemm_flops = 4.0 * (double)rows * h * h;
    {   // the GEMM's work quantum: one 256 x 256 output tile (2 * 256 * 256 * K flops) on each compute unit
        int dev = 0, n_cu = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n_cu > 0)
            p.gemm_round_flops = (int64_t)n_cu * 2 * 256 * 256 * h;
    }
    if (!rc) p.gemm_alone_flops_per_s = p.gemm_flops_per_s = gemm_flops / t;
    // v_gpu as the cost model uses it: Eq. 10's max() term has the GEMM and a cache copy running together, and the
    // copy's stream of HBM writes slows the GEMM measurably (up to 15 % at hidden 7168).  So the GEMM is timed
    // again while a cache-sized pinned copy is landing in a scratch buffer; median of 3 such runs.
    if (!rc) {
        void* dtmp = nullptr;
        hipEvent_t go = nullptr, e0 = nullptr, e1 = nullptr;
        if (hipMalloc(&dtmp, kv_bytes) != hipSuccess) rc = fail(KVPR_E_NOMEM, "profiler copy target");
        if (!rc && (hipEventCreate(&go) != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess))
            rc = fail(KVPR_E_HIP, "profiler events");
        const double t_copy = (double)kv_bytes / p.h2d_bytes_per_s;
        const int reps = std::max(1, std::min(64, (int)(0.8 * t_copy / t)));
        float ms[3] = {0.f, 0.f, 0.f};
        for (int r = 0; r < 3 && !rc; ++r) {
            auto run = [&]() -> int {
                KVPR_HIP(hipEventRecord(go, c->compute));
                KVPR_HIP(hipStreamWaitEvent(c->copy, go, 0));
                KVPR_HIP(hipMemcpyAsync(dtmp, hkv, kv_bytes, hipMemcpyHostToDevice, c->copy));
                KVPR_HIP(hipEventRecord(e0, c->compute));
                for (int i = 0; i < reps; ++i)
                    if (int q = c->llama ? kvpr::launch_gemm_rope(c->dx[0], wtmp, nullptr, dkv, rows, 2 * h, h, 2 * (int64_t)h, c->rope_tab,
                                                                  h, c->d.head_dim, c->d.batch, 0, c->compute)
                                         : kvpr::launch_gemm(c->dx[0], wtmp, nullptr, dkv, rows, 2 * h, h, 2 * (int64_t)h, c->compute))
                        return q;
                KVPR_HIP(hipEventRecord(e1, c->compute));
                KVPR_HIP(hipStreamSynchronize(c->compute));
                KVPR_HIP(hipStreamSynchronize(c->copy));
                KVPR_HIP(hipEventElapsedTime(&ms[r], e0, e1));
                return KVPR_OK;
            };
            rc = run();
        }
        if (!rc) {
            std::sort(ms, ms + 3);
            if (ms[1] > 0.f) p.gemm_flops_per_s = gemm_flops * reps / ((double)ms[1] * 1e-3);
        }
        if (go) (void)hipEventDestroy(go);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        if (dtmp) (void)hipFree(dtmp);
    }
    // attention read rate over the cache just produced (context batch, S = rows / batch positions)
    const int S = (int)(rows / c->d.batch);
    if (!rc && S >= 1) {
        rc = kvpr::launch_fill_random(c->z16, (size_t)c->d.batch * h, 1.0f, 3u, c->compute);   // any finite q source
        if (!rc) rc = hipMemsetAsync(c->q32, 0, (size_t)c->d.batch * h * sizeof(float), c->compute) == hipSuccess
                          ? KVPR_OK : fail(KVPR_E_HIP, "memset failed");
        if (!rc) rc = time_median(c->compute, 5, [&]() -> int {
                return kvpr::launch_attention(c->q32, dkv, c->z16, c->attn_ws, S, c->d.batch, h, c->d.n_heads, c->compute); }, &t);
        if (!rc) p.attn_bytes_per_s = (double)S * c->d.batch * 2 * h * sizeof(half) / t;
        // the rest of a layer's GPU work besides the recomputation: projections, attention, FFN (random weights)
        if (!rc) rc = time_median(c->compute, 5, [&]() -> int {
                const int b = c->d.batch, f = c->d.ffn_dim;
                if (int r = kvpr::launch_token_gemm_flags(c->z16, wtmp, nullptr, c->q32, dkv, b, 3 * h, h, h, 2 * (int64_t)h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return r;
                if (int r = kvpr::launch_attention(c->q32, dkv, c->z16, c->attn_ws, S, b, h, c->d.n_heads, c->compute)) return r;
                if (int r = kvpr::launch_token_gemm_flags(c->z16, wtmp, nullptr, nullptr, dkv, b, h, h, 0, h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return r;
                if (f > 0) {
                    const int f1 = (int)ffn_rows;
                    half* prod = c->ffn1 + (c->llama ? (size_t)b * 2 * f : 0);
                    if (int r = kvpr::launch_token_gemm_flags(c->z16, wtmp, nullptr, nullptr, c->ffn1, b, f1, h, 0, f1, 1, c->compute, c->tok_ws, c->tok_ws_bytes)) return r;
                    if (int r = kvpr::launch_token_gemm_flags(prod, wtmp, nullptr, nullptr, dkv, b, h, f, 0, h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return r;
                }
                return KVPR_OK; }, &t);
        if (!rc) p.layer_other_s = t;
    }
    (void)hipDeviceSynchronize();
    (void)hipFree(wtmp);
    if (rc) return rc;
    *out = p;
    return KVPR_OK;
}

// v_gpu as one decode step of one layer runs the GEMM (Eq. 9, Eq. 10): the step is rehearsed at the split the
// profile plans.  X-sized copy first (the GPU idles, or runs the clock keep-alive if the context has one), then
// the GEMM over batch*l rows while the rest of a cache-sized copy lands; full synchronisation between rehearsals,
// as between steps.  A GPU that works in such bursts runs the GEMM at other clocks than in the back-to-back
// launches kvpr_profile times, in both directions: lower out of a long idle stretch, higher while the board's
// power average is low.
extern "C" int kvpr_profile_step(kvpr_ctx* c, int batch, int seq, kvpr_profile_t* prof) {
    if (!c || !prof) return fail(KVPR_E_INVAL, "ctx / prof is null");
    if (batch < 1 || seq < 1) return fail(KVPR_E_RANGE, "batch and seq must be >= 1");
    if (batch > c->d.batch || seq > c->d.max_seq - 1)
        return fail(KVPR_E_RANGE, "batch %d / seq %d exceed the context's %d / %d", batch, seq, c->d.batch, c->d.max_seq - 1);
    if (!(prof->h2d_bytes_per_s > 0.0) || !(prof->gemm_flops_per_s > 0.0))
        return fail(KVPR_E_INVAL, "prof needs positive h2d_bytes_per_s and gemm_flops_per_s (run kvpr_profile first)");
    const int h = c->d.hidden;
    // bytes and flops per position at this batch (the context's own per-position sizes are for its full batch)
    const int64_t x_bpp = (int64_t)c->x_store_bytes() / c->d.batch * batch;
    const int64_t kv_bpp = (int64_t)c->kv_store_bytes() / c->d.batch * batch;
    const int64_t f_pp = 4 * (int64_t)batch * h * h;
    // copy target: any split's X part and cache part side by side (X rows can be the larger ones when only the cache is packed)
    const size_t kv_bytes = (size_t)seq * (size_t)std::max(x_bpp, kv_bpp);

    half* wtmp = nullptr;
    void* dtmp = nullptr;
    hipEvent_t go = nullptr, ev_x = nullptr, e0 = nullptr, e1 = nullptr;
    int rc = KVPR_OK;
    KVPR_HIP(hipDeviceSynchronize());
    if (hipMalloc((void**)&wtmp, (size_t)2 * h * h * sizeof(half)) != hipSuccess) rc = fail(KVPR_E_NOMEM, "profiler weight buffer");
    if (!rc && hipMalloc(&dtmp, kv_bytes) != hipSuccess) rc = fail(KVPR_E_NOMEM, "profiler copy target");
    if (!rc && (hipEventCreate(&go) != hipSuccess || hipEventCreate(&ev_x) != hipSuccess || hipEventCreate(&e0) != hipSuccess ||
                hipEventCreate(&e1) != hipSuccess))
        rc = fail(KVPR_E_HIP, "profiler events");
    if (!rc) rc = kvpr::launch_fill_random(wtmp, (size_t)2 * h * h, 0.035f, 1u, c->compute);
    if (!rc) rc = kvpr::launch_fill_random(c->dx[0], (size_t)batch * seq * h, 1.7f, 2u, c->compute);

    kvpr_profile_t p = *prof;
    int32_t l_prev = -1;
    for (int pass = 0; pass < 2 && !rc; ++pass) {
        int32_t l = 0;
        rc = kvpr_plan_split_linear(&p, KVPR_COST_EQ10, 1, seq, x_bpp, kv_bpp, f_pp, 64, &l, nullptr);
        if (rc) break;
        if (l < 64) l = seq >= 128 ? seq * 3 / 4 / 64 * 64 : seq;      // a plan without recomputation: rehearse a typical split
        if (l == l_prev) break;
        l_prev = l;
        const size_t x_bytes = (size_t)l * x_bpp, rest_bytes = (size_t)(seq - l) * kv_bpp;
        const int64_t rows = (int64_t)batch * l;
        const double t_act = (double)x_bytes / p.h2d_bytes_per_s;
        float ms[4] = {0.f, 0.f, 0.f, 0.f};
        for (int r = 0; r < 4 && !rc; ++r) {
            auto run = [&]() -> int {
                KVPR_HIP(hipEventRecord(go, c->compute));
                KVPR_HIP(hipStreamWaitEvent(c->copy, go, 0));
                KVPR_HIP(hipMemcpyAsync(dtmp, c->hx[0], x_bytes, hipMemcpyHostToDevice, c->copy));
                KVPR_HIP(hipEventRecord(ev_x, c->copy));
                if (rest_bytes)
                    KVPR_HIP(hipMemcpyAsync((char*)dtmp + x_bytes, c->hkv[0] + (size_t)l * kv_bpp, rest_bytes, hipMemcpyHostToDevice, c->copy));
                if (c->keep_warm > 0.0 && t_act * c->keep_warm > 200e-6)
                    if (int q = kvpr::launch_keep_warm(wtmp, (size_t)2 * h * h, t_act * c->keep_warm, c->wall_clock_hz, c->q32, c->compute))
                        return q;
                KVPR_HIP(hipStreamWaitEvent(c->compute, ev_x, 0));
                KVPR_HIP(hipEventRecord(e0, c->compute));
                if (int q = c->llama ? kvpr::launch_gemm_rope(c->dx[0], wtmp, nullptr, c->dkv[0], rows, 2 * h, h, 2 * (int64_t)h, c->rope_tab,
                                                              h, c->d.head_dim, batch, 0, c->compute)
                                     : kvpr::launch_gemm(c->dx[0], wtmp, nullptr, c->dkv[0], rows, 2 * h, h, 2 * (int64_t)h, c->compute))
                    return q;
                KVPR_HIP(hipEventRecord(e1, c->compute));
                KVPR_HIP(hipStreamSynchronize(c->compute));
                KVPR_HIP(hipStreamSynchronize(c->copy));
                KVPR_HIP(hipEventElapsedTime(&ms[r], e0, e1));
                return KVPR_OK;
            };
            rc = run();
        }
        if (rc) break;
        std::sort(ms + 1, ms + 4);                                       // the first rehearsal is the warm-up
        int64_t flops = f_pp * l;                                        // charged as the cost model charges it
        if (const int64_t q = p.gemm_round_flops; q > 0) flops = (flops + q - 1) / q * q;
        if (ms[2] > 0.f) p.gemm_flops_per_s = (double)flops / ((double)ms[2] * 1e-3);
    }
    (void)hipDeviceSynchronize();
    if (go) (void)hipEventDestroy(go);
    if (ev_x) (void)hipEventDestroy(ev_x);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (dtmp) (void)hipFree(dtmp);
    if (wtmp) (void)hipFree(wtmp);
    if (rc) return rc;
    prof->gemm_flops_per_s = p.gemm_flops_per_s;
    return KVPR_OK;
}

// ---- MFMA ceiling probe (debug hook, used by `bench.py --power-probe`) ----
// A register-only loop of the recompute GEMM's MFMA (v_mfma_f32_32x32x16_f16, a 4 x 2 tile of accumulators per wave,
// two k-steps of fragments) on operand fragments read once from a_dev / w_dev: no LDS, no memory traffic in the
// loop.  Its rate on given data is what the chip's power limit leaves to any fp16 GEMM on that data.
namespace {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(512) void mfma_loop_kernel(const _Float16* __restrict__ xa, const _Float16* __restrict__ xw,
                                                         size_t n_a, size_t n_w, float* __restrict__ out, int iters) {
    probe_half8 w[2][4], a[2][2];
    const size_t t = (size_t)blockIdx.x * 512 + threadIdx.x;
    for (int s = 0; s < 2; ++s) {
        for (int i = 0; i < 4; ++i) w[s][i] = *reinterpret_cast<const probe_half8*>(xw + ((((t * 8 + s * 4 + i) * 8) % (n_w - 7)) & ~(size_t)7));
        for (int j = 0; j < 2; ++j) a[s][j] = *reinterpret_cast<const probe_half8*>(xa + ((((t * 4 + s * 2 + j) * 8) % (n_a - 7)) & ~(size_t)7));
    }
    probe_floatx16 c[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w[s][i], a[s][j], c[i][j], 0, 0, 0);
    }
    float sum = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) sum += c[i][j][r];
    out[t] = sum;
}

}  // namespace

// a_dev / w_dev: float16 arrays of n_a / n_w elements (>= 8 each); out_dev: float32 [256 * 512]; flops = 256 * 8 * iters * 16 * 32768
extern "C" int kvpr_debug_mfma_loop(const void* a_dev, const void* w_dev, int64_t n_a, int64_t n_w, void* out_dev, int iters, void* stream) {
    if (!a_dev || !w_dev || !out_dev || n_a < 8 || n_w < 8 || iters < 1) return fail(KVPR_E_INVAL, "bad mfma loop arguments");
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(256), dim3(512), 0, (hipStream_t)stream, (const _Float16*)a_dev, (const _Float16*)w_dev,
                       (size_t)n_a, (size_t)n_w, (float*)out_dev, iters);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

// ---- clock keep-alive (kvpr_set_keep_warm) ----
// The same register-only MFMA loop, bounded by wall time: every wave leaves once `budget_ticks` of the constant-rate
// wall clock have passed since it started, and after max_iters iterations at the latest.
namespace {

__global__ __launch_bounds__(512) void keep_warm_kernel(const _Float16* __restrict__ xw, size_t n_w, long long budget_ticks,
                                                         int max_iters, float* __restrict__ sink) {
    probe_half8 w[2][4], a[2][2];
    const size_t t = (size_t)blockIdx.x * 512 + threadIdx.x;
    for (int s = 0; s < 2; ++s) {
        for (int i = 0; i < 4; ++i) w[s][i] = *reinterpret_cast<const probe_half8*>(xw + ((((t * 8 + s * 4 + i) * 8) % (n_w - 7)) & ~(size_t)7));
        for (int j = 0; j < 2; ++j) a[s][j] = *reinterpret_cast<const probe_half8*>(xw + ((((t * 4 + s * 2 + j) * 8 + 4096) % (n_w - 7)) & ~(size_t)7));
    }
    probe_floatx16 c[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
    const long long t0 = wall_clock64();
    for (int it = 0; it < max_iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w[s][i], a[s][j], c[i][j], 0, 0, 0);
        if ((it & 3) == 3 && wall_clock64() - t0 >= budget_ticks) break;
    }
    float sum = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) sum += c[i][j][r];
    if (sum == 12345.678f) sink[t & 255] = sum;     // keeps the loop alive; never true for these operands in practice
}

}  // namespace

namespace kvpr {

// w: any resident float16 array of n_w >= 8192 elements (a weight matrix); seconds of wall time to stay busy
int launch_keep_warm(const void* w, size_t n_w, double seconds, double wall_clock_hz, void* sink, hipStream_t st) {
    if (!w || n_w < 8192 || !(seconds > 0.0) || !(wall_clock_hz > 0.0)) return KVPR_OK;
    const long long ticks = (long long)(seconds * wall_clock_hz);
    // an iteration is 16 MFMAs per wave, two waves per SIMD: at least 1024 cycles, i.e. >= 0.4 us at any clock the chip runs;
    // the iteration bound is a backstop of a few times the requested time
    long long max_iters = (long long)(seconds / 0.4e-6) * 4 + 64;
    if (max_iters > 2000000) max_iters = 2000000;
    hipLaunchKernelGGL(keep_warm_kernel, dim3(256), dim3(512), 0, st, (const _Float16*)w, n_w, ticks, (int)max_iters, (float*)sink);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

}  // namespace kvpr
