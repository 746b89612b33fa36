// Runtime module (Sec. 3.3): context life cycle, copy / store streams, event-fenced overlap of transfer and
// recomputation, per-layer decode, the layer-pipelined decode step and the column-by-column schedule.
#include "context.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

namespace kvpr {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace kvpr

using kvpr::fail;

namespace kvpr {

int check_weights(const kvpr_ctx* c, const kvpr_layer_weights* w, bool need_ffn) {
    if (!w) return fail(KVPR_E_INVAL, "weights are null");
    if (!w->wqkv || !w->wo) return fail(KVPR_E_INVAL, "wqkv / wo must not be null");
    if (need_ffn && (!w->w1 || !w->w2 || !w->ln1_g || !w->ln2_g))
        return fail(KVPR_E_INVAL, "FFN / norm weights must not be null for a full decoder layer");
    if (need_ffn && !c->llama && (!w->ln1_b || !w->ln2_b))
        return fail(KVPR_E_INVAL, "LayerNorm offsets must not be null for a full decoder layer");
    return KVPR_OK;
}

}  // namespace kvpr

using kvpr::check_weights;

namespace {

int debug_sync(kvpr_ctx* c) {
    if (c->debug & KVPR_DEBUG_SYNC) {
        KVPR_HIP(hipStreamSynchronize(c->copy));
        KVPR_HIP(hipStreamSynchronize(c->compute));
        KVPR_HIP(hipStreamSynchronize(c->store));
    }
    return KVPR_OK;
}

int ensure_timing_events(kvpr_ctx* c, int slots) {
    while ((int)c->tev.size() < slots) {
        LayerEvents le{};
        for (int i = 0; i < LayerEvents::count; ++i) KVPR_HIP(hipEventCreate(&le.at[i]));
        c->tev.push_back(le);
    }
    return KVPR_OK;
}


int adapt_poll(kvpr_ctx* c);

int resolve_split(kvpr_ctx* c, int seq, int split, int32_t* out) {
    if (split == -1) {
        if (!c->have_prof) return fail(KVPR_E_STATE, "split = -1 needs kvpr_set_profile first");
        if (int rc = adapt_poll(c)) return rc;
        return kvpr_plan_split_linear(&c->prof, c->cost_model, c->plan_chunks(), seq, (int64_t)c->x_store_bytes(),
                                      (int64_t)c->kv_store_bytes(), c->flops_per_pos(), c->granularity, out, nullptr);
    }
    if (split < 0 || split > seq) return fail(KVPR_E_RANGE, "split %d outside [0, %d]", split, seq);
    *out = split;
    return KVPR_OK;
}

// Enqueue one attention layer's decode on the three streams.  ev may be null (no timing).
// wf (nullable): fences for weights that are themselves in flight from the host
struct WeightFence {
    hipEvent_t kv_ready;    // Wk|Wv and their bias have landed
    hipEvent_t all_ready;   // the whole layer has landed
};

int enqueue_layer(kvpr_ctx* c, int layer, int seq, int l, const kvpr_layer_weights* w, const half* x_new, half* out,
                  int buf, LayerEvents* ev, bool fence_copy_to_start, const WeightFence* wf = nullptr) {
    const int b = c->d.batch, h = c->d.hidden;
    const size_t xr = c->x_row_halfs(), kr = c->kv_row_halfs();
    const size_t xsb = c->x_store_bytes(), ksb = c->kv_store_bytes();
    half* dkv = c->dkv[buf];
    half* dx = c->dx[buf];
    // where copies from / to the store land on the device: the float16 buffers, or the packed staging buffers
    char* x_stage = c->qx ? c->dxq[buf] : (char*)dx;
    char* kv_stage = c->qkv ? c->dkvq[buf] : (char*)dkv;

    // adaptive profile: an untimed layer borrows a probe event set (if one is free) so that its copy and
    // GEMM durations can be read later without any synchronisation
    int probe_slot = -1;
    if (!ev && c->adapt_alpha > 0.0 && c->have_prof) {
        if (!c->probe_made) {
            for (auto& le : c->probe)
                for (int i = 0; i < LayerEvents::count; ++i) KVPR_HIP(hipEventCreate(&le.at[i]));
            c->probe_made = true;
        }
        if (!c->probe_pending[c->probe_next]) {
            probe_slot = c->probe_next;
            c->probe_next = (c->probe_next + 1) % kvpr_ctx::kProbes;
            ev = &c->probe[probe_slot];
        }
    }

    if (ev) {
        ev->seq = seq;
        ev->split = l;
        KVPR_HIP(hipEventRecord(ev->at[LayerEvents::start], c->compute));
    }
    if (c->debug & KVPR_DEBUG_POISON) {
        if (int rc = kvpr::launch_fill_u16(dkv, (size_t)(seq + 1) * kr, 0x7E00, c->compute)) return rc;
        if (int rc = kvpr::launch_fill_u16(dx, (size_t)seq * xr, 0x7E00, c->compute)) return rc;
        // packed staging: all-ones words decode to NaN scale and minimum
        if (c->qx) if (int rc = kvpr::launch_fill_u16(x_stage, (size_t)seq * xsb / 2, 0xFFFF, c->compute)) return rc;
        if (c->qkv) if (int rc = kvpr::launch_fill_u16(kv_stage, (size_t)seq * ksb / 2, 0xFFFF, c->compute)) return rc;
    }
    if (fence_copy_to_start || (c->debug & KVPR_DEBUG_POISON)) {
        KVPR_HIP(hipEventRecord(c->ev_begin, c->compute));
        KVPR_HIP(hipStreamWaitEvent(c->copy, c->ev_begin, 0));
    }

    // ---- copy stream: activations first, then the rest of the cache (the order Eq. 10 assumes) ----
    if (c->free_recorded[buf]) KVPR_HIP(hipStreamWaitEvent(c->copy, c->ev_free[buf], 0));
    // ... and the previous user's store-back, which reads its new row out of this device buffer
    if (c->buf_store_recorded[buf]) KVPR_HIP(hipStreamWaitEvent(c->copy, c->ev_buf_store[buf], 0));
    // the previous token's store-back wrote host row seq-1 of this slot, which the copies below may read
    if (c->slot_store_recorded[layer]) KVPR_HIP(hipStreamWaitEvent(c->copy, c->ev_slot_store[layer], 0));
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::c0], c->copy));
    // chunk boundaries: equal parts of [0, l) rounded down to multiples of 8 positions (whole GEMM tile rows
    // at batch 32); a single chunk is the paper's schedule
    int nchunk = (l > 0) ? std::min(c->chunks, std::max(1, l / 8)) : 0;
    int bound[kvpr_ctx::kMaxChunks + 1];
    for (int j = 0; j <= nchunk; ++j) bound[j] = (j == nchunk) ? l : (int)((int64_t)l * j / nchunk) / 8 * 8;
    for (int j = 0; j < nchunk; ++j) {
        if (bound[j + 1] > bound[j])
            KVPR_HIP(hipMemcpyAsync(x_stage + (size_t)bound[j] * xsb, c->hx[layer] + (size_t)bound[j] * xsb,
                                    (size_t)(bound[j + 1] - bound[j]) * xsb, hipMemcpyHostToDevice, c->copy));
        if (nchunk > 1) KVPR_HIP(hipEventRecord(c->ev_chunk[buf][j], c->copy));
    }
    KVPR_HIP(hipEventRecord(c->ev_x[buf], c->copy));
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::c_x], c->copy));
    if (l < seq)
        KVPR_HIP(hipMemcpyAsync(kv_stage + (size_t)l * ksb, c->hkv[layer] + (size_t)l * ksb, (size_t)(seq - l) * ksb,
                                hipMemcpyHostToDevice, c->copy));
    KVPR_HIP(hipEventRecord(c->ev_kv[buf], c->copy));
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::c_kv], c->copy));
    if (int rc = debug_sync(c)) return rc;

    // ---- new token's q (float32) and k|v row `seq` of the device cache (Eq. 1, Eq. 5), then the store-back ----
    auto project_and_store = [&]() -> int {
        if (wf) KVPR_HIP(hipStreamWaitEvent(c->compute, wf->all_ready, 0));
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::p0], c->compute));
        if (c->llama) {
            // q and k stay float32 until they are rotated with position seq; v goes straight into the cache row
            if (int rc = kvpr::launch_token_gemm_flags(x_new, w->wqkv, w->bqkv, c->qk32, dkv + (size_t)seq * kr + h, b, 3 * h, h,
                                                       2 * h, 2 * (int64_t)h, 0, c->compute, c->tok_ws, c->tok_ws_bytes))
                return rc;
            if (int rc = kvpr::launch_rope_token(c->qk32, c->rope_tab, seq, b, h, c->d.head_dim, c->q32, dkv + (size_t)seq * kr,
                                                 2 * (int64_t)h, c->compute))
                return rc;
        } else if (int rc = kvpr::launch_token_gemm_flags(x_new, w->wqkv, w->bqkv, c->q32, dkv + (size_t)seq * kr, b, 3 * h, h, h,
                                                          2 * (int64_t)h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) {
            return rc;
        }
        // a compressed store receives the new rows packed (Sec. 4.4); attention below still reads the exact row
        if (c->qkv)
            if (int rc = kvpr::launch_quant_int4(dkv + (size_t)seq * kr, kv_stage + (size_t)seq * ksb, b, 2 * h, c->compute)) return rc;
        if (c->qx)
            if (int rc = kvpr::launch_quant_int4(x_new, x_stage + (size_t)seq * xsb, b, h, c->compute)) return rc;
        KVPR_HIP(hipEventRecord(c->ev_proj, c->compute));
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::p1], c->compute));
        // store stream: write the new rows back to the host store.  A copy kernel writes them into the mapped pinned
        // arrays: with hipMemcpyAsync device-to-host copies here, layer decodes fed to the streams one at a time while
        // earlier ones ran had their host-to-device copies and the GEMM slowed down by up to 2x for steps at a time
        // (22 % per step on average; 3-6 % with the kernel)
        KVPR_HIP(hipStreamWaitEvent(c->store, c->ev_proj, 0));
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::s0], c->store));
        if (int rc = kvpr::launch_copy_bytes(kv_stage + (size_t)seq * ksb, c->hkv[layer] + (size_t)seq * ksb, ksb, c->store)) return rc;
        if (int rc = kvpr::launch_copy_bytes(c->qx ? (const void*)(x_stage + (size_t)seq * xsb) : (const void*)x_new,
                                             c->hx[layer] + (size_t)seq * xsb, xsb, c->store))
            return rc;
        KVPR_HIP(hipEventRecord(c->ev_store, c->store));
        KVPR_HIP(hipEventRecord(c->ev_slot_store[layer], c->store));
        c->slot_store_recorded[layer] = true;
        KVPR_HIP(hipEventRecord(c->ev_buf_store[buf], c->store));
        c->buf_store_recorded[buf] = true;
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::s1], c->store));
        return debug_sync(c);
    };
    // ---- recompute rows [0, l) as soon as their activations have landed (Eq. 7) ----
    auto recompute = [&]() -> int {
        if (wf) KVPR_HIP(hipStreamWaitEvent(c->compute, wf->kv_ready, 0));
        // single-layer latency path: the GPU would sit idle while X[0:l] is on the link and come out of that with its
        // clocks down; keep it busy for most of the predicted copy time instead (kvpr_set_keep_warm)
        if (fence_copy_to_start && !wf && c->keep_warm > 0.0 && c->have_prof && l > 0) {
            const double t_first = (double)bound[1] * (double)xsb / c->prof.h2d_bytes_per_s;
            if (t_first * c->keep_warm > 200e-6)
                if (int rc = kvpr::launch_keep_warm(w->wqkv, (size_t)3 * h * h, t_first * c->keep_warm, c->wall_clock_hz, c->q32, c->compute))
                    return rc;
        }
        if (nchunk <= 1) KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_x[buf], 0));
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::r0], c->compute));
        if (l > 0) {
            const half* wkv = (const half*)w->wqkv + (size_t)h * h;
            const half* bkv = w->bqkv ? (const half*)w->bqkv + h : nullptr;
            for (int j = 0; j < nchunk; ++j) {
                // with several chunks the GEMM of chunk j runs while chunks j+1.. and the cache are still on the link
                if (nchunk > 1) KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_chunk[buf][j], 0));
                const int64_t rows = (int64_t)(bound[j + 1] - bound[j]) * b;
                if (c->qx)
                    if (int rc = kvpr::launch_dequant_int4(x_stage + (size_t)bound[j] * xsb, dx + (size_t)bound[j] * xr, rows, h, c->compute))
                        return rc;
                // rotary models: the K half is rotated with the positions of its rows, bound[j] .. bound[j+1]-1
                if (int rc = c->llama
                                 ? kvpr::launch_gemm_rope(dx + (size_t)bound[j] * xr, wkv, bkv, dkv + (size_t)bound[j] * kr, rows, 2 * h, h,
                                                          2 * (int64_t)h, c->rope_tab, h, c->d.head_dim, b, bound[j], c->compute)
                                 : kvpr::launch_gemm(dx + (size_t)bound[j] * xr, wkv, bkv, dkv + (size_t)bound[j] * kr, rows, 2 * h, h,
                                                     2 * (int64_t)h, c->compute))
                    return rc;
            }
        }
        if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::r1], c->compute));
        return debug_sync(c);
    };
    if (wf) {
        // offloaded weights: Wk|Wv arrive first, so the recomputation goes first and the projections that need
        // Wq follow (fine-grained MHA pipeline, Sec. 3.3 "Hiding KV cache partial recomputation")
        if (int rc = recompute()) return rc;
        if (int rc = project_and_store()) return rc;
    } else {
        // resident weights: the token projection runs while the activations are still on the link
        if (int rc = project_and_store()) return rc;
        if (int rc = recompute()) return rc;
    }

    // ---- merge = wait for the transferred rows; then attention over all seq+1 rows (Eq. 2) ----
    // With a packed cache the attention runs in two phases: the recomputed rows and the new row (float16) before the
    // wait, the transferred rows straight from their packed form after it (dequantised in registers), one combine.
    // A float16 cache takes the same two phases in the latency-oriented single-layer call when enough rows are
    // recomputed: most of the attention then runs under the tail of the cache copy.  (In the layer pipeline the
    // attention is off the critical path and stays one launch.)
    const bool two_phase = c->qkv || (fence_copy_to_start && l >= 128);
    const void* packed = c->qkv ? kv_stage : nullptr;
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::e0], c->compute));
    if (two_phase)
        if (int rc = kvpr::launch_attention_mixed(c->q32, dkv, packed, c->z16, c->attn_ws, seq + 1, l, b, h, c->d.n_heads, 0, c->compute))
            return rc;
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::e1], c->compute));
    KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_kv[buf], 0));
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::a0], c->compute));
    if (int rc = two_phase ? kvpr::launch_attention_mixed(c->q32, dkv, packed, c->z16, c->attn_ws, seq + 1, l, b, h, c->d.n_heads, 1, c->compute)
                           : kvpr::launch_attention(c->q32, dkv, c->z16, c->attn_ws, seq + 1, b, h, c->d.n_heads, c->compute))
        return rc;
    KVPR_HIP(hipEventRecord(c->ev_free[buf], c->compute));
    c->free_recorded[buf] = true;
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::a1], c->compute));

    // ---- output projection (Eq. 3) ----
    if (int rc = kvpr::launch_token_gemm_flags(c->z16, w->wo, w->bo, nullptr, out, b, h, h, 0, h, 0, c->compute, c->tok_ws, c->tok_ws_bytes))
        return rc;
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::o1], c->compute));
    KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_store, 0));
    if (ev) KVPR_HIP(hipEventRecord(ev->at[LayerEvents::end], c->compute));
    if (int rc = debug_sync(c)) return rc;

    if (c->x_rows[layer] == seq) c->x_rows[layer] = seq + 1;
    if (c->kv_rows[layer] == seq) c->kv_rows[layer] = seq + 1;
    if (probe_slot >= 0) c->probe_pending[probe_slot] = true;
    return KVPR_OK;
}

// fold the probes that have finished into the profile (no waiting: unfinished probes stay pending)
int adapt_poll(kvpr_ctx* c) {
    if (!(c->adapt_alpha > 0.0) || !c->probe_made) return KVPR_OK;
    for (int i = 0; i < kvpr_ctx::kProbes; ++i) {
        if (!c->probe_pending[i]) continue;
        LayerEvents* ev = &c->probe[i];
        const hipError_t q1 = hipEventQuery(ev->at[LayerEvents::end]), q2 = hipEventQuery(ev->at[LayerEvents::c_kv]);
        if (q1 == hipErrorNotReady || q2 == hipErrorNotReady) continue;
        if (q1 != hipSuccess || q2 != hipSuccess) return fail(KVPR_E_HIP, "probe event query failed");
        c->probe_pending[i] = false;
        float ms_x = 0.f, ms_kv = 0.f, ms_rc = 0.f;
        KVPR_HIP(hipEventElapsedTime(&ms_x, ev->at[LayerEvents::c0], ev->at[LayerEvents::c_x]));
        KVPR_HIP(hipEventElapsedTime(&ms_kv, ev->at[LayerEvents::c_x], ev->at[LayerEvents::c_kv]));
        KVPR_HIP(hipEventElapsedTime(&ms_rc, ev->at[LayerEvents::r0], ev->at[LayerEvents::r1]));
        const int64_t l = ev->split, s = ev->seq;
        const int64_t link_bytes = (int64_t)c->x_store_bytes() * l + (int64_t)c->kv_store_bytes() * (s - l);
        // with a chunked activation copy the GEMM interval includes waiting for chunks: the link sample only
        // (whole rounds of work when the profile says the GEMM works in rounds, as the cost model charges them)
        int64_t flops = c->chunks > 1 ? 0 : c->flops_per_pos() * l;
        if (const int64_t r = c->prof.gemm_round_flops; r > 0) flops = (flops + r - 1) / r * r;
        if (int rc = kvpr_adapt_update(&c->prof, c->adapt_alpha, link_bytes, ((double)ms_x + (double)ms_kv) * 1e-3, flops,
                                       (double)ms_rc * 1e-3))
            return rc;
    }
    return KVPR_OK;
}

int read_timing(kvpr_ctx* c, LayerEvents* ev, int seq, int l, kvpr_layer_timing* t) {
    auto ms = [&](hipEvent_t a, hipEvent_t b, float* out) -> int {
        KVPR_HIP(hipEventElapsedTime(out, a, b));
        return KVPR_OK;
    };
    kvpr_layer_timing r{};
    float to_gemm = 0.f, to_kv = 0.f;
    if (int rc = ms(ev->at[LayerEvents::c0], ev->at[LayerEvents::c_x], &r.ms_act_copy)) return rc;
    if (int rc = ms(ev->at[LayerEvents::c_x], ev->at[LayerEvents::c_kv], &r.ms_kv_copy)) return rc;
    if (int rc = ms(ev->at[LayerEvents::r0], ev->at[LayerEvents::r1], &r.ms_recompute)) return rc;
    if (int rc = ms(ev->at[LayerEvents::p0], ev->at[LayerEvents::p1], &r.ms_proj)) return rc;
    if (int rc = ms(ev->at[LayerEvents::a0], ev->at[LayerEvents::a1], &r.ms_attn)) return rc;
    if (int rc = ms(ev->at[LayerEvents::a1], ev->at[LayerEvents::o1], &r.ms_out)) return rc;
    if (int rc = ms(ev->at[LayerEvents::s0], ev->at[LayerEvents::s1], &r.ms_store)) return rc;
    if (int rc = ms(ev->at[LayerEvents::start], ev->at[LayerEvents::r1], &to_gemm)) return rc;
    if (int rc = ms(ev->at[LayerEvents::start], ev->at[LayerEvents::c_kv], &to_kv)) return rc;
    if (int rc = ms(ev->at[LayerEvents::start], ev->at[LayerEvents::end], &r.ms_total)) return rc;
    // attention = the phase before the cache fence (empty unless it ran in two phases) + the phase after it
    float ms_early = 0.f;
    if (int rc = ms(ev->at[LayerEvents::e0], ev->at[LayerEvents::e1], &ms_early)) return rc;
    r.ms_attn += ms_early;
    r.ms_attn_early = ms_early;
    if (int rc = ms(ev->at[LayerEvents::start], ev->at[LayerEvents::r0], &r.ms_recompute_start)) return rc;
    if (ev->has_w_all) {
        if (int rc = ms(ev->at[LayerEvents::start], ev->at[LayerEvents::w_all], &r.ms_weights_landed)) return rc;
        r.weights_landed_valid = 1;
        ev->has_w_all = false;
    }
    r.ms_assemble = std::max(to_gemm, to_kv);
    r.split = l;
    if (c->have_prof)
        if (int rc = kvpr_cost_linear(&c->prof, c->cost_model, c->plan_chunks(), l, seq, (int64_t)c->x_store_bytes(),
                                      (int64_t)c->kv_store_bytes(), c->flops_per_pos(), &r.t_bound_s))
            return rc;
    *t = r;
    return KVPR_OK;
}

int check_decode_args(kvpr_ctx* c, int layer, int seq) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (layer < 0 || layer >= c->slots()) return fail(KVPR_E_RANGE, "layer %d outside [0, %d)", layer, c->slots());
    if (seq < 0 || seq + 1 > c->d.max_seq)
        return fail(KVPR_E_RANGE, "seq %d: need 0 <= seq and seq + 1 <= max_seq = %d", seq, c->d.max_seq);
    return KVPR_OK;
}

int check_rows(kvpr_ctx* c, int layer, int seq, int l) {
    if (c->x_rows[layer] < l)
        return fail(KVPR_E_STATE, "layer %d: activations of rows [%d, %d) were never written to the host store", layer,
                    c->x_rows[layer], l);
    if (c->kv_rows[layer] < seq && l < seq)
        return fail(KVPR_E_STATE, "layer %d: cache rows [%d, %d) were never written to the host store", layer,
                    c->kv_rows[layer], seq);
    return KVPR_OK;
}

void destroy_impl(kvpr_ctx* c) {
    if (!c) return;
    if (c->copy) (void)hipStreamSynchronize(c->copy);
    if (c->store) (void)hipStreamSynchronize(c->store);
    (void)hipStreamSynchronize(c->compute);
    for (hipEvent_t e : c->ev_slot_store) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev_step) if (e) (void)hipEventDestroy(e);
    for (auto p : c->hx) if (p) (void)hipHostFree(p);
    for (auto p : c->hkv) if (p) (void)hipHostFree(p);
    for (int i = 0; i < 2; ++i) {
        if (c->dx[i]) (void)hipFree(c->dx[i]);
        if (c->dkv[i]) (void)hipFree(c->dkv[i]);
        if (c->dxq[i]) (void)hipFree(c->dxq[i]);
        if (c->dkvq[i]) (void)hipFree(c->dkvq[i]);
        if (c->ev_x[i]) (void)hipEventDestroy(c->ev_x[i]);
        if (c->ev_kv[i]) (void)hipEventDestroy(c->ev_kv[i]);
        if (c->ev_free[i]) (void)hipEventDestroy(c->ev_free[i]);
        if (c->ev_buf_store[i]) (void)hipEventDestroy(c->ev_buf_store[i]);
        for (hipEvent_t e : c->ev_chunk[i]) if (e) (void)hipEventDestroy(e);
    }
    if (c->wstream) (void)hipStreamSynchronize(c->wstream);
    for (auto p : c->hw) if (p) (void)hipHostFree(p);
    if (c->hhid) (void)hipHostFree(c->hhid);
    for (int i = 0; i < 2; ++i) {
        if (c->hin[i]) (void)hipFree(c->hin[i]);
        if (c->hout[i]) (void)hipFree(c->hout[i]);
        hipEvent_t he[] = {c->ev_hin_loaded[i], c->ev_hin_free[i], c->ev_hout_ready[i], c->ev_hout_free[i]};
        for (hipEvent_t e : he) if (e) (void)hipEventDestroy(e);
    }
    for (int i = 0; i < 2; ++i) {
        hipEvent_t we[] = {c->ev_wkv[i], c->ev_wall[i], c->ev_wfree[i]};
        for (hipEvent_t e : we) if (e) (void)hipEventDestroy(e);
    }
    if (c->wstream) (void)hipStreamDestroy(c->wstream);
    void* dev[] = {c->qk32, c->rope_tab, c->q32, c->z16, c->attn_ws, c->tok_ws, c->hid, c->xn, c->attn_out, c->ffn1, c->ffn2, c->dw[0], c->dw[1], c->hid_all};
    for (void* p : dev) if (p) (void)hipFree(p);
    hipEvent_t evs[] = {c->ev_proj, c->ev_store, c->ev_begin};
    for (hipEvent_t e : evs) if (e) (void)hipEventDestroy(e);
    for (auto& le : c->tev)
        for (int i = 0; i < LayerEvents::count; ++i) (void)hipEventDestroy(le.at[i]);
    if (c->probe_made)
        for (auto& le : c->probe)
            for (int i = 0; i < LayerEvents::count; ++i) (void)hipEventDestroy(le.at[i]);
    if (c->copy) (void)hipStreamDestroy(c->copy);
    if (c->store) (void)hipStreamDestroy(c->store);
    delete c;
}

}  // namespace

extern "C" const char* kvpr_last_error(void) { return kvpr::g_err; }

namespace {

// The runtime binds streams to a few hardware queues (four per process by default), the least used one first, and a
// queue runs its packets in order.  When two streams share a queue, the marker that follows a long host-to-device copy
// on one of them holds back whatever the other enqueues after it: measured on the column schedule, the recomputation of
// a layer's first batch started 19 ms late, after the whole layer's weights instead of after [Wk;Wv], whenever the
// compute stream happened to share its queue with the weight stream (which depends on how many streams the process made
// before the context).  So every stream made here is checked against the streams it must run beside: a small kernel
// on the one has to finish while a 0.4 ms kernel is still running on the other.  (A copy would be the more direct
// blocker, but a lone copy at creation leaves both streams with the same preferred DMA engine, and the first step then
// runs its activation copy behind the weights: measured.)  A stream that fails is replaced; the rejected ones stay
// alive until the end so that the next one lands on another queue.  Best effort: after a few attempts the last stream
// is kept as it is.
int g_streams_replaced = 0;   // over the life of the process; read by tests through kvpr_debug_streams_replaced
int settle_streams(kvpr_ctx* c) {
    // the blocker: a register-only loop that runs for 0.4 ms of wall clock (bounded by an iteration count as well)
    const half* blk = (const half*)((char*)c->tok_ws + 4096);               // the partial-tile area: scratch, any contents
    const size_t blk_n = (c->tok_ws_bytes - 4096) / sizeof(half);
    if (!c->tok_ws || blk_n < 8192 || !(c->wall_clock_hz > 0.0)) return KVPR_OK;
    hipEvent_t e_busy = nullptr, e_probe = nullptr;
    KVPR_HIP(hipEventCreateWithFlags(&e_busy, hipEventDisableTiming));
    KVPR_HIP(hipEventCreateWithFlags(&e_probe, hipEventDisableTiming));
    std::vector<hipStream_t> rejected;
    // held: a small kernel on `probe` did not finish before the blocker running on `busy` did
    auto held_back = [&](hipStream_t busy, hipStream_t probe, bool* held) -> int {
        // first use binds a stream to its queue, which takes longer than the blocker runs: do that before the measurement
        for (hipStream_t st : {busy, probe}) {
            if (int rc = kvpr::launch_fill_u16(c->z16, 64, 0, st)) return rc;
            KVPR_HIP(hipStreamSynchronize(st));
        }
        if (int rc = kvpr::launch_keep_warm(blk, blk_n, 0.4e-3, c->wall_clock_hz, c->q32, busy)) return rc;
        KVPR_HIP(hipEventRecord(e_busy, busy));
        if (int rc = kvpr::launch_fill_u16(c->z16, 64, 0, probe)) return rc;
        KVPR_HIP(hipEventRecord(e_probe, probe));
        KVPR_HIP(hipEventSynchronize(e_probe));
        *held = hipEventQuery(e_busy) == hipSuccess;
        (void)hipGetLastError();                                             // "not ready" is the good answer here
        KVPR_HIP(hipEventSynchronize(e_busy));
        return KVPR_OK;
    };
    // `mine` carries copies (or, for the store stream, must not queue behind them): none of `beside` may share its queue
    auto settle = [&](hipStream_t* mine, bool mine_is_busy_side, std::initializer_list<hipStream_t> beside) -> int {
        for (int attempt = 0; attempt < 6; ++attempt) {
            bool shared = false;
            for (hipStream_t other : beside) {
                bool held = false;
                if (int rc = mine_is_busy_side ? held_back(*mine, other, &held) : held_back(other, *mine, &held)) return rc;
                shared = shared || held;
            }
            if (!shared || attempt == 5) break;
            rejected.push_back(*mine);
            ++g_streams_replaced;
            KVPR_HIP(hipStreamCreateWithFlags(mine, hipStreamNonBlocking));
        }
        return KVPR_OK;
    };
    int rc = settle(&c->copy, true, {c->compute});
    if (!rc && c->wstream) rc = settle(&c->wstream, true, {c->compute, c->copy});
    if (!rc) rc = c->wstream ? settle(&c->store, false, {c->copy, c->wstream}) : settle(&c->store, false, {c->copy});
    for (hipStream_t st : rejected) (void)hipStreamDestroy(st);
    (void)hipEventDestroy(e_busy);
    (void)hipEventDestroy(e_probe);
    return rc;
}

// element offsets (in halfs) of one layer's parameters inside a weight blob; the host (pinned) and
// device blobs share the layout so that a range of the blob is one contiguous copy.  [Wk;Wv], the
// q|k|v bias and the parameters of the norm in front of the attention block come right after Wq: the
// range [wkv, wo) is all that the pre-attention norm and the recomputation need.
struct BlobLayout {
    size_t wq, wkv, bqkv, wo, bo, ln1_g, ln1_b, ln2_g, ln2_b, w1, b1, w2, b2, total;
    BlobLayout(size_t h, size_t f, bool gated) {
        size_t o = 0;
        auto take = [&](size_t n) { size_t at = o; o += (n + 63) / 64 * 64; return at; };   // 128-byte aligned pieces
        wq = take(h * h);          // rows [0, h) of wqkv
        wkv = take(2 * h * h);     // rows [h, 3h): contiguous with wq because h*h is a multiple of 64
        bqkv = take(3 * h);
        ln1_g = take(h); ln1_b = take(h);
        wo = take(h * h);
        bo = take(h);
        ln2_g = take(h); ln2_b = take(h);
        w1 = take((gated ? 2 : 1) * f * h); b1 = take(f);   // gated FFN: [gate; up] stacked
        w2 = take(h * f); b2 = take(h);
        total = o;
    }
};

kvpr_layer_weights blob_weights(half* blob, const BlobLayout& L) {
    kvpr_layer_weights w{};
    w.wqkv = blob + L.wq; w.bqkv = blob + L.bqkv; w.wo = blob + L.wo; w.bo = blob + L.bo;
    w.ln1_g = blob + L.ln1_g; w.ln1_b = blob + L.ln1_b; w.ln2_g = blob + L.ln2_g; w.ln2_b = blob + L.ln2_b;
    w.w1 = blob + L.w1; w.b1 = blob + L.b1; w.w2 = blob + L.w2; w.b2 = blob + L.b2;
    return w;
}

int create_impl(const kvpr_model_desc* d, int n_gpu_batches, void* compute_stream, kvpr_ctx** out);

}  // namespace

extern "C" int kvpr_create(const kvpr_model_desc* d, void* compute_stream, kvpr_ctx** out) {
    return create_impl(d, 0, compute_stream, out);
}

extern "C" int kvpr_create_offload(const kvpr_model_desc* d, int n_gpu_batches, void* compute_stream, kvpr_ctx** out) {
    if (n_gpu_batches < 1 || n_gpu_batches > 64) return fail(KVPR_E_RANGE, "n_gpu_batches %d outside [1, 64]", n_gpu_batches);
    if (d && d->ffn_dim <= 0) return fail(KVPR_E_INVAL, "the column-by-column schedule needs a full decoder layer (ffn_dim > 0)");
    return create_impl(d, n_gpu_batches, compute_stream, out);
}

namespace {

int create_impl(const kvpr_model_desc* d, int n_gpu_batches, void* compute_stream, kvpr_ctx** out) {
    if (!d || !out) return fail(KVPR_E_INVAL, "desc / out is null");
    if ((d->dtype & ~KVPR_STORE_INT4) != KVPR_F16)
        return fail(KVPR_E_INVAL, "dtype must be KVPR_F16, optionally with KVPR_KV_INT4 / KVPR_X_INT4");
    if (d->n_layers < 1 || d->batch < 1 || d->max_seq < 1) return fail(KVPR_E_RANGE, "n_layers, batch, max_seq must be >= 1");
    if (d->batch > 64) return fail(KVPR_E_RANGE, "batch %d > 64 is not supported by the token GEMM", d->batch);
    if (d->head_dim != 64 && d->head_dim != 128) return fail(KVPR_E_INVAL, "head_dim must be 64 or 128");
    if (d->n_heads < 1 || d->hidden != d->n_heads * d->head_dim)
        return fail(KVPR_E_INVAL, "hidden (%d) != n_heads (%d) * head_dim (%d)", d->hidden, d->n_heads, d->head_dim);
    if (d->hidden % 128) return fail(KVPR_E_INVAL, "hidden must be a multiple of 128");
    if (d->ffn_dim < 0 || d->ffn_dim % 128) return fail(KVPR_E_INVAL, "ffn_dim must be 0 or a multiple of 128");
    if (d->arch != KVPR_ARCH_OPT && d->arch != KVPR_ARCH_LLAMA) return fail(KVPR_E_INVAL, "unknown arch %d", d->arch);
    if (d->arch == KVPR_ARCH_LLAMA && !(d->rope_base >= 0.f && std::isfinite(d->rope_base)))
        return fail(KVPR_E_INVAL, "rope_base must be finite and >= 0 (0 = 10000)");

    kvpr_ctx* c = new (std::nothrow) kvpr_ctx;
    if (!c) return fail(KVPR_E_NOMEM, "out of host memory");
    c->d = *d;
    c->nb = n_gpu_batches;
    c->llama = d->arch == KVPR_ARCH_LLAMA;
    c->qx = (d->dtype & KVPR_X_INT4) != 0;
    c->qkv = (d->dtype & KVPR_KV_INT4) != 0;
    c->compute = (hipStream_t)compute_stream;
    {
        int dev = 0, khz = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
            c->wall_clock_hz = (double)khz * 1e3;
    }
    const int slots = c->slots();
    c->nbuf = slots > 1 ? 2 : 1;
    const size_t x_bytes = (size_t)d->max_seq * c->x_row_halfs() * sizeof(half);
    const size_t kv_bytes = 2 * x_bytes;
    const size_t xs_bytes = (size_t)d->max_seq * c->x_store_bytes(), kvs_bytes = (size_t)d->max_seq * c->kv_store_bytes();
    auto bail = [&](int code, const char* what, hipError_t e) {
        int rc = fail(code, "%s: %s", what, hipGetErrorString(e));
        char keep[sizeof kvpr::g_err];
        memcpy(keep, kvpr::g_err, sizeof keep);
        destroy_impl(c);
        memcpy(kvpr::g_err, keep, sizeof keep);
        return rc;
    };
    hipError_t e;
    if ((e = hipStreamCreateWithFlags(&c->copy, hipStreamNonBlocking)) != hipSuccess) return bail(KVPR_E_HIP, "copy stream", e);
    if ((e = hipStreamCreateWithFlags(&c->store, hipStreamNonBlocking)) != hipSuccess) return bail(KVPR_E_HIP, "store stream", e);
    c->hx.assign(slots, nullptr);
    c->hkv.assign(slots, nullptr);
    c->x_rows.assign(slots, 0);
    c->kv_rows.assign(slots, 0);
    c->ev_slot_store.assign(slots, nullptr);
    c->slot_store_recorded.assign(slots, false);
    for (int i = 0; i < slots; ++i) {
        if ((e = hipEventCreateWithFlags(&c->ev_slot_store[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        if ((e = hipHostMalloc((void**)&c->hx[i], xs_bytes, hipHostMallocDefault)) != hipSuccess) return bail(KVPR_E_NOMEM, "pinned X store", e);
        if ((e = hipHostMalloc((void**)&c->hkv[i], kvs_bytes, hipHostMallocDefault)) != hipSuccess) return bail(KVPR_E_NOMEM, "pinned KV store", e);
    }
    for (int i = 0; i < c->nbuf; ++i) {
        if ((e = hipMalloc((void**)&c->dx[i], x_bytes)) != hipSuccess) return bail(KVPR_E_NOMEM, "device X buffer", e);
        if ((e = hipMalloc((void**)&c->dkv[i], kv_bytes)) != hipSuccess) return bail(KVPR_E_NOMEM, "device KV buffer", e);
        if (c->qx && (e = hipMalloc((void**)&c->dxq[i], xs_bytes)) != hipSuccess) return bail(KVPR_E_NOMEM, "device packed X buffer", e);
        if (c->qkv && (e = hipMalloc((void**)&c->dkvq[i], kvs_bytes)) != hipSuccess) return bail(KVPR_E_NOMEM, "device packed KV buffer", e);
    }
    for (int i = 0; i < 2; ++i) {
        if ((e = hipEventCreateWithFlags(&c->ev_x[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        if ((e = hipEventCreateWithFlags(&c->ev_kv[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        if ((e = hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        if ((e = hipEventCreateWithFlags(&c->ev_buf_store[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        for (int j = 0; j < kvpr_ctx::kMaxChunks; ++j)
            if ((e = hipEventCreateWithFlags(&c->ev_chunk[i][j], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
    }
    if ((e = hipEventCreateWithFlags(&c->ev_proj, hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
    if ((e = hipEventCreateWithFlags(&c->ev_store, hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
    if ((e = hipEventCreateWithFlags(&c->ev_begin, hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
    for (int i = 0; i < 2; ++i)
        if ((e = hipEventCreateWithFlags(&c->ev_step[i], hipEventDisableTiming | hipEventBlockingSync)) != hipSuccess)
            return bail(KVPR_E_HIP, "event", e);
    const size_t bh = (size_t)d->batch * d->hidden;
    if ((e = hipMalloc((void**)&c->q32, bh * sizeof(float))) != hipSuccess) return bail(KVPR_E_NOMEM, "q buffer", e);
    if ((e = hipMalloc((void**)&c->z16, bh * sizeof(half))) != hipSuccess) return bail(KVPR_E_NOMEM, "z buffer", e);
    if ((e = hipMalloc(&c->attn_ws, kvpr::attention_workspace_bytes(d->batch, d->hidden, d->n_heads, d->max_seq))) != hipSuccess)
        return bail(KVPR_E_NOMEM, "attention workspace", e);
    // K-slice partials of the token GEMMs with few output features (output projection, FFN down); its arrival
    // counters start at zero and every launch leaves them at zero
    c->tok_ws_bytes = kvpr::token_gemm_workspace_bytes(d->batch, d->hidden);
    if ((e = hipMalloc(&c->tok_ws, c->tok_ws_bytes)) != hipSuccess) return bail(KVPR_E_NOMEM, "token GEMM workspace", e);
    if ((e = hipMemset(c->tok_ws, 0, 4096)) != hipSuccess || (e = hipStreamSynchronize(nullptr)) != hipSuccess)
        return bail(KVPR_E_HIP, "token GEMM workspace", e);
    if (c->llama) {
        if ((e = hipMalloc((void**)&c->qk32, 2 * bh * sizeof(float))) != hipSuccess) return bail(KVPR_E_NOMEM, "q|k buffer", e);
        // (cos, sin)(p * theta_i), theta_i = base^(-2i/d): evaluated in double on the host, stored as float
        std::vector<float2> tab((size_t)d->max_seq * (d->head_dim / 2));
        if (kvpr_rope_table((float*)tab.data(), d->max_seq, d->head_dim, d->rope_base > 0.f ? (double)d->rope_base : 10000.0) != KVPR_OK) {
            destroy_impl(c);
            return KVPR_E_INVAL;
        }
        if ((e = hipMalloc((void**)&c->rope_tab, tab.size() * sizeof(float2))) != hipSuccess) return bail(KVPR_E_NOMEM, "rotary table", e);
        if ((e = hipMemcpy(c->rope_tab, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice)) != hipSuccess)
            return bail(KVPR_E_HIP, "rotary table upload", e);
    }
    if (d->ffn_dim > 0) {
        half** bufs[] = {&c->hid, &c->xn, &c->attn_out, &c->ffn2};
        for (half** p : bufs)
            if ((e = hipMalloc((void**)p, bh * sizeof(half))) != hipSuccess) return bail(KVPR_E_NOMEM, "hidden-state buffer", e);
        // gated FFN: [gate | up] (2 ffn columns) followed by their gated product (ffn columns)
        if ((e = hipMalloc((void**)&c->ffn1, (size_t)d->batch * d->ffn_dim * (c->llama ? 3 : 1) * sizeof(half))) != hipSuccess)
            return bail(KVPR_E_NOMEM, "FFN buffer", e);
    }
    if (c->nb > 0) {
        const BlobLayout L(d->hidden, d->ffn_dim, c->llama);
        if ((e = hipStreamCreateWithFlags(&c->wstream, hipStreamNonBlocking)) != hipSuccess) return bail(KVPR_E_HIP, "weight stream", e);
        c->hw.assign(d->n_layers, nullptr);
        c->w_written.assign(d->n_layers, false);
        for (int i = 0; i < d->n_layers; ++i)
            if ((e = hipHostMalloc((void**)&c->hw[i], L.total * sizeof(half), hipHostMallocDefault)) != hipSuccess)
                return bail(KVPR_E_NOMEM, "pinned weight store", e);
        for (int i = 0; i < 2; ++i) {
            if ((e = hipMalloc((void**)&c->dw[i], L.total * sizeof(half))) != hipSuccess) return bail(KVPR_E_NOMEM, "device weight buffer", e);
            if ((e = hipEventCreateWithFlags(&c->ev_wkv[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
            if ((e = hipEventCreateWithFlags(&c->ev_wall[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
            if ((e = hipEventCreateWithFlags(&c->ev_wfree[i], hipEventDisableTiming)) != hipSuccess) return bail(KVPR_E_HIP, "event", e);
        }
        if ((e = hipMalloc((void**)&c->hid_all, (size_t)c->nb * bh * sizeof(half))) != hipSuccess) return bail(KVPR_E_NOMEM, "hidden states", e);
    }
    if (int rc = settle_streams(c)) {
        destroy_impl(c);
        return rc;
    }
    *out = c;
    return KVPR_OK;
}

}  // namespace

extern "C" int kvpr_debug_streams_replaced(void) { return g_streams_replaced; }

extern "C" int kvpr_destroy(kvpr_ctx* c) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    destroy_impl(c);
    return KVPR_OK;
}

extern "C" int kvpr_set_debug(kvpr_ctx* c, int flags) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (flags & ~(KVPR_DEBUG_SYNC | KVPR_DEBUG_POISON)) return fail(KVPR_E_INVAL, "unknown debug flags 0x%x", flags);
    c->debug = flags;
    return KVPR_OK;
}

extern "C" int kvpr_set_weight_pipeline(kvpr_ctx* c, int fine_grained) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (c->nb <= 0) return fail(KVPR_E_STATE, "context was not created with kvpr_create_offload");
    c->weight_pipeline = fine_grained != 0;
    return KVPR_OK;
}

extern "C" int kvpr_set_hidden_offload(kvpr_ctx* c, int on) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (c->nb <= 0) return fail(KVPR_E_STATE, "context was not created with kvpr_create_offload");
    if (on && !c->hhid) {
        const size_t bh = (size_t)c->d.batch * c->d.hidden;
        KVPR_HIP(hipHostMalloc((void**)&c->hhid, (size_t)c->nb * bh * sizeof(half), hipHostMallocDefault));
        for (int i = 0; i < 2; ++i) {
            KVPR_HIP(hipMalloc((void**)&c->hin[i], bh * sizeof(half)));
            KVPR_HIP(hipMalloc((void**)&c->hout[i], bh * sizeof(half)));
            KVPR_HIP(hipEventCreateWithFlags(&c->ev_hin_loaded[i], hipEventDisableTiming));
            KVPR_HIP(hipEventCreateWithFlags(&c->ev_hin_free[i], hipEventDisableTiming));
            KVPR_HIP(hipEventCreateWithFlags(&c->ev_hout_ready[i], hipEventDisableTiming));
            KVPR_HIP(hipEventCreateWithFlags(&c->ev_hout_free[i], hipEventDisableTiming));
        }
    }
    // steps in flight keep the mode they were enqueued with; the staging buffers and events are reused across steps
    c->hid_offload = on != 0;
    return KVPR_OK;
}

extern "C" int kvpr_set_chunks(kvpr_ctx* c, int chunks) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (chunks < 1 || chunks > kvpr_ctx::kMaxChunks) return fail(KVPR_E_RANGE, "chunks %d outside [1, %d]", chunks, kvpr_ctx::kMaxChunks);
    c->chunks = chunks;
    return KVPR_OK;
}

extern "C" int kvpr_set_profile(kvpr_ctx* c, const kvpr_profile_t* p, int cost_model, int granularity) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    int32_t l;
    // validates the profile, the model and the granularity
    if (int rc = kvpr_plan_split(p, cost_model, c->d.batch, 1, c->d.hidden, 2, granularity, &l, nullptr)) return rc;
    if (c->chunks > 1 && cost_model == KVPR_COST_EQ10)
        if (int rc = kvpr_plan_split_chunked(p, c->chunks, c->d.batch, 1, c->d.hidden, 2, granularity, &l, nullptr)) return rc;
    c->prof = *p;
    c->cost_model = cost_model;
    c->granularity = granularity;
    c->have_prof = true;
    return KVPR_OK;
}

extern "C" int kvpr_set_adaptive(kvpr_ctx* c, double alpha) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(KVPR_E_RANGE, "alpha %g outside [0, 1]", alpha);
    c->adapt_alpha = alpha;
    return KVPR_OK;
}

extern "C" int kvpr_set_keep_warm(kvpr_ctx* c, double fraction) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (!(fraction >= 0.0 && fraction <= 0.95)) return fail(KVPR_E_RANGE, "fraction %g outside [0, 0.95]", fraction);
    if (fraction > 0.0 && !(c->wall_clock_hz > 0.0)) return fail(KVPR_E_STATE, "the device reports no wall clock rate");
    c->keep_warm = fraction;
    return KVPR_OK;
}

extern "C" int kvpr_get_profile(kvpr_ctx* c, kvpr_profile_t* out) {
    if (!c || !out) return fail(KVPR_E_INVAL, "ctx / out is null");
    if (!c->have_prof) return fail(KVPR_E_STATE, "no profile was set");
    if (int rc = adapt_poll(c)) return rc;
    *out = c->prof;
    return KVPR_OK;
}


extern "C" int kvpr_layer_decode(kvpr_ctx* c, int layer, int seq, int split, const kvpr_layer_weights* w,
                                 const void* x_new_dev, void* out_dev, kvpr_layer_timing* timing) {
    if (int rc = check_decode_args(c, layer, seq)) return rc;
    if (int rc = check_weights(c, w, false)) return rc;
    if (!x_new_dev || !out_dev) return fail(KVPR_E_INVAL, "x_new_dev / out_dev is null");
    int32_t l;
    if (int rc = resolve_split(c, seq, split, &l)) return rc;
    if (int rc = check_rows(c, layer, seq, l)) return rc;
    LayerEvents* ev = nullptr;
    if (timing) {
        if (int rc = ensure_timing_events(c, 1)) return rc;
        ev = &c->tev[0];
    }
    const int buf = layer % c->nbuf;
    if (int rc = enqueue_layer(c, layer, seq, l, w, (const half*)x_new_dev, (half*)out_dev, buf, ev, true)) return rc;
    if (timing) {
        KVPR_HIP(hipStreamSynchronize(c->compute));
        KVPR_HIP(hipStreamSynchronize(c->copy));
        KVPR_HIP(hipStreamSynchronize(c->store));
        return read_timing(c, ev, seq, l, timing);
    }
    return KVPR_OK;
}

extern "C" int kvpr_layer_decode_timed(kvpr_ctx* c, int layer, int seq, int split, const kvpr_layer_weights* w,
                                       const void* x_new_dev, void* out_dev, int slot) {
    if (int rc = check_decode_args(c, layer, seq)) return rc;
    if (int rc = check_weights(c, w, false)) return rc;
    if (!x_new_dev || !out_dev) return fail(KVPR_E_INVAL, "x_new_dev / out_dev is null");
    if (slot < 0 || slot >= 4096) return fail(KVPR_E_RANGE, "timing slot %d outside [0, 4096)", slot);
    int32_t l;
    if (int rc = resolve_split(c, seq, split, &l)) return rc;
    if (int rc = check_rows(c, layer, seq, l)) return rc;
    if (int rc = ensure_timing_events(c, slot + 1)) return rc;
    return enqueue_layer(c, layer, seq, l, w, (const half*)x_new_dev, (half*)out_dev, layer % c->nbuf, &c->tev[slot], true);
}

extern "C" int kvpr_timing_read(kvpr_ctx* c, int slot, kvpr_layer_timing* timing) {
    if (!c || !timing) return fail(KVPR_E_INVAL, "ctx / timing is null");
    if (slot < 0 || slot >= (int)c->tev.size() || c->tev[slot].seq < 0)
        return fail(KVPR_E_STATE, "timing slot %d holds no recording", slot);
    LayerEvents* ev = &c->tev[slot];
    KVPR_HIP(hipEventSynchronize(ev->at[LayerEvents::end]));
    KVPR_HIP(hipEventSynchronize(ev->at[LayerEvents::c_kv]));
    KVPR_HIP(hipEventSynchronize(ev->at[LayerEvents::s1]));
    return read_timing(c, ev, ev->seq, ev->split, timing);
}

namespace {

// the parts of a decoder layer around the attention block (c->xn = normalised input of the attention block)
int pre_attention_norm(kvpr_ctx* c, const kvpr_layer_weights* w, const half* hid_in) {
    const int b = c->d.batch, h = c->d.hidden;
    if (c->llama) return kvpr::launch_rmsnorm(hid_in, w->ln1_g, c->xn, b, h, c->compute);
    return kvpr::launch_layernorm(hid_in, w->ln1_g, w->ln1_b, c->xn, b, h, c->compute);
}

// hid_out = r + FFN(norm(r)),  r = hid_in + attn_out.  OPT: LayerNorm, ReLU FFN with biases (Eq. 4);
// LLaMA: RMSNorm, down(silu(gate) * up) with w1 = [gate; up] stacked
int residual_and_ffn(kvpr_ctx* c, const kvpr_layer_weights* w, const half* hid_in, half* hid_out) {
    const int b = c->d.batch, h = c->d.hidden, f = c->d.ffn_dim;
    const size_t bh = (size_t)b * h;
    if (int rc = kvpr::launch_add(hid_in, c->attn_out, c->ffn2, bh, c->compute)) return rc;      // ffn2 = residual stream
    if (c->llama) {
        half* prod = c->ffn1 + (size_t)b * 2 * f;
        if (int rc = kvpr::launch_rmsnorm(c->ffn2, w->ln2_g, c->xn, b, h, c->compute)) return rc;
        if (int rc = kvpr::launch_token_gemm_flags(c->xn, w->w1, nullptr, nullptr, c->ffn1, b, 2 * f, h, 0, 2 * (int64_t)f, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return rc;
        if (int rc = kvpr::launch_silu_mul(c->ffn1, prod, b, f, c->compute)) return rc;
        if (int rc = kvpr::launch_token_gemm_flags(prod, w->w2, nullptr, nullptr, c->attn_out, b, h, f, 0, h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return rc;
    } else {
        if (int rc = kvpr::launch_layernorm(c->ffn2, w->ln2_g, w->ln2_b, c->xn, b, h, c->compute)) return rc;
        if (int rc = kvpr::launch_token_gemm_flags(c->xn, w->w1, w->b1, nullptr, c->ffn1, b, f, h, 0, f, 1, c->compute, c->tok_ws, c->tok_ws_bytes)) return rc;
        if (int rc = kvpr::launch_token_gemm_flags(c->ffn1, w->w2, w->b2, nullptr, c->attn_out, b, h, f, 0, h, 0, c->compute, c->tok_ws, c->tok_ws_bytes)) return rc;
    }
    return kvpr::launch_add(c->ffn2, c->attn_out, hid_out, bh, c->compute);
}

}  // namespace

namespace {

// Bound on the run-ahead of a caller that enqueues token after token without synchronising: at most two whole-stack
// steps are in flight.  With more (a 40-layer step is ~2000 stream operations) the runtime itself stalls the host for
// a second at a time and steps in a deep queue ran up to twice as long (measured: 290 -> 330-590 ms per token).
int step_begin(kvpr_ctx* c) {
    if (c->steps_enqueued >= 2) KVPR_HIP(hipEventSynchronize(c->ev_step[c->steps_enqueued & 1]));
    return KVPR_OK;
}
int step_end(kvpr_ctx* c) {
    KVPR_HIP(hipEventRecord(c->ev_step[c->steps_enqueued & 1], c->compute));
    ++c->steps_enqueued;
    return KVPR_OK;
}

}  // namespace

extern "C" int kvpr_decode_step(kvpr_ctx* c, int seq, const kvpr_layer_weights* layers, const void* x_in_dev,
                                void* x_out_dev, const int32_t* splits_in, int32_t* splits_out,
                                kvpr_layer_timing* per_layer) {
    if (int rc = check_decode_args(c, 0, seq)) return rc;
    if (c->d.ffn_dim <= 0) return fail(KVPR_E_STATE, "kvpr_decode_step needs ffn_dim > 0");
    if (c->nb > 0) return fail(KVPR_E_STATE, "context was created for offloaded weights: use kvpr_decode_step_columns");
    if (!layers || !x_in_dev || !x_out_dev) return fail(KVPR_E_INVAL, "layers / x_in_dev / x_out_dev is null");
    const int L = c->d.n_layers, b = c->d.batch, h = c->d.hidden;
    std::vector<int32_t> ls(L);
    for (int i = 0; i < L; ++i) {
        if (int rc = check_weights(c, &layers[i], true)) return rc;
        if (int rc = resolve_split(c, seq, splits_in ? splits_in[i] : -1, &ls[i])) return rc;
        if (int rc = check_rows(c, i, seq, ls[i])) return rc;
    }
    if (per_layer)
        if (int rc = ensure_timing_events(c, L)) return rc;
    if (int rc = step_begin(c)) return rc;
    const size_t bh = (size_t)b * h;
    const half* hid_in = (const half*)x_in_dev;
    for (int i = 0; i < L; ++i) {
        const kvpr_layer_weights* w = &layers[i];
        half* hid_out = (i == L - 1) ? (half*)x_out_dev : c->hid;
        // pre-norm -> attention block -> residual -> norm -> FFN -> residual
        if (int rc = pre_attention_norm(c, w, hid_in)) return rc;
        if (int rc = enqueue_layer(c, i, seq, ls[i], w, c->xn, c->attn_out, i % c->nbuf, per_layer ? &c->tev[i] : nullptr, false))
            return rc;
        if (int rc = residual_and_ffn(c, w, hid_in, hid_out)) return rc;
        hid_in = hid_out;
    }
    if (int rc = step_end(c)) return rc;
    if (splits_out) std::copy(ls.begin(), ls.end(), splits_out);
    if (per_layer) {
        KVPR_HIP(hipStreamSynchronize(c->compute));
        KVPR_HIP(hipStreamSynchronize(c->copy));
        KVPR_HIP(hipStreamSynchronize(c->store));
        for (int i = 0; i < L; ++i)
            if (int rc = read_timing(c, &c->tev[i], seq, ls[i], &per_layer[i])) return rc;
    }
    return KVPR_OK;
}

extern "C" int kvpr_greedy_next(const void* hidden_dev, const void* w_lm_dev, const void* emb_dev, int batch, int hidden,
                                int vocab, void* logits_dev, int32_t* tokens_dev, void* x_next_dev, void* stream) {
    if (batch < 1 || batch > 64 || hidden < 1 || vocab < 1) return fail(KVPR_E_RANGE, "batch=%d (1..64) hidden=%d vocab=%d out of range", batch, hidden, vocab);
    if (hidden % 128) return fail(KVPR_E_INVAL, "hidden must be a multiple of 128");
    if (!hidden_dev || !w_lm_dev || !logits_dev || !tokens_dev) return fail(KVPR_E_INVAL, "null pointer");
    if ((emb_dev == nullptr) != (x_next_dev == nullptr)) return fail(KVPR_E_INVAL, "emb_dev and x_next_dev go together");
    hipStream_t st = (hipStream_t)stream;
    if (int rc = kvpr::launch_token_gemm_flags(hidden_dev, w_lm_dev, nullptr, logits_dev, nullptr, batch, vocab, hidden, vocab, 0, 0, st)) return rc;
    if (int rc = kvpr::launch_argmax_rows((const float*)logits_dev, batch, vocab, tokens_dev, st)) return rc;
    if (emb_dev) return kvpr::launch_gather_rows(emb_dev, tokens_dev, x_next_dev, batch, hidden, st);
    return KVPR_OK;
}

// ---- column-by-column schedule with offloaded weights (Sec. 3.2, Sec. 3.3, Algorithm 1) ----
extern "C" int kvpr_weights_write(kvpr_ctx* c, int layer, const kvpr_layer_weights* host) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (c->nb <= 0) return fail(KVPR_E_STATE, "context was not created with kvpr_create_offload");
    if (layer < 0 || layer >= c->d.n_layers) return fail(KVPR_E_RANGE, "layer %d outside [0, %d)", layer, c->d.n_layers);
    if (int rc = check_weights(c, host, true)) return rc;
    KVPR_HIP(hipStreamSynchronize(c->wstream));
    const size_t h = c->d.hidden, f = c->d.ffn_dim;
    const BlobLayout L(h, f, c->llama);
    half* blob = c->hw[layer];
    auto put = [&](size_t at, const void* src, size_t n) {
        if (src) memcpy(blob + at, src, n * sizeof(half));
        else memset(blob + at, 0, n * sizeof(half));            // absent bias = 0
    };
    put(L.wq, host->wqkv, 3 * h * h);                           // wq and wkv are adjacent: one fused [3h, h] block
    put(L.bqkv, host->bqkv, 3 * h);
    put(L.wo, host->wo, h * h);
    put(L.bo, host->bo, h);
    put(L.ln1_g, host->ln1_g, h); put(L.ln1_b, host->ln1_b, h);
    put(L.ln2_g, host->ln2_g, h); put(L.ln2_b, host->ln2_b, h);
    put(L.w1, host->w1, (c->llama ? 2 : 1) * f * h); put(L.b1, host->b1, f);
    put(L.w2, host->w2, h * f); put(L.b2, host->b2, h);
    c->w_written[layer] = true;
    return KVPR_OK;
}

extern "C" int kvpr_decode_step_columns(kvpr_ctx* c, int seq, const void* x_in_dev, void* x_out_dev,
                                        const int32_t* splits_in, int32_t* splits_out, kvpr_layer_timing* per_slot) {
    if (!c) return fail(KVPR_E_INVAL, "ctx is null");
    if (c->nb <= 0) return fail(KVPR_E_STATE, "context was not created with kvpr_create_offload");
    if (seq < 0 || seq + 1 > c->d.max_seq)
        return fail(KVPR_E_RANGE, "seq %d: need 0 <= seq and seq + 1 <= max_seq = %d", seq, c->d.max_seq);
    if (!x_in_dev || !x_out_dev) return fail(KVPR_E_INVAL, "x_in_dev / x_out_dev is null");
    const int L = c->d.n_layers, nb = c->nb, b = c->d.batch, h = c->d.hidden, f = c->d.ffn_dim;
    const int S = L * nb;
    std::vector<int32_t> ls(S);
    for (int j = 0; j < L; ++j)
        if (!c->w_written[j]) return fail(KVPR_E_STATE, "layer %d: weights were never written to the host store", j);
    for (int i = 0; i < S; ++i) {
        if (int rc = resolve_split(c, seq, splits_in ? splits_in[i] : -1, &ls[i])) return rc;
        if (int rc = check_rows(c, i, seq, ls[i])) return rc;
    }
    if (per_slot)
        if (int rc = ensure_timing_events(c, S)) return rc;
    if (int rc = step_begin(c)) return rc;
    const BlobLayout BL(h, f, c->llama);
    const size_t bh = (size_t)b * h;
    const size_t kv_part = (BL.wo - BL.wkv) * sizeof(half);       // [Wk;Wv] rows, the q|k|v bias, the first norm's parameters
    // weights of layer j into device blob j % 2: the part the recomputation needs first (fine-grained MHA
    // pipeline, Sec. 3.3), then Wq and everything else
    auto load_weights = [&](int j) -> int {
        const int wb = j & 1;
        if (c->wfree_recorded[wb]) KVPR_HIP(hipStreamWaitEvent(c->wstream, c->ev_wfree[wb], 0));
        KVPR_HIP(hipMemcpyAsync(c->dw[wb] + BL.wkv, c->hw[j] + BL.wkv, kv_part, hipMemcpyHostToDevice, c->wstream));
        KVPR_HIP(hipEventRecord(c->ev_wkv[wb], c->wstream));
        KVPR_HIP(hipMemcpyAsync(c->dw[wb] + BL.wq, c->hw[j] + BL.wq, (BL.wkv - BL.wq) * sizeof(half), hipMemcpyHostToDevice, c->wstream));
        KVPR_HIP(hipMemcpyAsync(c->dw[wb] + BL.wo, c->hw[j] + BL.wo, (BL.total - BL.wo) * sizeof(half), hipMemcpyHostToDevice, c->wstream));
        KVPR_HIP(hipEventRecord(c->ev_wall[wb], c->wstream));
        if (per_slot) {                                           // timing: when the whole layer had landed
            LayerEvents& le = c->tev[(size_t)j * nb];
            KVPR_HIP(hipEventRecord(le.at[LayerEvents::w_all], c->wstream));
            le.has_w_all = true;
        }
        return KVPR_OK;
    };
    // load_activation of slot t (layer t / nb >= 1, batch t % nb): host row -> device staging, on the store stream, behind
    // the store that wrote the row one layer earlier
    int next_hidden_load = nb;
    auto hidden_load = [&](int t) -> int {
        const int par = t & 1, k = t % nb;
        if (c->hin_free_rec[par]) KVPR_HIP(hipStreamWaitEvent(c->store, c->ev_hin_free[par], 0));
        if (int rc = kvpr::launch_copy_bytes(c->hhid + (size_t)k * bh, c->hin[par], bh * sizeof(half), c->store)) return rc;
        KVPR_HIP(hipEventRecord(c->ev_hin_loaded[par], c->store));
        return KVPR_OK;
    };
    if (int rc = load_weights(0)) return rc;
    for (int j = 0; j < L; ++j) {
        const int wb = j & 1;
        if (j + 1 < L)
            if (int rc = load_weights(j + 1)) return rc;          // next layer's weights travel while this layer's batches run
        const kvpr_layer_weights w = blob_weights(c->dw[wb], BL);
        const WeightFence wf{c->ev_wkv[wb], c->ev_wall[wb]};
        for (int k = 0; k < nb; ++k) {
            const int slot = j * nb + k, par = slot & 1;
            const half* hid_in = (j == 0) ? (const half*)x_in_dev + (size_t)k * bh : c->hid_all + (size_t)k * bh;
            half* hid_out = (j == L - 1) ? (half*)x_out_dev + (size_t)k * bh : c->hid_all + (size_t)k * bh;
            if (c->hid_offload) {
                // this slot's input, unless the previous slot already asked for it; then the next slot's, ahead of this
                // slot's own stores in the stream (load_activation(k+1) before compute(k) before store_activation(k-1)
                // in Algorithm 1): possible once the store that wrote it, one layer back, is already in the stream
                while (next_hidden_load <= slot)
                    if (int rc = hidden_load(next_hidden_load++)) return rc;
                if (nb >= 2 && next_hidden_load == slot + 1 && slot + 1 < S)
                    if (int rc = hidden_load(next_hidden_load++)) return rc;
                if (j > 0) {
                    KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_hin_loaded[par], 0));
                    hid_in = c->hin[par];
                }
                if (j < L - 1) {
                    if (c->hout_free_rec[par]) KVPR_HIP(hipStreamWaitEvent(c->compute, c->ev_hout_free[par], 0));
                    hid_out = c->hout[par];
                }
            }
            // the norm's parameters arrive with [Wk;Wv]: neither the norm nor the recomputation that follows it
            // waits for Wq, Wo and the FFN matrices, which may still be on the link (Sec. 3.3 fine-grained MHA pipeline)
            KVPR_HIP(hipStreamWaitEvent(c->compute, c->weight_pipeline ? c->ev_wkv[wb] : c->ev_wall[wb], 0));
            if (int rc = pre_attention_norm(c, &w, hid_in)) return rc;
            if (int rc = enqueue_layer(c, slot, seq, ls[slot], &w, c->xn, c->attn_out, slot % c->nbuf,
                                       per_slot ? &c->tev[slot] : nullptr, false, &wf))
                return rc;
            if (int rc = residual_and_ffn(c, &w, hid_in, hid_out)) return rc;
            if (c->hid_offload) {
                if (j > 0) {
                    KVPR_HIP(hipEventRecord(c->ev_hin_free[par], c->compute));
                    c->hin_free_rec[par] = true;
                }
                if (j < L - 1) {                                  // store_activation: this batch's output to its host row
                    KVPR_HIP(hipEventRecord(c->ev_hout_ready[par], c->compute));
                    KVPR_HIP(hipStreamWaitEvent(c->store, c->ev_hout_ready[par], 0));
                    if (int rc = kvpr::launch_copy_bytes(c->hout[par], c->hhid + (size_t)k * bh, bh * sizeof(half), c->store)) return rc;
                    KVPR_HIP(hipEventRecord(c->ev_hout_free[par], c->store));
                    c->hout_free_rec[par] = true;
                }
            }
        }
        KVPR_HIP(hipEventRecord(c->ev_wfree[wb], c->compute));
        c->wfree_recorded[wb] = true;
    }
    if (int rc = step_end(c)) return rc;
    if (splits_out) std::copy(ls.begin(), ls.end(), splits_out);
    if (per_slot) {
        KVPR_HIP(hipStreamSynchronize(c->compute));
        KVPR_HIP(hipStreamSynchronize(c->copy));
        KVPR_HIP(hipStreamSynchronize(c->store));
        for (int i = 0; i < S; ++i)
            if (int rc = read_timing(c, &c->tev[i], seq, ls[i], &per_slot[i])) return rc;
    }
    return KVPR_OK;
}
