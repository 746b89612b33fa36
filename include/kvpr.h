/*
 * kvpr.h - C ABI of libkvpr: KVPR's per-layer decode path on one AMD MI355X (gfx950).
 *
 * KVPR ("KV cache partial recomputation", Sec. 3) keeps every layer's KV cache and
 * attention-input activations in pinned host memory.  For a split point l the GPU
 * recomputes K/V of the first l positions from their activations (Eq. 7) while the
 * cache of the remaining positions streams host->device; both halves land in one
 * device buffer, the decode token's K/V row is appended (Eq. 5) and exact decode
 * attention (Eq. 2) runs over all s+1 positions.  A profiler measures the link and
 * GEMM rates, a scheduler picks l* by minimising the cost model (Eq. 10, Eq. 11).
 *
 * Conventions
 *   - Every function returns int: 0 = KVPR_OK, negative = error.  Nothing throws or
 *     aborts across this boundary.  kvpr_last_error() returns the text of the last
 *     error raised on the calling thread.  Out-parameters are written only on success.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host
 *     addresses.  The caller owns every pointer it passes in and the compute stream.
 *     The context owns the pinned host store, its copy/store streams, events, the
 *     device staging buffers for X / KV and the attention workspace; kvpr_destroy
 *     frees them.
 *   - Calls enqueue work and return without waiting for the GPU, except where a
 *     timing struct is requested or the text says "synchronises".
 *   - A context must be used from one host thread at a time.
 *   - The library also exports a few symbols whose names start with kvpr_debug_: hooks that tests and
 *     tuning sweeps use to force a kernel variant.  They are not part of this interface.  They set
 *     process-wide variables without any synchronisation: call them from one thread, while no other
 *     thread is inside the library.
 *   - dtype is IEEE float16 for all tensors; accumulation is float32.
 *
 * Layouts (token-major, row-major, innermost index contiguous)
 *   X   [seq, batch, hidden]        attention-input activations (the tensor that multiplies W)
 *   KV  [seq, batch, 2*hidden]      a row is [K(hidden) | V(hidden)]; head i = columns [i*d, (i+1)*d) of each half
 *   W*  [out_features, in_features] (in_features contiguous): y = x . W^T + b, i.e. the paper's  y = x . W  with W stored transposed
 *   wqkv [3*hidden, hidden] = rows of Wq^T, then Wk^T, then Wv^T;  bqkv [3*hidden]
 * With this layout X[0:l] is one contiguous [l*batch, hidden] GEMM operand, the GEMM
 * output is rows [0,l) of the device KV buffer, and KV[l:s] is one contiguous copy.
 */
#ifndef KVPR_H
#define KVPR_H

#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVPR_OK        0
#define KVPR_E_INVAL  -1   /* null pointer, bad enum, inconsistent description        */
#define KVPR_E_RANGE  -2   /* index / size outside the allowed range                  */
#define KVPR_E_NOMEM  -3   /* host or device allocation failed                        */
#define KVPR_E_HIP    -4   /* a HIP runtime call failed; text in kvpr_last_error()    */
#define KVPR_E_STATE  -5   /* call not valid in the current state (e.g. rows unwritten) */

#define KVPR_F16 1
/* Flags or-ed into kvpr_model_desc.dtype: keep the host store group-wise 4-bit compressed
 * (Sec. 4.4 "KV Cache Compression").  KV_INT4 compresses the cache rows, X_INT4 the stored
 * activations; KVPR_STORE_INT4 sets both.  All arithmetic stays float16 / float32: activation rows
 * are dequantised on the GPU after the copy, cache rows inside the attention kernel, and new rows
 * are quantised on the GPU before the store-back.
 * Compressing the cache alone makes a position's activations (2h bytes) larger than its cache
 * (9h/8 bytes), and Eq. 10 then never chooses to recompute; with both, the 1 : 2 ratio of Eq. 6
 * is kept (9h/16 against 9h/8 bytes per position and sequence). */
#define KVPR_KV_INT4    0x100
#define KVPR_X_INT4     0x200
#define KVPR_STORE_INT4 (KVPR_KV_INT4 | KVPR_X_INT4)

/* Layer family (kvpr_model_desc.arch).  OPT: biases, LayerNorm, two-matrix ReLU FFN (Eq. 4).
 * LLAMA (the paper's LLaMA-2 experiments): no biases needed, RMSNorm, gated FFN
 * down(silu(gate) * up), and rotary position embedding on q and k.  The cache holds K after the
 * rotation, so the partial recomputation (Eq. 7) rotates every recomputed K row with its own
 * position (row index / batch) and the decode token's q, k with position seq.  Pairing: element i
 * of a head with element i + head_dim/2, angle p * rope_base^(-2i/head_dim). */
#define KVPR_ARCH_OPT   0
#define KVPR_ARCH_LLAMA 1

/* Cost forms for the scheduler.  EQ10 is the paper's Eq. 10 (activations and cache
 * share one link, activations first).  ROW is Eq. 10 without its first term (the
 * paper's row-by-row case).  NS charges the activation copy to the compute arm only:
 * max(t_recomp + M_X/v_com, M_KV/v_com); it is not in the paper. */
#define KVPR_COST_EQ10 0
#define KVPR_COST_NS   1
#define KVPR_COST_ROW  2
/* Extension (not in the paper): steady state of the layer pipeline, where the next layer's
 * transfers overlap this layer's compute: max((M_X + M_KV)/v_com, t_recomp + layer_other_s). */
#define KVPR_COST_PIPE 3

/* debug flags for kvpr_set_debug */
#define KVPR_DEBUG_SYNC   1  /* synchronise every stream after every enqueue             */
#define KVPR_DEBUG_POISON 2  /* fill the device KV/X buffers with float16 NaN before each layer */

typedef struct kvpr_ctx kvpr_ctx;

/* User configuration (Sec. 3.1): model shape, batch and the longest sequence. */
typedef struct {
    int32_t n_layers;   /* >= 1                                                          */
    int32_t hidden;     /* h; multiple of 64                                             */
    int32_t n_heads;    /* hidden == n_heads * head_dim                                  */
    int32_t head_dim;   /* 64 or 128                                                     */
    int32_t ffn_dim;    /* 0 = attention block only (kvpr_decode_step then unavailable)  */
    int32_t batch;      /* b >= 1                                                        */
    int32_t max_seq;    /* rows per layer in the host store and device buffers; a decode at seq cached positions needs seq + 1 <= max_seq */
    int32_t dtype;      /* KVPR_F16, optionally | KVPR_KV_INT4 | KVPR_X_INT4             */
    int32_t arch;       /* KVPR_ARCH_OPT or KVPR_ARCH_LLAMA                              */
    float rope_base;    /* KVPR_ARCH_LLAMA: base of the rotary angles; 0 = 10000         */
} kvpr_model_desc;

/* Profiler output (Sec. 3.1 "profiler module"): the two constants of Eq. 9 / Eq. 10
 * plus figures that are only reported. */
typedef struct {
    double h2d_bytes_per_s;      /* v_com: pinned host->device rate at the full-KV copy size */
    double gemm_flops_per_s;     /* v_gpu: recompute GEMM rate at M = batch*seq, measured while a cache-sized
                                    host-to-device copy is in flight (the condition of Eq. 10's max term) */
    double h2d_latency_s;        /* optional fixed cost per non-empty copy (0 = paper's linear model) */
    double gemm_latency_s;       /* optional fixed cost per non-empty GEMM (0 = paper's linear model) */
    double d2h_bytes_per_s;      /* reported only */
    double attn_bytes_per_s;     /* reported only: decode attention's KV read rate           */
    double h2d_peak_bytes_per_s; /* reported only: best rate over a 64 KiB .. 1 GiB sweep    */
    double gemm_alone_flops_per_s; /* reported only: the same GEMM with nothing else running             */
    int64_t gemm_round_flops;    /* extension of Eq. 9 (0 = the paper's divisible work): the recompute GEMM runs in
                                    rounds of one 256 x 256 tile per compute unit; N_KV is charged rounded up to a
                                    multiple of this many flops.  kvpr_profile fills it (n_CU * 2*256*256*hidden) */
    double layer_other_s;        /* the rest of one layer's GPU work at this batch / context (token projections,
                                    attention, output projection, FFN if the context has one): used by
                                    KVPR_COST_PIPE only, where it shares the GPU with the recomputation; 0 = ignore */
} kvpr_profile_t;

/* Device pointers to one layer's parameters.  FFN / LayerNorm members may be null when ffn_dim == 0.
 * KVPR_ARCH_LLAMA: biases and ln*_b are ignored and may be null; ln*_g are the RMSNorm gains;
 * w1 is [2*ffn, h] = the gate matrix's rows followed by the up matrix's rows; w2 [h, ffn] is the down matrix. */
typedef struct {
    const void *wqkv, *bqkv;   /* [3h, h], [3h]                       (Eq. 1)  */
    const void *wo, *bo;       /* [h, h], [h]                         (Eq. 3)  */
    const void *ln1_g, *ln1_b; /* [h] LayerNorm before attention               */
    const void *w1, *b1;       /* [ffn, h], [ffn]                     (Eq. 4)  */
    const void *w2, *b2;       /* [h, ffn], [h]                                */
    const void *ln2_g, *ln2_b; /* [h] LayerNorm before the FFN                 */
} kvpr_layer_weights;

/* Per-layer timing, milliseconds from HIP events (same categories as the paper's
 * runtime breakdown figure: load-activation, load-cache, compute, store). */
typedef struct {
    float ms_act_copy;   /* H2D of X[0:l]                                              */
    float ms_kv_copy;    /* H2D of KV[l:s]                                             */
    float ms_recompute;  /* recompute GEMM (Eq. 7)                                     */
    float ms_proj;       /* new-token q/k/v projection (Eq. 1, Eq. 5)                  */
    float ms_attn;       /* decode attention (Eq. 2): both phases when it ran in two           */
    float ms_out;        /* output projection (Eq. 3)                                  */
    float ms_store;      /* the new X / KV rows written into the pinned host store    */
    float ms_assemble;   /* first enqueue -> both KV halves resident: what Eq. 10 models */
    float ms_total;      /* first enqueue -> output projection and store-back done     */
    double t_bound_s;    /* cost-model prediction for the split used (0 if no profile) */
    int32_t split;       /* the split l actually used                                   */
    float ms_attn_early; /* the part of ms_attn that ran before the cache fence: attention over the recomputed
                            rows and the new row, issued while the cache copy is still in flight (always with
                            KVPR_KV_INT4, whose transferred rows are then read in packed form; with a float16
                            cache only in kvpr_layer_decode[_timed] at split >= 128); 0 when one launch did it all */
    float ms_recompute_start; /* first enqueue -> the recompute GEMM may begin (its fences have passed)           */
    float ms_weights_landed;  /* column schedule, first batch of a layer: first enqueue of this slot -> the layer's
                                 whole weight blob has landed (negative: it had landed before); valid only when
                                 weights_landed_valid != 0.  ms_recompute_start < ms_weights_landed shows the
                                 recomputation running while Wq / Wo / FFN weights are still on the link */
    int32_t weights_landed_valid;
} kvpr_layer_timing;

const char* kvpr_last_error(void);

/* Create a context for `desc`.  compute_stream is a hipStream_t (may be null = the
 * null stream) owned by the caller; all kernels are launched on it.  Allocates the
 * pinned host store: n_layers * max_seq * batch * 3*hidden * 2 bytes (9/32 of that for
 * an array kept 4-bit compressed), and device staging buffers for min(n_layers, 2)
 * layers (float16 X and KV, plus packed copies of the arrays kept compressed).
 * KVPR_E_NOMEM if that fails.  kvpr_destroy waits for the context's streams and
 * frees everything the context owns.
 * The context makes its own copy and store streams (and a weight stream in kvpr_create_offload).  The runtime
 * shares a few hardware queues among all streams of a process, and two streams on one queue run in order, so
 * creation launches a few short kernels (about 3 ms in all) on compute_stream and on its own streams and replaces
 * any of its streams that turns out to sit behind one it has to overlap with; compute_stream must be idle or
 * short of work at that time for the check to mean anything, and is synchronised by it (so a context cannot be
 * created while compute_stream is being captured into a graph). */
int kvpr_create(const kvpr_model_desc* desc, void* compute_stream, kvpr_ctx** out);
int kvpr_destroy(kvpr_ctx* ctx);
/* Debug modes (KVPR_DEBUG_*), results are unchanged by them. */
int kvpr_set_debug(kvpr_ctx* ctx, int flags);
/* Gives the context the constants of Eq. 10 (from kvpr_profile or the caller), the cost form and the
 * granularity of l that split = -1 plans with.  Validates the profile like kvpr_plan_split. */
int kvpr_set_profile(kvpr_ctx* ctx, const kvpr_profile_t* prof, int cost_model, int granularity);

/* Host store (Sec. 3.3 "pinned memory").  Copies rows [t0, t1) of `layer` from
 * ordinary host memory; x_host is [t1-t0, batch, hidden], kv_host [t1-t0, batch, 2*hidden],
 * both float16; either may be null to leave that array untouched.  An array that the context
 * keeps compressed is quantised on the GPU on the way (the call then synchronises the device). */
int kvpr_store_write(kvpr_ctx* ctx, int layer, int t0, int t1, const void* x_host, const void* kv_host);
/* Borrowed pointers to a layer's pinned arrays X[max_seq,batch,hidden] and KV[max_seq,batch,2*hidden]
 * (float16), or, for an array kept compressed, its packed form [max_seq, batch, kvpr_int4_row_bytes(cols)]
 * with cols = hidden for X and 2*hidden for KV. */
int kvpr_store_ptrs(kvpr_ctx* ctx, int layer, void** x_host, void** kv_host);
/* Stand-in for prefill: computes KV[0:seq] of `layer` from the stored X[0:seq] on the
 * GPU (Eq. 1 for K and V) and writes it into the host store.  Synchronises. */
int kvpr_store_prefill_kv(kvpr_ctx* ctx, int layer, int seq, const kvpr_layer_weights* w);

/* Profiler (Sec. 3.1): measures on this machine, for this ctx's hidden size, the pinned
 * H2D rate at the size of a full KV copy of [seq, batch] and the recompute GEMM rate at
 * M = batch*seq (median of 5 after warm-up; the GEMM once alone and once under a concurrent copy).  Synchronises.  batch*seq must not exceed
 * the context's batch*max_seq. */
int kvpr_profile(kvpr_ctx* ctx, int batch, int seq, kvpr_profile_t* out);
/* Refinement of v_gpu (Sec. 3.1, Eq. 9) for a context that decodes one layer at a time (kvpr_layer_decode) with
 * the GPU idle between steps: rehearses the copy / GEMM sequence of one step at the split that *prof plans with
 * Eq. 10 (activation-sized pinned copy first, under the clock keep-alive if kvpr_set_keep_warm was given; then the
 * recompute GEMM over batch*l rows of random operands while the rest of a cache-sized copy lands), four times with
 * a full synchronisation in between, and replaces prof->gemm_flops_per_s by (flops as the cost model charges them)
 * / (median GEMM time of the last three); re-plans once and repeats if the split moved.  No other field changes.
 * A GPU that works in such bursts clocks the GEMM differently from the back-to-back launches kvpr_profile times.
 * prof must hold positive h2d_bytes_per_s and gemm_flops_per_s.  Reads the first layer's host activations and cache as
 * copy sources (contents irrelevant), overwrites device staging buffers, allocates and frees its own scratch, synchronises.
 * KVPR_E_RANGE if batch or seq exceed the context's. */
int kvpr_profile_step(kvpr_ctx* ctx, int batch, int seq, kvpr_profile_t* prof);

/* Scheduler (Sec. 3.2, Eq. 6-11).  Pure host arithmetic, no context.  Evaluates the
 * cost for every l in {0, g, 2g, ...} U {seq} (g = granularity >= 1) in ascending order
 * and returns the first strict minimum.  Byte / flop counts are formed in int64 and
 * converted to double once; each rate enters through one double division. */
int kvpr_plan_split(const kvpr_profile_t* prof, int cost_model, int batch, int seq, int hidden,
                    int elem_bytes, int granularity, int32_t* l_star, double* t_pred);
/* The cost model itself at one split (Eq. 10 or a variant). */
int kvpr_cost(const kvpr_profile_t* prof, int cost_model, int split, int batch, int seq, int hidden,
              int elem_bytes, double* t_pred);

/* Extension (not in the paper): the activation copy X[0:l] is cut into `chunks` equal parts
 * (1..32; 1 = the paper's schedule) and the recomputation of part j starts as soon as part j has
 * landed, while the later parts and then the cache are still on the link.  Results are unchanged.
 * kvpr_cost_chunked / kvpr_plan_split_chunked are Eq. 10 / Eq. 11 for that schedule: with
 * t_act, t_kv, t_rc as in Eq. 10, part j's GEMM starts at max(j*t_act/chunks, end of part j-1)
 * and takes t_rc/chunks; t = max(end of the last GEMM, t_act + t_kv).  chunks = 1 gives Eq. 10. */
int kvpr_set_chunks(kvpr_ctx* ctx, int chunks);
int kvpr_cost_chunked(const kvpr_profile_t* prof, int chunks, int split, int batch, int seq, int hidden,
                      int elem_bytes, double* t_pred);
int kvpr_plan_split_chunked(const kvpr_profile_t* prof, int chunks, int batch, int seq, int hidden,
                            int elem_bytes, int granularity, int32_t* l_star, double* t_pred);

/* The same scheduler on per-position sizes (Eq. 6 and Eq. 8 are linear in the number of positions):
 * M_X = x_bytes_per_pos * l, M_KV = kv_bytes_per_pos * (seq - l), N_KV = flops_per_pos * l.  With
 * b*h*p, 2*b*h*p and 4*b*h*h these are kvpr_cost / kvpr_plan_split; a compressed store (Sec. 4.4)
 * passes its own byte rates.  chunks > 1 selects the chunked schedule above (KVPR_COST_EQ10 only). */
int kvpr_cost_linear(const kvpr_profile_t* prof, int cost_model, int chunks, int split, int seq,
                     int64_t x_bytes_per_pos, int64_t kv_bytes_per_pos, int64_t flops_per_pos, double* t_pred);
int kvpr_plan_split_linear(const kvpr_profile_t* prof, int cost_model, int chunks, int seq,
                           int64_t x_bytes_per_pos, int64_t kv_bytes_per_pos, int64_t flops_per_pos,
                           int granularity, int32_t* l_star, double* t_pred);

/* Extension (the paper profiles once, at start-up, and names run-time adaptation as future work in its
 * Limitations section): keep the two constants of Eq. 10 current while decoding.
 * kvpr_adapt_update: host arithmetic.  v' = (1 - alpha) v + alpha (work / seconds) for the link rate
 * (link_bytes over link_seconds) and the GEMM rate (gemm_flops over gemm_seconds); a sample with no work or
 * no time is skipped.
 * kvpr_set_adaptive: alpha in (0, 1] makes every layer that is decoded without a timing request record HIP
 * events around its copies and its recompute GEMM (no waiting); the next planned split (split = -1) first
 * folds the samples of all finished layers into the context's profile with kvpr_adapt_update.  alpha = 0
 * (the default) turns it off.  With a chunked activation copy only the link rate is adapted.
 * kvpr_get_profile: the context's current profile, after folding in finished samples. */
int kvpr_adapt_update(kvpr_profile_t* prof, double alpha, int64_t link_bytes, double link_seconds,
                      int64_t gemm_flops, double gemm_seconds);
int kvpr_set_adaptive(kvpr_ctx* ctx, double alpha);
int kvpr_get_profile(kvpr_ctx* ctx, kvpr_profile_t* out);

/* Extension (not in the paper): clock keep-alive for the single-layer latency path.  In the paper's schedule the GPU
 * has nothing to do while X[0:l] is on the link (the first term of Eq. 10), and a GPU that has idled for a few
 * milliseconds starts the recompute GEMM with its clocks down (measured: 10-15 % slower at hidden >= 5120).  With
 * fraction in (0, 0.95], kvpr_layer_decode[_timed] on a context that has a profile puts a register-only MFMA loop
 * on the compute stream, between the token projection and the wait for the activations, that runs for
 * fraction * (bytes of the first activation chunk) / h2d_bytes_per_s of wall time (its waves watch the constant-rate
 * wall clock; an iteration count bounds it as well).  It reads 192 bytes of wqkv per lane and writes nothing; results
 * are unchanged.  If the link turns out faster than the profile says, the GEMM starts late by at most the
 * difference.  0 (the default) turns it off.  kvpr_decode_step and the column schedule never use it: there the GPU is
 * busy with the neighbouring layers. */
int kvpr_set_keep_warm(kvpr_ctx* ctx, double fraction);

/* One decode step of one attention layer (Sec. 3.2 row-by-row pipeline with partial
 * recomputation; Eq. 1, 2, 3, 5, 7).  `seq` = cached positions s already in the host
 * store; split in [0, seq], or -1 to use the plan from kvpr_set_profile.
 * x_new_dev [batch, hidden] is the decode token's attention input; out_dev [batch, hidden]
 * receives z . Wo^T + bo.  Side effects: rows `seq` of the layer's host X and KV are
 * written (store-back).  If timing is non-null the call synchronises and fills it.
 * Asynchronous otherwise.  Measured on MI355X: decodes fed to the streams one at a time while earlier ones are still
 * running run 3-6 % slower per step than decodes enqueued several at a time (or by kvpr_decode_step, which enqueues a
 * whole token's layers in one go). */
int kvpr_layer_decode(kvpr_ctx* ctx, int layer, int seq, int split, const kvpr_layer_weights* w,
                      const void* x_new_dev, void* out_dev, kvpr_layer_timing* timing);

/* As kvpr_layer_decode, but records HIP events around every category into timing slot
 * `slot` (0 .. 4095) and does not wait; kvpr_timing_read waits for that slot's events and
 * converts them.  Lets a timed loop stay asynchronous. */
int kvpr_layer_decode_timed(kvpr_ctx* ctx, int layer, int seq, int split, const kvpr_layer_weights* w,
                            const void* x_new_dev, void* out_dev, int slot);
int kvpr_timing_read(kvpr_ctx* ctx, int slot, kvpr_layer_timing* timing);

/* One decode step through all n_layers OPT-style decoder layers (pre-LayerNorm,
 * attention block, residual, LayerNorm, ReLU FFN (Eq. 4), residual), with the next
 * layer's transfers prefetched into the other device buffer while this layer computes
 * (Sec. 4 "Implementation": double buffering across decoder layers).
 * x_in_dev / x_out_dev [batch, hidden] hidden states; splits_in [n_layers] or null (= plan).
 * Asynchronous, with bounded run-ahead: at most two steps of a context are in flight; a further call (this one or
 * kvpr_decode_step_columns) first blocks the calling thread until the step before the previous one has finished on
 * the GPU.  Deeper queues gain nothing and made steps slower (the runtime stalls the caller by itself, later and
 * for longer). */
int kvpr_decode_step(kvpr_ctx* ctx, int seq, const kvpr_layer_weights* layers, const void* x_in_dev,
                     void* x_out_dev, const int32_t* splits_in, int32_t* splits_out, kvpr_layer_timing* per_layer);

/* ---- column-by-column schedule with offloaded weights (Sec. 3.2 "Column-by-column schedule",
 * Sec. 3.3, Algorithm 1): the throughput-oriented mode.  The weights live in pinned host memory too;
 * a layer's weights are loaded once and used for n_gpu_batches batches before the next layer.
 *
 * kvpr_create_offload: as kvpr_create (ffn_dim > 0 required) plus a pinned weight store for n_layers
 * layers, two device weight buffers (the next layer's weights load while this layer's batches run)
 * and a weight stream.  The X / KV store has n_layers * n_gpu_batches slots; the store functions and
 * the splits arrays address slot = layer * n_gpu_batches + batch_index in place of `layer`.
 * kvpr_weights_write: copies one layer's parameters from ordinary host memory (pointers in `host`,
 * same shapes as the device struct; null biases mean 0) into the pinned weight store.
 * kvpr_decode_step_columns: one decode token for all batches.  x_in_dev / x_out_dev are
 * [n_gpu_batches, batch, hidden] float16 hidden states.  Per layer the part of the weights the
 * recomputation needs ([Wk;Wv], bias) is loaded first and the recomputation runs before the
 * projections that need Wq ("fine-grained MHA pipeline").  kvpr_decode_step is not available on
 * such a context. */
int kvpr_create_offload(const kvpr_model_desc* desc, int n_gpu_batches, void* compute_stream, kvpr_ctx** out);

/* Column schedule only, optional (off by default): keep the hidden states that pass from layer to layer in pinned host
 * memory, as Algorithm 1 does with load_activation / store_activation.  After a batch's layer its output goes to the
 * batch's host row (store stream); the next layer fetches it into one of two device staging buffers, one batch ahead
 * of the computation when n_gpu_batches >= 2.  The device then holds the hidden states of four batches at most instead
 * of n_gpu_batches.  Results are unchanged bit for bit.  x_in_dev / x_out_dev of kvpr_decode_step_columns stay device
 * arrays.  KVPR_E_STATE on a context without offloaded weights. */
int kvpr_set_hidden_offload(kvpr_ctx* ctx, int on);

/* Column schedule only.  fine_grained != 0 (the default) is the paper's fine-grained MHA pipeline (Sec. 3.3 "Hiding KV
 * cache partial recomputation"): the recomputation of a layer's batches is released by [Wk;Wv] and runs while Wq, Wo
 * and the FFN matrices are still on the link.  0 makes every batch wait for the layer's whole weight blob first: the
 * "without hiding" arm of the paper's ablation (Table 2), for measurements.  Results are the same either way. */
int kvpr_set_weight_pipeline(kvpr_ctx* ctx, int fine_grained);
int kvpr_weights_write(kvpr_ctx* ctx, int layer, const kvpr_layer_weights* host);
int kvpr_decode_step_columns(kvpr_ctx* ctx, int seq, const void* x_in_dev, void* x_out_dev,
                             const int32_t* splits_in, int32_t* splits_out, kvpr_layer_timing* per_slot);

/* Greedy sampling step of the row-by-row schedule: logits = hidden . W_lm^T in float32
 * (logits_dev: scratch [batch, vocab] float32), tokens_dev[n] = argmax over the vocabulary (lowest
 * index on ties), and, if emb_dev is non-null, x_next_dev[n] = emb_dev[tokens_dev[n]] (float16
 * [vocab, hidden] table).  hidden_dev float16 [batch, hidden], w_lm_dev float16 [vocab, hidden]. */
int kvpr_greedy_next(const void* hidden_dev, const void* w_lm_dev, const void* emb_dev, int batch, int hidden,
                     int vocab, void* logits_dev, int32_t* tokens_dev, void* x_next_dev, void* stream);

/* ---- individual kernels, exposed for parity tests and roofline measurement ---- */

/* C[M, N] (row stride ldc halfs) = A[M, K] . W[N, K]^T + bias[N]   (Eq. 7 when W = [Wk^T ; Wv^T]).
 * float16 in, float32 accumulate on MFMA, float16 out.  K % 64 == 0, N % 8 == 0, ldc >= N, ldc % 8 == 0
 * (rows are written in 16-byte pieces; c_dev 16-byte aligned).
 * bias may be null.  M == 0 is a no-op.  stream is a hipStream_t. */
int kvpr_recompute_gemm(const void* a_dev, const void* w_dev, const void* bias_dev, void* c_dev,
                        int64_t M, int N, int K, int64_t ldc, void* stream);

/* Exact decode attention (Eq. 2): q_dev float32 [batch, hidden] (unscaled), kv_dev float16
 * [S, batch, 2*hidden], z_dev float16 [batch, hidden].  ws_dev is scratch of at least
 * kvpr_attention_workspace_bytes(batch, hidden, n_heads, S) bytes.  S >= 1. */
int kvpr_decode_attention(const void* q_dev, const void* kv_dev, void* z_dev, void* ws_dev,
                          int S, int batch, int hidden, int n_heads, void* stream);
size_t kvpr_attention_workspace_bytes(int batch, int hidden, int n_heads, int S);
/* kvpr_decode_attention for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as kvpr_decode_attention, but the partial results of a launch that splits the positions
 * across workgroups go to a static device array of KVPR_ATTENTION_STATIC_SCRATCH_BYTES that every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing.  A shape whose
 * partials (splits * batch * hidden * 5 bytes, splits as kvpr_decode_attention chooses them; 0 when one
 * workgroup per sequence and column group suffices) exceed the array is refused with KVPR_E_RANGE; the
 * split choice keeps them below 1.3 MiB for every shape, so only a forced split count gets there.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two threads)
 * race; calls on one stream are ordered.  Nothing in the array needs clearing between calls: every slot
 * that a launch reads was written by that launch. */
#define KVPR_ATTENTION_STATIC_SCRATCH_BYTES (2u << 20)
int kvpr_decode_attention_static(const void* q_dev, const void* kv_dev, void* z_dev,
                                 int S, int batch, int hidden, int n_heads, void* stream);
/* The same attention (Eq. 2) over a cache whose rows [split, S-1) are still in the packed 4-bit form of the
 * host store (Sec. 4.4): rows [0, split) and row S-1 are read from kv16_dev (float16 [S, batch, 2*hidden]),
 * rows [split, S-1) from kvq_dev ([S, batch, kvpr_int4_row_bytes(2*hidden)], indexed by position) and
 * used as the codec's code * scale + minimum without kvpr_dequant_int4's final rounding to float16 (at most 2^-11
 * relative per element; the affine map is applied to the sums, not per element).  Same workspace size as above.
 * split in [0, S-1].  With kvq_dev null every row comes from kv16_dev: the same two launches (rows [0, split)
 * and S-1, then rows [split, S-1)) and one combine, which is how kvpr_layer_decode overlaps the attention
 * over the recomputed rows with the tail of the cache copy. */
int kvpr_decode_attention_mixed(const void* q_dev, const void* kv16_dev, const void* kvq_dev, void* z_dev, void* ws_dev,
                                int S, int split, int batch, int hidden, int n_heads, void* stream);

/* y[M, N] = x[M, K] . W[N, K]^T + bias for small M (the decode token's projections).
 * out_f32_cols: the first out_f32_cols columns are written as float32 to y32_dev [M, out_f32_cols]
 * (used for q), the remaining N - out_f32_cols columns as float16 to y16_dev with row stride ld16. */
int kvpr_token_gemm(const void* x_dev, const void* w_dev, const void* bias_dev, void* y32_dev, void* y16_dev,
                    int M, int N, int K, int out_f32_cols, int64_t ld16, void* stream);

/* The same operation (Eq. 1 / 3 / 4 / 5 for the decode token) with a device workspace.  When the output has too few
 * features to give every compute unit a block of them (the output projection and the FFN's second matrix: N = hidden),
 * the sum over K is cut into up to 8 slices computed by different workgroups; the float32 partial tiles meet in the
 * workspace and are added in slice order, so a given (shape, workspace size) always rounds the same way.
 * ws_dev: 16-byte aligned device memory of ws_bytes, owned by the caller; kvpr_token_gemm_workspace_bytes(M, N) is
 * enough for 8 slices (less workspace: fewer slices; null or at most 4096 bytes: exactly kvpr_token_gemm).  Its first
 * 4096 bytes (arrival counters) must be zero before the first call and are zero again when a call has finished;
 * calls that share a workspace must run one after the other (same stream, or ordered by events).
 * kvpr_token_gemm_workspace_bytes returns 0 for M outside 1..64 or N < 1. */
size_t kvpr_token_gemm_workspace_bytes(int M, int N);
int kvpr_token_gemm_ws(const void* x_dev, const void* w_dev, const void* bias_dev, void* y32_dev, void* y16_dev,
                       int M, int N, int K, int out_f32_cols, int64_t ld16, void* ws_dev, size_t ws_bytes, void* stream);

/* ---- rotary models (KVPR_ARCH_LLAMA), exposed for parity tests ----
 * kvpr_rope_table: host arithmetic only.  out_host [n_pos, head_dim/2, 2] float32 = (cos, sin) of
 * p * base^(-2i/head_dim), evaluated in double.  head_dim 64 or 128.
 * kvpr_recompute_gemm_rope: kvpr_recompute_gemm with columns [0, rope_cols) (the K half, a multiple of
 * 128) rotated in float32 before the float16 conversion; row r has position pos0 + r / batch, which
 * must stay below n_pos (the table's rows).  table_dev is the device copy of kvpr_rope_table's output.
 * kvpr_rope_token: qk32_dev float32 [batch, 2*hidden] = [q | k] of the decode token before rotation;
 * writes the rotated q as float32 [batch, hidden] and the rotated k as float16 with row stride ldk. */
int kvpr_rope_table(float* out_host, int n_pos, int head_dim, double base);
int kvpr_recompute_gemm_rope(const void* a_dev, const void* w_dev, const void* bias_dev, void* c_dev, int64_t M, int N, int K,
                             int64_t ldc, const void* table_dev, int n_pos, int rope_cols, int head_dim, int batch,
                             int pos0, void* stream);
int kvpr_rope_token(const void* qk32_dev, const void* table_dev, int n_pos, int pos, int batch, int hidden, int head_dim,
                    void* q32_dev, void* k16_dev, int64_t ldk, void* stream);

/* Group-wise 4-bit codec of the compressed store (Sec. 4.4; the paper fixes no format, this is the
 * library's): rows of `cols` float16 columns (cols % 64 == 0) in groups of 64 columns; per group
 * mn = min, scale = float16((max - mn) / 15), code = clamp(rint((x - mn) / scale), 0, 15) in float32
 * (all codes 0 when scale == 0), value = float16(code * scale + mn).  A packed row is cols/2 code bytes
 * (element 2k in the low nibble of byte k) followed by cols/64 float16 pairs (scale, mn):
 * kvpr_int4_row_bytes(cols) = 9*cols/16 bytes.  src_dev / dst_dev hold `rows` contiguous rows. */
size_t kvpr_int4_row_bytes(int cols);
int kvpr_quant_int4(const void* src_dev, void* dst_dev, int64_t rows, int cols, void* stream);
int kvpr_dequant_int4(const void* src_dev, void* dst_dev, int64_t rows, int cols, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVPR_H */
