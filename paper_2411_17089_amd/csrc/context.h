// Runtime state shared by the translation units of libkvpr (not part of the ABI): the context, its
// per-layer timing events, and the few helpers more than one file needs.
#pragma once
#include "kvpr_internal.h"

#include <vector>

namespace kvpr {

typedef _Float16 half;

// events bracketing each category of one layer (timing enabled)
struct LayerEvents {
    // e0..e1: early attention phase; w_all: the layer's whole weight blob has landed (offloaded weights only)
    enum Id { start, c0, c_x, c_kv, p0, p1, r0, r1, e0, e1, a0, a1, o1, s0, s1, end, w_all, count };
    hipEvent_t at[count]{};
    int seq = -1, split = -1;            // what the slot last recorded
    bool has_w_all = false;              // w_all was recorded for the step being timed
};

}  // namespace kvpr

using kvpr::half;
using kvpr::LayerEvents;

struct kvpr_ctx {
    kvpr_model_desc d{};
    hipStream_t compute = nullptr, copy = nullptr, store = nullptr;
    std::vector<char*> hx, hkv;          // pinned, per layer: float16 rows, or packed 4-bit rows (Sec. 4.4)
    bool qx = false, qkv = false;        // which of the two arrays the store keeps 4-bit compressed
    char* dxq[2] = {nullptr, nullptr};   // device staging for packed rows (only when compressed)
    char* dkvq[2] = {nullptr, nullptr};
    std::vector<int> x_rows, kv_rows;    // contiguous prefix of rows known to hold data
    std::vector<hipEvent_t> ev_slot_store;   // per slot: "the last store-back into this slot's host rows is done"
    std::vector<bool> slot_store_recorded;
    int nbuf = 0;
    half* dx[2] = {nullptr, nullptr};
    half* dkv[2] = {nullptr, nullptr};
    float* q32 = nullptr;
    half* z16 = nullptr;
    // rotary models (KVPR_ARCH_LLAMA): q|k of the decode token before rotation, and the (cos, sin) table
    bool llama = false;
    float* qk32 = nullptr;
    float2* rope_tab = nullptr;          // [max_seq][head_dim / 2]
    void* attn_ws = nullptr;
    void* tok_ws = nullptr;              // token GEMM K-slice workspace (tickets, then partial tiles)
    size_t tok_ws_bytes = 0;
    // hidden-state scratch of the full decoder layer
    half *hid = nullptr, *xn = nullptr, *attn_out = nullptr, *ffn1 = nullptr, *ffn2 = nullptr;
    // fences (timing disabled)
    hipEvent_t ev_x[2]{}, ev_kv[2]{}, ev_free[2]{}, ev_proj = nullptr, ev_store = nullptr, ev_begin = nullptr;
    static constexpr int kMaxChunks = 32;
    hipEvent_t ev_chunk[2][kMaxChunks]{};   // per device buffer: "activation chunk j has landed"
    int chunks = 1;                          // 1 = the paper's schedule: all of X[0:l], then one GEMM
    // column-by-column schedule with offloaded weights (n_gpu_batches > 0)
    int nb = 0;                              // GPU batches per layer; the store then has n_layers * nb slots
    hipStream_t wstream = nullptr;           // weight loads
    std::vector<half*> hw;                   // pinned weight blob per layer
    half* dw[2] = {nullptr, nullptr};        // device weight blobs (ping-pong across layers)
    half* hid_all = nullptr;                 // [nb, batch, hidden] hidden states of all GPU batches
    // optional (kvpr_set_hidden_offload): the hidden states between layers live in pinned host memory, as Algorithm 1's
    // load_activation / store_activation have it; the device then holds two input and two output batches at a time
    bool weight_pipeline = true;             // recompute released by [Wk;Wv] alone (Sec. 3.3); false: by the whole layer's weights
    bool hid_offload = false;
    half* hhid = nullptr;                    // pinned [nb, batch, hidden]
    half* hin[2] = {nullptr, nullptr};       // device: input of this slot and of the next one
    half* hout[2] = {nullptr, nullptr};      // device: output of this slot and of the previous one
    hipEvent_t ev_hin_loaded[2]{}, ev_hin_free[2]{}, ev_hout_ready[2]{}, ev_hout_free[2]{};
    bool hin_free_rec[2] = {false, false}, hout_free_rec[2] = {false, false};
    hipEvent_t ev_wkv[2]{}, ev_wall[2]{}, ev_wfree[2]{};
    bool wfree_recorded[2] = {false, false};
    std::vector<bool> w_written;
    int slots() const { return nb > 0 ? d.n_layers * nb : d.n_layers; }
    bool free_recorded[2] = {false, false};
    hipEvent_t ev_buf_store[2]{};        // per device buffer: "the last store-back that read a row of this buffer is done"
    bool buf_store_recorded[2] = {false, false};
    // whole-stack steps in flight: a step's end is recorded on the compute stream, and a new step first waits (on the
    // host) for the end of the step before the previous one
    hipEvent_t ev_step[2]{};
    uint64_t steps_enqueued = 0;
    std::vector<LayerEvents> tev;        // lazily created timing events, one set per layer slot
    kvpr_profile_t prof{};
    bool have_prof = false;
    // run-time adaptation of prof (alpha > 0): a small ring of event sets recorded on untimed layers
    double adapt_alpha = 0.0;
    static constexpr int kProbes = 8;
    LayerEvents probe[kProbes]{};
    bool probe_made = false, probe_pending[kProbes] = {};
    int probe_next = 0;
    // clock keep-alive: fraction of the predicted activation-copy time that the compute stream spends in a register-only
    // MFMA loop before it waits for the activations (0 = off)
    double keep_warm = 0.0;
    double wall_clock_hz = 0.0;
    int cost_model = KVPR_COST_EQ10, granularity = 1;
    int debug = 0;

    size_t x_row_halfs() const { return (size_t)d.batch * d.hidden; }
    size_t kv_row_halfs() const { return (size_t)d.batch * 2 * d.hidden; }
    // bytes of one position (all sequences of the batch) as the host store holds it and as it crosses the link
    size_t x_store_bytes() const { return qx ? d.batch * kvpr::int4_row_bytes(d.hidden) : x_row_halfs() * sizeof(half); }
    size_t kv_store_bytes() const { return qkv ? d.batch * kvpr::int4_row_bytes(2 * d.hidden) : kv_row_halfs() * sizeof(half); }
    int64_t flops_per_pos() const { return 4 * (int64_t)d.batch * d.hidden * d.hidden; }   // Eq. 8
    int plan_chunks() const { return (chunks > 1 && cost_model == KVPR_COST_EQ10) ? chunks : 1; }
};

namespace kvpr {

// wqkv / wo always; FFN and norm parameters when a full decoder layer is about to run
int check_weights(const kvpr_ctx* c, const kvpr_layer_weights* w, bool need_ffn);

}  // namespace kvpr
