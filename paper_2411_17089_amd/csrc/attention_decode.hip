// Exact decode attention for gfx950 (Eq. 2): one query per sequence over S positions of a
// token-major float16 KV buffer  kv[S, batch, 2h]  (row = [K(h) | V(h)], head i = columns [i*d, (i+1)*d)).
//
// The kernel is bound by the single pass over KV in HBM (about 1 flop per byte), so everything is
// arranged around 16-byte lane loads of contiguous 1 KiB wave segments:
//   - a workgroup owns (sequence n, a group of 512 columns, a range of positions); lane L of every
//     wave owns columns [512*cg + 8L, +8), i.e. 8 consecutive halfs of one head, for both K and V;
//   - the waves of a workgroup take interleaved runs of UNROLL positions, so 2*UNROLL independent
//     1 KiB loads are in flight per wave (UNROLL = 8, 4 waves measured best); loads are non-temporal:
//     the cache is streamed exactly once, and bypassing the caches raised the measured read rate
//     from 5.4 to 6.2 TB/s;
//   - q.k is a lane-local 8-term dot product followed by an add-butterfly over the d/8 lanes of the
//     head with DPP row operations (no LDS, no ds_bpermute);
//   - softmax is the usual running (max, sum) recurrence in float32 with exp2 and q pre-scaled by
//     log2(e)/sqrt(d); the rescale is applied once per UNROLL positions;
//   - waves are merged through LDS; only when (column groups x batch) workgroups cannot fill the
//     chip are positions also split across workgroups ("splits"), merged through a float32
//     workspace and a small combine kernel.
//
// Mixed-source variant for a 4-bit host store (Sec. 4.4): attention_partial_ranged takes a range of
// positions (plus, optionally, one extra position) from either the float16 buffer or the packed staging
// buffer [position][batch][9h/8 bytes] and always leaves a partial (m, l, acc) in the workspace.  The
// runtime launches it over the recomputed rows [0, l) and the new row as soon as they exist, and over the
// packed rows [l, s) once they have landed (attention_partial_packed: 16 bytes of K codes and 16 of V codes per
// lane, dequantised in registers to float16(code * scale + mn) exactly as the standalone codec), so they are never
// expanded in HBM.  One combine kernel merges all partials, or, when both phases run one workgroup per sequence
// and column group, the second phase merges the first one's partial itself.
#include "kvpr_internal.h"
#include <math.h>
#include <mutex>

namespace kvpr {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int COLS_PER_GROUP = 64 * 8;   // columns one wave covers

template <int CTRL>
__device__ __forceinline__ float dpp_xchg_add(float v) {
    const int o = __builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(o);
}

// sum over the D/8 consecutive lanes that hold one head; every lane of the group gets the sum
template <int D>
__device__ __forceinline__ float head_sum(float v) {
    v = dpp_xchg_add<0xB1>(v);     // quad_perm [1,0,3,2]
    v = dpp_xchg_add<0x4E>(v);     // quad_perm [2,3,0,1]
    v = dpp_xchg_add<0x141>(v);    // row_half_mirror: 8 lanes
    if (D == 128) v = dpp_xchg_add<0x140>(v);   // row_mirror: 16 lanes
    return v;
}

template <int D, int UNROLL, int ATT_WAVES>
__global__ __launch_bounds__(ATT_WAVES * 64) void attention_partial(
    const float* __restrict__ q, const _Float16* __restrict__ kv, float* __restrict__ ws_acc,
    float* __restrict__ ws_ml, _Float16* __restrict__ z, int S, int batch, int h, int chunk, int splits,
    float scale_log2) {
    const int cg = blockIdx.x, n = blockIdx.y, sp = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = cg * COLS_PER_GROUP + lane * 8;
    const bool active = col < h;
    const int ccol = active ? col : 0;            // inactive lanes shadow column 0 and never store
    const int64_t row_stride = (int64_t)batch * 2 * h;
    const _Float16* kbase = kv + (int64_t)n * 2 * h + ccol;
    const _Float16* vbase = kbase + h;

    float qf[8];
    {
        const float4 q0 = *reinterpret_cast<const float4*>(q + (int64_t)n * h + ccol);
        const float4 q1 = *reinterpret_cast<const float4*>(q + (int64_t)n * h + ccol + 4);
        qf[0] = q0.x * scale_log2; qf[1] = q0.y * scale_log2; qf[2] = q0.z * scale_log2; qf[3] = q0.w * scale_log2;
        qf[4] = q1.x * scale_log2; qf[5] = q1.y * scale_log2; qf[6] = q1.z * scale_log2; qf[7] = q1.w * scale_log2;
    }

    const int j0 = sp * chunk;
    const int j1 = min(S, j0 + chunk);

    float m_run = -INFINITY, l_run = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    for (int j = j0 + wave * UNROLL; j < j1; j += ATT_WAVES * UNROLL) {
        half8 kf[UNROLL], vf[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int jj = min(j + u, j1 - 1);    // clamp: tail slots re-read the last valid row and are masked below
            kf[u] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(kbase + jj * row_stride));
            vf[u] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(vbase + jj * row_stride));
        }
        float sc[UNROLL];
        float m_new = m_run;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf((float)kf[u][e], qf[e], d);
            d = head_sum<D>(d);
            sc[u] = (j + u < j1) ? d : -INFINITY;
            m_new = fmaxf(m_new, sc[u]);
        }
        const float rescale = exp2f(m_run - m_new);   // first round: exp2(-inf) = 0
        l_run *= rescale;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= rescale;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const float p = exp2f(sc[u] - m_new);
            l_run += p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, (float)vf[u][e], acc[e]);
        }
        m_run = m_new;
    }

    // ---- merge the 4 waves (wave 0 always has at least one position) ----
    __shared__ float sm[ATT_WAVES][10][64];
    sm[wave][0][lane] = m_run;
    sm[wave][1][lane] = l_run;
#pragma unroll
    for (int e = 0; e < 8; ++e) sm[wave][2 + e][lane] = acc[e];
    __syncthreads();
    if (wave != 0) return;
    float m_tot = m_run;
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) m_tot = fmaxf(m_tot, sm[w][0][lane]);
    float l_tot = 0.f;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) {
        const float mw = sm[w][0][lane];
        const float wt = (mw == -INFINITY) ? 0.f : exp2f(mw - m_tot);
        l_tot += sm[w][1][lane] * wt;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += sm[w][2 + e][lane] * wt;
    }
    if (!active) return;
    if (splits == 1) {
        const float inv = 1.f / l_tot;
        half8 out;
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (_Float16)(o[e] * inv);
        *reinterpret_cast<half8*>(z + (int64_t)n * h + col) = out;
    } else {
        float* a = ws_acc + ((int64_t)sp * batch + n) * h + col;
        *reinterpret_cast<float4*>(a) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4*>(a + 4) = make_float4(o[4], o[5], o[6], o[7]);
        float* ml = ws_ml + (((int64_t)sp * batch + n) * (h / 8) + col / 8) * 2;
        *reinterpret_cast<float2*>(ml) = make_float2(m_tot, l_tot);
    }
}

// one thread per 8 columns: merge the per-split partials
__global__ __launch_bounds__(256) void attention_combine(const float* __restrict__ ws_acc,
                                                         const float* __restrict__ ws_ml,
                                                         _Float16* __restrict__ z, int batch, int h, int splits) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int chunks = h / 8;
    if (t >= (int64_t)batch * chunks) return;
    const int n = (int)(t / chunks), c = (int)(t % chunks);
    float m_tot = -INFINITY;
    for (int sp = 0; sp < splits; ++sp) m_tot = fmaxf(m_tot, ws_ml[(((int64_t)sp * batch + n) * chunks + c) * 2]);
    float l_tot = 0.f;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < splits; ++sp) {
        const float* ml = ws_ml + (((int64_t)sp * batch + n) * chunks + c) * 2;
        const float wt = (ml[0] == -INFINITY) ? 0.f : exp2f(ml[0] - m_tot);
        l_tot += ml[1] * wt;
        const float* a = ws_acc + ((int64_t)sp * batch + n) * h + c * 8;
        const float4 a0 = *reinterpret_cast<const float4*>(a), a1 = *reinterpret_cast<const float4*>(a + 4);
        o[0] += a0.x * wt; o[1] += a0.y * wt; o[2] += a0.z * wt; o[3] += a0.w * wt;
        o[4] += a1.x * wt; o[5] += a1.y * wt; o[6] += a1.z * wt; o[7] += a1.w * wt;
    }
    const float inv = 1.f / l_tot;
    half8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (_Float16)(o[e] * inv);
    *reinterpret_cast<half8*>(z + (int64_t)n * h + c * 8) = out;
}

// merge the waves' running (max, sum, acc) through LDS; wave 0 returns the workgroup's partial in (m, l, o)
template <int ATT_WAVES>
__device__ __forceinline__ bool merge_waves(float (*sm)[10][64], int wave, int lane, float& m_run, float& l_run, float (&acc)[8]) {
    sm[wave][0][lane] = m_run;
    sm[wave][1][lane] = l_run;
#pragma unroll
    for (int e = 0; e < 8; ++e) sm[wave][2 + e][lane] = acc[e];
    __syncthreads();
    if (wave != 0) return false;
    float m_tot = m_run;
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) m_tot = fmaxf(m_tot, sm[w][0][lane]);
    float l_tot = 0.f;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) {
        const float mw = sm[w][0][lane];
        const float wt = (mw == -INFINITY) ? 0.f : exp2f(mw - m_tot);
        l_tot += sm[w][1][lane] * wt;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += sm[w][2 + e][lane] * wt;
    }
    m_run = m_tot;
    l_run = l_tot;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = o[e];
    return true;
}

// Positions pos0 .. pos0 + n_pos - 1, then extra_pos if it is >= 0, rows of kv16 [*, batch, 2h] float16.  Writes partial
// slot split_base + blockIdx.z, or (fuse_slot >= 0) merges the partial in that slot and writes z.
template <int D, int UNROLL, int ATT_WAVES>
__global__ __launch_bounds__(ATT_WAVES * 64) void attention_partial_ranged(
    const float* __restrict__ q, const _Float16* __restrict__ kv16,
    float* __restrict__ ws_acc, float* __restrict__ ws_ml, int pos0, int n_pos, int extra_pos, int batch, int h,
    int chunk, int split_base, float scale_log2, int fuse_slot, _Float16* __restrict__ z) {
    const int cg = blockIdx.x, n = blockIdx.y, sp = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = cg * COLS_PER_GROUP + lane * 8;
    const bool active = col < h;
    const int ccol = active ? col : 0;
    float qf[8];
    {
        const float4 q0 = *reinterpret_cast<const float4*>(q + (int64_t)n * h + ccol);
        const float4 q1 = *reinterpret_cast<const float4*>(q + (int64_t)n * h + ccol + 4);
        qf[0] = q0.x * scale_log2; qf[1] = q0.y * scale_log2; qf[2] = q0.z * scale_log2; qf[3] = q0.w * scale_log2;
        qf[4] = q1.x * scale_log2; qf[5] = q1.y * scale_log2; qf[6] = q1.z * scale_log2; qf[7] = q1.w * scale_log2;
    }
    const int n_total = n_pos + (extra_pos >= 0 ? 1 : 0);
    const int j0 = sp * chunk;
    const int j1 = min(n_total, j0 + chunk);
    auto position = [&](int j) { return j < n_pos ? pos0 + j : extra_pos; };

    const int64_t row_stride = (int64_t)batch * 2 * h;
    const _Float16* kbase = kv16 + (int64_t)n * 2 * h + ccol;
    float m_run = -INFINITY, l_run = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = j0 + wave * UNROLL; j < j1; j += ATT_WAVES * UNROLL) {
        float kf[UNROLL][8], vf[UNROLL][8];
        {
            half8 kh[UNROLL], vh[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const _Float16* row = kbase + (int64_t)position(min(j + u, j1 - 1)) * row_stride;
                kh[u] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(row));
                vh[u] = __builtin_nontemporal_load(reinterpret_cast<const half8*>(row + h));
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    kf[u][e] = (float)kh[u][e];
                    vf[u][e] = (float)vh[u][e];
                }
        }
        float sc[UNROLL];
        float m_new = m_run;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(kf[u][e], qf[e], d);
            d = head_sum<D>(d);
            sc[u] = (j + u < j1) ? d : -INFINITY;
            m_new = fmaxf(m_new, sc[u]);
        }
        const float rescale = exp2f(m_run - m_new);
        l_run *= rescale;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= rescale;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const float p = exp2f(sc[u] - m_new);
            l_run += p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(p, vf[u][e], acc[e]);
        }
        m_run = m_new;
    }
    __shared__ float sm[ATT_WAVES][10][64];
    if (!merge_waves<ATT_WAVES>(sm, wave, lane, m_run, l_run, acc) || !active) return;
    if (fuse_slot >= 0) {
        // this launch has one workgroup per (sequence, column group) and so has the earlier one whose partial sits in
        // slot fuse_slot: merge the two here and write z, instead of a combine launch
        const float* a = ws_acc + ((int64_t)fuse_slot * batch + n) * h + col;
        const float2 ml = *reinterpret_cast<const float2*>(ws_ml + (((int64_t)fuse_slot * batch + n) * (h / 8) + col / 8) * 2);
        const float4 a0 = *reinterpret_cast<const float4*>(a), a1 = *reinterpret_cast<const float4*>(a + 4);
        const float m_tot = fmaxf(m_run, ml.x);
        const float w_mine = (m_run == -INFINITY) ? 0.f : exp2f(m_run - m_tot);
        const float w_prev = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - m_tot);
        const float inv = 1.f / (l_run * w_mine + ml.y * w_prev);
        const float prev[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        half8 out;
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (_Float16)((acc[e] * w_mine + prev[e] * w_prev) * inv);
        *reinterpret_cast<half8*>(z + (int64_t)n * h + col) = out;
        return;
    }
    const int slot = split_base + sp;
    float* a = ws_acc + ((int64_t)slot * batch + n) * h + col;
    *reinterpret_cast<float4*>(a) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(a + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    float* ml = ws_ml + (((int64_t)slot * batch + n) * (h / 8) + col / 8) * 2;
    *reinterpret_cast<float2*>(ml) = make_float2(m_run, l_run);
}

// The 8 codes of one word as floats: nibble e of the word is element e.  Even and odd nibbles are separated first so that
// every element is one byte-to-float conversion.
__device__ __forceinline__ void unpack_codes(uint32_t word, float (&c)[8]) {
    const uint32_t lo = word & 0x0F0F0F0Fu, hi = (word >> 4) & 0x0F0F0F0Fu;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        c[2 * b] = (float)((lo >> (8 * b)) & 0xFFu);
        c[2 * b + 1] = (float)((hi >> (8 * b)) & 0xFFu);
    }
}

// Packed rows of kvq [*, batch, 9h/8] (h bytes of codes: K then V, then h/32 + h/32 (scale, mn) float16 pairs, one per
// 64 columns), positions pos0 .. pos0 + n_pos - 1.  A lane owns 32 consecutive columns of one head: its K codes and its
// V codes are 16 bytes each, so every wave load is one contiguous KiB of codes (2048 columns).
// The first version read 4 bytes of codes per lane (256-byte segments) and reached 1.8 TB/s.
// The codec's value of an element is code * scale + mn with one (scale, mn) per 64 columns, i.e. per lane here, so the
// affine map is taken out of the sums: q . k = scale * sum_e q_e code_e + mn * sum_e q_e, and
// sum_t p_t v_te = sum_t (p_t scale_t) code_te + sum_t p_t mn_t.  That is a conversion and one fma per element where
// dequantising first (with the codec's rounding to float16) cost six instructions, and the kernel is bound by those.
// The values differ from kvpr_dequant_int4's by that rounding: at most 2^-11 relative per element.
template <int D, int ATT_WAVES>
__global__ __launch_bounds__(ATT_WAVES * 64) void attention_partial_packed(
    const float* __restrict__ q, const uint8_t* __restrict__ kvq, float* __restrict__ ws_acc, float* __restrict__ ws_ml,
    int pos0, int n_pos, int batch, int h, int chunk, int split_base, float scale_log2, int fuse_slot,
    _Float16* __restrict__ z) {
    constexpr int PU = 4;                                   // positions in flight per wave
    const int cg = blockIdx.x, n = blockIdx.y, sp = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = cg * 2048 + lane * 32;
    const bool active = col < h;
    const int ccol = active ? col : 0;
    float qf[32];
#pragma unroll
    for (int e = 0; e < 32; e += 4) {
        const float4 v = *reinterpret_cast<const float4*>(q + (int64_t)n * h + ccol + e);
        qf[e] = v.x * scale_log2; qf[e + 1] = v.y * scale_log2; qf[e + 2] = v.z * scale_log2; qf[e + 3] = v.w * scale_log2;
    }
    const int j0 = sp * chunk;
    const int j1 = min(n_pos, j0 + chunk);
    const int64_t qrow_stride = (int64_t)batch * (h + h / 8);
    const uint8_t* qbase = kvq + (int64_t)n * (h + h / 8);
    const int k_code = ccol / 2, v_code = (h + ccol) / 2;
    const int k_meta = h + (ccol / 64) * 4, v_meta = h + ((h + ccol) / 64) * 4;

    float qsum = 0.f;
#pragma unroll
    for (int e = 0; e < 32; ++e) qsum += qf[e];
    float m_run = -INFINITY, l_run = 0.f, pm_run = 0.f;      // pm_run: sum_t p_t mn_t, the same for the lane's 32 columns
    float acc[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) acc[e] = 0.f;
    for (int j = j0 + wave * PU; j < j1; j += ATT_WAVES * PU) {
        uint4v kc[PU], vc[PU];
        uint32_t km[PU], vm[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const uint8_t* row = qbase + (int64_t)(pos0 + min(j + u, j1 - 1)) * qrow_stride;   // tail slots re-read the last row, masked below
            kc[u] = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(row + k_code));
            vc[u] = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(row + v_code));
            km[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(row + k_meta));
            vm[u] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(row + v_meta));
        }
        float sc[PU];
        float m_new = m_run;
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            union { uint32_t w; _Float16 hh[2]; } a;
            a.w = km[u];
            const float ks = (float)a.hh[0], kmn = (float)a.hh[1];
            float dc = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float c8[8];
                unpack_codes(kc[u][w], c8);
#pragma unroll
                for (int e = 0; e < 8; ++e) dc = fmaf(c8[e], qf[8 * w + e], dc);
            }
            float d = fmaf(ks, dc, kmn * qsum);
            // sum over the D/32 consecutive lanes of the head
            d = dpp_xchg_add<0xB1>(d);
            if (D == 128) d = dpp_xchg_add<0x4E>(d);
            sc[u] = (j + u < j1) ? d : -INFINITY;
            m_new = fmaxf(m_new, sc[u]);
        }
        const float rescale = exp2f(m_run - m_new);
        l_run *= rescale;
        pm_run *= rescale;
#pragma unroll
        for (int e = 0; e < 32; ++e) acc[e] *= rescale;
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            union { uint32_t w; _Float16 hh[2]; } b;
            b.w = vm[u];
            const float vs = (float)b.hh[0], vmn = (float)b.hh[1];
            const float p = exp2f(sc[u] - m_new);
            l_run += p;
            pm_run = fmaf(p, vmn, pm_run);
            const float ps = p * vs;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float c8[8];
                unpack_codes(vc[u][w], c8);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[8 * w + e] = fmaf(ps, c8[e], acc[8 * w + e]);
            }
        }
        m_run = m_new;
    }
#pragma unroll
    for (int e = 0; e < 32; ++e) acc[e] += pm_run;
    // ---- merge the waves (wave 0 always has at least one position)
    __shared__ float sm[ATT_WAVES][34][64];
    sm[wave][0][lane] = m_run;
    sm[wave][1][lane] = l_run;
#pragma unroll
    for (int e = 0; e < 32; ++e) sm[wave][2 + e][lane] = acc[e];
    __syncthreads();
    if (wave != 0 || !active) return;
    float m_tot = m_run;
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) m_tot = fmaxf(m_tot, sm[w][0][lane]);
    float l_tot = 0.f;
    float o[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) o[e] = 0.f;
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) {
        const float mw = sm[w][0][lane];
        const float wt = (mw == -INFINITY) ? 0.f : exp2f(mw - m_tot);
        l_tot += sm[w][1][lane] * wt;
#pragma unroll
        for (int e = 0; e < 32; ++e) o[e] += sm[w][2 + e][lane] * wt;
    }
    if (fuse_slot >= 0) {
        // one workgroup per (sequence, column group) here and in the earlier float16 phase: merge its partial, write z
        const float* a = ws_acc + ((int64_t)fuse_slot * batch + n) * h + col;
        const float2 ml = *reinterpret_cast<const float2*>(ws_ml + (((int64_t)fuse_slot * batch + n) * (h / 8) + col / 8) * 2);
        const float m_all = fmaxf(m_tot, ml.x);
        const float w_mine = (m_tot == -INFINITY) ? 0.f : exp2f(m_tot - m_all);
        const float w_prev = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - m_all);
        const float inv = 1.f / (l_tot * w_mine + ml.y * w_prev);
#pragma unroll
        for (int e = 0; e < 32; e += 8) {
            const float4 a0 = *reinterpret_cast<const float4*>(a + e), a1 = *reinterpret_cast<const float4*>(a + e + 4);
            const float prev[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            half8 out;
#pragma unroll
            for (int t = 0; t < 8; ++t) out[t] = (_Float16)((o[e + t] * w_mine + prev[t] * w_prev) * inv);
            *reinterpret_cast<half8*>(z + (int64_t)n * h + col + e) = out;
        }
        return;
    }
    const int slot = split_base + sp;
    float* a = ws_acc + ((int64_t)slot * batch + n) * h + col;
#pragma unroll
    for (int e = 0; e < 32; e += 4) *reinterpret_cast<float4*>(a + e) = make_float4(o[e], o[e + 1], o[e + 2], o[e + 3]);
    float* ml = ws_ml + (((int64_t)slot * batch + n) * (h / 8) + col / 8) * 2;
#pragma unroll
    for (int g = 0; g < 4; ++g) *reinterpret_cast<float2*>(ml + 2 * g) = make_float2(m_tot, l_tot);   // one (m, l) per 8 columns
}

int g_attn_target_blocks = 256;   // one workgroup per CU: the fewest position splits that fill the chip
int g_attn_cfg = 1;       // (unroll, waves per workgroup) choice, see launch_attention
int g_attn_force_splits = 0;

struct SplitPlan { int chunk, splits; };
SplitPlan plan_splits(int batch, int hidden, int S, int cols_per_group = COLS_PER_GROUP) {
    const int groups = (hidden + cols_per_group - 1) / cols_per_group;
    int64_t base = (int64_t)groups * batch;
    int want = g_attn_force_splits > 0 ? g_attn_force_splits : (int)((g_attn_target_blocks + base - 1) / base);
    const int max_splits = (S + 63) / 64;              // keep at least 64 positions per workgroup
    if (g_attn_force_splits <= 0 && want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    if (want > S) want = S;
    const int chunk = (S + want - 1) / want;
    return {chunk, (S + chunk - 1) / chunk};           // no empty split
}

}  // namespace

size_t attention_workspace_bytes(int batch, int hidden, int n_heads, int S) {
    (void)n_heads;
    // upper bound over any split choice plan_splits can make for this shape (splits <= S, capped)
    int64_t splits = S < 1 ? 1 : S;
    if (splits > 512) splits = 512;
    return (size_t)(splits * batch * (int64_t)hidden * 4 + splits * batch * (int64_t)(hidden / 8) * 8);
}

namespace {

// the split choice launch_attention makes, with the workspace bound applied
SplitPlan attention_plan(int batch, int hidden, int S) {
    SplitPlan sp = plan_splits(batch, hidden, S);
    if (sp.splits > 512) {                            // workspace bound above
        sp.chunk = (S + 511) / 512;
        sp.splits = (S + sp.chunk - 1) / sp.chunk;
    }
    return sp;
}

}  // namespace

int launch_attention(const void* q, const void* kv, void* z, void* ws, int S, int batch, int hidden, int n_heads,
                     hipStream_t st) {
    const int d = hidden / n_heads;
    const SplitPlan sp = attention_plan(batch, hidden, S);
    const int groups = (hidden + COLS_PER_GROUP - 1) / COLS_PER_GROUP;
    float* ws_acc = (float*)ws;
    float* ws_ml = ws_acc + (int64_t)sp.splits * batch * hidden;
    const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)d));
    dim3 grid(groups, batch, sp.splits);
#define KVPR_LAUNCH_PART(D_, U_, W_)                                                                                \
    hipLaunchKernelGGL((attention_partial<D_, U_, W_>), grid, dim3(64 * W_), 0, st, (const float*)q, (const _Float16*)kv, \
                       ws_acc, ws_ml, (_Float16*)z, S, batch, hidden, sp.chunk, sp.splits, scale_log2)
    if (d == 128) {
        switch (g_attn_cfg) {
            case 1: KVPR_LAUNCH_PART(128, 8, 4); break;
            case 2: KVPR_LAUNCH_PART(128, 4, 8); break;
            case 3: KVPR_LAUNCH_PART(128, 8, 8); break;
            case 4: KVPR_LAUNCH_PART(128, 4, 16); break;
            case 5: KVPR_LAUNCH_PART(128, 8, 16); break;
            default: KVPR_LAUNCH_PART(128, 4, 4); break;
        }
    } else {
        switch (g_attn_cfg) {
            case 0: KVPR_LAUNCH_PART(64, 4, 4); break;
            case 2: KVPR_LAUNCH_PART(64, 4, 8); break;
            default: KVPR_LAUNCH_PART(64, 8, 4); break;
        }
    }
#undef KVPR_LAUNCH_PART
    KVPR_HIP(hipGetLastError());
    if (sp.splits > 1) {
        const int64_t threads = (int64_t)batch * (hidden / 8);
        hipLaunchKernelGGL(attention_combine, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ws_acc, ws_ml,
                           (_Float16*)z, batch, hidden, sp.splits);
        KVPR_HIP(hipGetLastError());
    }
    return KVPR_OK;
}

// ---- mixed float16 / packed attention in two phases (see the header comment) ----
namespace {

struct MixedPlan { SplitPlan a, b; int total; };
constexpr int PACKED_COLS_PER_GROUP = 64 * 32;   // columns one wave of the packed-row kernel covers

MixedPlan plan_mixed(int batch, int hidden, int S, int split, bool packed) {
    MixedPlan p;
    p.a = plan_splits(batch, hidden, split + 1);                    // rows [0, split) and the new row
    const int nb = S - 1 - split;                                   // transferred rows
    p.b = nb > 0 ? plan_splits(batch, hidden, nb, packed ? PACKED_COLS_PER_GROUP : COLS_PER_GROUP) : SplitPlan{0, 0};
    auto cap = [](SplitPlan& sp, int n) {                           // 256 + 256 partial slots fit the workspace bound
        if (sp.splits > 256) { sp.chunk = (n + 255) / 256; sp.splits = (n + sp.chunk - 1) / sp.chunk; }
    };
    cap(p.a, split + 1);
    if (nb > 0) cap(p.b, nb);
    p.total = p.a.splits + p.b.splits;
    return p;
}

int launch_ranged(const void* q, const void* kv16, float* ws_acc, float* ws_ml, int pos0, int n_pos,
                  int extra_pos, int batch, int hidden, int d, SplitPlan sp, int split_base, hipStream_t st,
                  int fuse_slot = -1, void* z = nullptr) {
    const int groups = (hidden + COLS_PER_GROUP - 1) / COLS_PER_GROUP;
    const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)d));
    dim3 grid(groups, batch, sp.splits);
    if (d == 128)
        hipLaunchKernelGGL((attention_partial_ranged<128, 8, 4>), grid, dim3(256), 0, st, (const float*)q,
                           (const _Float16*)kv16, ws_acc, ws_ml, pos0, n_pos, extra_pos, batch, hidden,
                           sp.chunk, split_base, scale_log2, fuse_slot, (_Float16*)z);
    else
        hipLaunchKernelGGL((attention_partial_ranged<64, 8, 4>), grid, dim3(256), 0, st, (const float*)q,
                           (const _Float16*)kv16, ws_acc, ws_ml, pos0, n_pos, extra_pos, batch, hidden,
                           sp.chunk, split_base, scale_log2, fuse_slot, (_Float16*)z);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

int launch_packed(const void* q, const void* kvq, float* ws_acc, float* ws_ml, int pos0, int n_pos, int batch, int hidden,
                  int d, SplitPlan sp, int split_base, hipStream_t st, int fuse_slot, void* z) {
    const int groups = (hidden + PACKED_COLS_PER_GROUP - 1) / PACKED_COLS_PER_GROUP;
    const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)d));
    dim3 grid(groups, batch, sp.splits);
    if (d == 128)
        hipLaunchKernelGGL((attention_partial_packed<128, 8>), grid, dim3(512), 0, st, (const float*)q, (const uint8_t*)kvq,
                           ws_acc, ws_ml, pos0, n_pos, batch, hidden, sp.chunk, split_base, scale_log2, fuse_slot, (_Float16*)z);
    else
        hipLaunchKernelGGL((attention_partial_packed<64, 8>), grid, dim3(512), 0, st, (const float*)q, (const uint8_t*)kvq,
                           ws_acc, ws_ml, pos0, n_pos, batch, hidden, sp.chunk, split_base, scale_log2, fuse_slot, (_Float16*)z);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

}  // namespace

// phase 0: float16 rows [0, split) and row S-1 of kv16.  phase 1: rows [split, S-1), packed from kvq if it is not null
// and float16 from kv16 otherwise, then the combine into z.  Both phases of one attention must be given the same S,
// split, batch and hidden.
int launch_attention_mixed(const void* q, const void* kv16, const void* kvq, void* z, void* ws, int S, int split, int batch,
                           int hidden, int n_heads, int phase, hipStream_t st) {
    const int d = hidden / n_heads;
    const MixedPlan p = plan_mixed(batch, hidden, S, split, kvq != nullptr);
    float* ws_acc = (float*)ws;
    float* ws_ml = ws_acc + (int64_t)p.total * batch * hidden;
    if (phase == 0)
        return launch_ranged(q, kv16, ws_acc, ws_ml, 0, split, S - 1, batch, hidden, d, p.a, 0, st);
    // one workgroup per (sequence, column group) in both phases: the second phase merges the first one's partial itself
    const bool fuse = p.a.splits == 1 && p.b.splits == 1;
    if (p.b.splits > 0)
        if (int rc = kvq ? launch_packed(q, kvq, ws_acc, ws_ml, split, S - 1 - split, batch, hidden, d, p.b, p.a.splits, st,
                                         fuse ? 0 : -1, z)
                         : launch_ranged(q, kv16, ws_acc, ws_ml, split, S - 1 - split, -1, batch, hidden, d, p.b, p.a.splits, st,
                                         fuse ? 0 : -1, z))
            return rc;
    if (fuse) return KVPR_OK;
    const int64_t threads = (int64_t)batch * (hidden / 8);
    hipLaunchKernelGGL(attention_combine, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ws_acc, ws_ml,
                       (_Float16*)z, batch, hidden, p.total);
    KVPR_HIP(hipGetLastError());
    return KVPR_OK;
}

}  // namespace kvpr

// ---- decode attention for callers that cannot allocate ----
// The partial results of a launch that splits the positions across workgroups live in a file-scope device array
// instead of a caller workspace.  Every GPU holds its own copy of the array at its own address; the address is
// looked up once per device (with that device current) and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[KVPR_ATTENTION_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int scratch_for_current_device(void** out) {
    int dev = -1;
    KVPR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return kvpr::fail(KVPR_E_RANGE, "device %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        KVPR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return kvpr::fail(KVPR_E_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return KVPR_OK;
}

}  // namespace

extern "C" int kvpr_decode_attention_static(const void* q, const void* kv, void* z, int S, int batch, int hidden,
                                            int n_heads, void* stream) {
    if (S < 1 || batch < 1 || n_heads < 1) return kvpr::fail(KVPR_E_RANGE, "S=%d batch=%d n_heads=%d out of range", S, batch, n_heads);
    if (hidden % n_heads || (hidden / n_heads != 64 && hidden / n_heads != 128))
        return kvpr::fail(KVPR_E_INVAL, "head_dim must be 64 or 128");
    if (!q || !kv || !z) return kvpr::fail(KVPR_E_INVAL, "q / kv / z is null");
    // what this launch would keep in the workspace: (acc[h] float32 + (m, l) per 8 columns) per split and sequence
    const kvpr::SplitPlan sp = kvpr::attention_plan(batch, hidden, S);
    const int64_t need = sp.splits > 1 ? (int64_t)sp.splits * batch * ((int64_t)hidden * 4 + (int64_t)(hidden / 8) * 8) : 0;
    if (need > (int64_t)KVPR_ATTENTION_STATIC_SCRATCH_BYTES)
        return kvpr::fail(KVPR_E_RANGE, "this shape needs %lld bytes of partial results, the static scratch holds %lld: use "
                          "kvpr_decode_attention with a workspace", (long long)need, (long long)KVPR_ATTENTION_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (int rc = scratch_for_current_device(&ws)) return rc;
    return kvpr::launch_attention(q, kv, z, ws, S, batch, hidden, n_heads, (hipStream_t)stream);
}

extern "C" int kvpr_debug_set_attention_kernel(int v) {
    kvpr::g_attn_cfg = v;
    return KVPR_OK;
}

extern "C" int kvpr_debug_set_attention_splits(int force_splits, int target_blocks) {
    kvpr::g_attn_force_splits = force_splits;
    if (target_blocks > 0) kvpr::g_attn_target_blocks = target_blocks;
    return KVPR_OK;
}
