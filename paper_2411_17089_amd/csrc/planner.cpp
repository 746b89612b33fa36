// Split-point scheduler (Sec. 3.2, Eq. 6-11).  Pure host arithmetic; compiled with
// -ffp-contract=off so that every operation is one IEEE-754 double operation.
//
// Eq. 6 and Eq. 8 are linear in the number of positions, so the model is evaluated on
// per-position sizes: M_X = x_bpp * l, M_KV = kv_bpp * (s - l), N_KV = flops_pp * l.  The entry
// points that take (batch, hidden, elem_bytes) fill in the paper's sizes; a compressed store
// (Sec. 4.4) passes its own byte rates through the *_linear entry points.
#include <cmath>
#include <cstdint>
#include "kvpr.h"

namespace kvpr {
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}

namespace {

struct Sizes {
    int64_t x_bpp, kv_bpp, flops_pp;
};

bool rate_ok(double v) { return std::isfinite(v) && v > 0.0; }
bool lat_ok(double v) { return std::isfinite(v) && v >= 0.0; }

int check_profile(const kvpr_profile_t* p, int model, int chunks) {
    if (!p) return kvpr::fail(KVPR_E_INVAL, "profile is null");
    if (model != KVPR_COST_EQ10 && model != KVPR_COST_NS && model != KVPR_COST_ROW && model != KVPR_COST_PIPE)
        return kvpr::fail(KVPR_E_INVAL, "unknown cost model %d", model);
    if (chunks < 1) return kvpr::fail(KVPR_E_RANGE, "chunks %d < 1", chunks);
    if (chunks > 1 && model != KVPR_COST_EQ10)
        return kvpr::fail(KVPR_E_INVAL, "the chunked schedule is modelled for KVPR_COST_EQ10 only");
    if (!rate_ok(p->h2d_bytes_per_s) || !rate_ok(p->gemm_flops_per_s))
        return kvpr::fail(KVPR_E_INVAL, "profile rates must be finite and > 0 (v_com=%g, v_gpu=%g)",
                          p->h2d_bytes_per_s, p->gemm_flops_per_s);
    if (!lat_ok(p->h2d_latency_s) || !lat_ok(p->gemm_latency_s) || !lat_ok(p->layer_other_s))
        return kvpr::fail(KVPR_E_INVAL, "profile latencies must be finite and >= 0");
    if (p->gemm_round_flops < 0) return kvpr::fail(KVPR_E_INVAL, "gemm_round_flops must be >= 0");
    return KVPR_OK;
}

// every count must stay below 2^53 so that the int64 -> double conversion is exact
int check_sizes(const Sizes& z, int seq) {
    if (seq < 0) return kvpr::fail(KVPR_E_RANGE, "seq=%d out of range", seq);
    if (z.x_bpp < 0 || z.kv_bpp < 0 || z.flops_pp < 0)
        return kvpr::fail(KVPR_E_RANGE, "per-position sizes must be >= 0");
    const long double lim = 9007199254740992.0L;
    if ((long double)z.x_bpp * seq >= lim || (long double)z.kv_bpp * seq >= lim || (long double)z.flops_pp * seq >= lim / 2)
        return kvpr::fail(KVPR_E_RANGE, "problem too large for exact byte / flop counts");
    return KVPR_OK;
}

int paper_sizes(int batch, int seq, int hidden, int elem_bytes, Sizes* z) {
    if (batch < 1 || seq < 0 || hidden < 1 || elem_bytes < 1)
        return kvpr::fail(KVPR_E_RANGE, "batch=%d seq=%d hidden=%d elem_bytes=%d out of range", batch, seq, hidden,
                          elem_bytes);
    const long double flops = 4.0L * batch * (long double)seq * hidden * (long double)hidden;
    if (flops >= 9007199254740992.0L) return kvpr::fail(KVPR_E_RANGE, "problem too large for exact flop count");
    z->x_bpp = (int64_t)batch * hidden * elem_bytes;            // Eq. 6
    z->kv_bpp = 2 * (int64_t)batch * hidden * elem_bytes;       // Eq. 6
    z->flops_pp = 4 * (int64_t)batch * hidden * hidden;         // Eq. 8
    return KVPR_OK;
}

// Eq. 8, charged in whole rounds of work when the profile says the GPU works in rounds
int64_t recompute_flops(const kvpr_profile_t* p, int64_t l, const Sizes& z) {
    const int64_t n = z.flops_pp * l;
    const int64_t r = p->gemm_round_flops;
    return r > 0 ? (n + r - 1) / r * r : n;
}

// Eq. 10 (or a variant) at one split
double cost_at(const kvpr_profile_t* p, int model, int64_t l, int64_t s, const Sizes& z) {
    double t_act = (double)(z.x_bpp * l) / p->h2d_bytes_per_s;
    double t_kv = (double)(z.kv_bpp * (s - l)) / p->h2d_bytes_per_s;
    double t_rc = (double)recompute_flops(p, l, z) / p->gemm_flops_per_s;   // Eq. 9
    if (l > 0) {
        t_act = t_act + p->h2d_latency_s;
        t_rc = t_rc + p->gemm_latency_s;
    }
    if (l < s) t_kv = t_kv + p->h2d_latency_s;
    switch (model) {
        case KVPR_COST_ROW: return t_rc > t_kv ? t_rc : t_kv;
        case KVPR_COST_NS: {
            const double arm = t_rc + t_act;
            return arm > t_kv ? arm : t_kv;
        }
        case KVPR_COST_PIPE: {
            const double link = t_act + t_kv, gpu = t_rc + p->layer_other_s;
            return link > gpu ? link : gpu;
        }
        default: return t_act + (t_rc > t_kv ? t_rc : t_kv);
    }
}

// Extension of Eq. 10 to a chunked activation copy: X[0:l] travels as `chunks` equal parts, the GEMM of
// part j starts when part j has landed and part j-1 has been recomputed; the cache follows X on the link.
double cost_chunked_at(const kvpr_profile_t* p, int chunks, int64_t l, int64_t s, const Sizes& z) {
    const double t_act = (double)(z.x_bpp * l) / p->h2d_bytes_per_s;
    double t_kv = (double)(z.kv_bpp * (s - l)) / p->h2d_bytes_per_s;
    const double t_rc = (double)recompute_flops(p, l, z) / p->gemm_flops_per_s;
    if (l < s) t_kv = t_kv + p->h2d_latency_s;
    double done = 0.0;                                   // end of the GEMM of the parts so far
    if (l > 0) {
        for (int j = 1; j <= chunks; ++j) {
            const double landed = t_act * (double)j / (double)chunks + p->h2d_latency_s;
            const double start = landed > done ? landed : done;
            done = start + (t_rc / (double)chunks + p->gemm_latency_s);
        }
    }
    const double link = (l > 0 ? t_act + p->h2d_latency_s : 0.0) + t_kv;
    return done > link ? done : link;
}

double cost_any(const kvpr_profile_t* p, int model, int chunks, int64_t l, int64_t s, const Sizes& z) {
    return chunks > 1 ? cost_chunked_at(p, chunks, l, s, z) : cost_at(p, model, l, s, z);
}

int cost_impl(const kvpr_profile_t* prof, int model, int chunks, int split, int seq, const Sizes& z, double* t_pred) {
    if (!t_pred) return kvpr::fail(KVPR_E_INVAL, "t_pred is null");
    if (split < 0 || split > seq) return kvpr::fail(KVPR_E_RANGE, "split %d outside [0, %d]", split, seq);
    *t_pred = cost_any(prof, model, chunks, split, seq, z);
    return KVPR_OK;
}

// Eq. 11 by enumeration: multiples of the granularity in ascending order, then seq itself; the first strict minimum wins
int plan_impl(const kvpr_profile_t* prof, int model, int chunks, int seq, const Sizes& z, int granularity,
              int32_t* l_star, double* t_pred) {
    if (granularity < 1) return kvpr::fail(KVPR_E_RANGE, "granularity %d < 1", granularity);
    if (!l_star) return kvpr::fail(KVPR_E_INVAL, "l_star is null");
    int32_t best_l = -1;
    double best_t = INFINITY;
    auto visit = [&](int64_t l) {
        const double t = cost_any(prof, model, chunks, l, seq, z);
        if (t < best_t) {
            best_t = t;
            best_l = (int32_t)l;
        }
    };
    for (int64_t l = 0; l <= seq; l += granularity) visit(l);
    if (seq % granularity != 0) visit(seq);
    *l_star = best_l;
    if (t_pred) *t_pred = best_t;
    return KVPR_OK;
}

}  // namespace

extern "C" int kvpr_cost(const kvpr_profile_t* prof, int cost_model, int split, int batch, int seq, int hidden,
                         int elem_bytes, double* t_pred) {
    Sizes z;
    if (int rc = check_profile(prof, cost_model, 1)) return rc;
    if (int rc = paper_sizes(batch, seq, hidden, elem_bytes, &z)) return rc;
    return cost_impl(prof, cost_model, 1, split, seq, z, t_pred);
}

extern "C" int kvpr_plan_split(const kvpr_profile_t* prof, int cost_model, int batch, int seq, int hidden,
                               int elem_bytes, int granularity, int32_t* l_star, double* t_pred) {
    Sizes z;
    if (int rc = check_profile(prof, cost_model, 1)) return rc;
    if (int rc = paper_sizes(batch, seq, hidden, elem_bytes, &z)) return rc;
    return plan_impl(prof, cost_model, 1, seq, z, granularity, l_star, t_pred);
}

extern "C" int kvpr_cost_chunked(const kvpr_profile_t* prof, int chunks, int split, int batch, int seq, int hidden,
                                 int elem_bytes, double* t_pred) {
    Sizes z;
    if (int rc = check_profile(prof, KVPR_COST_EQ10, chunks)) return rc;
    if (int rc = paper_sizes(batch, seq, hidden, elem_bytes, &z)) return rc;
    if (!t_pred) return kvpr::fail(KVPR_E_INVAL, "t_pred is null");
    if (split < 0 || split > seq) return kvpr::fail(KVPR_E_RANGE, "split %d outside [0, %d]", split, seq);
    *t_pred = cost_chunked_at(prof, chunks, split, seq, z);   // chunks = 1 goes through the chunked form too
    return KVPR_OK;
}

extern "C" int kvpr_plan_split_chunked(const kvpr_profile_t* prof, int chunks, int batch, int seq, int hidden,
                                       int elem_bytes, int granularity, int32_t* l_star, double* t_pred) {
    Sizes z;
    if (int rc = check_profile(prof, KVPR_COST_EQ10, chunks)) return rc;
    if (int rc = paper_sizes(batch, seq, hidden, elem_bytes, &z)) return rc;
    // chunks = 1 evaluates the chunked recurrence as well (it equals Eq. 10 up to rounding order)
    if (granularity < 1) return kvpr::fail(KVPR_E_RANGE, "granularity %d < 1", granularity);
    if (!l_star) return kvpr::fail(KVPR_E_INVAL, "l_star is null");
    int32_t best_l = -1;
    double best_t = INFINITY;
    auto visit = [&](int64_t l) {
        const double t = cost_chunked_at(prof, chunks, l, seq, z);
        if (t < best_t) {
            best_t = t;
            best_l = (int32_t)l;
        }
    };
    for (int64_t l = 0; l <= seq; l += granularity) visit(l);
    if (seq % granularity != 0) visit(seq);
    *l_star = best_l;
    if (t_pred) *t_pred = best_t;
    return KVPR_OK;
}

extern "C" int kvpr_cost_linear(const kvpr_profile_t* prof, int cost_model, int chunks, int split, int seq,
                                int64_t x_bytes_per_pos, int64_t kv_bytes_per_pos, int64_t flops_per_pos, double* t_pred) {
    const Sizes z{x_bytes_per_pos, kv_bytes_per_pos, flops_per_pos};
    if (int rc = check_profile(prof, cost_model, chunks)) return rc;
    if (int rc = check_sizes(z, seq)) return rc;
    return cost_impl(prof, cost_model, chunks, split, seq, z, t_pred);
}

extern "C" int kvpr_plan_split_linear(const kvpr_profile_t* prof, int cost_model, int chunks, int seq,
                                      int64_t x_bytes_per_pos, int64_t kv_bytes_per_pos, int64_t flops_per_pos,
                                      int granularity, int32_t* l_star, double* t_pred) {
    const Sizes z{x_bytes_per_pos, kv_bytes_per_pos, flops_per_pos};
    if (int rc = check_profile(prof, cost_model, chunks)) return rc;
    if (int rc = check_sizes(z, seq)) return rc;
    return plan_impl(prof, cost_model, chunks, seq, z, granularity, l_star, t_pred);
}

// Extension: run-time adaptation of the two profiled constants (the paper profiles once, at start-up):
// exponential moving average over what finished layers achieved.  A sample with no work or no time is skipped.
extern "C" int kvpr_adapt_update(kvpr_profile_t* prof, double alpha, int64_t link_bytes, double link_seconds,
                                 int64_t gemm_flops, double gemm_seconds) {
    if (!prof) return kvpr::fail(KVPR_E_INVAL, "profile is null");
    if (!(alpha >= 0.0 && alpha <= 1.0)) return kvpr::fail(KVPR_E_RANGE, "alpha %g outside [0, 1]", alpha);
    if (link_bytes > 0 && link_seconds > 0.0)
        prof->h2d_bytes_per_s = (1.0 - alpha) * prof->h2d_bytes_per_s + alpha * ((double)link_bytes / link_seconds);
    if (gemm_flops > 0 && gemm_seconds > 0.0)
        prof->gemm_flops_per_s = (1.0 - alpha) * prof->gemm_flops_per_s + alpha * ((double)gemm_flops / gemm_seconds);
    return KVPR_OK;
}
