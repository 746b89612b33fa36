// Split-point scheduler (Sec. 3.2, Eq. 6-11).  Pure host arithmetic; compiled with
// -ffp-contract=off so that every operation is one IEEE-754 double operation.
#include <cmath>
#include <cstdint>
#include "kvpr.h"

namespace kvpr {
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}

namespace {

bool rate_ok(double v) { return std::isfinite(v) && v > 0.0; }
bool lat_ok(double v) { return std::isfinite(v) && v >= 0.0; }

int check(const kvpr_profile_t* p, int model, int batch, int seq, int hidden, int elem_bytes) {
    if (!p) return kvpr::fail(KVPR_E_INVAL, "profile is null");
    if (model != KVPR_COST_EQ10 && model != KVPR_COST_NS && model != KVPR_COST_ROW && model != KVPR_COST_PIPE)
        return kvpr::fail(KVPR_E_INVAL, "unknown cost model %d", model);
    if (batch < 1 || seq < 0 || hidden < 1 || elem_bytes < 1)
        return kvpr::fail(KVPR_E_RANGE, "batch=%d seq=%d hidden=%d elem_bytes=%d out of range", batch, seq, hidden,
                          elem_bytes);
    if (!rate_ok(p->h2d_bytes_per_s) || !rate_ok(p->gemm_flops_per_s))
        return kvpr::fail(KVPR_E_INVAL, "profile rates must be finite and > 0 (v_com=%g, v_gpu=%g)",
                          p->h2d_bytes_per_s, p->gemm_flops_per_s);
    if (!lat_ok(p->h2d_latency_s) || !lat_ok(p->gemm_latency_s))
        return kvpr::fail(KVPR_E_INVAL, "profile latencies must be finite and >= 0");
    // 4*b*s*h*h must stay below 2^53 so that the int64 -> double conversion is exact
    const long double flops = 4.0L * batch * (long double)seq * hidden * (long double)hidden;
    if (flops >= 9007199254740992.0L) return kvpr::fail(KVPR_E_RANGE, "problem too large for exact flop count");
    return KVPR_OK;
}

// Eq. 10 (or a variant) at one split
double cost_at(const kvpr_profile_t* p, int model, int64_t l, int64_t b, int64_t s, int64_t h, int64_t eb) {
    const int64_t m_x = b * l * h * eb;                 // Eq. 6
    const int64_t m_kv = 2 * b * (s - l) * h * eb;      // Eq. 6
    const int64_t n_kv = 4 * b * l * h * h;             // Eq. 8
    double t_act = (double)m_x / p->h2d_bytes_per_s;
    double t_kv = (double)m_kv / p->h2d_bytes_per_s;
    double t_rc = (double)n_kv / p->gemm_flops_per_s;   // Eq. 9
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
            const double link = t_act + t_kv;
            return link > t_rc ? link : t_rc;
        }
        default: return t_act + (t_rc > t_kv ? t_rc : t_kv);
    }
}

// Extension of Eq. 10 to a chunked activation copy: X[0:l] travels as `chunks` equal parts, the GEMM of
// part j starts when part j has landed and part j-1 has been recomputed; the cache follows X on the link.
double cost_chunked_at(const kvpr_profile_t* p, int chunks, int64_t l, int64_t b, int64_t s, int64_t h, int64_t eb) {
    const int64_t m_x = b * l * h * eb, m_kv = 2 * b * (s - l) * h * eb, n_kv = 4 * b * l * h * h;
    const double t_act = (double)m_x / p->h2d_bytes_per_s;
    double t_kv = (double)m_kv / p->h2d_bytes_per_s;
    const double t_rc = (double)n_kv / p->gemm_flops_per_s;
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

}  // namespace

extern "C" int kvpr_cost_chunked(const kvpr_profile_t* prof, int chunks, int split, int batch, int seq, int hidden,
                                 int elem_bytes, double* t_pred) {
    if (int rc = check(prof, KVPR_COST_EQ10, batch, seq, hidden, elem_bytes)) return rc;
    if (chunks < 1) return kvpr::fail(KVPR_E_RANGE, "chunks %d < 1", chunks);
    if (!t_pred) return kvpr::fail(KVPR_E_INVAL, "t_pred is null");
    if (split < 0 || split > seq) return kvpr::fail(KVPR_E_RANGE, "split %d outside [0, %d]", split, seq);
    *t_pred = cost_chunked_at(prof, chunks, split, batch, seq, hidden, elem_bytes);
    return KVPR_OK;
}

extern "C" int kvpr_plan_split_chunked(const kvpr_profile_t* prof, int chunks, int batch, int seq, int hidden,
                                       int elem_bytes, int granularity, int32_t* l_star, double* t_pred) {
    if (int rc = check(prof, KVPR_COST_EQ10, batch, seq, hidden, elem_bytes)) return rc;
    if (chunks < 1) return kvpr::fail(KVPR_E_RANGE, "chunks %d < 1", chunks);
    if (granularity < 1) return kvpr::fail(KVPR_E_RANGE, "granularity %d < 1", granularity);
    if (!l_star) return kvpr::fail(KVPR_E_INVAL, "l_star is null");
    int32_t best_l = -1;
    double best_t = INFINITY;
    auto visit = [&](int64_t l) {
        const double t = cost_chunked_at(prof, chunks, l, batch, seq, hidden, elem_bytes);
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

extern "C" int kvpr_cost(const kvpr_profile_t* prof, int cost_model, int split, int batch, int seq, int hidden,
                         int elem_bytes, double* t_pred) {
    if (int rc = check(prof, cost_model, batch, seq, hidden, elem_bytes)) return rc;
    if (!t_pred) return kvpr::fail(KVPR_E_INVAL, "t_pred is null");
    if (split < 0 || split > seq) return kvpr::fail(KVPR_E_RANGE, "split %d outside [0, %d]", split, seq);
    *t_pred = cost_at(prof, cost_model, split, batch, seq, hidden, elem_bytes);
    return KVPR_OK;
}

extern "C" int kvpr_plan_split(const kvpr_profile_t* prof, int cost_model, int batch, int seq, int hidden,
                               int elem_bytes, int granularity, int32_t* l_star, double* t_pred) {
    if (int rc = check(prof, cost_model, batch, seq, hidden, elem_bytes)) return rc;
    if (granularity < 1) return kvpr::fail(KVPR_E_RANGE, "granularity %d < 1", granularity);
    if (!l_star) return kvpr::fail(KVPR_E_INVAL, "l_star is null");
    int32_t best_l = -1;
    double best_t = INFINITY;
    // Eq. 11 by enumeration: multiples of the granularity in ascending order, then seq itself
    auto visit = [&](int64_t l) {
        const double t = cost_at(prof, cost_model, l, batch, seq, hidden, elem_bytes);
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
