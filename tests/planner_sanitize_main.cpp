// Host-only driver for the scheduler (planner.cpp) built with -fsanitize=address,undefined: walks the entry
// points over ordinary, extreme and invalid arguments.  Any sanitizer report makes the process fail.
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <initializer_list>
#include <limits>
#include "kvpr.h"

namespace kvpr {
int fail(int code, const char* fmt, ...) {
    char buf[256];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace kvpr

int main() {
    long ok = 0, refused = 0;
    auto tally = [&](int rc) { (rc == KVPR_OK ? ok : refused)++; };
    const double inf = std::numeric_limits<double>::infinity(), nan = std::nan("");
    const double rates[] = {1.0, 57e9, 1e15, 1e-300, 1e300, 0.0, -1.0, inf, nan};
    const int seqs[] = {0, 1, 7, 1024, 4096, 1 << 16, -1};
    const int grans[] = {1, 8, 64, 1 << 30, 0, -3};
    for (double vc : rates)
        for (double vg : rates)
            for (double other : {0.0, 1e-3, nan}) {
                kvpr_profile_t p{vc, vg, 1e-5, 2e-5, 0, 0, 0, 0, (other > 0) ? (int64_t)1 << 33 : 0, other};
                for (int model = -1; model <= 4; ++model)
                    for (int s : seqs)
                        for (int g : grans) {
                            int32_t l = -7;
                            double t = 0;
                            tally(kvpr_plan_split(&p, model, 32, s, 4096, 2, g, &l, &t));
                            tally(kvpr_plan_split(&p, model, 64, s, 7168, 2, g, &l, nullptr));
                            tally(kvpr_plan_split_linear(&p, model, 1, s, 9 * 4096 / 16 * 32, 9 * 4096 / 8 * 32, 4LL * 32 * 4096 * 4096, g, &l, &t));
                            tally(kvpr_plan_split_linear(&p, model, 3, s, INT64_MAX / 2, 1, 1, g, &l, &t));
                            tally(kvpr_plan_split_chunked(&p, 5, 16, s, 5120, 2, g, &l, &t));
                            tally(kvpr_cost(&p, model, s / 2, 32, s, 4096, 2, &t));
                            tally(kvpr_cost(&p, model, s + 1, 32, s, 4096, 2, &t));
                            tally(kvpr_cost_chunked(&p, 32, s / 3, 1, s, 768, 2, &t));
                            tally(kvpr_cost_linear(&p, model, 2, s / 2, s, 0, 0, 0, &t));
                        }
                tally(kvpr_adapt_update(&p, 0.5, 1 << 20, 1e-3, 1LL << 40, 2e-3));
                tally(kvpr_adapt_update(&p, 1.5, 1, 1.0, 1, 1.0));
            }
    int32_t l;
    tally(kvpr_plan_split(nullptr, 0, 1, 1, 64, 2, 1, &l, nullptr));
    kvpr_profile_t good{1e9, 1e12, 0, 0, 0, 0, 0, 0, 0, 0};
    tally(kvpr_plan_split(&good, 0, 1, 1, 64, 2, 1, nullptr, nullptr));
    tally(kvpr_plan_split(&good, 0, 2000000000, 2000000000, 2000000000, 2, 1, &l, nullptr));
    tally(kvpr_cost(&good, 0, 0, 1, 1, 64, 2, nullptr));
    tally(kvpr_adapt_update(nullptr, 0.5, 1, 1.0, 1, 1.0));
    printf("ok=%ld refused=%ld\n", ok, refused);
    return (ok > 0 && refused > 0) ? 0 : 1;
}
