// Workload analysis unit (Section 3.2.1): the number of GPUs d that minimises Eq. 1,
//   t_estimate(d) = sum over layers l of { t_c(l, d) + t_s(l, d) },
// with t_c measured (wap_profile_layer) and t_s the ring all-reduce cost of Section 3.2.3.  Host code only.
#include <cmath>
#include <limits>

#include "wap_internal.h"

using namespace wap;

extern "C" int wap_choose_gpus(int32_t n_layers, int32_t max_gpus, const double* t_c, const double* grad_bytes,
                               const wap_link_model* link, const uint8_t* allowed, double* t_estimate_out,
                               int32_t* best_d_out) {
    if (!t_c || !grad_bytes || !link || !t_estimate_out || !best_d_out)
        return set_error(WAP_EINVAL, "choose_gpus: NULL argument");
    if (n_layers < 1 || max_gpus < 1) return set_error(WAP_EINVAL, "choose_gpus: n_layers and max_gpus must be >= 1");
    if (!(link->link_bytes_per_s > 0.0) || !std::isfinite(link->link_bytes_per_s))
        return set_error(WAP_EINVAL, "choose_gpus: link bandwidth must be positive and finite");
    if (!(link->latency_s >= 0.0) || !std::isfinite(link->latency_s))
        return set_error(WAP_EINVAL, "choose_gpus: link latency must be >= 0 and finite");
    for (int l = 0; l < n_layers; ++l) {
        if (!(grad_bytes[l] >= 0.0) || !std::isfinite(grad_bytes[l]))
            return set_error(WAP_EINVAL, "choose_gpus: grad_bytes[%d] must be >= 0 and finite", l);
        for (int d = 1; d <= max_gpus; ++d) {
            if (allowed && !allowed[d - 1]) continue;
            const double t = t_c[(size_t)l * max_gpus + (d - 1)];
            if (!(t >= 0.0) || !std::isfinite(t))
                return set_error(WAP_EINVAL, "choose_gpus: t_c[%d][%d] must be >= 0 and finite", l, d - 1);
        }
    }
    int best = 0;
    double best_t = std::numeric_limits<double>::infinity();
    for (int d = 1; d <= max_gpus; ++d) {
        if (allowed && !allowed[d - 1]) {
            t_estimate_out[d - 1] = std::numeric_limits<double>::infinity();
            continue;
        }
        // ring all-reduce: every GPU sends and receives 2 (d-1)/d of the gradient in 2 (d-1) steps
        const double traffic = d == 1 ? 0.0 : 2.0 * (d - 1) / d;
        const double steps = d == 1 ? 0.0 : 2.0 * (d - 1);
        double total = 0.0;
        for (int l = 0; l < n_layers; ++l)
            total += t_c[(size_t)l * max_gpus + (d - 1)] +
                     (traffic * grad_bytes[l] / link->link_bytes_per_s + steps * link->latency_s);
        t_estimate_out[d - 1] = total;
        if (total < best_t) {  // strict: a tie keeps the smaller d
            best_t = total;
            best = d;
        }
    }
    if (best == 0) return set_error(WAP_EINVAL, "choose_gpus: no allowed division");
    *best_d_out = best;
    return WAP_OK;
}
