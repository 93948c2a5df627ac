// The control loop of the paper's Sec. 3.3 as a pure host function: one period moves the reserved
// share r of the latency-critical (prefill) class and its flush time-out tau_pre.  The paper states the
// directions -- KV-link utilisation below target: raise r or shorten tau_pre; decode stalls rising:
// lower r -- and that the loop also works on the prefill P95 wait; amounts and order are parameters and
// a reading of this implementation (see the header).  No GPU code in this file.
#include "../../include/trinity_ivf.h"

#include <cmath>

extern "C" int tri_policy_feedback(const tri_feedback_cfg *c, const tri_feedback_signals *sg, tri_policy *pol, uint32_t *rules)
{
    if (rules) *rules = 0;
    if (!c || !sg || !pol) return TRI_EINVAL;
    if (!(c->r_min >= 0.0f && c->r_min <= c->r_max && c->r_max <= 1.0f && c->r_step > 0.0f)) return TRI_EINVAL;
    if (!(c->tau_factor > 1.0f) || !(c->tau_min_s >= 0.0 && c->tau_min_s <= c->tau_max_s)) return TRI_EINVAL;
    float r = std::fmin(std::fmax(pol->high_share, c->r_min), c->r_max);
    double tau = std::fmin(std::fmax(pol->flush_timeout_high_s, c->tau_min_s), c->tau_max_s);
    uint32_t applied = 0;
    const bool link_starved = !std::isnan(sg->u_kv) && sg->u_kv < c->u_kv_target - c->u_kv_band;
    if (link_starved) {                                        // rule 1
        if (r < c->r_max) r = std::fmin(c->r_max, r + c->r_step);
        else tau = std::fmax(c->tau_min_s, tau / c->tau_factor);
        applied |= 1u;
    }
    const bool waited = !std::isnan(sg->wait_p95_s);
    if (waited && sg->wait_p95_s > c->wait_p95_budget_s) {     // rule 2
        tau = std::fmax(c->tau_min_s, tau / c->tau_factor);
        applied |= 2u;
    }
    if (!link_starved && !std::isnan(sg->decode_stall) && sg->decode_stall > c->stall_target &&
        !std::isnan(sg->decode_stall_prev) && sg->decode_stall > sg->decode_stall_prev) {   // rule 3
        r = std::fmax(c->r_min, r - c->r_step);
        applied |= 4u;
    }
    if (!applied && (!waited || sg->wait_p95_s <= 0.5 * c->wait_p95_budget_s)) {            // rule 4
        tau = std::fmin(c->tau_max_s, tau * c->tau_factor);
        applied |= 8u;
    }
    pol->high_share = r;
    pol->flush_timeout_high_s = tau;
    if (rules) *rules = applied;
    return TRI_OK;
}
