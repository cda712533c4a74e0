// Host-side adaptive-compression controller (Alg. 1: epsilon switch, UpdateStep, CheckGraVAC; scaling
// policies of Sec. IV-B).  Pure host code; see gravac_controller.h for the contract and for the readings
// taken where the listing and the text disagree.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <new>
#include <utility>
#include <vector>

#include "gravac.h"
#include "gravac_controller.h"

namespace {

// Exponentially weighted moving average started at its first sample.
struct Ewma {
    double value = 0.0;
    bool started = false;
    double push(double x, double alpha)
    {
        value = started ? alpha * x + (1.0 - alpha) * value : x;
        started = true;
        return value;
    }
};

}  // namespace

struct gravac_controller {
    gravac_controller_config cfg;
    double theta_min;
    double theta_s;
    int64_t iteration = 0;       // iterations finished
    Ewma gain_min, gain_c;
    std::map<double, double> t_compress;  // CF -> compression throughput, last value recorded
    bool decided = false;        // decide() called, finish_iteration() pending
    int32_t choice = GRAVAC_SEND_DENSE;

    double candidate() const { return std::min(theta_s * theta_min, cfg.theta_max); }

    double scaled(double s) const
    {
        return cfg.policy == GRAVAC_POLICY_EXPONENTIAL ? s * s : 2.0 * s;
    }

    // CheckGraVAC at the end of a window
    void evaluate()
    {
        const double evaluated = candidate();
        theta_s = scaled(theta_s);
        const double dmin = gain_min.value, dc = gain_c.value;
        if (dmin > 0.0 && cfg.omega >= std::fabs(dmin - dc) / dmin && evaluated > theta_min) {
            theta_min = evaluated;   // the minimum CF moves up to the CF just evaluated
            gain_min = gain_c;       // whose gain history it inherits
        }
        if (t_compress.size() >= 2) {
            // the two largest throughputs; among equal values the lower CF counts as the larger entry
            std::vector<std::pair<double, double>> ct;  // (throughput, CF)
            for (const auto& e : t_compress) ct.emplace_back(e.second, e.first);
            std::sort(ct.begin(), ct.end(), [](const std::pair<double, double>& a, const std::pair<double, double>& b) {
                return a.first < b.first || (a.first == b.first && a.second > b.second);
            });
            const auto& top = ct[ct.size() - 1];
            const auto& second = ct[ct.size() - 2];
            if (second.first > 0.0 && std::fabs((top.first - second.first) / second.first) <= cfg.omega) {
                const double ideal = std::min(top.second, second.second);
                theta_s = std::max(1.0, ideal / theta_min);
            }
        }
        if (candidate() != evaluated) gain_c = Ewma();  // a new candidate CF starts its own average
    }
};

extern "C" {

int gravac_controller_create(const gravac_controller_config* c, gravac_controller** out)
{
    if (out) *out = nullptr;
    if (!c || !out) return GRAVAC_ERR_INVALID_ARG;
    const bool ok = std::isfinite(c->theta_min) && std::isfinite(c->theta_max) && c->theta_min >= 1.0 &&
                    c->theta_max >= c->theta_min && c->epsilon > 0.0 && c->epsilon <= 1.0 && std::isfinite(c->omega) &&
                    c->omega >= 0.0 && std::isfinite(c->theta_s) && c->theta_s >= 1.0 && c->alpha > 0.0 &&
                    c->alpha <= 1.0 && std::isfinite(c->samples_per_iteration) && c->samples_per_iteration > 0.0 &&
                    c->window >= 1 &&
                    (c->policy == GRAVAC_POLICY_EXPONENTIAL || c->policy == GRAVAC_POLICY_GEOMETRIC) && c->reserved == 0;
    if (!ok) return GRAVAC_ERR_INVALID_ARG;
    gravac_controller* g = new (std::nothrow) gravac_controller();
    if (!g) return GRAVAC_ERR_INVALID_ARG;
    g->cfg = *c;
    g->theta_min = c->theta_min;
    g->theta_s = c->theta_s;
    *out = g;
    return GRAVAC_OK;
}

void gravac_controller_destroy(gravac_controller* c) { delete c; }

int gravac_controller_candidates(const gravac_controller* c, double* theta_min, double* theta_c, double* cf_rel)
{
    if (!c) return GRAVAC_ERR_INVALID_ARG;
    const double cand = c->candidate();
    if (theta_min) *theta_min = c->theta_min;
    if (theta_c) *theta_c = cand;
    if (cf_rel) *cf_rel = cand / c->theta_min;
    return GRAVAC_OK;
}

int gravac_controller_decide(gravac_controller* c, double gain_min, double gain_c, int32_t* choice, double* delta_min,
                             double* delta_c)
{
    if (!c || !choice || c->decided) return GRAVAC_ERR_INVALID_ARG;
    if (!std::isfinite(gain_min) || !std::isfinite(gain_c) || gain_min < 0.0 || gain_c < 0.0) return GRAVAC_ERR_INVALID_ARG;
    const double dmin = c->gain_min.push(gain_min, c->cfg.alpha);
    const double dc = c->gain_c.push(gain_c, c->cfg.alpha);
    if (dc >= c->cfg.epsilon)
        c->choice = GRAVAC_SEND_CANDIDATE;
    else if (dmin >= c->cfg.epsilon)
        c->choice = GRAVAC_SEND_MIN;
    else
        c->choice = GRAVAC_SEND_DENSE;
    c->decided = true;
    *choice = c->choice;
    if (delta_min) *delta_min = dmin;
    if (delta_c) *delta_c = dc;
    return GRAVAC_OK;
}

int gravac_controller_finish_iteration(gravac_controller* c, double t_iter, double* theta_s_out)
{
    if (!c || !c->decided || !(t_iter > 0.0) || !std::isfinite(t_iter)) return GRAVAC_ERR_INVALID_ARG;
    // UpdateStep
    const double t_sys = c->cfg.samples_per_iteration / t_iter;
    if (c->choice == GRAVAC_SEND_CANDIDATE)
        c->t_compress[c->candidate()] = t_sys * c->gain_c.value;
    else if (c->choice == GRAVAC_SEND_MIN)
        c->t_compress[c->theta_min] = t_sys * c->gain_min.value;
    else
        c->t_compress[1.0] = t_sys;
    c->decided = false;
    c->iteration += 1;
    if (c->iteration % c->cfg.window == 0) c->evaluate();
    if (theta_s_out) *theta_s_out = c->theta_s;
    return GRAVAC_OK;
}

int gravac_controller_throughput(const gravac_controller* c, double cf, double* t_compress)
{
    if (!c || !t_compress) return GRAVAC_ERR_INVALID_ARG;
    const auto it = c->t_compress.find(cf);
    if (it == c->t_compress.end()) return GRAVAC_ERR_INVALID_ARG;
    *t_compress = it->second;
    return GRAVAC_OK;
}

int64_t gravac_controller_iteration(const gravac_controller* c) { return c ? c->iteration : -1; }

}  // extern "C"
