// Host-side time-cost model of CD-SGD (Sec. 2.1-2.3 eq. 2, 4, 5; Sec. 3.3 eq. 6-9).
// The savings are taken from the case tables of eq. 8 and eq. 9 as printed, not
// as differences of the iteration times, so that the two can be checked
// against each other.
#include <cmath>

#include "cdsgd_cost_model.h"

namespace {

bool ok_time(double x) { return std::isfinite(x) && x >= 0.0; }

bool ok_params(const cdsgd_cost_params *p)
{
    return p && p->k >= 1 && ok_time(p->tau) && ok_time(p->phi) && ok_time(p->psi) && ok_time(p->delta);
}

}  // namespace

extern "C" {

int cdsgd_cost_iteration(const cdsgd_cost_params *p, long i, cdsgd_cost *out)
{
    if (!ok_params(p) || !out || i < 0) return 3;
    const double tau = p->tau, phi = p->phi, comp = p->delta + p->psi;
    const bool correction = (i % p->k) == 0;
    out->t_ssgd = tau + phi;
    out->t_loc = tau > phi ? tau : phi;
    out->t_bit = tau + p->delta + p->psi;  // eq. 5, summed as written
    out->phi_cd = correction ? phi : comp;
    out->t_cd = tau > out->phi_cd ? tau : out->phi_cd;
    out->eq9_assumption_holds = comp <= phi ? 1 : 0;
    // eq. 8
    if (tau > out->phi_cd) {
        out->case_bit = 1;
        out->save_vs_bit = comp;
    } else if (!correction) {
        out->case_bit = 2;
        out->save_vs_bit = tau;
    } else {
        out->case_bit = 3;
        out->save_vs_bit = tau + comp - phi;
    }
    // eq. 9 (cases are tried in the printed order)
    if (tau > phi) {
        out->case_loc = 1;
        out->save_vs_loc = 0.0;
    } else if (tau > out->phi_cd) {
        out->case_loc = 2;
        out->save_vs_loc = phi - tau;
    } else if (!correction) {
        out->case_loc = 3;
        out->save_vs_loc = phi - comp;
    } else {
        out->case_loc = 4;
        out->save_vs_loc = 0.0;
    }
    return 0;
}

int cdsgd_cost_period_mean(const cdsgd_cost_params *p, cdsgd_cost *out)
{
    if (!ok_params(p) || !out) return 3;
    cdsgd_cost acc = {};
    for (long i = 0; i < p->k; ++i) {
        cdsgd_cost c;
        const int rc = cdsgd_cost_iteration(p, i, &c);
        if (rc) return rc;
        acc.t_ssgd += c.t_ssgd;
        acc.t_loc += c.t_loc;
        acc.t_bit += c.t_bit;
        acc.phi_cd += c.phi_cd;
        acc.t_cd += c.t_cd;
        acc.save_vs_bit += c.save_vs_bit;
        acc.save_vs_loc += c.save_vs_loc;
        acc.eq9_assumption_holds = c.eq9_assumption_holds;
    }
    const double k = (double)p->k;
    out->t_ssgd = acc.t_ssgd / k;
    out->t_loc = acc.t_loc / k;
    out->t_bit = acc.t_bit / k;
    out->phi_cd = acc.phi_cd / k;
    out->t_cd = acc.t_cd / k;
    out->save_vs_bit = acc.save_vs_bit / k;
    out->save_vs_loc = acc.save_vs_loc / k;
    out->case_bit = 0;
    out->case_loc = 0;
    out->eq9_assumption_holds = acc.eq9_assumption_holds;
    return 0;
}

}  // extern "C"
