// Goodput-efficiency planner (paper Sec. 3.3.1): host-only code.
//
// Per control window the global scheduler scores, for every SLO tier and every
// (prefill TP, decode TP) pair of a small TP set, a balanced block of P prefill
// and D decode instances with Eq. 1, GE = min(P*THP, rps) / (P*TPi + D*TPj), and
// hands out the GPU pool greedily by the weighted score GE * rps / served_rps.
// The integer details the paper leaves open are fixed as follows: a block is the
// (P, D) in 1..max_inst with the closest stage rates (ties: fewer instances, then
// smaller P) and serves min(P*THP, D*THD); Eq. 1 is taken as printed (prefill rate
// only in the numerator) on the block's P, D with the tier's unmet rate; a
// tier that has been given nothing yet outranks the others; ties go to larger GE,
// then lower tier, lower prefill TP, lower decode TP; a step gives one block to
// the best configuration that fits, until no demand is unmet or nothing fits.
// The paper's scheduler is multi-threaded; this search is a few thousand scalar
// evaluations, so one thread finishes it in microseconds.
#include <math.h>

#include <vector>

#include "nitsum_kvmig.h"

namespace {

const int kTp[NTS_TP_LEVELS] = {1, 2, 4, 8};

void balanced_block(double thp, double thd, int max_inst, int *P_out, int *D_out)
{
    double best_gap = 0;
    int best_P = 0, best_D = 0;
    for (int P = 1; P <= max_inst; ++P)
        for (int D = 1; D <= max_inst; ++D) {
            const double a = P * thp, b = D * thd;
            const double gap = fabs(a - b) / (a > b ? a : b);
            bool better = best_P == 0;
            if (!better) {
                if (gap != best_gap) better = gap < best_gap;
                else if (P + D != best_P + best_D) better = P + D < best_P + best_D;
                else better = P < best_P;
            }
            if (better) {
                best_gap = gap;
                best_P = P;
                best_D = D;
            }
        }
    *P_out = best_P;
    *D_out = best_D;
}

inline double block_rate(double thp, double thd, int P, int D)
{
    const double a = P * thp, b = D * thd;
    return a < b ? a : b;
}

}  // namespace

extern "C" {

int nts_balanced_block(double thp, double thd, int max_inst, int *P, int *D)
{
    if (!P || !D || !(thp > 0) || !(thd > 0) || max_inst < 1) return NTS_EINVAL;
    balanced_block(thp, thd, max_inst, P, D);
    return NTS_OK;
}

int nts_goodput_efficiency(double thp, int tpi, double thd, int tpj, int P, int D, double rps, double *ge)
{
    if (!ge || tpi < 1 || tpj < 1 || P < 1 || D < 1 || !(thp > 0) || !(thd > 0) || !(rps >= 0)) return NTS_EINVAL;
    const double r = P * thp;                       // Eq. 1: the prefill rate only
    *ge = (r < rps ? r : rps) / double(P * tpi + D * tpj);
    return NTS_OK;
}

int nts_plan_cluster(int n_gpus, int n_tiers, const nts_tier *tiers, int max_inst, nts_alloc *out,
                     int max_out, int *n_out, int *gpus_left)
{
    if (n_gpus < 0 || n_tiers < 0 || (n_tiers > 0 && !tiers) || max_inst < 1 || !n_out || !gpus_left ||
        max_out < 0 || (max_out > 0 && !out))
        return NTS_EINVAL;
    for (int k = 0; k < n_tiers; ++k) {
        if (!(tiers[k].rps >= 0)) return NTS_EINVAL;
        for (int i = 0; i < NTS_TP_LEVELS; ++i)
            if (!(tiers[k].thp[i] >= 0) || !(tiers[k].thd[i] >= 0)) return NTS_EINVAL;
    }
    struct Cfg { int k, i, j, P, D, gpus; double rate, prefill; };   // rate: what a block serves
    std::vector<Cfg> cfgs;
    std::vector<double> served;
    try {
        served.assign(size_t(n_tiers), 0.0);
        for (int k = 0; k < n_tiers; ++k)
            for (int i = 0; i < NTS_TP_LEVELS; ++i)
                for (int j = 0; j < NTS_TP_LEVELS; ++j) {
                    const double thp = tiers[k].thp[i], thd = tiers[k].thd[j];
                    if (!(thp > 0) || !(thd > 0)) continue;
                    Cfg c;
                    c.k = k; c.i = i; c.j = j;
                    balanced_block(thp, thd, max_inst, &c.P, &c.D);
                    c.gpus = c.P * kTp[i] + c.D * kTp[j];
                    c.rate = block_rate(thp, thd, c.P, c.D);
                    c.prefill = c.P * thp;
                    cfgs.push_back(c);
                }
    } catch (...) {
        return NTS_ENOMEM;
    }
    int left = n_gpus, n = 0;
    for (;;) {
        const Cfg *best = nullptr;
        bool b_fresh = false;
        double b_wge = 0, b_ge = 0;
        for (const Cfg &c : cfgs) {               // enumeration order = (tier, prefill TP, decode TP) ascending
            const double unmet = tiers[c.k].rps - served[c.k];
            if (!(unmet > 0) || c.gpus > left) continue;
            const double ge = (c.prefill < unmet ? c.prefill : unmet) / double(c.gpus);
            const bool fresh = served[c.k] == 0.0;
            const double wge = fresh ? ge : ge * (tiers[c.k].rps / served[c.k]);
            bool better = best == nullptr;
            if (!better) {
                if (fresh != b_fresh) better = fresh;
                else if (wge != b_wge) better = wge > b_wge;
                else better = ge > b_ge;          // full tie: the earlier (lower tier / TP) one stays
            }
            if (better) {
                best = &c;
                b_fresh = fresh;
                b_wge = wge;
                b_ge = ge;
            }
        }
        if (!best) break;
        const double unmet = tiers[best->k].rps - served[best->k];
        const double got = best->rate < unmet ? best->rate : unmet;
        if (n < max_out) {
            nts_alloc a;
            a.tier = best->k;
            a.tp_prefill = kTp[best->i];
            a.tp_decode = kTp[best->j];
            a.P = best->P;
            a.D = best->D;
            a.gpus = best->gpus;
            a.served_rps = got;
            out[n] = a;
        }
        ++n;
        served[best->k] += got;
        left -= best->gpus;
    }
    *n_out = n;
    *gpus_left = left;
    return n > max_out ? NTS_ERANGE : NTS_OK;
}

}  // extern "C"
