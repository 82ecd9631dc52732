// Host-only planner: cost model and strategy search of MoNTA's section "Network-traffic-aware"
// (Eq. 8-11, Algorithms 1-3).  No GPU work; included by monta.hip so that it ships in the same library.
#pragma once

#include <cmath>
#include <limits>

#include "monta.h"

namespace monta_planner {

inline bool curve_ok(const monta_curve &c)
{
    if (!c.volume || !c.eff || c.n < 1) return false;
    for (int i = 0; i < c.n; ++i) {
        if (!(c.eff[i] > 0.0) || !std::isfinite(c.eff[i]) || !std::isfinite(c.volume[i])) return false;
        if (i && !(c.volume[i] > c.volume[i - 1])) return false;
    }
    return true;
}

// efficiency at a volume: linear between samples, constant outside them
inline double lookup(const monta_curve &c, double v)
{
    if (v <= c.volume[0]) return c.eff[0];
    if (v >= c.volume[c.n - 1]) return c.eff[c.n - 1];
    int hi = 1;
    while (c.volume[hi] <= v) ++hi;
    const double x0 = c.volume[hi - 1], x1 = c.volume[hi];
    return c.eff[hi - 1] + (c.eff[hi] - c.eff[hi - 1]) * (v - x0) / (x1 - x0);
}

inline int validate(const monta_plan_in *in)
{
    if (!in) return MONTA_ERR_NULL;
    if (!(in->traffic > 0.0) || !std::isfinite(in->traffic) || in->t < 1 || in->e < 1 || in->n_max < 1)
        return MONTA_ERR_INVALID;
    if (!(in->b1 > 0.0) || !(in->b2 > 0.0) || !(in->b3 > 0.0) || !(in->i_minimal >= 0.0)) return MONTA_ERR_INVALID;
    if (!curve_ok(in->r1) || !curve_ok(in->r2) || !curve_ok(in->r3)) return MONTA_ERR_INVALID;
    return MONTA_OK;
}

struct Chunk {
    double aa, ag, d2d;
};

// Eq. 8, 9, 10: one of n chunks; r1 is looked up at I/(n*t), r2 and r3 at I/n
inline Chunk chunk_times(const monta_plan_in &in, int n)
{
    const double I = in.traffic, t = in.t, e = in.e;
    Chunk c;
    c.aa = I / (n * t) * (e - 1.0) / e / (in.b1 * lookup(in.r1, I / (n * t)));
    c.ag = I / n * (t - 1.0) / t / (in.b2 * lookup(in.r2, I / n));
    c.d2d = I / n / (in.b3 * lookup(in.r3, I / n));
    return c;
}

// total time of the n-chunk pipeline; Algorithm 1 keeps the D2D copy inside the gather stage,
// Algorithm 2 pipelines it as well and pays it once
inline double chunked_time(const monta_plan_in &in, int n, bool o3)
{
    const Chunk c = chunk_times(in, n);
    if (!o3) return c.aa < c.ag + c.d2d ? c.aa + (c.ag + c.d2d) * n : c.aa * n + c.ag + c.d2d;
    return c.aa < c.ag ? c.aa + c.ag * n + c.d2d : c.aa * n + c.ag + c.d2d;
}

inline void search(const monta_plan_in &in, bool o3, int *best_n, double *best_t)
{
    *best_n = 0;
    *best_t = std::numeric_limits<double>::infinity();
    for (int n = 1; n <= in.n_max; ++n) {
        if (in.traffic / ((double)n * in.t) < in.i_minimal || in.traffic / n < in.i_minimal) break;
        const double tt = chunked_time(in, n, o3);
        if (tt < *best_t) {
            *best_t = tt;
            *best_n = n;
        }
    }
}

}  // namespace monta_planner

extern "C" int monta_plan_chunk_times(const monta_plan_in *in, int n, double *aa, double *ag, double *d2d)
{
    int rc = monta_planner::validate(in);
    if (rc) return rc;
    if (n < 1) return MONTA_ERR_INVALID;
    const monta_planner::Chunk c = monta_planner::chunk_times(*in, n);
    if (aa) *aa = c.aa;
    if (ag) *ag = c.ag;
    if (d2d) *d2d = c.d2d;
    return MONTA_OK;
}

extern "C" int monta_plan_strategy(const monta_plan_in *in, monta_plan_out *out)
{
    int rc = monta_planner::validate(in);
    if (rc) return rc;
    if (!out) return MONTA_ERR_NULL;
    const double I = in->traffic, t = in->t, e = in->e;
    out->t_base = I * (e - 1.0) / e / (in->b1 * monta_planner::lookup(in->r1, I));
    // Eq. 11: r1 at I/t, r2 at I
    out->t_o1 = I / t * (e - 1.0) / e / (in->b1 * monta_planner::lookup(in->r1, I / t)) +
                I * (t - 1.0) / t / (in->b2 * monta_planner::lookup(in->r2, I));
    monta_planner::search(*in, false, &out->n_o2, &out->t_o2);
    monta_planner::search(*in, true, &out->n_o3, &out->t_o3);
    out->strategy = 1;
    out->chunks = 1;
    out->t_best = out->t_o1;
    if (out->t_o2 < out->t_best) {
        out->strategy = 2;
        out->chunks = out->n_o2;
        out->t_best = out->t_o2;
    }
    if (out->t_o3 < out->t_best) {
        out->strategy = 3;
        out->chunks = out->n_o3;
        out->t_best = out->t_o3;
    }
    return MONTA_OK;
}
