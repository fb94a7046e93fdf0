// Performance model and plan search of decoupled speculation (paper: Section 4.1, "Modeling TGS" and
// Algorithm 1).  Host-only: a few hundred double-precision operations per call.
#include <cmath>
#include <limits>
#include <vector>
#include "../../include/specverify_plan.h"

namespace {

inline bool prob_ok(double p) { return p >= 0.0 && p <= 1.0; }
inline double at(const sv_affine& f, double b) { return b * f.slope + f.icpt; }

double tau_of(double p, int w) {
    double partial = 0.0;
    for (int a = 0; a < w; ++a) partial += std::pow(p, a) * (1.0 - p) * ((a + 1) / 2.0);
    return partial + w * std::pow(p, w);
}

inline double tgs_of(double p, int w, const sv_affine& D, const sv_affine& V, double b) {
    const double draft = w * at(D, b), verify = at(V, b);
    return tau_of(p, w) / (draft > verify ? draft : verify);
}

int window_bound(const sv_affine& D, const sv_affine& V_largest, int W) {
    bool any = false;
    double m = 0.0;
    if (D.slope > 0) { m = std::ceil(V_largest.slope / D.slope); any = true; }
    if (D.icpt > 0) {
        const double c = std::ceil(V_largest.icpt / D.icpt);
        m = any ? (c > m ? c : m) : c;
        any = true;
    }
    if (!any) return W;
    if (m < 1.0) return 1;
    return m > W ? W : (int)m;
}

}  // namespace

extern "C" double sv_plan_accept_prob(double p, int a, int w) {
    if (w < 1 || a < 0 || a > w) return std::numeric_limits<double>::quiet_NaN();
    return a < w ? std::pow(p, a) * (1.0 - p) : std::pow(p, w);
}

extern "C" double sv_plan_tau(double p, int w) {
    if (w < 1) return std::numeric_limits<double>::quiet_NaN();
    return tau_of(p, w);
}

// The plan search (what Algorithm 1 of Section 4.1 computes): every (verifier configuration, drafter size) pair
// fixes a per-worker batch; every such pair is expanded into the draft windows worth trying; each resulting
// candidate is scored by the speed model; the best-scoring candidate wins, the earliest among equals.
namespace {

struct Deployment {        // a verifier configuration paired with a drafter size
    int config, g_d, g_v, batch, windows;
};

// All deployments in visiting order (configurations as given, drafter sizes ascending), each with the per-worker
// batch it implies and the number of windows to try for it.
std::vector<Deployment> enumerate_deployments(const sv_plan_input& in) {
    std::vector<Deployment> all;
    for (int c = 0; c < in.n_configs; ++c) {
        const sv_affine& widest = in.V[(long long)c * in.W + in.W - 1];
        for (int g_d = 1; g_d <= in.g_v[c]; ++g_d) {
            const long long workers_times_batch = (long long)(g_d + in.g_v[c]) * in.B;
            all.push_back({c, g_d, in.g_v[c], (int)((workers_times_batch + in.G - 1) / in.G),
                           window_bound(in.D[g_d - 1], widest, in.W)});
        }
    }
    return all;
}

}  // namespace

extern "C" int sv_plan_decoupled(const sv_plan_input* in, sv_plan* out) {
    if (!in || !out || !in->g_v || !in->D || !in->V) return SV_EINVAL;
    if (in->B < 1 || in->G < 1 || in->W < 1 || in->n_configs < 1 || !prob_ok(in->p)) return SV_EINVAL;
    for (int c = 0; c < in->n_configs; ++c)
        if (in->g_v[c] < 1) return SV_EINVAL;
    struct Scored { const Deployment* d; int w; double speed; };
    const std::vector<Deployment> deployments = enumerate_deployments(*in);
    std::vector<Scored> scored;
    for (const Deployment& d : deployments)
        for (int w = 1; w <= d.windows; ++w)
            scored.push_back({&d, w, tgs_of(in->p, w, in->D[d.g_d - 1], in->V[(long long)d.config * in->W + w - 1], (double)d.batch)});
    const Scored* winner = nullptr;                       // first of the largest positive speeds
    for (const Scored& s : scored)
        if (s.speed > (winner ? winner->speed : 0.0)) winner = &s;
    if (winner) *out = {winner->d->g_d, winner->d->g_v, winner->w, winner->d->batch, winner->speed};
    else *out = {0, 0, 0, 0, 0.0};
    return SV_OK;
}

extern "C" int sv_plan_best_window(double p, sv_affine D, const sv_affine* V, int W, double b, int* w_out, double* tgs_out) {
    if (!V || !w_out || !tgs_out || W < 1 || !prob_ok(p)) return SV_EINVAL;
    int bw = 0;
    double bt = 0.0;
    for (int w = 1; w <= W; ++w) {
        const double t = tgs_of(p, w, D, V[w - 1], b);
        if (t > bt) { bw = w; bt = t; }
    }
    *w_out = bw;
    *tgs_out = bt;
    return SV_OK;
}

extern "C" int sv_fit_affine(const double* b, const double* t, int n, sv_affine* out) {
    if (!b || !t || !out || n < 2) return SV_EINVAL;
    double mb = 0.0, mt = 0.0;
    for (int i = 0; i < n; ++i) { mb += b[i]; mt += t[i]; }
    mb /= n; mt /= n;
    double sbb = 0.0, sbt = 0.0;
    for (int i = 0; i < n; ++i) { sbb += (b[i] - mb) * (b[i] - mb); sbt += (b[i] - mb) * (t[i] - mt); }
    if (sbb == 0.0) return SV_EINVAL;
    out->slope = sbt / sbb;
    out->icpt = mt - out->slope * mb;
    return SV_OK;
}
