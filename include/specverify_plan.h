/*
 * specverify_plan -- the performance model and plan search that decide how a verifier built on this
 * library is fed: how many workers draft, how many verify, and how many drafts a verification window holds.
 *
 * Host-only arithmetic in double precision; no device work, no allocation, no state.  All pointers are HOST
 * pointers, borrowed for the duration of the call.  Return values are sv_status codes (specverify.h) unless
 * the function returns a double, in which case invalid arguments give NaN.
 *
 * The model is the one of the paper's Section 4.1 ("Modeling TGS"): with b requests in a batch, one token
 * of drafting takes D(b) = b D' + alpha and the verification of a window of w drafts V_w(b) = b V'_w + beta_w
 * (affine in b, fitted offline); drafter and verifier run concurrently, so a window costs
 * IL = max{ w D(b), V_w(b) }; each draft is accepted with probability p; and the expected number of tokens a
 * window yields is tau_w.  Token generation speed is TGS = tau_w / IL.
 */
#ifndef SPECVERIFY_PLAN_H
#define SPECVERIFY_PLAN_H

#include "specverify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* time(b) = slope * b + icpt */
typedef struct { double slope, icpt; } sv_affine;

/* P(a, w) of Section 4.1: exactly a of the w drafts of a window are accepted,
 *   p^a (1 - p) for 0 <= a <= w - 1,   p^w for a = w.   NaN unless 0 <= a <= w, w >= 1. */
double sv_plan_accept_prob(double p, int a, int w);

/* tau_w of Section 4.1, as printed: sum_{a=0}^{w-1} p^a (1-p) (a+1)/2 + w p^w, summed in ascending a.
 * NaN unless w >= 1. */
double sv_plan_tau(double p, int w);

/* Algorithm 1 (plan generation at the start of a rollout).
 *   B          global batch size;  G  GPUs in the cluster;  p  acceptance probability of one draft
 *   n_configs  size of the set of verifier configurations;  g_v[c]  GPUs of configuration c (>= 1)
 *   W          largest profiled draft window (>= 1)
 *   D[g-1]     drafting model of g drafter GPUs, g = 1 .. max_c g_v[c]
 *   V[c*W+w-1] verification model of configuration c for a window of w drafts
 * For every configuration c (in the given order), every g_d = 1 .. g_v[c] and every w = 1 .. w_max:
 * b = ceil((g_d + g_v) B / G), TGS = tau_w / max{ w D_{g_d}(b), V_{c,w}(b) }; the triple with the largest TGS
 * is returned, the first one met among equals.  w_max = max{ ceil(V'/D'), ceil(beta/alpha) } with V', beta
 * those of the largest profiled window W of the configuration (the printed bound refers to the window it
 * bounds), clipped to 1 .. W; a term whose denominator is not positive is left out, and with both left out
 * w_max = W.
 * out: the chosen g_d, g_v, w, the batch b it implies, and its TGS (all zero if no TGS is positive).
 * SV_EINVAL on null pointers, B, G, W, n_configs < 1, a g_v < 1, or p outside [0, 1]. */
typedef struct {
    int B, G;
    double p;
    int n_configs;
    const int *g_v;
    int W;
    const sv_affine *D;
    const sv_affine *V;
} sv_plan_input;
typedef struct { int g_d, g_v, w, b; double tgs; } sv_plan;
int sv_plan_decoupled(const sv_plan_input *in, sv_plan *out);

/* The window that maximises the decoupled TGS for acceptance probability p at batch b, w = 1 .. W, V[w-1]
 * the verification model of window w (what Algorithm 2 evaluates, at b = 1, for a request whose acceptance
 * rate has fallen behind the batch's).  First of equal maxima.  SV_EINVAL on null pointers, W < 1, p outside
 * [0, 1]. */
int sv_plan_best_window(double p, sv_affine D, const sv_affine *V, int W, double b, int *w_out, double *tgs_out);

/* Ordinary least-squares line through n >= 2 measured points (b[i], t[i]) with at least two distinct b:
 * how D', alpha, V', beta are obtained from a profile.  SV_EINVAL otherwise. */
int sv_fit_affine(const double *b, const double *t, int n, sv_affine *out);

#ifdef __cplusplus
}
#endif
#endif
