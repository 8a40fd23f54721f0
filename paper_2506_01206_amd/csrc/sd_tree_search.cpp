// Host-side test-time tree search (UCB bandit over tree configurations, Sec. 4.2 Eq. 1-2) and the
// draft verification rule (appendix, verification algorithm).  No GPU work.
#include "../../include/sd_tree_search.h"

#include <math.h>

namespace {
constexpr int kOk = 0, kNull = -1, kBadShape = -2;

int64_t argmax_row(const float *row, int64_t V)
{
    int64_t best = 0;
    for (int64_t v = 1; v < V; ++v)
        if (row[v] > row[best]) best = v;
    return best;
}

// inverse CDF over weights w[v] >= 0 in index order; u in [0, 1)
template <typename F> int64_t draw(F weight, int64_t V, double u)
{
    double total = 0.0;
    for (int64_t v = 0; v < V; ++v) total += weight(v);
    if (!(total > 0.0)) return -1;
    const double target = u * total;
    double acc = 0.0;
    int64_t last = 0;
    for (int64_t v = 0; v < V; ++v) {
        const double w = weight(v);
        if (w <= 0.0) continue;
        acc += w;
        last = v;
        if (target < acc) return v;
    }
    return last;  // u == 1 or rounding at the end of the table
}
}  // namespace

extern "C" {

int sd_bandit_init(sd_bandit_t *b, int n_arms, double lambda_ucb, double lambda_gamma)
{
    if (!b) return kNull;
    if (n_arms < 1 || n_arms > SD_MAX_ARMS || !(lambda_ucb >= 0.0) || !(lambda_gamma >= 0.0)) return kBadShape;
    b->n_arms = n_arms;
    b->t = 0;
    for (int k = 0; k < SD_MAX_ARMS; ++k) {
        b->n[k] = 0;
        b->reward_sum[k] = 0.0;
    }
    b->lambda_ucb = lambda_ucb;
    b->lambda_gamma = lambda_gamma;
    return kOk;
}

int sd_bandit_select(const sd_bandit_t *b, int32_t *arm)
{
    if (!b || !arm) return kNull;
    if (b->n_arms < 1 || b->n_arms > SD_MAX_ARMS) return kBadShape;
    for (int k = 0; k < b->n_arms; ++k)
        if (b->n[k] == 0) {
            *arm = k;
            return kOk;
        }
    const double t = (double)(b->t + 1);
    int best = 0;
    double best_score = 0.0;
    for (int k = 0; k < b->n_arms; ++k) {
        const double mean = b->reward_sum[k] / (double)b->n[k];
        const double score = mean + b->lambda_ucb * sqrt(2.0 * log(t) / (double)b->n[k]);
        if (k == 0 || score > best_score) {
            best = k;
            best_score = score;
        }
    }
    *arm = best;
    return kOk;
}

int sd_reward(int64_t n_accept, int32_t gamma, double lambda_gamma, double *reward)
{
    if (!reward) return kNull;
    if (n_accept < 1 || gamma < 1) return kBadShape;
    *reward = -(1.0 / (double)n_accept + lambda_gamma * (double)gamma / (double)n_accept);
    return kOk;
}

int sd_bandit_update(sd_bandit_t *b, int32_t arm, int64_t n_accept, int32_t gamma)
{
    if (!b) return kNull;
    if (arm < 0 || arm >= b->n_arms) return kBadShape;
    double r;
    const int st = sd_reward(n_accept, gamma, b->lambda_gamma, &r);
    if (st != kOk) return st;
    b->t += 1;
    b->n[arm] += 1;
    b->reward_sum[arm] += r;
    return kOk;
}

int sd_verify(const float *p, const float *q, const int32_t *draft, const float *u_accept,
              float u_sample, int32_t gamma, int64_t V, int greedy, int32_t *out_tokens, int32_t *n_out)
{
    if (!p || !q || !draft || !u_accept || !out_tokens || !n_out) return kNull;
    if (gamma < 1 || V < 1) return kBadShape;
    for (int32_t t = 0; t < gamma; ++t)
        if (draft[t] < 0 || draft[t] >= V) return kBadShape;
    int32_t n = 0;
    for (int32_t t = 0; t < gamma; ++t) {
        const float *pr = p + (int64_t)t * V, *qr = q + (int64_t)t * V;
        const int64_t tok = draft[t];
        const double pt = greedy ? (argmax_row(pr, V) == tok ? 1.0 : 0.0) : (double)pr[tok];
        const double qt = (double)qr[tok];
        // u < min(1, p_t / q_t); a token the drafter gave zero probability cannot have been drafted
        const double ratio = qt > 0.0 ? pt / qt : (pt > 0.0 ? 1.0 : 0.0);
        if ((double)u_accept[t] < (ratio < 1.0 ? ratio : 1.0)) {
            out_tokens[n++] = (int32_t)tok;
            continue;
        }
        int64_t repl;
        if (greedy) {
            repl = argmax_row(pr, V);
        } else {
            repl = draw([&](int64_t v) { const double d = (double)pr[v] - (double)qr[v]; return d > 0.0 ? d : 0.0; },
                        V, (double)u_sample);
            if (repl < 0) repl = draw([&](int64_t v) { return (double)pr[v]; }, V, (double)u_sample);  // p == q
            if (repl < 0) return kBadShape;
        }
        out_tokens[n++] = (int32_t)repl;
        *n_out = n;
        return kOk;
    }
    const float *pr = p + (int64_t)gamma * V;
    int64_t extra = greedy ? argmax_row(pr, V) : draw([&](int64_t v) { return (double)pr[v]; }, V, (double)u_sample);
    if (extra < 0) return kBadShape;
    out_tokens[n++] = (int32_t)extra;
    *n_out = n;
    return kOk;
}

}  // extern "C"
