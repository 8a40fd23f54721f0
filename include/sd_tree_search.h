/*
 * sd_tree_search.h - host-side logic of test-time tree search and draft verification.
 *
 * Plain host arithmetic (no GPU work, HOST pointers only) for the part of the paper that picks
 * the draft tree and accepts draft tokens:
 *   - the multi-armed bandit over a set of tree configurations with the UCB policy (Sec. 4.2,
 *     Eq. 1): k* = argmax_k  rhat_k + lambda_UCB * sqrt(2 ln t / n_k);
 *   - the reward of a round (Sec. 4.2, Eq. 2 and the appendix on reward modeling):
 *     r = -(1 / N_accept + lambda_gamma * gamma / N_accept), the negated inverse speed-up;
 *   - the verification of a draft sequence against the target model's probabilities, greedy or
 *     sampling (appendix, verification algorithm): accept token t while u_t < min(1, p_t / q_t);
 *     at the first rejection draw from the one-hot target (greedy) or from (p - q)_+ normalized
 *     (sampling) and stop; if every token is accepted draw one more from p_{gamma+1}.
 * Readings where the paper is silent: rhat_k is the MEAN reward of the rounds in which arm k was
 * played; an arm never played yet is played first (lowest index first), which is what the UCB
 * bonus going to infinity means; ties go to the lowest index; lambda_UCB and lambda_gamma are
 * parameters (the paper gives no values); N_accept = 0 cannot occur (a round always yields at
 * least the token drawn at the first rejection), so N_accept counts that token too and the
 * functions reject N_accept < 1.  All random numbers are inputs.
 * Return values: 0 on success, the negative mamba_status_t codes of mamba_hip.h on bad arguments.
 */
#ifndef SD_TREE_SEARCH_H
#define SD_TREE_SEARCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SD_MAX_ARMS 32

typedef struct {
    int32_t n_arms;                 /* K tree configurations                      */
    int64_t t;                      /* rounds played so far                       */
    int64_t n[SD_MAX_ARMS];         /* n_k: rounds in which arm k was played      */
    double reward_sum[SD_MAX_ARMS]; /* sum of the rewards arm k received          */
    double lambda_ucb;
    double lambda_gamma;
} sd_bandit_t;

int sd_bandit_init(sd_bandit_t *b, int n_arms, double lambda_ucb, double lambda_gamma);

/* Eq. 1 at round t + 1 (the round about to be played).  Writes the chosen arm to *arm. */
int sd_bandit_select(const sd_bandit_t *b, int32_t *arm);

/* Eq. 2 for the arm that was played: -(1 + lambda_gamma * gamma) / n_accept.  */
int sd_reward(int64_t n_accept, int32_t gamma, double lambda_gamma, double *reward);

/* Record a finished round: arm played, tokens it yielded, draft length of its tree. */
int sd_bandit_update(sd_bandit_t *b, int32_t arm, int64_t n_accept, int32_t gamma);

/*
 * Verification of one draft sequence.
 *   p: (gamma + 1, V) target probabilities, row t for position t (row gamma = the extra token);
 *   q: (gamma, V) drafter probabilities; draft: int32[gamma] draft tokens;
 *   u_accept: float[gamma] uniforms of the acceptance tests;
 *   u_sample: one uniform used for the token drawn at a rejection or as the extra token
 *             (inverse-CDF over the vocabulary in index order; unused when greedy);
 *   greedy: nonzero = the target is taken one-hot at its argmax (lowest index on ties).
 * Writes the accepted tokens followed by the drawn token to out_tokens (room for gamma + 1)
 * and their count to *n_out (1 .. gamma + 1).
 */
int sd_verify(const float *p, const float *q, const int32_t *draft, const float *u_accept,
              float u_sample, int32_t gamma, int64_t V, int greedy, int32_t *out_tokens,
              int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* SD_TREE_SEARCH_H */
