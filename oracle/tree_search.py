"""Plain-Python oracle of the paper's test-time tree search and draft verification (test
infrastructure only; shares nothing with the library).

Sec. 4.2, Eq. 1: at round t the policy plays k* = argmax_k rhat_k + lambda_UCB sqrt(2 ln t / n_k),
rhat_k the mean reward of arm k so far.  Eq. 2 and the appendix on reward modeling: the reward of
the played arm is the negated inverse speed-up, r = -(1/N_accept + lambda_gamma gamma/N_accept).
Appendix, verification algorithm: token t is accepted when u < min(1, p_t/q_t); at the first
rejection a token is drawn from (p - q)_+ (sampling) or from the one-hot target (greedy) and the
loop stops; when all gamma tokens are accepted one more is drawn from the target's next
distribution.  Readings: an arm that was never played is played first (lowest index first); ties
go to the lowest index; a draw uses the inverse CDF in vocabulary order with the uniform passed in.
"""
import math


def reward(n_accept, gamma, lambda_gamma):
    return -(1.0 / n_accept + lambda_gamma * gamma / n_accept)


class Bandit:
    def __init__(self, n_arms, lambda_ucb, lambda_gamma):
        self.n_arms, self.lambda_ucb, self.lambda_gamma = n_arms, lambda_ucb, lambda_gamma
        self.t = 0
        self.n = [0] * n_arms
        self.reward_sum = [0.0] * n_arms

    def select(self):
        for k in range(self.n_arms):
            if self.n[k] == 0:
                return k
        t = self.t + 1
        scores = [self.reward_sum[k] / self.n[k] + self.lambda_ucb * math.sqrt(2.0 * math.log(t) / self.n[k])
                  for k in range(self.n_arms)]
        return max(range(self.n_arms), key=lambda k: (scores[k], -k))

    def update(self, arm, n_accept, gamma):
        self.t += 1
        self.n[arm] += 1
        self.reward_sum[arm] += reward(n_accept, gamma, self.lambda_gamma)


def _draw(weights, u):
    total = float(sum(weights))
    acc, last = 0.0, 0
    for v, w in enumerate(weights):
        if w <= 0.0:
            continue
        acc += float(w)
        last = v
        if u * total < acc:
            return v
    return last


def verify(p, q, draft, u_accept, u_sample, greedy):
    """p: (gamma+1) rows of V probabilities, q: gamma rows, draft: gamma tokens -> list of tokens."""
    gamma = len(draft)
    out = []
    for t in range(gamma):
        pr, qr, tok = list(map(float, p[t])), list(map(float, q[t])), int(draft[t])
        top = max(range(len(pr)), key=lambda v: (pr[v], -v))
        pt = (1.0 if top == tok else 0.0) if greedy else pr[tok]
        qt = qr[tok]
        ratio = pt / qt if qt > 0.0 else (1.0 if pt > 0.0 else 0.0)
        if float(u_accept[t]) < min(1.0, ratio):
            out.append(tok)
            continue
        if greedy:
            out.append(top)
        else:
            resid = [max(a - b, 0.0) for a, b in zip(pr, qr)]
            out.append(_draw(resid if sum(resid) > 0.0 else pr, float(u_sample)))
        return out
    last = list(map(float, p[gamma]))
    out.append(max(range(len(last)), key=lambda v: (last[v], -v)) if greedy else _draw(last, float(u_sample)))
    return out
