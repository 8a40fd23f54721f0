"""Host-side tree search (Sec. 4.2, Eq. 1 and Eq. 2) and verification (appendix algorithm): the
plain-Python oracle is pinned by hand-worked values and by the property that makes speculative
sampling exact, then the C implementation in the library is compared with the oracle."""
import math

import numpy as np
import pytest

from oracle import tree_search as ots


@pytest.fixture(scope="module")
def ts():
    from paper_2506_01206_amd import tree_search
    return tree_search


# ---------------------------------------------------------------- pins for the oracle
def test_reward_is_negated_inverse_speedup():
    # Eq. 2 with N_accept = 4, gamma = 5, lambda_gamma = 0.1: -(1/4 + 0.1 * 5/4) = -0.375
    assert ots.reward(4, 5, 0.1) == pytest.approx(-0.375, abs=1e-15)
    # appendix: 1/speedup = (1/N) T_target(gamma)/T_target + (gamma/N) T_draft/T_target with the first
    # ratio ~ 1 and the second = lambda_gamma; speedup for T_target = 10, T_draft = 1, gamma = 5, N = 3
    t_target, t_draft, gamma, n = 10.0, 1.0, 5, 3
    speedup = n * t_target / (t_target + gamma * t_draft)
    assert ots.reward(n, gamma, t_draft / t_target) == pytest.approx(-1.0 / speedup, rel=1e-14)
    # more accepted tokens or a shorter draft is better (larger reward)
    assert ots.reward(5, 5, 0.1) > ots.reward(4, 5, 0.1) > ots.reward(4, 6, 0.1)


def test_ucb_selection_hand_worked():
    # Eq. 1 at t = 5 with means (-0.4, -0.3), counts (3, 1), lambda_UCB = 0.5:
    #   arm 0: -0.4 + 0.5 sqrt(2 ln 5 / 3) = -0.4 + 0.5 * 1.03583 = 0.11792
    #   arm 1: -0.3 + 0.5 sqrt(2 ln 5 / 1) = -0.3 + 0.5 * 1.79412 = 0.59706   -> arm 1
    b = ots.Bandit(2, 0.5, 0.1)
    b.t, b.n, b.reward_sum = 4, [3, 1], [-1.2, -0.3]
    assert b.select() == 1
    assert -0.4 + 0.5 * math.sqrt(2 * math.log(5) / 3) == pytest.approx(0.11792, abs=1e-5)
    # with lambda_UCB = 0 it is pure exploitation; a huge bonus favours the least-played arm
    b.lambda_ucb = 0.0
    b.reward_sum = [-0.6, -0.5]            # means -0.2, -0.5
    assert b.select() == 0
    b.lambda_ucb = 100.0
    assert b.select() == 1
    # arms that were never played go first, in index order
    c = ots.Bandit(3, 0.5, 0.1)
    order = []
    for _ in range(3):
        k = c.select()
        order.append(k)
        c.update(k, 3, 5)
    assert order == [0, 1, 2] and c.t == 3 and c.n == [1, 1, 1]
    assert c.reward_sum[0] == pytest.approx(ots.reward(3, 5, 0.1))


def test_bandit_converges_to_the_best_arm():
    # arm 1 always yields more tokens for the same draft length: it must get most of the plays
    b = ots.Bandit(3, 0.2, 0.1)
    accepted = [2, 4, 3]
    for _ in range(300):
        k = b.select()
        b.update(k, accepted[k], 5)
    assert b.n[1] > 200 and sum(b.n) == 300


def output_distribution(verify, p, q, bins=200):
    """Exact-in-the-limit distribution of the first emitted token: the draft token is drawn from q
    (weights q[x]), u_accept and u_sample run over bin midpoints."""
    V = len(q[0])
    us = (np.arange(bins) + 0.5) / bins
    dist = np.zeros(V)
    for x in range(V):
        if q[0][x] == 0:
            continue
        for ua in us:
            # the rejection branch does not depend on ua beyond the accept test: one pass over u_sample
            first = verify(p, q, [x], [ua], 0.5, False)
            if first == [x, first[-1]] and len(first) == 2:        # accepted, extra token follows
                dist[x] += q[0][x] / bins
            else:
                for ub in us:
                    tok = verify(p, q, [x], [ua], ub, False)[0]
                    dist[tok] += q[0][x] / bins / bins
    return dist


def test_sampling_verification_reproduces_the_target_distribution():
    # speculative sampling emits tokens distributed exactly as the target p, whatever q is
    p = [[0.5, 0.2, 0.2, 0.1], [0.25, 0.25, 0.25, 0.25]]
    q = [[0.1, 0.6, 0.1, 0.2]]
    dist = output_distribution(ots.verify, p, q, bins=100)
    np.testing.assert_allclose(dist, p[0], atol=0.02)
    # acceptance probability of token x is min(1, p/q): token 1 (p/q = 1/3) at u = 0.30 and 0.40
    assert ots.verify(p, q, [1], [0.30], 0.0, False)[0] == 1
    assert ots.verify(p, q, [1], [0.40], 0.0, False)[0] != 1
    # the replacement comes from (p - q)_+ = (0.4, 0, 0.1, 0) / 0.5: u_sample 0.79 -> token 0, 0.81 -> token 2
    assert ots.verify(p, q, [1], [0.9], 0.79, False) == [0]
    assert ots.verify(p, q, [1], [0.9], 0.81, False) == [2]


def test_greedy_verification_follows_the_argmax():
    p = [[0.1, 0.7, 0.2], [0.6, 0.3, 0.1], [0.2, 0.2, 0.6]]
    q = [[0.3, 0.4, 0.3], [0.5, 0.25, 0.25]]
    # both draft tokens equal the target's argmax: both accepted (ratio 1/q >= 1), extra = argmax of row 2
    assert ots.verify(p, q, [1, 0], [0.99, 0.99], 0.3, True) == [1, 0, 2]
    # second token differs from the argmax: rejected whatever u is, replaced by the argmax, stop
    assert ots.verify(p, q, [1, 2], [0.0, 0.0], 0.3, True) == [1, 0]
    assert ots.verify(p, q, [0, 0], [0.0, 0.0], 0.3, True) == [1]


# ---------------------------------------------------------------- the library against the oracle
def test_library_bandit_matches_oracle(ts):
    rng = np.random.default_rng(5)
    for trial in range(20):
        K = int(rng.integers(1, 6))
        lam_u, lam_g = float(rng.uniform(0, 1)), float(rng.uniform(0, 0.3))
        ob, lb = ots.Bandit(K, lam_u, lam_g), ts.sd_bandit_init(K, lam_u, lam_g)
        for _ in range(60):
            k = ob.select()
            assert ts.sd_bandit_select(lb) == k
            n_acc, gamma = int(rng.integers(1, 7)), int(rng.integers(4, 7))
            assert ts.sd_reward(n_acc, gamma, lam_g) == pytest.approx(ots.reward(n_acc, gamma, lam_g), rel=1e-15)
            ob.update(k, n_acc, gamma)
            ts.sd_bandit_update(lb, k, n_acc, gamma)
        assert list(lb.n[:K]) == ob.n and lb.t == ob.t
        np.testing.assert_allclose(list(lb.reward_sum[:K]), ob.reward_sum, rtol=1e-14)


def test_library_verify_matches_oracle(ts):
    rng = np.random.default_rng(6)
    for trial in range(300):
        gamma, V = int(rng.integers(1, 7)), int(rng.integers(2, 12))
        p = rng.dirichlet(np.ones(V) * 0.5, gamma + 1).astype(np.float32)
        q = rng.dirichlet(np.ones(V) * 0.5, gamma).astype(np.float32)
        if trial % 5 == 0:
            q[0] = p[0]                                         # identical distributions: always accept
        draft = np.array([rng.choice(V, p=q[t] / q[t].sum()) for t in range(gamma)], dtype=np.int32)
        ua = rng.uniform(0, 1, gamma).astype(np.float32)
        us = float(np.float32(rng.uniform(0, 1)))
        for greedy in (False, True):
            assert ts.sd_verify(p, q, draft, ua, us, greedy) == ots.verify(p, q, draft, ua, us, greedy)


def test_library_rejects_bad_arguments(ts):
    from paper_2506_01206_amd.binding import MambaError
    with pytest.raises(MambaError):
        ts.sd_bandit_init(0, 0.1, 0.1)
    with pytest.raises(MambaError):
        ts.sd_bandit_init(33, 0.1, 0.1)
    with pytest.raises(MambaError):
        ts.sd_reward(0, 5, 0.1)
    b = ts.sd_bandit_init(2, 0.1, 0.1)
    with pytest.raises(MambaError):
        ts.sd_bandit_update(b, 2, 3, 5)
    with pytest.raises(MambaError):
        ts.sd_verify(np.full((2, 3), 1 / 3), np.full((1, 3), 1 / 3), [5], [0.5], 0.5, False)
