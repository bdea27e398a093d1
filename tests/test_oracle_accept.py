"""Pins for the acceptance rule (Sec. 2.1 for temperature > 0; Sec. 3.1 footnote for greedy)."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats

from .helpers import dp, f32, fp, ip
import ctypes as C


def _greedy(orc, logits, ids):
    k, V = len(ids), logits.shape[1]
    na, b = C.c_int(), C.c_int32()
    ids = np.ascontiguousarray(ids, np.int32)
    lg = f32(logits)
    orc.orc_accept_greedy(fp(lg), V, k, ip(ids), C.byref(na), C.byref(b))
    return na.value, b.value


def _sample(orc, tl, dl, ids, T, u):
    k, V = len(ids), tl.shape[1]
    na, b = C.c_int(), C.c_int32()
    ids = np.ascontiguousarray(ids, np.int32)
    tl, dl, u = f32(tl), f32(dl), np.ascontiguousarray(u, np.float64)
    orc.orc_accept_sample(fp(tl), fp(dl), V, k, ip(ids), T, dp(u), C.byref(na), C.byref(b))
    return na.value, b.value


def test_greedy_brute_force_three_token_vocab(orc):
    rng = np.random.default_rng(0)
    for k in range(0, 4):
        logits = rng.standard_normal((k + 1, 3)).astype(np.float32)
        best = [int(np.argmax(r)) for r in logits]
        for ids in itertools.product(range(3), repeat=k):
            # definition: longest prefix with no incorrect token, then the target's own token
            want = 0
            while want < k and ids[want] == best[want]:
                want += 1
            assert _greedy(orc, logits, list(ids) if k else np.zeros(0, np.int32)) == (want, best[want])


def test_greedy_tie_resolves_to_lowest_id(orc):
    logits = np.array([[1.0, 1.0, 0.0], [0.0, 2.0, 2.0]], np.float32)
    assert _greedy(orc, logits, [0]) == (1, 1)
    assert _greedy(orc, logits, [1]) == (0, 0)


P = np.array([0.5, 0.3, 0.2])
PH = np.array([0.2, 0.5, 0.3])


def test_worked_example_accept_probabilities_and_residual(orc):
    """p = [.5,.3,.2], p_hat = [.2,.5,.3]: accept w.p. min(1, p/p_hat) = [1, .6, 2/3];
    residual max(0, p - p_hat) normalised = [1, 0, 0]; sum_t p_hat(t) a_t = .7."""
    tl = np.log(P)[None].repeat(2, 0)
    dl = np.log(PH)[None]
    grid = (np.arange(2000) + 0.5) / 2000
    acc = []
    for t in range(3):
        hits = sum(_sample(orc, tl, dl, [t], 1.0, [u, 0.5])[0] for u in grid)
        acc.append(hits / len(grid))
    np.testing.assert_allclose(acc, [1.0, 0.6, 2 / 3], atol=1e-3)
    assert abs(float(np.dot(PH, acc)) - 0.7) < 1e-3
    # rejected (u0 = 0.999 rejects tokens 1 and 2): the resample always lands on token 0
    for t in (1, 2):
        for u in (0.0, 0.3, 0.999):
            assert _sample(orc, tl, dl, [t], 1.0, [0.999, u]) == (0, 0)
    # output law = sum_t p_hat(t) [a_t delta_t + (1 - a_t) residual] must be p
    law = np.array([PH[0] * acc[0], PH[1] * acc[1], PH[2] * acc[2]])
    law[0] += 1 - float(np.dot(PH, acc))
    np.testing.assert_allclose(law, P, atol=2e-3)


def test_token_the_target_excludes_is_never_accepted(orc):
    """Sec. 2.1: acceptance probability min(1, p/p_hat) is 0 when the target gives the token no mass;
    the strict comparison u < ratio rejects it even for u = 0, and the replacement comes from the
    target (the residual max(0, p - p_hat) has no mass on the rejected token)."""
    V = 6
    tl = np.zeros((2, V), np.float32)
    tl[0, 2] = -5000.0                           # exp underflows: p(2) = 0 exactly
    dl = np.zeros((1, V), np.float32)
    dl[0, 2] = 5.0                               # the draft is confident in token 2
    for u1 in (0.0, 0.3, 0.999):
        na, b = _sample(orc, tl, dl, [2], 1.0, [0.0, u1])
        assert na == 0 and b != 2
    # with any target mass at all and u = 0 it is accepted
    tl[0, 2] = -20.0
    na, _ = _sample(orc, tl, dl, [2], 1.0, [0.0, 0.5])
    assert na == 1


def test_all_accepted_bonus_follows_target_row_k(orc):
    tl = np.log(np.array([[0.25, 0.25, 0.5], [0.1, 0.6, 0.3]]))
    dl = tl[:1]
    grid = (np.arange(1000) + 0.5) / 1000
    cnt = np.zeros(3)
    for u in grid:
        na, b = _sample(orc, tl, dl, [2], 1.0, [0.5, u])   # p == p_hat: always accepted
        assert na == 1
        cnt[b] += 1
    np.testing.assert_allclose(cnt / len(grid), [0.1, 0.6, 0.3], atol=2e-3)


def test_identical_laws_accept_everything_and_disjoint_reject(orc):
    rng = np.random.default_rng(1)
    V, k = 8, 4
    tl = rng.standard_normal((k + 1, V)).astype(np.float32)
    ids = rng.integers(0, V, k)
    for _ in range(50):
        u = rng.random(k + 1)
        assert _sample(orc, tl, tl[:k], ids, 0.7, u)[0] == k
    # draft puts all its mass on token 0, target gives it (almost) none: always rejected, bonus ~ p
    tl2 = np.array([[-80.0, 0.0, math.log(3.0)], [0, 0, 0]], np.float32)
    dl2 = np.array([[0.0, -80.0, -80.0]], np.float32)
    cnt = np.zeros(3)
    for u in (np.arange(400) + 0.5) / 400:
        na, b = _sample(orc, tl2, dl2, [0], 1.0, [u * 0.999 + 1e-6, u])
        assert na == 0
        cnt[b] += 1
    np.testing.assert_allclose(cnt / 400, [0, 0.25, 0.75], atol=5e-3)


def test_temperature_scales_logits(orc):
    # softmax(l / T): with T = 2 the ratio p/p_hat for token 0 becomes sqrt of the T = 1 ratio
    tl = np.log(np.array([[0.2, 0.8], [0.5, 0.5]]))
    dl = np.log(np.array([[0.8, 0.2]]))
    def acc_rate(T):
        g = (np.arange(4000) + 0.5) / 4000
        return sum(_sample(orc, tl, dl, [0], T, [u, 0.1])[0] for u in g) / 4000
    p1, ph1 = 0.2, 0.8
    assert abs(acc_rate(1.0) - p1 / ph1) < 1e-3
    p2 = math.sqrt(0.2) / (math.sqrt(0.2) + math.sqrt(0.8))
    ph2 = math.sqrt(0.8) / (math.sqrt(0.2) + math.sqrt(0.8))
    assert abs(acc_rate(2.0) - p2 / ph2) < 1e-3


@pytest.mark.parametrize("V,k,seed", [(5, 1, 0), (8, 4, 1), (6, 3, 2)])
def test_chi_square_first_two_tokens_follow_target(orc, V, k, seed):
    """Lossless sampling: the emitted tokens are distributed as if drawn from the target.
    Row-i logits here do not depend on earlier tokens, so the joint law of the first two
    emitted tokens must be p_1 x p_2."""
    rng = np.random.default_rng(seed)
    tl = (rng.standard_normal((k + 1, V)) * 1.2).astype(np.float32)
    dl = (rng.standard_normal((k, V)) * 1.2).astype(np.float32)
    T = 0.9
    sm = lambda l: np.exp(l.astype(np.float64) / T) / np.exp(l.astype(np.float64) / T).sum()
    ph = [sm(dl[i]) for i in range(k)]
    n = 120000
    first = np.zeros(V)
    joint = np.zeros((V, V))
    n_joint = 0
    for _ in range(n):
        ids = [rng.choice(V, p=ph[i]) for i in range(k)]     # draft tokens MUST be sampled from p_hat
        na, b = _sample(orc, tl, dl, ids, T, rng.random(k + 1))
        seq = ids[:na] + [b]
        first[seq[0]] += 1
        if k >= 2 or len(seq) >= 2:
            if len(seq) >= 2:
                joint[seq[0], seq[1]] += 1
                n_joint += 1
    p1, p2 = sm(tl[0]), sm(tl[1])
    assert stats.chisquare(first, p1 * n).pvalue > 1e-3
    if k >= 2:
        # a second token exists iff the first draft token was accepted; conditioned on the first
        # emitted token x, that happens w.p. min(p1, ph1)(x)/p1(x) independent of the second, so
        # the second token given "exists" is still ~ p_2
        row = joint.sum(0)
        assert stats.chisquare(row, p2 * n_joint).pvalue > 1e-3


def test_gaussian_logit_acceptance_rate_closed_form(orc):
    """iid N(0, s^2) target and draft logits, large V: E[accept] = sum min(p, p_hat) ->
    2 Phi(-s / sqrt 2)."""
    rng = np.random.default_rng(5)
    V, s, trials = 4096, 0.4135, 1500
    hits = 0
    for _ in range(trials):
        tl = (rng.standard_normal((2, V)) * s).astype(np.float32)
        dl = (rng.standard_normal((1, V)) * s).astype(np.float32)
        ph = np.exp(dl[0].astype(np.float64))
        t = rng.choice(V, p=ph / ph.sum())
        hits += _sample(orc, tl, dl, [t], 1.0, rng.random(2))[0]
    want = 2 * stats.norm.cdf(-s / math.sqrt(2))
    assert abs(hits / trials - want) < 0.035, (hits / trials, want)
