"""Pins for the oracle's acceptance rule, samplers and metrics (CPU only)."""
import itertools
import os

import numpy as np
import pytest
import scipy.special

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------- library / brute-force pins of the pieces ----------

def test_softmax_T_matches_library():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(300) * 4).astype(np.float32)
    for T in (1.0, 0.7, 2.5):
        ref = scipy.special.softmax(x.astype(np.float64) / T)
        np.testing.assert_allclose(oracle.softmax_T(x, T), ref, rtol=2e-7, atol=1e-12)


def test_sample_cdf_matches_searchsorted_and_edges():
    rng = np.random.default_rng(1)
    w = rng.random(37)
    w[[3, 4, 36]] = 0.0
    cdf = np.cumsum(w)
    for u in np.concatenate([rng.random(500), [0.0, 1.0 - 2.0 ** -24]]):
        k, _ = oracle.sample_cdf(w, u)
        assert k == int(np.searchsorted(cdf, u * cdf[-1], side="right"))
        assert w[k] > 0
    # exact dyadic edges: cdf > u*Z is strict, so u on an edge goes to the next token
    w = np.array([0.25, 0.25, 0.0, 0.5])
    assert oracle.sample_cdf(w, 0.25)[0] == 1
    assert oracle.sample_cdf(w, 0.5)[0] == 3
    assert oracle.sample_cdf(w, 0.4999)[0] == 1
    assert oracle.sample_cdf(w, 0.0)[0] == 0
    k, mg = oracle.sample_cdf(w, 0.3)
    assert k == 1 and abs(mg - 0.05) < 1e-12


def test_argmax_ties_to_lowest_index():
    k, gap = oracle.argmax(np.array([1.0, 3.0, 3.0, 2.0], np.float32))
    assert k == 1 and gap == 0.0
    k, gap = oracle.argmax(np.array([1.0, 3.0, 2.5], np.float32))
    assert k == 1 and abs(gap - 0.5) < 1e-12


# ---------- exact law of the emitted tokens by enumeration ----------

def _accept_threshold(logits, q, cand, pos, T):
    """Largest-measure set {u_pos : candidate pos accepted}, found by bisection on
    the oracle's own decision (earlier candidates are forced accepted with u=0)."""
    gamma = len(cand)
    lo, hi = 0.0, 1.0  # accepted at lo (if at all), rejected at hi
    u = np.zeros(gamma + 1, np.float32)
    u[pos] = 0.0
    if oracle.accept(logits, q, cand, u, T)[0] <= pos:
        return 0.0
    u[pos] = np.float32(1.0 - 2.0 ** -24)
    if oracle.accept(logits, q, cand, u, T)[0] > pos:
        return 1.0
    for _ in range(30):
        mid = 0.5 * (lo + hi)
        u[pos] = np.float32(mid)
        if oracle.accept(logits, q, cand, u, T)[0] > pos:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _next_token_law(logits, q, cand, n_acc, T, V):
    """P(next = x | exactly n_acc accepted) as lengths of u-intervals, by bisection
    for each change point of the (monotone) map u -> next token."""
    gamma = len(cand)
    u = np.zeros(gamma + 1, np.float32)
    if n_acc < gamma:
        u[n_acc] = np.float32(1.0 - 2.0 ** -24)  # force the rejection at n_acc

    def tok(x):
        u[gamma] = np.float32(x)
        na, nx, _ = oracle.accept(logits, q, cand, u, T)
        assert na == n_acc
        return nx

    law = np.zeros(V)
    edges = [(0.0, tok(0.0))]
    top = 1.0 - 2.0 ** -24

    def split(a, ta, b, tb):
        if ta == tb:
            return
        if b - a < 2.0 ** -23:
            edges.append((b, tb))
            return
        m = 0.5 * (a + b)
        tm = tok(m)
        split(a, ta, m, tm)
        split(m, tm, b, tb)

    split(0.0, edges[0][1], top, tok(top))
    edges.sort()
    for i, (a, t) in enumerate(edges):
        b = edges[i + 1][0] if i + 1 < len(edges) else 1.0
        law[t] += b - a
    return law


@pytest.mark.parametrize("V,T", [(4, 1.0), (7, 0.7), (16, 1.0)])
def test_single_candidate_emits_target_law(V, T):
    """gamma = 1: sum_c q(c) [a(c) 1{x=c} + (1-a(c)) r(x|c)] = p(x), and after an
    accepted candidate the bonus token follows the second row's p."""
    rng = np.random.default_rng(V)
    logits = (rng.standard_normal((2, V)) * 2).astype(np.float32)
    q = scipy.special.softmax(rng.standard_normal(V) * 2).astype(np.float32)[None]
    q[0, 1] = 0.0  # a token the draft can never propose
    q[0] /= q[0].sum()
    p = scipy.special.softmax(logits.astype(np.float64) / T, axis=1)
    law = np.zeros(V)
    for c in range(V):
        if q[0, c] == 0:
            continue
        a = _accept_threshold(logits, q, [c], 0, T)
        assert abs(a - min(1.0, p[0, c] / q[0, c])) < 1e-6
        law[c] += q[0, c] * a
        if a < 1.0:
            law += q[0, c] * (1 - a) * _next_token_law(logits, q, [c], 0, T, V)
        if a > 0:
            bonus = _next_token_law(logits, q, [c], 1, T, V)
            np.testing.assert_allclose(bonus, p[1], atol=2e-6)
    np.testing.assert_allclose(law, p[0], atol=2e-6)


def test_two_candidates_joint_law_is_target_autoregressive_law():
    """gamma = 2 on a toy conditional model p(.|prefix), q(.|prefix): the joint law
    of the first two emitted tokens (second one completed by the target law when
    the step emitted only one) equals p(x1) p(x2|x1)."""
    V, T = 4, 1.0
    rng = np.random.default_rng(11)
    lg0 = (rng.standard_normal(V) * 1.5).astype(np.float32)            # target row after ctx
    lg1 = (rng.standard_normal((V, V)) * 1.5).astype(np.float32)       # target row after ctx+x1
    lg2 = (rng.standard_normal((V, V, V)) * 1.5).astype(np.float32)    # after ctx+x1+x2
    q0 = scipy.special.softmax(rng.standard_normal(V)).astype(np.float32)
    q1 = scipy.special.softmax(rng.standard_normal((V, V)), axis=1).astype(np.float32)
    p0 = scipy.special.softmax(lg0.astype(np.float64))
    p1 = scipy.special.softmax(lg1.astype(np.float64), axis=1)
    joint = np.zeros((V, V))
    for c1, c2 in itertools.product(range(V), range(V)):
        logits = np.stack([lg0, lg1[c1], lg2[c1, c2]])
        q = np.stack([q0, q1[c1]])
        w = float(q0[c1]) * float(q1[c1, c2])
        a1 = _accept_threshold(logits, q, [c1, c2], 0, T)
        a2 = _accept_threshold(logits, q, [c1, c2], 1, T)
        # reject c1: one token emitted, the next step would draw x2 ~ p(.|x1)
        if a1 < 1:
            r = _next_token_law(logits, q, [c1, c2], 0, T, V)
            joint += w * (1 - a1) * r[:, None] * p1
        # accept c1, reject c2: emits c1 then the residual draw
        if a1 > 0 and a2 < 1:
            joint[c1] += w * a1 * (1 - a2) * _next_token_law(logits, q, [c1, c2], 1, T, V)
        # accept both: emits c1, c2 (and a bonus token not examined here)
        joint[c1, c2] += w * a1 * a2
    np.testing.assert_allclose(joint, p0[:, None] * p1, atol=5e-6)


# ---------- Equation 1's numerator as a closed form ----------

@pytest.mark.parametrize("gamma", [3, 5, 8])
@pytest.mark.parametrize("rho", [0.0, 0.5, 0.9])
def test_expected_tokens_per_step_matches_equation_1(gamma, rho):
    """Position-independent p and q: every candidate is accepted with probability
    alpha = sum_x min(p, q), so tokens per step is truncated geometric with mean
    (1 - alpha^(gamma+1)) / (1 - alpha), and Equation 2's rate is
    alpha (1 - alpha^gamma) / ((1 - alpha) gamma)."""
    V, N = 64, 20000
    rng = np.random.default_rng(100 + gamma)
    lt = (rng.standard_normal(V) * 1.5).astype(np.float32)
    zq = rho * lt + (1 - rho) * 4.0 * rng.standard_normal(V).astype(np.float32)
    q1 = oracle.softmax_T(zq, 1.0)
    p1 = oracle.softmax_T(lt, 1.0).astype(np.float64)
    alpha = float(np.minimum(p1, q1.astype(np.float64)).sum())
    logits = np.tile(lt, (gamma + 1, 1))
    q = np.tile(q1, (gamma, 1))
    cdf = np.cumsum(q1.astype(np.float64))
    n_accs = []
    for _ in range(N):
        cand = np.minimum(np.searchsorted(cdf, rng.random(gamma) * cdf[-1], side="right"), V - 1)
        u = (rng.integers(0, 1 << 24, gamma + 1) * 2.0 ** -24).astype(np.float32)
        n_accs.append(oracle.accept(logits, q, cand, u, 1.0)[0])
    n_accs = np.array(n_accs)
    tau = oracle.mean_tau(n_accs)
    sigma = np.std(n_accs + 1) / np.sqrt(N)
    assert abs(tau - oracle.expected_tau(alpha, gamma)) < 4 * sigma + 1e-9
    rate_cf = alpha * (1 - alpha ** gamma) / ((1 - alpha) * gamma)
    assert abs(oracle.acceptance_rate(n_accs, gamma) - rate_cf) < 4 * sigma / gamma + 1e-9
    assert abs(oracle.alpha_hat(n_accs, gamma) - alpha) < 0.02
    # Equation 2's rate is decreasing in gamma at fixed alpha (Section 3.2.1 observes this)
    assert rate_cf <= alpha + 1e-12


def test_metric_definitions_against_table_1():
    """Table 1's rows satisfy tau = gamma * rate + 1 to the printed precision, which
    fixes that tau counts the token the target adds; and speedup <= tau always."""
    rows = {}
    for line in open(os.path.join(GOLD, "table1.txt")):
        if line.startswith("#") or not line.strip():
            continue
        g, method, metric, *vals = line.split()
        rows[(int(g), method, metric)] = [float(v) for v in vals]
    assert len(rows) == 12
    for (g, method, metric), rates in rows.items():
        if metric != "rate":
            continue
        taus = rows[(g, method, "tau")]
        spd = rows[(g, method, "speedup")]
        for r, t, s in zip(rates, taus, spd):
            assert abs(g * r + 1 - t) <= 0.005 * g + 0.005 + 1e-9  # printed-precision bound
            assert s < t
            # Equation 1 with tau as numerator implies a draft/target cost ratio in (0, 1)
            c = (t / s - 1) / g
            assert 0.0 < c < 0.3
    # our definitions reproduce the identity exactly
    n_acc = [0, 3, 9, 2, 9, 1]
    assert abs(oracle.mean_tau(n_acc) - (9 * oracle.acceptance_rate(n_acc, 9) + 1)) < 1e-12
    assert abs(oracle.eq1_speedup(0.8, 5, 0.1) - (1 - 0.8 ** 6) / (0.2 * 1.5)) < 1e-12
    assert oracle.expected_tau(1.0, 5) == 6.0
    assert abs(oracle.alpha_hat([5, 5], 5) - 1.0) < 1e-12 and oracle.alpha_hat([0, 0], 5) == 0.0


# ---------- special cases ----------

def test_identical_distributions_accept_everything():
    rng = np.random.default_rng(5)
    V, gamma = 33, 4
    logits = (rng.standard_normal((gamma + 1, V)) * 3).astype(np.float32)
    q = np.stack([oracle.softmax_T(logits[i], 0.7) for i in range(gamma)])
    for _ in range(50):
        cand = rng.integers(0, V, gamma)
        u = (rng.integers(0, 1 << 24, gamma + 1) * 2.0 ** -24).astype(np.float32)
        na, nx, _ = oracle.accept(logits, q, cand, u, 0.7)
        assert na == gamma
        w = oracle.softmax_T(logits[gamma], 0.7).astype(np.float64)
        assert nx == oracle.sample_cdf(w, float(u[gamma]))[0]


def test_impossible_candidate_is_rejected_and_residual_excludes_overdrafted_tokens():
    V = 8
    logits = np.zeros((2, V), np.float32)
    logits[0, 3] = -1e4  # p(3) = 0
    q = np.full((1, V), 0.0, np.float32)
    q[0, 3] = 0.5
    q[0, 5] = 0.5        # q(5) = .5 > p(5) = 1/7: residual mass there is 0
    for uu in (0.0, 0.3, 0.999):
        na, nx, _ = oracle.accept(logits, q, [3], np.array([0.0, uu], np.float32), 1.0)
        assert na == 0 and nx not in (3, 5)
    na, nx, _ = oracle.accept(logits, q, [5], np.array([0.99, 0.5], np.float32), 1.0)
    assert na == 0 and nx not in (3, 5)
    na, _, mg = oracle.accept(logits, q, [5], np.array([0.25, 0.5], np.float32), 1.0)
    assert na == 1 and abs(mg[0] - abs(0.25 - (1 / 7) / 0.5)) < 1e-6


def test_greedy_rule_is_argmax_matching():
    logits = np.array([[0, 5, 1], [7, 0, 0], [0, 0, 9], [1, 2, 3]], np.float32)
    assert oracle.accept(logits, None, [1, 0, 2], np.zeros(4, np.float32), 0.0)[:2] == (3, 2)
    assert oracle.accept(logits, None, [1, 1, 2], np.zeros(4, np.float32), 0.0)[:2] == (1, 0)
    assert oracle.accept(logits, None, [0, 0, 2], np.zeros(4, np.float32), 0.0)[:2] == (0, 1)
    # gamma = 0: plain next-token choice
    assert oracle.accept(logits[:1], None, [], np.zeros(1, np.float32), 0.0)[:2] == (0, 1)


def test_route_is_argmax_of_linear_scores():
    rng = np.random.default_rng(3)
    W, b, e = rng.standard_normal((4, 16)), rng.standard_normal(4), rng.standard_normal((20, 16))
    ref = np.argmax(e.astype(np.float32).astype(np.float64) @ W.astype(np.float32).astype(np.float64).T
                    + b.astype(np.float32), axis=1)
    np.testing.assert_array_equal(oracle.route(W, b, e), ref)
    # ties go to the lowest id
    assert oracle.route(np.ones((3, 2)), np.zeros(3), np.ones((1, 2)))[0] == 0


def test_cdf_distance_and_next_weights():
    w = np.array([0.25, 0.25, 0.0, 0.5])
    assert oracle.cdf_distance(w, 0.3, 1) == 0.0
    assert abs(oracle.cdf_distance(w, 0.3, 0) - 0.05) < 1e-12
    assert abs(oracle.cdf_distance(w, 0.3, 3) - 0.2) < 1e-12
    assert oracle.cdf_distance(w, 0.5, 1) == 0.0 and oracle.cdf_distance(w, 0.5, 3) == 0.0  # on the edge
    rng = np.random.default_rng(8)
    logits = (rng.standard_normal((3, 12)) * 2).astype(np.float32)
    q = scipy.special.softmax(rng.standard_normal((2, 12)), axis=1).astype(np.float32)
    p = scipy.special.softmax(logits.astype(np.float64) / 0.7, axis=1)
    np.testing.assert_allclose(oracle.next_weights(logits, q, 1, 0.7), np.maximum(p[1] - q[1], 0), atol=1e-7)
    np.testing.assert_allclose(oracle.next_weights(logits, q, 2, 0.7), p[2], atol=1e-7)
    for u in (0.1, 0.6, 0.95):   # the token the rule picks is the one at distance 0
        na, nx, _ = oracle.accept(logits, q, [0, 1], np.array([0.999999, 0.0, u], np.float32), 0.7)
        if na == 0:
            assert oracle.cdf_distance(oracle.next_weights(logits, q, 0, 0.7), u, nx) == 0.0
