"""Pins of the fp64 oracle against what the paper and the mathematics fix.

None of these tests re-types the oracle's formulas: the reference side is either
textbook softmax attention differentiated numerically, a dense linear-algebra
solution of the paper's Newton system, a brute-force minimiser, a brute-force
sort, or an invariant.
"""

import itertools

import numpy as np
import pytest
from scipy.optimize import minimize_scalar

from oracle import kvs_oracle as O


def softmax_attention(q, K, V):
    """Textbook attention of one query (Sec. 4.1, Eq. attn_def_vec), written independently."""
    e = K @ q / np.sqrt(q.shape[0])
    w = np.exp(e - e.max())
    a = w / w.sum()
    return a, a @ V


def tiny_head(seed, n=6, d=4, dv=None, spread=1.0):
    rng = np.random.default_rng(seed)
    dv = dv or d
    return (rng.standard_normal(d), spread * rng.standard_normal((n, d)), rng.standard_normal((n, dv)))


# --------------------------------------------------------------------------------------------
# O1-O4
def test_score_single_row_is_textbook_attention():
    q, K, V = tiny_head(0, n=9, d=5)
    a, o = softmax_attention(q, K, V)
    ab, ob = O.score(q[None, :], K, V)
    np.testing.assert_allclose(ab, a, rtol=1e-14)
    np.testing.assert_allclose(ob, o, rtol=1e-13, atol=1e-15)


def test_score_is_mean_over_rows_and_normalised():
    rng = np.random.default_rng(1)
    Q = rng.standard_normal((3, 4, 8))            # [G, W, D]
    K = rng.standard_normal((50, 8)) * 3.0
    V = rng.standard_normal((50, 8))
    ab, ob = O.score(Q, K, V)
    rows = [softmax_attention(q, K, V) for q in Q.reshape(-1, 8)]
    np.testing.assert_allclose(ab, np.mean([r[0] for r in rows], axis=0), rtol=1e-13)
    np.testing.assert_allclose(ob, np.mean([r[1] for r in rows], axis=0), rtol=1e-12, atol=1e-15)
    assert abs(ab.sum() - 1.0) < 1e-14


def test_score_shift_invariance_and_large_logits():
    # softmax must be computed stably: logits around +-4000 overflow a naive exp.
    rng = np.random.default_rng(2)
    K = rng.standard_normal((20, 4)) * 100.0
    Q = rng.standard_normal((2, 4)) * 100.0
    V = rng.standard_normal((20, 4))
    ab, _ = O.score(Q, K, V)
    assert np.isfinite(ab).all() and abs(ab.sum() - 1) < 1e-12
    # adding a vector to every Key shifts each row's logits by a constant: alpha unchanged
    ab2, _ = O.score(Q, K + 0.01 * rng.standard_normal(4)[None, :], V)
    np.testing.assert_allclose(ab2, ab, rtol=1e-9, atol=1e-300)


# --------------------------------------------------------------------------------------------
# O8: the forward-only vectors are the derivatives of s_i = alpha_i (v_i - o) w.r.t. the logits
def s_of_logits(e, V):
    w = np.exp(e - e.max())
    a = w / w.sum()
    o = a @ V
    return a[:, None] * (V - o[None, :])


def fd_ds_de(q, K, V, h=1e-5):
    """J[i, j, :] = d s_i / d e_j by central differences on the logits."""
    e0 = K @ q / np.sqrt(q.shape[0])
    n = K.shape[0]
    J = np.zeros((n, n, V.shape[1]))
    for j in range(n):
        ep, em = e0.copy(), e0.copy()
        ep[j] += h
        em[j] -= h
        J[:, j, :] = (s_of_logits(ep, V) - s_of_logits(em, V)) / (2 * h)
    return J


@pytest.mark.parametrize("seed", [3, 4, 5])
def test_norms_match_finite_difference_of_s(seed):
    q, K, V = tiny_head(seed, n=6, d=4, dv=5, spread=1.5)
    J = fd_ds_de(q, K, V)
    ab, ob = O.score(q[None, :], K, V)
    A, C = O.token_and_edge_norms(ab, V, ob)
    np.testing.assert_allclose(A, [np.linalg.norm(J[i, i]) for i in range(6)], rtol=1e-7)
    np.testing.assert_allclose(C, [np.linalg.norm(J[i, i + 1]) for i in range(5)], rtol=1e-7)
    # the coupling is symmetric (h^{m+1,m} = h^{m,m+1}, Sec. 4.1)
    np.testing.assert_allclose(J[1, 2], J[2, 1], atol=1e-9)


def test_hessian_blocks_are_rank_one_with_forward_only_scalars():
    """Central-difference Hessian of f(K) = E^T o(K) w.r.t. (k_i, k_j) equals
    (1/d_k)(E^T ds_i/de_j) q q^T (Eq. hessian_rank1), with the same vectors whose norms the oracle uses."""
    q, K, V = tiny_head(7, n=5, d=3, dv=4)
    rng = np.random.default_rng(70)
    E = rng.standard_normal(4)
    d = 3

    def f(Kx):
        return E @ softmax_attention(q, Kx, V)[1]

    h = 1e-4
    J = fd_ds_de(q, K, V)

    def hess_block(i, j):
        H = np.zeros((d, d))
        for a in range(d):
            for b in range(d):
                acc = 0.0
                for sa, sb in itertools.product((1, -1), (1, -1)):
                    Kx = K.copy()
                    Kx[i, a] += sa * h
                    Kx[j, b] += sb * h
                    acc += sa * sb * f(Kx)
                H[a, b] = acc / (4 * h * h)
        return H

    for (i, j) in [(1, 1), (1, 2), (2, 1), (0, 3)]:
        want = (E @ J[i, j]) / d * np.outer(q, q)
        np.testing.assert_allclose(hess_block(i, j), want, atol=2e-6)


def test_softmax_second_derivative_signs():
    """App. C: the off-diagonal second derivatives of softmax are negative; the diagonal of ds_i/de_i
    keeps the direction of (v_i - o) while alpha_i < 1/2 and flips it above (the oracle takes the norm,
    so its A_t must stay correct on both sides: covered by test_norms_match_finite_difference_of_s)."""
    q, K, V = tiny_head(8, n=7, d=4)
    a, o = softmax_attention(q, K, V)
    assert a.max() > 0.5 > np.sort(a)[-2]     # this head has one dominant token: both signs occur
    J = fd_ds_de(q, K, V)
    for i in range(7):
        cos = J[i, i] @ (V[i] - o) / (np.linalg.norm(J[i, i]) * np.linalg.norm(V[i] - o))
        assert abs(cos - np.sign(1 - 2 * a[i])) < 1e-8
    for i in range(6):
        rsum = (V[i] - o) + (V[i + 1] - o)
        cos = J[i, i + 1] @ rsum / (np.linalg.norm(J[i, i + 1]) * np.linalg.norm(rsum))
        assert cos < -1 + 1e-8


# --------------------------------------------------------------------------------------------
# O9 for a pair: dense Newton system of Eq. optimal_k_cn, then the surrogate
def test_pair_weight_form_equals_dense_pseudo_inverse_along_q():
    q, K, V = tiny_head(9, n=6, d=4, dv=4)
    rng = np.random.default_rng(90)
    E = rng.standard_normal(4)
    J = fd_ds_de(q, K, V)
    m = 2
    g11, g12, g22 = E @ J[m, m], E @ J[m, m + 1], E @ J[m + 1, m + 1]
    qq = np.outer(q, q) / 4.0
    h11, h12, h22 = g11 * qq, g12 * qq, g22 * qq
    k_dense = np.linalg.pinv(h11 + 2 * h12 + h22) @ (h11 @ K[m] + h12 @ (K[m] + K[m + 1]) + h22 @ K[m + 1])
    wm = (g11 + g12) / (g11 + 2 * g12 + g22)
    k_weight = wm * K[m] + (1 - wm) * K[m + 1]
    # the two expressions differ only by a vector orthogonal to q (Eqs. kstar_proj_form vs kstar_weight_final_rewrite)
    assert abs(q @ k_dense - q @ k_weight) < 1e-8 * max(1.0, abs(q @ k_weight))


def run_oracle_on_mask(q, K, V, mask):
    ab, ob = O.score(q[None, :], K, V)
    mask = np.asarray(mask, dtype=np.uint8)
    starts = np.ones(len(mask), dtype=int)
    starts[1:] = 1 - mask[:-1]
    slot = (np.cumsum(starts) - 1).astype(np.int32)
    return ab, ob, O.merge_compact(K, V, ab, ob, mask, slot)


def surrogate_objective_minimiser(q, K, J, t0, t1):
    """Brute-force minimiser (over x = q.k) of the second-order objective
       sum_ab g_ab (q.(k - k_a)) (q.(k - k_b)),  a, b in the run,
    with the gradient-free surrogate g_aa = ||ds_a/de_a||, g_{a,a+1} = -||ds_a/de_{a+1}|| and all other
    blocks dropped.  The norms come from finite differences, not from the oracle."""
    idx = list(range(t0, t1 + 1))
    L = len(idx)
    g = np.zeros((L, L))
    for a in range(L):
        g[a, a] = np.linalg.norm(J[idx[a], idx[a]])
        if a + 1 < L:
            g[a, a + 1] = g[a + 1, a] = -np.linalg.norm(J[idx[a], idx[a + 1]])
    x = K[idx] @ q

    def obj(z):
        dz = z - x
        return dz @ g @ dz

    lo, hi = x.min() - 5 * (np.ptp(x) + 1), x.max() + 5 * (np.ptp(x) + 1)
    grid = np.linspace(lo, hi, 20001)
    z0 = grid[np.argmin([obj(z) for z in grid])]
    step = grid[1] - grid[0]
    res = minimize_scalar(obj, bracket=(z0 - step, z0, z0 + step), tol=1e-14)
    return res.x, g


@pytest.mark.parametrize("seed,L", [(10, 2), (11, 2), (12, 3), (13, 4), (16, 3), (17, 4)])
def test_merged_key_minimises_second_order_objective(seed, L):
    n = 8
    q, K, V = tiny_head(seed, n=n, d=4, dv=6, spread=1.2)
    t0 = 2
    t1 = t0 + L - 1
    mask = np.zeros(n, dtype=np.uint8)
    mask[t0:t1] = 1
    ab, ob, res = run_oracle_on_mask(q, K, V, mask)
    J = fd_ds_de(q, K, V)
    xstar, g = surrogate_objective_minimiser(q, K, J, t0, t1)
    assert g.sum() > 0            # convex along q
    S = t0                        # tokens before t0 are singletons
    assert res.counts[S] == L
    got = q @ res.K_out[S]
    assert abs(got - xstar) < 2e-6 * max(1.0, abs(xstar))
    # random perturbations of the merged Key never lower the objective
    rng = np.random.default_rng(seed)
    x = K[t0:t1 + 1] @ q
    base = (got - x) @ g @ (got - x)
    for _ in range(50):
        z = q @ (res.K_out[S] + 0.1 * rng.standard_normal(4))
        assert (z - x) @ g @ (z - x) >= base - 1e-12


def test_pair_rule_is_the_printed_closed_form():
    """|S| = 2 evaluated through the finite-difference norms reproduces Eq. kstar_final term by term."""
    q, K, V = tiny_head(15, n=7, d=4, dv=5)
    J = fd_ds_de(q, K, V)
    m = 3
    mask = np.zeros(7, dtype=np.uint8)
    mask[m] = 1
    _, _, res = run_oracle_on_mask(q, K, V, mask)
    n11, n22, n12 = (np.linalg.norm(J[m, m]), np.linalg.norm(J[m + 1, m + 1]), np.linalg.norm(J[m, m + 1]))
    want = ((n11 - n12) * K[m] + (n22 - n12) * K[m + 1]) / (n11 - 2 * n12 + n22)
    np.testing.assert_allclose(res.K_out[m], want, rtol=1e-6, atol=1e-9)
    # the coupling term is visible at this size: dropping it moves the Key measurably
    no_coupling = (n11 * K[m] + n22 * K[m + 1]) / (n11 + n22)
    assert np.linalg.norm(no_coupling - want) > 1e-3 * np.linalg.norm(want)


def test_identical_keys_merge_to_themselves():
    q, K, V = tiny_head(16, n=10, d=4)
    K[3:7] = K[3]
    mask = np.zeros(10, dtype=np.uint8)
    mask[3:6] = 1          # run 3..6
    mask[7] = 1            # pair 7, 8 with distinct Keys
    _, _, res = run_oracle_on_mask(q, K, V, mask)
    np.testing.assert_allclose(res.K_out[3], K[3], rtol=1e-13)
    assert res.counts.tolist() == [1, 1, 1, 4, 2, 1]


def test_lossless_values_when_merged_keys_identical():
    """Sum-merged Values with cardinality normalisation reproduce full attention exactly when
    the Keys of every run coincide (Sec. 3.1: replacing (k_m, k_{m+1}) by (k, k))."""
    rng = np.random.default_rng(17)
    n, d = 12, 4
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    K[2:5] = K[2]
    K[8:10] = K[8]
    mask = np.zeros(n, dtype=np.uint8)
    mask[2:4] = 1
    mask[8] = 1
    q = rng.standard_normal(d)
    _, _, res = run_oracle_on_mask(q, K, V, mask)
    for _ in range(5):
        qn = rng.standard_normal(d)
        want = softmax_attention(qn, K, V)[1]
        got = O.merged_attention(qn, res.K_out, res.V_out, res.counts)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_fallback_mean_when_denominator_vanishes():
    # all Values equal => every residual v_t - o is zero => A = C = 0 => U = 0 => arithmetic mean
    rng = np.random.default_rng(18)
    K = rng.standard_normal((6, 4))
    V = np.ones((6, 4))
    q = rng.standard_normal(4)
    mask = np.array([0, 1, 1, 0, 0, 0], dtype=np.uint8)
    _, _, res = run_oracle_on_mask(q, K, V, mask)
    assert res.fallback[1] and not res.fallback[0]
    np.testing.assert_allclose(res.K_out[1], K[1:4].mean(axis=0), rtol=1e-14)


def test_fallback_mean_when_surrogate_is_not_convex():
    # a token at alpha = 1/2 has A = 0: the run's denominator goes negative, the quadratic has no minimiser
    q, K, V = tiny_head(14, n=8, d=4, dv=6, spread=1.2)
    mask = np.zeros(8, dtype=np.uint8)
    mask[2:4] = 1
    ab, _, res = run_oracle_on_mask(q, K, V, mask)
    assert abs(ab[3] - 0.5) < 1e-2 and res.U[2] < 0 and res.fallback[2]
    np.testing.assert_allclose(res.K_out[2], K[2:5].mean(axis=0), rtol=1e-14)


# --------------------------------------------------------------------------------------------
# O5-O7
def brute_force_select(alpha, budget, s, nr):
    n = len(alpha)
    r = n - budget
    edges = [(alpha[m] + alpha[m + 1], m) for m in range(s, n - 1 - nr)]
    edges.sort()
    chosen = {m for _, m in edges[:max(r, 0)]}
    mask = np.array([1 if m in chosen else 0 for m in range(n)], dtype=np.uint8)
    slot, cur = [], -1
    for t in range(n):
        if t == 0 or not mask[t - 1]:
            cur += 1
        slot.append(cur)
    return mask, np.array(slot, dtype=np.int32)


@pytest.mark.parametrize("n,budget,s,nr,seed", [
    (40, 20, 4, 0, 0), (40, 5, 4, 0, 1), (64, 33, 32, 0, 2), (50, 25, 3, 7, 3), (33, 33, 2, 0, 4),
    (33, 40, 2, 0, 5), (200, 50, 32, 0, 6), (10, 3, 0, 0, 7), (10, 1, 0, 0, 8)])
def test_select_matches_brute_force(n, budget, s, nr, seed):
    rng = np.random.default_rng(seed)
    alpha = rng.dirichlet(np.ones(n) * 0.3)
    mask, slot = O.select(alpha, budget, s, nr)
    bm, bs = brute_force_select(alpha, budget, s, nr)
    assert (mask == bm).all() and (slot == bs).all()
    assert slot[-1] + 1 == max(min(budget, n), n - max(n - budget, 0))
    assert mask[-1] == 0 and (mask[:s] == 0).all()
    if nr:
        assert (mask[n - 1 - nr:] == 0).all()


def test_select_ties_go_to_lower_index():
    alpha = np.full(16, 1 / 16)
    mask, slot = O.select(alpha, 12, 2, 0)
    assert mask.tolist() == [0, 0, 1, 1, 1, 1] + [0] * 10
    # float32 decision: ties created by rounding also resolve to the lower index
    a64 = np.array([0.1, 0.2, 0.1 - 1e-9, 0.25, 0.1, 0.3], dtype=np.float64)
    m64, _ = O.select(a64, 5, 0, 0)
    m32, _ = O.select(a64.astype(np.float32), 5, 0, 0, sigma_dtype=np.float32)
    assert m64.tolist() == [0, 1, 0, 0, 0, 0]     # exact sums: edge 1 is strictly smallest
    assert m32.tolist() == [1, 0, 0, 0, 0, 0]     # edges 0 and 1 are equal in fp32: the lower index wins


def test_select_many_ties_large_n():
    rng = np.random.default_rng(30)
    n = 5000
    alpha = rng.integers(1, 6, size=n).astype(np.float64)       # only 9 distinct edge scores
    alpha /= alpha.sum()
    for budget in (600, 2500, 4900):
        mask, slot = O.select(alpha, budget, 32, 0)
        bm, bs = brute_force_select(alpha, budget, 32, 0)
        assert (mask == bm).all() and (slot == bs).all()


def test_select_rejects_impossible_budget():
    with pytest.raises(ValueError):
        O.select(np.full(10, 0.1), 3, 4, 0)


# --------------------------------------------------------------------------------------------
# whole step: invariants and order-freedom (Sec. 3.1: the pairs are merged in parallel)
@pytest.mark.parametrize("seed,n,budget,R", [(20, 96, 48, 3), (21, 300, 64, 8), (22, 128, 127, 1)])
def test_step_invariants(seed, n, budget, R):
    rng = np.random.default_rng(seed)
    d = 8
    K = np.cumsum(rng.standard_normal((n, d)), axis=0) * 0.3
    V = rng.standard_normal((n, d))
    Q = rng.standard_normal((R, d))
    s = 4
    r = O.step(Q, K, V, budget, s, 0)
    m = r.merged
    assert abs(r.alpha_bar.sum() - 1) < 1e-13
    assert m.K_out.shape == (budget, d) and m.counts.sum() == n
    np.testing.assert_allclose(m.V_out.sum(axis=0), V.sum(axis=0), rtol=1e-12, atol=1e-12)
    inc = np.diff(r.slot)
    assert set(np.unique(inc)) <= {0, 1} and r.slot[0] == 0
    assert (m.counts[:s] == 1).all()
    single = np.flatnonzero(m.counts == 1)
    first_token = np.searchsorted(r.slot, np.arange(budget))
    assert (m.K_out[single] == K[first_token[single]]).all()       # bit-identical copies
    assert (m.V_out[single] == V[first_token[single]]).all()
    # every merged Key is an affine combination of its run with weights summing to one:
    # it reproduces any affine functional of the Keys when all run members agree on it
    assert not m.fallback.any()


def test_partition_is_independent_of_edge_processing_order():
    rng = np.random.default_rng(23)
    n, d, budget = 80, 4, 30
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    Q = rng.standard_normal((2, d))
    r = O.step(Q, K, V, budget, 2, 0)
    edges = np.flatnonzero(r.mask)
    for trial in range(5):
        parent = list(range(n))

        def find(x):
            while parent[x] != x:
                parent[x] = parent[parent[x]]
                x = parent[x]
            return x

        for m in rng.permutation(edges):
            a, b = find(int(m)), find(int(m) + 1)
            parent[max(a, b)] = min(a, b)
        roots = np.array([find(t) for t in range(n)])
        _, relabel = np.unique(roots, return_inverse=True)
        assert (relabel == r.slot).all()


def test_isolated_pairs_equal_sequential_pair_merges_in_any_order():
    """When no two selected edges touch, the step is exactly the paper's pair merge applied to
    each pair with the ORIGINAL alpha and o, whatever the order."""
    rng = np.random.default_rng(24)
    n, d = 20, 4
    q, K, V = rng.standard_normal(d), rng.standard_normal((n, d)), rng.standard_normal((n, d))
    mask = np.zeros(n, dtype=np.uint8)
    mask[[2, 5, 9, 14]] = 1
    ab, ob, res = run_oracle_on_mask(q, K, V, mask)
    J = fd_ds_de(q, K, V)
    merged = {}
    for m in rng.permutation([2, 5, 9, 14]):
        n11, n22, n12 = (np.linalg.norm(J[m, m]), np.linalg.norm(J[m + 1, m + 1]), np.linalg.norm(J[m, m + 1]))
        merged[int(m)] = ((n11 - n12) * K[m] + (n22 - n12) * K[m + 1]) / (n11 - 2 * n12 + n22)
    slot_of = {2: 2, 5: 4, 9: 7, 14: 11}
    for m, S in slot_of.items():
        np.testing.assert_allclose(res.K_out[S], merged[m], rtol=1e-6, atol=1e-9)
        np.testing.assert_allclose(res.V_out[S], V[m] + V[m + 1], rtol=1e-14)


def test_pair_denominator_positive_when_mass_below_half():
    """With alpha_m + alpha_{m+1} < 1/2 the pair denominator A_m - 2 C_m + A_{m+1} is positive
    (triangle inequality), so Eq. kstar_final never divides by a non-positive number there."""
    rng = np.random.default_rng(25)
    for _ in range(200):
        n = 6
        q, K, V = rng.standard_normal(4), rng.standard_normal((n, 4)) * 2, rng.standard_normal((n, 4))
        ab, ob = O.score(q[None, :], K, V)
        A, C = O.token_and_edge_norms(ab, V, ob)
        for m in range(n - 1):
            if ab[m] + ab[m + 1] < 0.5:
                assert A[m] - 2 * C[m] + A[m + 1] > 0


# --------------------------------------------------------------------------------------------
# Streaming regime: rows that are already merged slots (k, V, c)
def expanded_cache(K, V, c):
    """The cache a merged one stands for: slot t becomes c[t] tokens with Key K[t]; their Values are
    unknown one by one, only their sum V[t] is, so every copy gets V[t] / c[t]."""
    return np.repeat(K, c, axis=0), np.repeat(V / c[:, None], c, axis=0), np.repeat(np.arange(len(c)), c)


def test_counts_of_one_change_nothing():
    rng = np.random.default_rng(40)
    Q, K, V = rng.standard_normal((3, 8)), rng.standard_normal((60, 8)) * 2.0, rng.standard_normal((60, 8))
    a = O.step(Q, K, V, budget=25, n_sink=2)
    b = O.step(Q, K, V, budget=25, n_sink=2, counts=np.ones(60, dtype=np.int32))
    assert np.array_equal(a.alpha_bar, b.alpha_bar) and np.array_equal(a.mask, b.mask)
    assert np.array_equal(a.merged.K_out, b.merged.K_out) and np.array_equal(a.merged.V_out, b.merged.V_out)
    assert np.array_equal(a.merged.counts, b.merged.counts)


@pytest.mark.parametrize("seed", [41, 42])
def test_slot_of_cardinality_c_attends_like_c_copies(seed):
    rng = np.random.default_rng(seed)
    n, d = 9, 5
    K, V = rng.standard_normal((n, d)) * 1.5, rng.standard_normal((n, d)) * 3.0
    c = rng.integers(1, 6, size=n)
    Ke, Ve, owner = expanded_cache(K, V, c)
    Q = rng.standard_normal((4, d))
    ab, ob = O.score(Q, K, V, counts=c)
    rows = [softmax_attention(q, Ke, Ve) for q in Q]            # textbook attention over the expanded cache
    a_exp = np.mean([r[0] for r in rows], axis=0)
    mass = np.array([a_exp[owner == t].sum() for t in range(n)])
    np.testing.assert_allclose(ab, mass, rtol=1e-13)
    np.testing.assert_allclose(ob, np.mean([r[1] for r in rows], axis=0), rtol=1e-12, atol=1e-15)
    # and the consumer formula for merged caches (pinned above) gives the same output for one query
    np.testing.assert_allclose(O.score(Q[:1], K, V, counts=c)[1], O.merged_attention(Q[0], K, V, c), rtol=1e-12)


@pytest.mark.parametrize("seed", [43, 44])
def test_norms_with_counts_match_finite_difference_of_s(seed):
    """A slot is one token with logit e + ln c and value V / c: the c-vectors are the logit derivatives of
    s_t = alpha_t (V_t / c_t - o) with alpha the softmax of the shifted logits (textbook side: s_of_logits)."""
    q, K, V = tiny_head(seed, n=6, d=4, dv=5, spread=1.5)
    c = np.array([1, 3, 2, 1, 4, 2])
    e0 = K @ q / np.sqrt(q.shape[0]) + np.log(c)
    Vs = V / c[:, None]
    h = 1e-5
    J = np.zeros((6, 6, 5))
    for j in range(6):
        ep, em = e0.copy(), e0.copy()
        ep[j] += h
        em[j] -= h
        J[:, j, :] = (s_of_logits(ep, Vs) - s_of_logits(em, Vs)) / (2 * h)
    ab, ob = O.score(q[None, :], K, V, counts=c)
    A, C = O.token_and_edge_norms(ab, V, ob, counts=c)
    np.testing.assert_allclose(A, [np.linalg.norm(J[i, i]) for i in range(6)], rtol=1e-7)
    np.testing.assert_allclose(C, [np.linalg.norm(J[i, i + 1]) for i in range(5)], rtol=1e-7)


def test_merge_with_counts_invariants_and_lossless_chain():
    """Cardinalities add up, Values stay sums, single rows are copied, and when the Keys of every run
    coincide the re-merged cache attends exactly like the cache it was made from (Sec. 3.1)."""
    rng = np.random.default_rng(45)
    n, d = 14, 4
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d)) * 2.0
    c = rng.integers(1, 5, size=n)
    K[3:6] = K[3]
    K[9:11] = K[9]
    mask = np.zeros(n, dtype=np.uint8)
    mask[3:5] = 1
    mask[9] = 1
    slot = np.concatenate([[0], np.cumsum(mask[:-1] == 0)]).astype(np.int32)
    q = rng.standard_normal(d)
    ab, ob = O.score(q[None, :], K, V, counts=c)
    res = O.merge_compact(K, V, ab, ob, mask, slot, counts_in=c)
    assert res.counts.sum() == c.sum() and res.counts[3] == c[3:6].sum() and res.n_rows[3] == 3
    np.testing.assert_allclose(res.V_out.sum(axis=0), V.sum(axis=0), rtol=1e-13)
    assert np.array_equal(res.K_out[0], K[0]) and np.array_equal(res.V_out[0], V[0]) and res.counts[0] == c[0]
    Ke, Ve, _ = expanded_cache(K, V, c)
    for _ in range(5):
        qn = rng.standard_normal(d)
        want = softmax_attention(qn, Ke, Ve)[1]                  # the tokens the input stood for
        np.testing.assert_allclose(O.merged_attention(qn, res.K_out, res.V_out, res.counts), want,
                                   rtol=1e-12, atol=1e-14)


def test_fallback_with_counts_is_the_mean_over_the_tokens_the_rows_stand_for():
    rng = np.random.default_rng(46)
    K = rng.standard_normal((6, 4))
    c = np.array([2, 1, 3, 2, 1, 1])
    V = np.ones((6, 4)) * c[:, None]                             # V / c identical: every residual vanishes
    q = rng.standard_normal(4)
    mask = np.array([0, 1, 1, 0, 0, 0], dtype=np.uint8)
    slot = np.concatenate([[0], np.cumsum(mask[:-1] == 0)]).astype(np.int32)
    ab, ob = O.score(q[None, :], K, V, counts=c)
    res = O.merge_compact(K, V, ab, ob, mask, slot, counts_in=c)
    assert res.fallback[1] and not res.fallback[0]
    Ke, _, owner = expanded_cache(K, V, c)
    np.testing.assert_allclose(res.K_out[1], Ke[(owner >= 1) & (owner <= 3)].mean(axis=0), rtol=1e-14)


# --------------------------------------------------------------------------------------------
# Ablation rules of the merged Key
def test_mean_rule_is_the_arithmetic_mean_of_the_tokens():
    rng = np.random.default_rng(50)
    n, d = 10, 4
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    c = rng.integers(1, 4, size=n)
    mask = np.zeros(n, dtype=np.uint8)
    mask[2:5] = 1
    slot = np.concatenate([[0], np.cumsum(mask[:-1] == 0)]).astype(np.int32)
    q = rng.standard_normal(d)
    ab, ob = O.score(q[None, :], K, V)
    res = O.merge_compact(K, V, ab, ob, mask, slot, rule="mean")
    np.testing.assert_allclose(res.K_out[2], K[2:6].mean(axis=0), rtol=1e-14)
    ab, ob = O.score(q[None, :], K, V, counts=c)
    res = O.merge_compact(K, V, ab, ob, mask, slot, counts_in=c, rule="mean")
    Ke, _, owner = expanded_cache(K, V, c)
    np.testing.assert_allclose(res.K_out[2], Ke[(owner >= 2) & (owner <= 5)].mean(axis=0), rtol=1e-14)
    full = O.merge_compact(K, V, ab, ob, mask, slot, counts_in=c)
    assert np.array_equal(full.V_out, res.V_out) and np.array_equal(full.counts, res.counts)


@pytest.mark.parametrize("seed,L", [(51, 2), (52, 3), (53, 4)])
def test_diagonal_rule_minimises_the_objective_without_coupling(seed, L):
    """C := 0: the minimiser of sum_a g_aa (q.(k - k_a))^2 with g_aa from finite differences."""
    n = 8
    q, K, V = tiny_head(seed, n=n, d=4, dv=6, spread=1.2)
    t0, t1 = 2, 2 + L - 1
    mask = np.zeros(n, dtype=np.uint8)
    mask[t0:t1] = 1
    slot = np.concatenate([[0], np.cumsum(mask[:-1] == 0)]).astype(np.int32)
    ab, ob = O.score(q[None, :], K, V)
    res = O.merge_compact(K, V, ab, ob, mask, slot, rule="diagonal")
    J = fd_ds_de(q, K, V)
    g = np.array([np.linalg.norm(J[t, t]) for t in range(t0, t1 + 1)])
    x = K[t0:t1 + 1] @ q
    xstar = minimize_scalar(lambda z: ((z - x) ** 2 * g).sum(), bracket=(x.min() - 1, x.mean(), x.max() + 1),
                            tol=1e-14).x
    assert abs(q @ res.K_out[t0] - xstar) < 2e-6 * max(1.0, abs(xstar))
    # and it differs from the full rule: the coupling term is visible on a tiny head
    full = O.merge_compact(K, V, ab, ob, mask, slot)
    assert np.linalg.norm(full.K_out[t0] - res.K_out[t0]) > 1e-4 * np.linalg.norm(full.K_out[t0])


# --------------------------------------------------------------------------------------------
# The consumer of a merged cache
def test_decode_attention_over_a_merged_cache_is_attention_over_the_tokens_it_stands_for():
    rng = np.random.default_rng(60)
    n, d = 11, 6
    K, V = rng.standard_normal((n, d)) * 1.5, rng.standard_normal((n, d)) * 2.0
    c = rng.integers(1, 5, size=n)
    Ke, Ve, _ = expanded_cache(K, V, c)
    Q = rng.standard_normal((2, 3, d))
    got = O.decode_attention(Q, K, V, c)
    want = np.stack([softmax_attention(q, Ke, Ve)[1] for q in Q.reshape(-1, d)])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    plain = O.decode_attention(Q, K, V)
    np.testing.assert_allclose(plain, np.stack([softmax_attention(q, K, V)[1] for q in Q.reshape(-1, d)]), rtol=1e-12)


# --------------------------------------------------------------------------------------------
# per-query aggregation: every query row keeps its own attention and output; the norms are averaged
def test_per_query_norms_are_the_mean_of_single_query_finite_difference_norms():
    """Each row q by itself is the paper's single-query case: its blocks d s_i / d e_j come from central
    differences of textbook attention (nothing of the oracle), and the aggregate is their norms' mean."""
    rng = np.random.default_rng(60)
    n, d, dv, R = 6, 4, 5, 3
    Q = rng.standard_normal((R, d)) * 1.5
    K = rng.standard_normal((n, d)) * 1.5
    V = rng.standard_normal((n, dv))
    A_want = np.zeros(n)
    C_want = np.zeros(n - 1)
    for q in Q:
        J = fd_ds_de(q, K, V)
        A_want += [np.linalg.norm(J[i, i]) for i in range(n)]
        C_want += [np.linalg.norm(J[i, i + 1]) for i in range(n - 1)]
    A, C = O.per_query_norms(Q, K, V)
    np.testing.assert_allclose(A, A_want / R, rtol=1e-7)
    np.testing.assert_allclose(C, C_want / R, rtol=1e-7)


def test_per_query_norms_special_cases():
    rng = np.random.default_rng(61)
    n, d = 40, 8
    K = rng.standard_normal((n, d)) * 2.0
    V = rng.standard_normal((n, d))
    q = rng.standard_normal(d)
    # identical rows: every row has the mean attention and the mean output, the two aggregations agree
    Q = np.tile(q, (5, 1))
    ab, ob = O.score(Q, K, V)
    A0, C0 = O.token_and_edge_norms(ab, V, ob)
    A, C = O.per_query_norms(Q, K, V)
    np.testing.assert_allclose(A, A0, rtol=1e-12)
    np.testing.assert_allclose(C, C0, rtol=1e-12)
    # the order of the rows does not matter; [G, W, D] is read as G*W rows
    Q = rng.standard_normal((2, 3, d))
    A1, C1 = O.per_query_norms(Q, K, V)
    A2, C2 = O.per_query_norms(Q.reshape(6, d)[::-1], K, V)
    np.testing.assert_allclose(A1, A2, rtol=1e-13)
    np.testing.assert_allclose(C1, C2, rtol=1e-13)
    # rows that disagree: the aggregate differs from the mean-first norms (the mode is not a no-op)
    ab, ob = O.score(Q, K, V)
    A0, _ = O.token_and_edge_norms(ab, V, ob)
    assert np.max(np.abs(A1 - A0) / A0) > 1e-3


def test_per_query_norms_closed_forms_of_rows_that_concentrate():
    """Closed forms.  A row with all its weight on token t has o = v_t: it adds nothing to any A or C.  A row that
    splits its weight evenly between t and t + 1 has o = (v_t + v_{t+1}) / 2: alpha (1 - 2 alpha) = 0, so it adds
    nothing to A, and ||v_t + v_{t+1} - 2 o|| = 0, so nothing to C either.  A row with weights (a, 1 - a) on the two
    adds a |1 - 2a| (1 - a) ||v_t - v_{t+1}|| to A_t, the same with a and 1 - a exchanged to A_{t+1}, and
    a (1 - a) |1 - 2a| ||v_t - v_{t+1}|| to C_t.  Identical Values give zero norms whatever the weights."""
    rng = np.random.default_rng(66)
    n, d = 12, 6
    V = rng.standard_normal((n, d))
    big = 60.0                                       # logit gap: the other tokens' weights are below 1e-25
    K = np.zeros((n, n))
    np.fill_diagonal(K, 1.0)                         # token t answers to query e_t alone
    scale = 1.0 / np.sqrt(n)

    def row(weights):
        """A query whose logits are ln(weight) on the named tokens and -big elsewhere."""
        e = np.full(n, -big)
        for t, w in weights.items():
            e[t] = np.log(w)
        return e / scale

    t = 4
    one_hot = row({t: 1.0})
    halves = row({t: 0.5, t + 1: 0.5})
    a = 0.8
    uneven = row({t: a, t + 1: 1 - a})
    A, C = O.per_query_norms(np.stack([one_hot, halves]), K, V)
    assert np.max(A) < 1e-15 and np.max(C) < 1e-15     # (the halves' o carries fp64 rounding)
    A, C = O.per_query_norms(uneven[None, :], K, V)
    gap = np.linalg.norm(V[t] - V[t + 1])
    want_A = np.zeros(n)
    want_A[t] = a * abs(1 - 2 * a) * (1 - a) * gap
    want_A[t + 1] = (1 - a) * abs(1 - 2 * (1 - a)) * a * gap
    want_C = np.zeros(n - 1)
    want_C[t] = a * (1 - a) * abs(1 - 2 * a) * gap
    np.testing.assert_allclose(A, want_A, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(C, want_C, rtol=1e-12, atol=1e-15)
    # the three rows together: the mean of their shares
    A3, C3 = O.per_query_norms(np.stack([one_hot, halves, uneven]), K, V)
    np.testing.assert_allclose(A3, want_A / 3, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(C3, want_C / 3, rtol=1e-12, atol=1e-15)
    # identical Values
    Q = rng.standard_normal((5, n))
    A, C = O.per_query_norms(Q, K, np.tile(V[0], (n, 1)))
    assert np.max(A) < 1e-15 and np.max(C) < 1e-15


def test_per_query_norms_with_counts():
    """Streaming regime, every query row apart.  Each row by itself is the single-query case with slots of
    cardinality c: the blocks d s_t / d e_j of s_t = alpha_t (V_t / c_t - o) at logits e + ln c, by central
    differences of textbook attention; cardinalities of one change nothing; one row is the averaged rule; and a
    row's output is textbook attention over the cache the slots stand for."""
    rng = np.random.default_rng(64)
    n, d, dv, R = 6, 4, 5, 3
    Q = rng.standard_normal((R, d)) * 1.5
    K = rng.standard_normal((n, d)) * 1.5
    V = rng.standard_normal((n, dv)) * 2.0
    c = np.array([2, 1, 3, 1, 4, 2])
    Vs = V / c[:, None]
    A_want, C_want = np.zeros(n), np.zeros(n - 1)
    h = 1e-5
    for q in Q:
        e0 = K @ q / np.sqrt(d) + np.log(c)
        J = np.zeros((n, n, dv))
        for j in range(n):
            ep, em = e0.copy(), e0.copy()
            ep[j] += h
            em[j] -= h
            J[:, j, :] = (s_of_logits(ep, Vs) - s_of_logits(em, Vs)) / (2 * h)
        A_want += [np.linalg.norm(J[i, i]) for i in range(n)]
        C_want += [np.linalg.norm(J[i, i + 1]) for i in range(n - 1)]
    A, C = O.per_query_norms(Q, K, V, counts=c)
    np.testing.assert_allclose(A, A_want / R, rtol=1e-7)
    np.testing.assert_allclose(C, C_want / R, rtol=1e-7)
    # cardinalities of one: bit for bit the plain call
    A1, C1 = O.per_query_norms(Q, K, V, counts=np.ones(n, dtype=np.int32))
    A0, C0 = O.per_query_norms(Q, K, V)
    assert np.array_equal(A1, A0) and np.array_equal(C1, C0)
    # one row: the averaged rule with cardinalities
    ab, ob = O.score(Q[:1], K, V, counts=c)
    Aa, Ca = O.token_and_edge_norms(ab, V, ob, counts=c)
    Ar, Cr = O.per_query_norms(Q[:1], K, V, counts=c)
    np.testing.assert_allclose(Ar, Aa, rtol=1e-13)
    np.testing.assert_allclose(Cr, Ca, rtol=1e-13)
    # the step with both switches uses these norms
    st = O.step(Q, K, V, budget=4, n_sink=1, counts=c, per_query=True)
    ref = O.merge_compact(K, V, st.alpha_bar, st.o_bar, st.mask, st.slot, counts_in=c, norms=(A, C))
    assert np.array_equal(st.merged.K_out, ref.K_out) and np.array_equal(st.merged.counts, ref.counts)


@pytest.mark.parametrize("seed,L", [(62, 2), (63, 3)])
def test_per_query_merged_key_minimises_the_summed_surrogate(seed, L):
    """With norms=(A, C) the merged Key of a run minimises, along q-independent weights, the surrogate
    sum_ab g_ab (k - k_a).(k - k_b)-type objective whose blocks are the AVERAGED norms: the stationary point
    is K' = sum_a w_a k_a with w_a = sum_b g_ab / sum_ab g_ab, g_tt = A_t, g_{t,t+1} = -C_t, written here as
    a dense solve."""
    rng = np.random.default_rng(seed)
    n, d, R = L + 3, 4, 4
    Q = rng.standard_normal((R, d)) * 0.3
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    mask = np.zeros(n, dtype=np.uint8)
    t0 = 1
    mask[t0:t0 + L - 1] = 1
    starts = np.ones(n, dtype=np.int64)
    starts[1:] = 1 - mask[:-1]
    slot = (np.cumsum(starts) - 1).astype(np.int32)
    A, C = O.per_query_norms(Q, K, V)
    ab, ob = O.score(Q, K, V)
    res = O.merge_compact(K, V, ab, ob, mask, slot, norms=(A, C))
    G = np.diag(A[t0:t0 + L])
    for i in range(L - 1):
        G[i, i + 1] = G[i + 1, i] = -C[t0 + i]
    w = G.sum(axis=1) / G.sum()
    assert G.sum() > 0
    np.testing.assert_allclose(res.K_out[t0], w @ K[t0:t0 + L], rtol=1e-12)
    # the other rows and all Values do not depend on the aggregation
    base = O.merge_compact(K, V, ab, ob, mask, slot)
    np.testing.assert_array_equal(res.V_out, base.V_out)
    np.testing.assert_array_equal(res.counts, base.counts)
    keep = np.ones(res.K_out.shape[0], dtype=bool)
    keep[t0] = False
    np.testing.assert_array_equal(res.K_out[keep], base.K_out[keep])


def test_step_per_query_with_one_row_is_the_plain_step():
    rng = np.random.default_rng(64)
    n, d = 96, 8
    Q = rng.standard_normal((1, d))
    K = rng.standard_normal((n, d)) * 2
    V = rng.standard_normal((n, d))
    a = O.step(Q, K, V, 48, n_sink=4)
    b = O.step(Q, K, V, 48, n_sink=4, per_query=True)
    np.testing.assert_array_equal(a.mask, b.mask)
    np.testing.assert_allclose(a.merged.K_out, b.merged.K_out, rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------------------------
# causal mask inside the window
def test_causal_rows_are_textbook_attention_over_the_cache_up_to_their_position():
    rng = np.random.default_rng(70)
    n, d, G, W = 40, 8, 2, 5
    Q = rng.standard_normal((G, W, d))
    K = rng.standard_normal((n, d)) * 2.0
    V = rng.standard_normal((n, d))
    alpha = O.attention_rows(Q, K, causal_window=W)
    for g in range(G):
        for w in range(W):
            seen = n - W + w + 1                         # the query at window position w sits at row n - W + w
            a, _ = softmax_attention(Q[g, w], K[:seen], V[:seen])
            np.testing.assert_allclose(alpha[g * W + w, :seen], a, rtol=1e-13)
            assert (alpha[g * W + w, seen:] == 0).all()
    # the last position sees everything: same as without the mask
    full = O.attention_rows(Q, K)
    np.testing.assert_allclose(alpha[W - 1::W], full[W - 1::W], rtol=1e-14)
    # score and the per-query norms are built on these rows
    ab, ob = O.score(Q, K, V, causal_window=W)
    np.testing.assert_allclose(ab, alpha.mean(axis=0), rtol=1e-14)
    np.testing.assert_allclose(ob, alpha.mean(axis=0) @ V, rtol=1e-13)
    A, C = O.per_query_norms(Q, K, V, causal_window=W)
    A_want = np.zeros(n)
    for q in range(G * W):
        seen = n - W + q % W + 1
        a_q, o_q = softmax_attention(Q.reshape(-1, d)[q], K[:seen], V[:seen])
        Aq, _ = O.token_and_edge_norms(a_q, V[:seen], o_q)   # (pinned by finite differences above)
        A_want[:seen] += Aq
    np.testing.assert_allclose(A, A_want / (G * W), rtol=1e-12)
    assert C[-1] > 0 and A[-1] > 0                       # the last token is seen by the last position only


def test_causal_window_of_one_and_with_counts():
    rng = np.random.default_rng(71)
    n, d = 30, 4
    Q = rng.standard_normal((3, 1, d))
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    np.testing.assert_array_equal(O.attention_rows(Q, K, causal_window=1), O.attention_rows(Q, K))
    # a masked row of cardinality c: c copies of the row, all masked or all seen
    c = rng.integers(1, 4, size=n)
    c[-4:] = 1                                           # the window's own rows are fresh tokens
    Q4 = rng.standard_normal((1, 4, d))
    a = O.attention_rows(Q4, K, counts=c, causal_window=4)
    Kx = np.repeat(K, c, axis=0)
    ax = O.attention_rows(Q4, Kx, causal_window=4)
    ends = np.cumsum(c)
    for t in range(n):
        np.testing.assert_allclose(a[:, t], ax[:, ends[t] - c[t]:ends[t]].sum(axis=1), rtol=1e-12, atol=1e-300)


# ------------------------------------------------------------------------------------------------
# The two helpers that decide which seeded units the GPU tests see (the acceptance rule of tests/helpers.py)
def test_boundary_gap_worked_example_and_brute_force():
    """boundary_gap is the relative distance between the r-th and the (r+1)-th smallest eligible edge score
    (App. C (i): pairs ranked by accumulated attention mass; Sec. 3.1: r = n - budget of them merge).  A worked
    example by hand, then plain Python loops (no numpy sorting, no shared helper) on random tiny inputs, then what
    the number means: a relative change of the scores below half the gap cannot change the selected set, and
    there is one of the size of the gap that does."""
    # tokens 0..5, one sink token, one recent token: eligible edges 1, 2, 3 with scores .15, .25, .45
    a = np.array([0.30, 0.10, 0.05, 0.20, 0.25, 0.10])
    assert O.boundary_gap(a, budget=4, n_sink=1, n_recent=1) == pytest.approx((0.45 - 0.25) / 0.45, rel=1e-12)
    assert O.boundary_gap(a, budget=5, n_sink=1, n_recent=1) == pytest.approx((0.25 - 0.15) / 0.25, rel=1e-12)
    assert O.boundary_gap(a, budget=6, n_sink=1, n_recent=1) == float("inf")      # nothing to merge
    assert O.boundary_gap(a, budget=3, n_sink=1, n_recent=1) == float("inf")      # every eligible edge merges
    # without the recent token edge 4 (score .35) is eligible too: sorted .15 .25 .35 .45
    assert O.boundary_gap(a, budget=4, n_sink=1, n_recent=0) == pytest.approx((0.35 - 0.25) / 0.35, rel=1e-12)
    # the sink moves the first eligible edge: with n_sink = 0 edge 0 (score .40) joins: .15 .25 .40 .45, r = 3
    assert O.boundary_gap(a, budget=3, n_sink=0, n_recent=1) == pytest.approx((0.45 - 0.40) / 0.45, rel=1e-12)

    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(4, 14))
        s, nr = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        a = rng.dirichlet(np.ones(n))
        edges = [m for m in range(n - 1) if s <= m <= n - 2 - nr]
        if len(edges) < 2:
            continue
        r = int(rng.integers(1, len(edges)))
        scores = [float(a[m]) + float(a[m + 1]) for m in edges]
        ranked = []
        pool = list(scores)
        while pool:                                        # selection sort by hand
            lo = min(range(len(pool)), key=lambda i: pool[i])
            ranked.append(pool.pop(lo))
        want = (ranked[r] - ranked[r - 1]) / ranked[r]
        got = O.boundary_gap(a, budget=n - r, n_sink=s, n_recent=nr)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-300)
        # meaning: scores perturbed by a relative eps < gap / 2 select the same edges ...
        if want > 1e-6:
            sel = set(np.flatnonzero(O.select(a, n - r, s, nr)[0]))
            for sign in (+1, -1):
                sig = np.array(scores) * (1 + sign * 0.49 * want * rng.uniform(-1, 1, len(scores)))
                order = sorted(range(len(sig)), key=lambda i: (sig[i], i))[:r]
                assert {edges[i] for i in order} == sel


def test_conditioning_worked_example_and_brute_force():
    """conditioning is the smallest ratio, over the slots of several rows, of the weight denominator of Eq. kstar_final
    (A_m - 2 C_m + A_{m+1} for a pair; sum of the u_t for a run) to the slot's sum of A_t.  A pair by hand with the
    vectors of Eqs. c11_def-c12_def written out, slots of one row ignored, then loops over explicit c-vectors."""
    # one dimension, o = 0: residuals 1 and 3, masses .1 and .2
    #   c11 = .1 (1 - .2) 1 = .08, c22 = .2 (1 - .4) 3 = .36, c12 = -.1 .2 (1 + 3) = -.08
    #   denominator .08 - 2 (.08) + .36 = .28, sum of A = .44
    K = np.array([[1.0], [2.0], [5.0]])
    V = np.array([[1.0], [3.0], [7.0]])
    alpha = np.array([0.1, 0.2, 0.7])
    mask = np.array([1, 0, 0], dtype=np.uint8)
    slot = np.array([0, 0, 1], dtype=np.int32)
    res = O.merge_compact(K, V, alpha, np.zeros(1), mask, slot)
    assert O.conditioning(res) == pytest.approx(0.28 / 0.44, rel=1e-12)
    # the single row's own ratio (1) is not what is reported, and without merged slots the value is 1
    assert O.conditioning(O.merge_compact(K, V, alpha, np.zeros(1), np.zeros(3, np.uint8), np.arange(3, dtype=np.int32))) == 1.0
    # a non-positive denominator shows as a non-positive ratio (masses of one half: A = 0, C > 0)
    res = O.merge_compact(K, V, np.array([0.5, 0.5, 0.0]), np.zeros(1), mask, slot)
    assert res.fallback[0] and res.U[0] == pytest.approx(-2.0) and O.conditioning(res) == -np.inf

    rng = np.random.default_rng(9)
    for _ in range(100):
        n, D = int(rng.integers(3, 12)), int(rng.integers(1, 4))
        K, V = rng.standard_normal((n, D)), rng.standard_normal((n, D))
        alpha = rng.dirichlet(np.ones(n))
        o = alpha @ V
        mask = (rng.random(n) < 0.5).astype(np.uint8)
        mask[-1] = 0
        starts = [t for t in range(n) if t == 0 or mask[t - 1] == 0]
        slot = np.cumsum([1 if t in starts else 0 for t in range(n)]).astype(np.int32) - 1
        ratios = []
        for i, t0 in enumerate(starts):
            t1 = (starts[i + 1] if i + 1 < len(starts) else n) - 1
            if t1 == t0:
                continue
            c_diag = [alpha[t] * (1 - 2 * alpha[t]) * (V[t] - o) for t in range(t0, t1 + 1)]
            c_off = [-alpha[t] * alpha[t + 1] * (V[t] + V[t + 1] - 2 * o) for t in range(t0, t1)]
            a_sum = sum(float(np.sqrt(c @ c)) for c in c_diag)
            denom = a_sum - 2 * sum(float(np.sqrt(c @ c)) for c in c_off)
            ratios.append(denom / a_sum)
        res = O.merge_compact(K, V, alpha, o, mask, slot)
        want = min(ratios) if ratios else 1.0
        assert O.conditioning(res) == pytest.approx(want, rel=1e-10, abs=1e-12)
