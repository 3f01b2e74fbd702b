"""Pins for the float64 oracle against things that are not the oracle: definitions written out as loops,
numpy's least-squares routine, brute force over all supports, closed forms and special cases.
Citations are to the paper's sections / equations."""
import itertools
import math
import os

import numpy as np
import pytest

import osscar_inputs as inp
from oracle import osscar_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_problem(p, q, m, n, seed, corr=0.6, lam=1e-3):
    rng = np.random.default_rng(seed)
    d1 = p * q
    Z = rng.standard_normal((n, d1))
    # correlated columns so that swaps are non-trivial
    A = np.eye(d1) + corr * rng.standard_normal((d1, d1)) / math.sqrt(d1)
    X = Z @ A
    W = rng.standard_normal((d1, m)) / math.sqrt(d1)
    H, G, c0, lam_used = orc.gram(X, W, lam_abs=lam)
    return X, W, H, G, c0, lam_used


# ---------------------------------------------------------------- Gram / objective (Section 3)
def test_gram_is_sum_of_outer_products():
    X, W, H, G, c0, lam = make_problem(6, 1, 3, 20, 0, lam=0.25)
    H_loop = np.zeros((6, 6))
    for i in range(X.shape[0]):
        for a in range(6):
            for b in range(6):
                H_loop[a, b] += X[i, a] * X[i, b]
    for a in range(6):
        H_loop[a, a] += 0.25
    assert np.allclose(H, H_loop, rtol=1e-13, atol=1e-13)
    assert np.allclose(H, H.T)
    assert np.min(np.linalg.eigvalsh(H)) > 0
    assert np.allclose(G, H_loop @ W)
    assert np.isclose(c0, np.trace(W.T @ H_loop @ W))


def test_lambda_rel_uses_diag_before_ridge():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((50, 5))
    W = rng.standard_normal((5, 2))
    H, G, c0, lam = orc.gram(X, W, lam_abs=0.5, lam_rel=0.1)
    want = 0.5 + 0.1 * np.mean(np.sum(X * X, axis=0))
    assert np.isclose(lam, want, rtol=1e-14)
    assert np.allclose(H - X.T @ X, lam * np.eye(5), atol=1e-12)


def test_quadratic_objective_equals_reconstruction_loss():
    # pins the minus sign of the linear term (eq. (MIQP)) and c0
    X, W, H, G, c0, lam = make_problem(8, 1, 4, 40, 2)
    rng = np.random.default_rng(3)
    What = rng.standard_normal(W.shape)
    assert np.isclose(orc.objective_direct(X, W, What, lam), orc.objective_quadratic(H, G, c0, What), rtol=1e-11)
    assert abs(orc.objective_quadratic(H, G, c0, W)) < 1e-9 * c0


def test_objective_of_a_state_equals_the_pruned_rows_form():
    """With G = H W the optimum on a support K (Appendix A.1) can be written without the constant: obj(K) = <W_c, R_c>,
    R_c = G_c - H_cK B over the pruned rows, instead of c0 - <G_K, B>, a difference of two numbers of the size of c0.
    The library reports the first form; here both are held against the reconstruction loss of the solved weights."""
    for q, seed in ((1, 11), (3, 12)):
        p, m, n = 7, 5, 50
        X, W, H, G, c0, lam = make_problem(p, q, m, n, seed, lam=0.2)
        groups = [1, 2, 4, 6]
        What, obj = orc.solve_support(H, G, c0, groups, q)
        K = orc.rows_of(groups, q)
        Cc = np.setdiff1d(np.arange(p * q), K)
        B = np.linalg.solve(H[np.ix_(K, K)], G[K])
        R = G[Cc] - H[np.ix_(Cc, K)] @ B
        pruned_form = float(np.sum(W[Cc] * R))
        assert np.isclose(pruned_form, obj, rtol=1e-10)
        assert np.isclose(pruned_form, c0 - float(np.sum(G[K] * B)), rtol=1e-10)
        assert np.isclose(pruned_form, orc.objective_direct(X, W, What, lam), rtol=1e-10)


# ---------------------------------------------------------------- optimum for a fixed support (eq. (optf))
@pytest.mark.parametrize("q", [1, 3])
def test_solve_support_matches_ridge_least_squares(q):
    p, m, n = 6, 4, 60
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 4, lam=0.3)
    groups = [0, 2, 5]
    What, obj = orc.solve_support(H, G, c0, groups, q)
    rows = orc.rows_of(groups, q)
    # textbook ridge LS on the stacked system [X_K; sqrt(lam) I_K; 0] What_K ~ [X W; sqrt(lam) W]
    d1 = p * q
    A = np.vstack([X[:, rows], math.sqrt(lam) * np.eye(d1)[:, rows]])
    Y = np.vstack([X @ W, math.sqrt(lam) * W])
    sol, *_ = np.linalg.lstsq(A, Y, rcond=None)
    assert np.allclose(What[rows], sol, rtol=1e-8, atol=1e-10)
    other = np.setdiff1d(np.arange(d1), rows)
    assert np.all(What[other] == 0)
    assert np.isclose(obj, orc.objective_direct(X, W, What, lam), rtol=1e-10)
    # normal equations on the kept rows; eq. (optf): f = -1/2 Tr(G_K^T H_KK^-1 G_K)
    assert np.allclose(H[np.ix_(rows, rows)] @ What[rows], G[rows], rtol=1e-9, atol=1e-9)
    f = -0.5 * np.trace(G[rows].T @ np.linalg.inv(H[np.ix_(rows, rows)]) @ G[rows])
    assert np.isclose(obj, c0 + 2 * f, rtol=1e-10)


def test_keep_everything_recovers_dense_weights():
    X, W, H, G, c0, lam = make_problem(5, 2, 3, 30, 5)
    What, obj = orc.solve_support(H, G, c0, range(5), 2)
    assert np.allclose(What, W, atol=1e-10)
    assert abs(obj) < 1e-9 * c0


def test_residual_identity_on_pruned_rows():
    # obj(K) = <W_Kc, R>, R = G_Kc - H_{Kc,K} What_K  (follows from G = H W and the normal equations)
    X, W, H, G, c0, lam = make_problem(7, 2, 3, 50, 6)
    groups = [1, 3, 4]
    What, obj = orc.solve_support(H, G, c0, groups, 2)
    rows = orc.rows_of(groups, 2)
    crow = np.setdiff1d(np.arange(14), rows)
    R = G[crow] - H[np.ix_(crow, rows)] @ What[rows]
    assert np.isclose(obj, np.sum(W[crow] * R), rtol=1e-10)


# ---------------------------------------------------------------- enumeration (Section 4.1)
def test_combination_counter_matches_paper_count():
    with open(os.path.join(GOLDEN, "paper_counts.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    for name, n, k, lower, exact in rows:
        c = orc.n_choose_k(int(n), int(k))
        assert c > int(lower)
        assert c == int(exact) == math.comb(int(n), int(k))
    assert orc.n_choose_k(16, 8) == 12870


def test_brute_force_enumerates_everything_and_search_is_bounded_by_it():
    cfg = inp.CONFIGS["cfg1x"]
    X = inp.gen_X(cfg).double().numpy()
    W = inp.gen_W(cfg).double().numpy()
    H, G, c0, lam = orc.gram(X, W, cfg.lam_abs, cfg.lam_rel)
    best, best_obj, objs = orc.brute_force(H, G, c0, cfg.p, cfg.q, cfg.k)
    assert len(objs) == 12870
    assert best_obj == objs.min()
    # spot-check three enumerated objectives against the reconstruction loss itself
    combos = list(itertools.combinations(range(cfg.p), cfg.k))
    for idx in (0, 6000, 12869):
        What, o = orc.solve_support(H, G, c0, combos[idx], cfg.q)
        assert np.isclose(objs[idx], orc.objective_direct(X, W, What, lam), rtol=1e-9)
    # search from the magnitude support cannot beat the global optimum, and never gets worse than its start
    K0 = orc.magnitude_support(W, cfg.p, cfg.q, cfg.k)
    res = orc.local_search(H, G, c0, K0, cfg.p, cfg.q, cfg.swaps)
    assert res.obj_final >= best_obj * (1 - 1e-12)
    assert res.obj_final <= res.obj_initial
    # the global optimum is a fixed point: no 1-out/1-in swap improves it, so nothing is accepted
    res2 = orc.local_search(H, G, c0, best, cfg.p, cfg.q, 10)
    assert res2.accepted == 0 and res2.support == sorted(best)
    # and whatever the search returns is 1-swap-stable only w.r.t. its selected pair; check its objective
    _, o = orc.solve_support(H, G, c0, res.support, cfg.q)
    assert np.isclose(o, res.obj_final, rtol=1e-9)


# ---------------------------------------------------------------- impact scores (eq. (impact), Prop. 4.1)
@pytest.mark.parametrize("q", [1, 2, 4])
def test_scores_equal_differences_of_full_resolves(q):
    p, m, n, k = 9, 5, 80, 5
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 7 + q)
    K = [0, 2, 3, 6, 8]
    st = orc.init_state(H, G, K, q)
    _, objK = orc.solve_support(H, G, c0, K, q)
    assert np.isclose(c0 + 2 * st.f, objK, rtol=1e-10)
    rem = orc.removal_scores(st, p, q)
    add = orc.addition_scores(st, H, G, p, q)
    for g in range(p):
        if g in K:
            _, o = orc.solve_support(H, G, c0, [x for x in K if x != g], q)
            assert np.isclose(rem[g], o - objK, rtol=1e-8), ("rem", g)
            assert rem[g] >= 0 and add[g] == -np.inf
        else:
            _, o = orc.solve_support(H, G, c0, K + [g], q)
            assert np.isclose(add[g], objK - o, rtol=1e-8), ("add", g)
            assert add[g] >= 0 and rem[g] == np.inf
            # the one-candidate Case-2 formula agrees with the batched evaluation
            assert np.isclose(orc.addition_score(st, H, G, g, q), add[g], rtol=1e-9)


@pytest.mark.parametrize("q", [1, 3])
def test_updates_match_fresh_state_and_are_involutive(q):
    p, m, n = 8, 4, 70
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 20 + q)
    K = [1, 2, 4, 7]
    st = orc.init_state(H, G, K, q)
    rows = orc.rows_of(K, q)
    assert np.allclose(st.P @ H[np.ix_(rows, rows)], np.eye(len(rows)), atol=1e-9)
    # Case 1: remove group 4 (slot 2)
    mid = orc.remove_group(st, 2, q)
    fresh = orc.init_state(H, G, [1, 2, 7], q)
    assert mid.groups == [1, 2, 7]
    assert np.allclose(mid.P, fresh.P, rtol=1e-8, atol=1e-11)
    assert np.allclose(mid.What_K, fresh.What_K, rtol=1e-8, atol=1e-11)
    assert np.isclose(mid.f, fresh.f, rtol=1e-10)
    assert mid.f > st.f                      # removing rows raises f (sign reading of the f update)
    # Case 2: add group 5
    new = orc.add_group(mid, H, G, 5, q)
    fresh2 = orc.init_state(H, G, [1, 2, 7, 5], q)
    assert new.groups == [1, 2, 7, 5]
    assert np.allclose(new.P, fresh2.P, rtol=1e-8, atol=1e-11)
    assert np.allclose(new.What_K, fresh2.What_K, rtol=1e-8, atol=1e-11)
    assert np.isclose(new.f, fresh2.f, rtol=1e-10)
    assert new.f < mid.f                     # adding rows lowers f
    # involution: remove 4 then add 4 gives back the state (up to the slot permutation)
    back = orc.add_group(mid, H, G, 4, q)
    ref = orc.init_state(H, G, [1, 2, 7, 4], q)
    assert np.allclose(back.P, ref.P, rtol=1e-8, atol=1e-11)
    assert np.isclose(back.f, st.f, rtol=1e-10)
    # the optimal weights are the solution of the normal equations on the kept rows
    r2 = orc.rows_of(new.groups, q)
    assert np.allclose(H[np.ix_(r2, r2)] @ new.What_K, G[r2], rtol=1e-8, atol=1e-9)


@pytest.mark.parametrize("q", [1, 3])
def test_swap_delta_equals_resolve_difference(q):
    p, m, n = 8, 4, 70
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 30 + q)
    K = [0, 3, 5, 6]
    st = orc.init_state(H, G, K, q)
    _, objK = orc.solve_support(H, G, c0, K, q)
    for g in K:
        for j in (1, 2, 4, 7):
            delta, _ = orc.swap_delta(st, H, G, g, j, q)
            _, o = orc.solve_support(H, G, c0, [x for x in K if x != g] + [j], q)
            assert np.isclose(delta, o - objK, rtol=1e-7, atol=1e-9 * objK)


# ---------------------------------------------------------------- search invariants
@pytest.mark.parametrize("q,seed", [(1, 40), (2, 41), (1, 42)])
def test_search_objective_is_monotone_and_tracked_exactly(q, seed):
    p, m, n, k = 24, 6, 200, 10
    X, W, H, G, c0, lam = make_problem(p, q, m, n, seed, corr=1.5)
    K0 = orc.magnitude_support(W, p, q, k)
    res = orc.local_search(H, G, c0, K0, p, q, 40)
    objs = [res.obj_initial] + [r.obj_after for r in res.trace if r.accepted]
    assert all(b < a for a, b in zip(objs, objs[1:]))
    assert res.accepted >= 1                                  # the planted correlation makes swaps pay
    for r in res.trace:
        if r.accepted:
            assert r.delta < 0
    _, o = orc.solve_support(H, G, c0, res.support, q)
    assert np.isclose(o, res.obj_final, rtol=1e-9)
    What, _ = orc.solve_support(H, G, c0, res.support, q)
    assert np.isclose(o, orc.objective_direct(X, W, What, lam), rtol=1e-9)
    assert len(res.support) == k and len(set(res.support)) == k
    # the last record is the rejected one (or the budget ran out)
    assert res.iters == res.accepted or (res.iters == res.accepted + 1 and not res.trace[-1].accepted)


@pytest.mark.parametrize("q,seed", [(1, 60), (3, 61), (1, 62)])
def test_exact_entering_rule_is_the_best_pair_by_brute_force(q, seed):
    """With the leaving group fixed, the exact rule must pick the j that minimises obj(K - g + j) solved from scratch,
    its score must be that objective's drop from the state without g, and its first move can only be at least as
    good as the separable rule's."""
    p, m, n, k = 12, 4, 120, 5
    X, W, H, G, c0, lam = make_problem(p, q, m, n, seed, corr=1.5)
    K0 = orc.magnitude_support(W, p, q, k)
    st = orc.init_state(H, G, sorted(K0), q)
    g = int(np.argmin(orc.removal_scores(st, p, q)))
    res = orc.local_search(H, G, c0, K0, p, q, 1, exact_in=True, always_accept=True)
    r = res.trace[0]
    assert r.g_out == g
    Kg = [x for x in sorted(K0) if x != g]
    _, obj_mid = orc.solve_support(H, G, c0, Kg, q)
    objs = {j: orc.solve_support(H, G, c0, sorted(Kg + [j]), q)[1] for j in range(p) if j not in K0}
    best = min(objs, key=objs.get)
    assert r.j_in == best
    assert np.isclose(r.add, obj_mid - objs[best], rtol=1e-8)
    _, objK = orc.solve_support(H, G, c0, sorted(K0), q)
    assert np.isclose(r.delta, objs[best] - objK, rtol=1e-7, atol=1e-9 * objK)
    sep = orc.local_search(H, G, c0, K0, p, q, 1, always_accept=True).trace[0]
    assert sep.g_out == g and r.delta <= sep.delta + 1e-12 * objK
    # a whole run: monotone, and the tracked objective is the fresh solve's
    run = orc.local_search(H, G, c0, K0, p, q, 30, exact_in=True)
    o = [run.obj_initial] + [x.obj_after for x in run.trace if x.accepted]
    assert all(b < a for a, b in zip(o, o[1:]))
    assert np.isclose(orc.solve_support(H, G, c0, run.support, q)[1], run.obj_final, rtol=1e-9)
    # follow mode on its own trajectory: zero deficits
    pairs = [(x.g_out, x.j_in) for x in run.trace if x.accepted]
    fol = orc.local_search(H, G, c0, K0, p, q, len(pairs), follow=pairs, exact_in=True)
    assert all(x.deficit_rem == 0 and x.deficit_add == 0 for x in fol.trace)
    assert fol.support == run.support


def test_follow_mode_reproduces_free_run_with_zero_deficit():
    p, q, m, n, k = 20, 1, 5, 150, 8
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 50, corr=1.5)
    K0 = orc.magnitude_support(W, p, q, k)
    free = orc.local_search(H, G, c0, K0, p, q, 30)
    pairs = [(r.g_out, r.j_in) for r in free.trace if r.accepted]
    fol = orc.local_search(H, G, c0, K0, p, q, 30, follow=pairs)
    assert fol.support == free.support
    assert np.isclose(fol.obj_final, free.obj_final, rtol=1e-12)
    assert all(r.deficit_rem == 0 and r.deficit_add == 0 for r in fol.trace)
    # a deliberately second-best choice shows up as a positive deficit
    st = orc.init_state(H, G, K0, q)
    rem = orc.removal_scores(st, p, q)
    second = int(np.argsort(rem)[1])
    bad = orc.local_search(H, G, c0, K0, p, q, 1, follow=[(second, pairs[0][1])])
    assert bad.trace[0].deficit_rem > 0


def test_diagonal_H_closed_form():
    # orthogonal columns: rem_g = add_g = H_gg ||W_g||^2, the optimum keeps the k largest, search reaches it
    rng = np.random.default_rng(60)
    p, m, k = 12, 4, 5
    Qm, _ = np.linalg.qr(rng.standard_normal((40, p)))
    X = Qm * rng.uniform(0.5, 3.0, size=p)[None, :]
    W = rng.standard_normal((p, m))
    H, G, c0, lam = orc.gram(X, W, lam_abs=0.1)
    assert np.allclose(H, np.diag(np.diag(H)), atol=1e-12)
    imp = np.diag(H) * np.sum(W * W, axis=1)
    K0 = orc.magnitude_support(W, p, 1, k)
    st = orc.init_state(H, G, K0, 1)
    rem = orc.removal_scores(st, p, 1)
    add = orc.addition_scores(st, H, G, p, 1)
    for g in range(p):
        assert np.isclose(rem[g] if g in K0 else add[g], imp[g], rtol=1e-9)
    res = orc.local_search(H, G, c0, K0, p, 1, 50)
    want = sorted(int(i) for i in np.argsort(-imp)[:k])
    assert res.support == want
    best, best_obj, _ = orc.brute_force(H, G, c0, p, 1, k)
    assert sorted(best) == want and np.isclose(res.obj_final, best_obj, rtol=1e-10)


def test_huge_ridge_makes_magnitude_support_optimal():
    X, W, H, G, c0, lam = make_problem(10, 1, 4, 50, 70, lam=1e9)
    K0 = orc.magnitude_support(W, 10, 1, 4)
    res = orc.local_search(H, G, c0, K0, 10, 1, 20)
    assert res.accepted == 0 and res.support == K0
    best, _, _ = orc.brute_force(H, G, c0, 10, 1, 4)
    assert sorted(best) == K0


def test_magnitude_support_definition_and_ties():
    W = np.array([[3.0, 4.0], [0.0, 5.0], [5.0, 0.0], [1.0, 1.0], [0.0, 0.0], [4.0, 3.0]])
    assert np.allclose(orc.group_magnitudes(W, 6, 1), [5, 5, 5, math.sqrt(2), 0, 5])
    assert orc.magnitude_support(W, 6, 1, 3) == [0, 1, 2]          # four-way tie: lower indices stay
    assert np.allclose(orc.group_magnitudes(W, 3, 2), [math.sqrt(50), math.sqrt(27), 5.0])
    assert orc.magnitude_support(W, 3, 2, 2) == [0, 1]


def test_always_accept_runs_the_printed_algorithm():
    p, q, m, n, k = 16, 1, 4, 100, 6
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 80, corr=1.0)
    K0 = orc.magnitude_support(W, p, q, k)
    res = orc.local_search(H, G, c0, K0, p, q, 12, always_accept=True)
    assert res.iters == 12 and res.accepted == 12
    _, o = orc.solve_support(H, G, c0, res.support, q)
    assert np.isclose(o, res.obj_final, rtol=1e-8)


# ---------------------------------------------------------------- convolutional layers (Section 3)
def test_unfold_matches_the_library_routine_and_reproduces_the_convolution():
    import torch
    rng = np.random.default_rng(71)
    for (B, C, Hin, Win, kh, kw, stride, pad) in ((2, 3, 5, 6, 3, 3, 1, 1), (1, 2, 7, 5, 3, 2, 2, 0), (2, 4, 4, 4, 1, 1, 1, 0)):
        F = rng.standard_normal((B, C, Hin, Win))
        X = orc.unfold(F, kh, kw, stride, pad)
        ref = torch.nn.functional.unfold(torch.from_numpy(F), (kh, kw), padding=pad, stride=stride)   # (B, C*kh*kw, L)
        ref = ref.permute(0, 2, 1).reshape(-1, C * kh * kw).numpy()
        assert X.shape == ref.shape and np.array_equal(X, ref)
        # X W is the convolution with the filters stored as the columns of W
        Cout = 3
        Wm = rng.standard_normal((C * kh * kw, Cout))
        filt = torch.from_numpy(Wm.T.reshape(Cout, C, kh, kw).copy())
        y = torch.nn.functional.conv2d(torch.from_numpy(F), filt, padding=pad, stride=stride)        # (B, Cout, Hout, Wout)
        assert np.allclose(X @ Wm, y.permute(0, 2, 3, 1).reshape(-1, Cout).numpy(), atol=1e-12)
    # a 1 x 1 kernel: the rows are the pixels, the columns the channels
    F = rng.standard_normal((2, 3, 2, 2))
    assert np.array_equal(orc.unfold(F, 1, 1), F.transpose(0, 2, 3, 1).reshape(-1, 3))


# ---------------------------------------------------------------- block moves (Section 4.2, t-hat = 2 s, p-hat = 0)
def test_block_search_with_one_pair_is_the_swap_search():
    X, W, H, G, c0, lam = make_problem(10, 2, 4, 90, 41)
    K0 = orc.magnitude_support(W, 10, 2, 5)
    a = orc.local_search(H, G, c0, K0, 10, 2, 30)
    b = orc.block_search(H, G, c0, K0, 10, 2, 30, 1)
    assert a.support == b.support and a.iters == b.iters and a.accepted == b.accepted
    assert [(r.g_out, r.j_in) for r in a.trace] == [(r.out[0], r.inn[0]) for r in b.trace]
    assert np.allclose([r.delta for r in a.trace], [r.delta for r in b.trace], rtol=1e-9)
    assert np.isclose(a.obj_final, b.obj_final, rtol=1e-12)


@pytest.mark.parametrize("q,s", [(1, 2), (1, 3), (2, 2)])
def test_block_moves_by_definition(q, s):
    # every iteration: the sets are the s best of each side by re-solve differences, delta is the re-solve difference of
    # the whole move, the objective never rises, and the search ends where no block move of its own choice improves
    p, m, n, k = 11, 4, 100, 5
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 50 + 3 * q + s)
    K0 = orc.magnitude_support(W, p, q, k)
    res = orc.block_search(H, G, c0, K0, p, q, 40, s)
    K = sorted(K0)
    for rec in res.trace:
        take = min(s, len(K), p - len(K))
        _, objK = orc.solve_support(H, G, c0, K, q)
        cost = {g: orc.solve_support(H, G, c0, [x for x in K if x != g], q)[1] - objK for g in K}
        gain = {j: objK - orc.solve_support(H, G, c0, K + [j], q)[1] for j in range(p) if j not in K}
        assert rec.out == sorted(K, key=lambda g: (cost[g], g))[:take]
        assert rec.inn == sorted(gain, key=lambda j: (-gain[j], j))[:take]
        Kn = sorted([g for g in K if g not in rec.out] + rec.inn)
        _, objn = orc.solve_support(H, G, c0, Kn, q)
        assert np.isclose(rec.delta, objn - objK, rtol=1e-7, atol=1e-10 * c0)
        assert rec.deficit_rem == 0.0 and rec.deficit_add == 0.0
        if rec.accepted:
            assert rec.delta < 0 and np.isclose(rec.obj_after, objn, rtol=1e-9)
            K = Kn
        else:
            assert rec.delta >= 0
    assert res.support == K and len(K) == k
    assert res.accepted == sum(r.accepted for r in res.trace) and res.iters == len(res.trace)
    assert res.iters == res.accepted + (0 if res.trace[-1].accepted else 1)


def test_block_moves_cut_to_what_is_there_and_follow_mode():
    X, W, H, G, c0, lam = make_problem(8, 1, 3, 60, 57)
    K0 = [0, 1, 2, 3, 4, 5]                                  # two groups outside: a move of 4 is cut to 2
    res = orc.block_search(H, G, c0, K0, 8, 1, 3, 4, always_accept=True)
    assert all(len(r.out) == 2 and len(r.inn) == 2 for r in res.trace)
    free = orc.block_search(H, G, c0, K0, 8, 1, 5, 2)
    again = orc.block_search(H, G, c0, K0, 8, 1, 5, 2, follow=[(r.out[::-1], r.inn[::-1]) for r in free.trace if r.accepted])
    assert again.support == free.support and all(r.deficit_rem == 0.0 and r.deficit_add == 0.0 for r in again.trace)
    with pytest.raises(ValueError):
        orc.block_search(H, G, c0, K0, 8, 1, 1, 2, follow=[([0, 6], [7, 1])])


# ---------------------------------------------------------------- sequential-pipeline target (Appendix B.1)
def test_target_form_reduces_to_the_plain_form_and_matches_its_definition():
    rng = np.random.default_rng(31)
    n, d1, m, lam = 50, 9, 4, 0.3
    X = rng.standard_normal((n, d1))
    Xhat = X + 0.2 * rng.standard_normal((n, d1))          # the dense model's input differs from the pruned model's
    W = rng.standard_normal((d1, m))
    # same inputs on both sides: the plain quadratic form
    H0, G0, c00, lam0 = orc.gram(X, W, lam_abs=lam)
    H1, G1, c01, lam1 = orc.gram_target(X, X @ W, W, lam_abs=lam)
    assert np.allclose(H0, H1) and np.allclose(G0, G1, rtol=1e-12, atol=1e-12) and np.isclose(c00, c01) and lam0 == lam1
    # different inputs: the quadratic form equals the loss written out, for any weights
    Y = Xhat @ W
    H, G, c0, lam_u = orc.gram_target(X, Y, W, lam_abs=0.1, lam_rel=0.05)
    assert np.isclose(lam_u, 0.1 + 0.05 * np.mean(np.sum(X * X, axis=0)))
    for _ in range(3):
        What = rng.standard_normal((d1, m))
        What[[1, 4, 7]] = 0
        assert np.isclose(orc.objective_quadratic(H, G, c0, What), orc.objective_target(X, Y, W, What, lam_u), rtol=1e-10)


def test_target_form_optimum_is_ridge_least_squares_onto_the_dense_output():
    rng = np.random.default_rng(32)
    n, p, q, m = 60, 6, 2, 3
    d1 = p * q
    X = rng.standard_normal((n, d1))
    Y = (X + 0.3 * rng.standard_normal((n, d1))) @ rng.standard_normal((d1, m))
    W = rng.standard_normal((d1, m))
    H, G, c0, lam = orc.gram_target(X, Y, W, lam_abs=0.2)
    K = [0, 2, 5]
    rows = orc.rows_of(K, q)
    What, obj = orc.solve_support(H, G, c0, K, q)
    A = np.vstack([X[:, rows], math.sqrt(lam) * np.eye(d1)[:, rows]])
    Bm = np.vstack([Y, math.sqrt(lam) * W])
    sol, *_ = np.linalg.lstsq(A, Bm, rcond=None)
    assert np.allclose(What[rows], sol, rtol=1e-8, atol=1e-10)
    assert np.isclose(obj, orc.objective_target(X, Y, W, What, lam), rtol=1e-10)
    # the dense layer no longer reproduces the target exactly: the nested schedule starts from a positive objective
    dense, obj_dense = orc.solve_support(H, G, c0, list(range(p)), q)
    assert obj_dense > 1e-6 * c0 and np.isclose(obj_dense, orc.objective_target(X, Y, W, dense, lam), rtol=1e-10)
    res = orc.greedy_from_dense(H, G, c0, p, q, 3, 2)
    _, o = orc.solve_support(H, G, c0, res.support, q)
    assert np.isclose(res.obj_final, o, rtol=1e-10)


# ---------------------------------------------------------------- nested schedule from the dense layer (Algorithm 1)
def test_dense_start_is_the_dense_layer():
    # S_0 empty: every group kept, the optimal weights are W itself and the objective is zero
    X, W, H, G, c0, lam = make_problem(7, 2, 5, 60, 81)
    st = orc.init_state(H, G, list(range(7)), 2)
    assert np.allclose(st.What_K, W, atol=1e-9)
    assert abs(c0 + 2 * st.f) < 1e-9 * c0
    res = orc.greedy_from_dense(H, G, c0, 7, 2, 7, 3)
    assert res.trace == [] and res.support == list(range(7))


@pytest.mark.parametrize("q,t_hat", [(1, 1), (1, 3), (2, 2), (3, 4)])
def test_greedy_picks_the_cheapest_removals_by_definition(q, t_hat):
    # every iteration: the chosen set is the t_hat smallest of obj(K - g) - obj(K) computed by full re-solves,
    # the tracked objective equals the re-solved one, and the final state equals a fresh state on the final support
    p, m, n, k = 10, 4, 90, 3
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 90 + 7 * q + t_hat)
    res = orc.greedy_from_dense(H, G, c0, p, q, k, t_hat)
    K = list(range(p))
    want_iters = math.ceil((p - k) / t_hat)
    assert len(res.trace) == want_iters
    prev_obj = 0.0
    for it, rec in enumerate(res.trace):
        take = min(t_hat, len(K) - k)
        _, objK = orc.solve_support(H, G, c0, K, q)
        cost = {g: orc.solve_support(H, G, c0, [x for x in K if x != g], q)[1] - objK for g in K}
        order = sorted(K, key=lambda g: (cost[g], g))
        assert rec.removed == order[:take]
        assert np.allclose(rec.costs, [cost[g] for g in rec.removed], rtol=1e-7, atol=1e-9 * c0)
        assert rec.deficit == 0.0 and rec.gap >= 0.0
        K = [g for g in K if g not in rec.removed]
        _, objn = orc.solve_support(H, G, c0, K, q)
        assert np.isclose(rec.obj_after, objn, rtol=1e-9)
        assert rec.obj_after >= prev_obj - 1e-12 * c0          # pruning never lowers the loss
        prev_obj = rec.obj_after
    assert res.support == sorted(K) and len(K) == k
    fresh = orc.init_state(H, G, res.support, q)
    order = np.argsort(res.state.groups)
    rows = np.concatenate([np.arange(s * q, (s + 1) * q) for s in order])
    assert np.allclose(res.state.P[np.ix_(rows, rows)], fresh.P, rtol=1e-8, atol=1e-10)
    assert np.allclose(res.state.What_K[rows], fresh.What_K, rtol=1e-8, atol=1e-10)


def test_greedy_first_iteration_closed_form_and_one_shot_case():
    # at the dense layer the cost of pruning row g (q = 1) is ||W_g||^2 / (H^-1)_gg; with t_hat = p - k the
    # schedule is one iteration that prunes the p - k smallest of these
    p, m, n, k = 12, 6, 100, 5
    X, W, H, G, c0, lam = make_problem(p, 1, m, n, 97)
    cost = np.sum(W * W, axis=1) / np.diag(np.linalg.inv(H))
    res = orc.greedy_from_dense(H, G, c0, p, 1, k, p - k)
    assert len(res.trace) == 1
    assert res.trace[0].removed == [int(i) for i in np.argsort(cost, kind="stable")[:p - k]]
    assert np.allclose(res.trace[0].costs, np.sort(cost)[:p - k], rtol=1e-9)


def test_greedy_on_diagonal_H_reaches_the_optimum_and_is_bounded_by_brute_force():
    rng = np.random.default_rng(61)
    p, m, k = 12, 4, 5
    Qm, _ = np.linalg.qr(rng.standard_normal((40, p)))
    X = Qm * rng.uniform(0.5, 3.0, size=p)[None, :]
    W = rng.standard_normal((p, m))
    H, G, c0, lam = orc.gram(X, W, lam_abs=0.1)
    imp = np.diag(H) * np.sum(W * W, axis=1)
    for t_hat in (1, 2, 7):
        res = orc.greedy_from_dense(H, G, c0, p, 1, k, t_hat)
        assert res.support == sorted(int(i) for i in np.argsort(-imp)[:k])
    # correlated columns: greedy is a heuristic, never better than the enumerated optimum
    X, W, H, G, c0, lam = make_problem(12, 1, 4, 60, 98)
    _, best_obj, _ = orc.brute_force(H, G, c0, 12, 1, 6)
    for t_hat in (1, 2, 3):
        res = orc.greedy_from_dense(H, G, c0, 12, 1, 6, t_hat)
        _, o = orc.solve_support(H, G, c0, res.support, 1)
        assert np.isclose(o, res.obj_final, rtol=1e-9) and res.obj_final >= best_obj * (1 - 1e-12)


def test_greedy_follow_mode_reports_deficit():
    X, W, H, G, c0, lam = make_problem(9, 1, 4, 70, 99)
    free = orc.greedy_from_dense(H, G, c0, 9, 1, 4, 2)
    again = orc.greedy_from_dense(H, G, c0, 9, 1, 4, 2, follow=[r.removed[::-1] for r in free.trace])
    assert again.support == free.support and all(r.deficit == 0.0 for r in again.trace)
    # forcing the costliest removal first shows up as a positive deficit
    st = orc.init_state(H, G, list(range(9)), 1)
    rem = orc.removal_scores(st, 9, 1)
    bad = [int(np.argmax(rem)), int(np.argmin(rem))]
    forced = orc.greedy_from_dense(H, G, c0, 9, 1, 7, 2, follow=[bad])
    assert forced.trace[0].deficit > 0.0
    with pytest.raises(ValueError):
        orc.greedy_from_dense(H, G, c0, 9, 1, 7, 2, follow=[[0, 0]])


def test_prune_layer_end_to_end_on_cfg1():
    cfg = inp.CONFIGS["cfg1"]
    X = inp.gen_X(cfg).double().numpy()
    W = inp.gen_W(cfg).double().numpy()
    out = orc.prune_layer(X, W, cfg.p, cfg.q, cfg.k, cfg.swaps, cfg.lam_abs, cfg.lam_rel)
    assert len(out["support"]) == cfg.k
    assert out["obj"] <= out["search"].obj_initial
    assert np.isclose(out["obj"], orc.objective_direct(X, W, out["What"], out["lam"]), rtol=1e-9)
    pruned = np.setdiff1d(np.arange(cfg.d1), orc.rows_of(out["support"], cfg.q))
    assert np.all(out["What"][pruned] == 0)


# ---------------------------------------------------------------- gaps and deficits (the quantities the GPU parity rule reads)
def _diagonal_form(scores, m=1):
    """A quadratic form with H = I and one weight column scaled so that the impact of group g (eq. (impact), doubled by the
    missing 1/2) is exactly scores[g] whether it is kept or not: H_gg ||W_g||^2 with orthogonal columns
    (pinned to re-solves in test_diagonal_H_closed_form)."""
    s = np.asarray(scores, dtype=np.float64)
    p = len(s)
    W = np.zeros((p, m))
    W[:, 0] = np.sqrt(s)
    H = np.eye(p)
    G = H @ W
    return H, G, float(np.sum(W * G)), p


def test_gap_helpers_on_hand_values():
    inf = np.inf
    # best and second-best of the finite entries, relative to the best
    assert orc._gap_low(np.array([1.0, 1.5, 4.0])) == pytest.approx(0.5, rel=1e-15)
    assert orc._gap_low(np.array([inf, 4.0, inf, 1.5, 1.0])) == pytest.approx(0.5, rel=1e-15)
    assert orc._gap_high(np.array([1.0, 1.5, 4.0])) == pytest.approx(0.625, rel=1e-15)
    assert orc._gap_high(np.array([-inf, 8.0, 6.0, -inf, 2.0])) == pytest.approx(0.25, rel=1e-15)
    assert orc._gap_low(np.array([2.0, 2.0, 9.0])) == 0.0 and orc._gap_high(np.array([3.0, 7.0, 7.0])) == 0.0
    # fewer than two finite values: no second-best, the gap is infinite
    assert orc._gap_low(np.array([inf, 3.0])) == inf and orc._gap_high(np.array([-inf, 3.0])) == inf
    assert orc._gap_low(np.array([inf, inf])) == inf and orc._gap_high(np.array([])) == inf


def test_swap_record_gaps_and_deficits_on_a_diagonal_form():
    # kept {0, 1, 2} with removal costs 1, 1.5, 4; outside {3, 4, 5} with gains 8, 6, 2 (Section 4.2 selection rule)
    H, G, c0, p = _diagonal_form([1.0, 1.5, 4.0, 8.0, 6.0, 2.0])
    free = orc.local_search(H, G, c0, [0, 1, 2], p, 1, 1)
    x = free.trace[0]
    assert (x.g_out, x.j_in) == (0, 3) and x.accepted
    assert x.rem == pytest.approx(1.0) and x.add == pytest.approx(8.0) and x.delta == pytest.approx(1.0 - 8.0)
    assert x.gap_rem == pytest.approx(0.5) and x.gap_add == pytest.approx(0.25)
    assert x.deficit_rem == 0.0 and x.deficit_add == 0.0
    # forced second-best on both sides: shortfalls (1.5 - 1) / 1 and (8 - 6) / 8; the gaps still describe the oracle's own best
    y = orc.local_search(H, G, c0, [0, 1, 2], p, 1, 1, follow=[(1, 4)]).trace[0]
    assert y.deficit_rem == pytest.approx(0.5) and y.deficit_add == pytest.approx(0.25)
    assert y.gap_rem == pytest.approx(0.5) and y.gap_add == pytest.approx(0.25)
    assert y.delta == pytest.approx(1.5 - 6.0)
    # forced worst on the entering side only
    z = orc.local_search(H, G, c0, [0, 1, 2], p, 1, 1, follow=[(0, 5)]).trace[0]
    assert z.deficit_rem == 0.0 and z.deficit_add == pytest.approx(0.75)
    # the exact entering rule scores the candidates at the state without the leaving group; on a diagonal form the same numbers
    w = orc.local_search(H, G, c0, [0, 1, 2], p, 1, 1, follow=[(0, 4)], exact_in=True).trace[0]
    assert w.deficit_add == pytest.approx(0.25) and w.gap_add == pytest.approx(0.25)
    # a correlated form: the deficit of a forced second-best entering group, from scores obtained by full re-solves
    X, W, Hc, Gc, c0c, lam = make_problem(10, 1, 3, 80, 123, corr=1.2)
    K0 = [0, 2, 4, 6, 8]
    base = orc.solve_support(Hc, Gc, c0c, K0, 1)[1]
    gains = {j: base - orc.solve_support(Hc, Gc, c0c, K0 + [j], 1)[1] for j in range(10) if j not in K0}
    order = sorted(gains, key=lambda j: -gains[j])
    costs = {g: orc.solve_support(Hc, Gc, c0c, [h for h in K0 if h != g], 1)[1] - base for g in K0}
    gmin = min(costs, key=lambda g: costs[g])
    r = orc.local_search(Hc, Gc, c0c, K0, 10, 1, 1, follow=[(gmin, order[1])]).trace[0]
    assert r.deficit_add == pytest.approx((gains[order[0]] - gains[order[1]]) / gains[order[0]], rel=1e-8)
    assert r.gap_add == pytest.approx((gains[order[0]] - gains[order[1]]) / gains[order[0]], rel=1e-8)
    assert r.deficit_rem == 0.0
    rs = sorted(costs.values())
    assert r.gap_rem == pytest.approx((rs[1] - rs[0]) / rs[0], rel=1e-8)


def test_block_record_gaps_and_deficits_on_a_diagonal_form():
    # kept {0..3} with costs 1, 1.5, 4, 7; outside {4..7} with gains 8, 6, 2, 1; two out, two in
    H, G, c0, p = _diagonal_form([1.0, 1.5, 4.0, 7.0, 8.0, 6.0, 2.0, 1.0])
    own = orc.block_search(H, G, c0, [0, 1, 2, 3], p, 1, 1, 2).trace[0]
    assert own.out == [0, 1] and own.inn == [4, 5]
    assert own.gap_rem == pytest.approx((4.0 - 1.5) / 1.5) and own.gap_add == pytest.approx((6.0 - 2.0) / 6.0)
    assert own.deficit_rem == 0.0 and own.deficit_add == 0.0
    assert own.delta == pytest.approx((1.0 + 1.5) - (8.0 + 6.0))
    forced = orc.block_search(H, G, c0, [0, 1, 2, 3], p, 1, 1, 2, follow=[([0, 2], [4, 6])]).trace[0]
    assert forced.deficit_rem == pytest.approx((4.0 - 1.5) / 1.5) and forced.deficit_add == pytest.approx((6.0 - 2.0) / 6.0)
    assert forced.gap_rem == pytest.approx((4.0 - 1.5) / 1.5) and forced.gap_add == pytest.approx((6.0 - 2.0) / 6.0)
    # every group of a side taken: nothing is left out, the gap is infinite
    allof = orc.block_search(H, G, c0, [0, 1], p, 1, 1, 2).trace[0]
    assert allof.gap_rem == np.inf and np.isfinite(allof.gap_add)


def test_greedy_record_gap_and_deficit_on_a_diagonal_form():
    # dense start, removal costs 3, 1, 2, 5, 4; two per iteration down to two kept
    H, G, c0, p = _diagonal_form([3.0, 1.0, 2.0, 5.0, 4.0])
    own = orc.greedy_from_dense(H, G, c0, p, 1, 2, 2)
    assert [r.removed for r in own.trace] == [[1, 2], [0]]
    assert own.trace[0].gap == pytest.approx((3.0 - 2.0) / 2.0) and own.trace[0].deficit == 0.0
    assert own.trace[1].gap == pytest.approx((4.0 - 3.0) / 3.0)
    assert own.trace[0].costs == pytest.approx([1.0, 2.0])
    assert own.obj_final == pytest.approx(1.0 + 2.0 + 3.0)
    forced = orc.greedy_from_dense(H, G, c0, p, 1, 2, 2, follow=[[1, 0], [2]])
    assert forced.trace[0].deficit == pytest.approx((3.0 - 2.0) / 2.0) and forced.trace[0].gap == pytest.approx(0.5)
    assert forced.trace[1].deficit == 0.0                       # 2 is now the cheapest of what is left
    last = orc.greedy_from_dense(H, G, c0, p, 1, 0, 5).trace[0]
    assert last.gap == np.inf                                   # nothing left out


def test_search_from_a_given_start_state_is_the_same_search():
    p, q, m, n, k = 14, 1, 4, 90, 6
    X, W, H, G, c0, lam = make_problem(p, q, m, n, 77, corr=1.3)
    K0 = orc.magnitude_support(W, p, q, k)
    a = orc.local_search(H, G, c0, K0, p, q, 10)
    st = orc.init_state(H, G, sorted(K0), q)
    b = orc.local_search(H, G, c0, K0, p, q, 10, start=st)
    assert [(x.g_out, x.j_in, x.delta) for x in a.trace] == [(x.g_out, x.j_in, x.delta) for x in b.trace]
    assert st.groups == sorted(K0) and np.array_equal(st.P, orc.init_state(H, G, sorted(K0), q).P)      # the caller's state is not touched
    # keep_scores: the arrays of each record are the scores at the state its iteration started from
    c = orc.local_search(H, G, c0, K0, p, q, 10, keep_scores=True)
    assert [(x.g_out, x.j_in) for x in c.trace] == [(x.g_out, x.j_in) for x in a.trace]
    kept = sorted(K0)
    for x in c.trace:
        stx = orc.init_state(H, G, kept, q)
        assert np.allclose(x.rem_all, orc.removal_scores(stx, p, q), rtol=1e-9) and np.allclose(x.add_all, orc.addition_scores(stx, H, G, p, q), rtol=1e-9)
        assert x.rem_all[x.g_out] == x.rem and x.add_all[x.j_in] == x.add
        if x.accepted:
            kept = sorted(set(kept) - {x.g_out} | {x.j_in})
    with pytest.raises(ValueError):
        orc.local_search(H, G, c0, K0[:-1] + [max(set(range(p)) - set(K0))], p, q, 1, start=st)
