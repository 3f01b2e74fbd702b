"""Plain float64 CPU oracle for the OSSCAR per-layer structured-pruning solver.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the HIP library
must compute.  It shares no code with the GPU path and is imported only by tests/, by
__graft_entry__.smoke() and by bench.py's cpu_baseline leg.  The product path never calls it.

Everything is numpy float64.  A matmul, a Cholesky factorisation and a linear solve are used as library
steps; nothing is blocked, fused or reordered beyond what the cited passage states.

Notation.  The paper writes S for the set of PRUNED groups and I_S for the rows that stay.  This file,
like the library's C interface, works with the complementary KEPT set K (|K| = k, the paper's p - p')
and writes
    H = X^T X + lam*I,  G = H W            (Section 3, dense-layer paragraph; lam is this build's ridge)
    P = (H_KK)^-1,      What_K = P G_K     (eq. (optf) and the closed-form optimum in Appendix A.1)
    L(What) = 1/2 Tr(What^T H What) - Tr(G^T What)        (eq. (MIQP))
    f(K)   = min L = -1/2 Tr(G_K^T P G_K)                 (eq. (optf))
    obj(What) = ||X W - X What||_F^2 + lam ||W - What||_F^2 = c0 + 2 L(What),  c0 = Tr(W^T H W).
The paper's dense weights "W-hat" are called W here and its solved weights "W" are called What.

Readings of the paper taken here (each pinned by a test against a re-solve or brute force):
  * sign of the f update: removing rows RAISES f by 1/2 Tr(What_r^T C^-1 What_r), adding rows LOWERS it
    by the same expression (the last lines of the two f derivations in Appendix A.1 print the opposite
    orientation of f(S), f(S'));
  * the linear term of L carries a minus sign (eq. (MIQP)), not the plus printed in eq. (obj-ver2);
  * A = P + B C^-1 B^T in Case 2 (the transpose is missing in print);
  * selection (Section 4.2, after eq. (impact)): in kept-set terms the kept group whose removal costs
    least leaves and the outside group whose addition gains most enters;
  * Algorithm 1 prints no acceptance test: here a swap is applied only if its exact effect, computed by
    Case 3 (= Case 1 then Case 2), lowers the objective by more than rel_tol*obj; otherwise the search
    stops.  always_accept=True applies every selected swap, as the printed algorithm does;
  * ties: lowest group index wins (argmin, argmax, top-k).
"""
from __future__ import annotations

import dataclasses
import itertools
from typing import List, Optional, Sequence, Tuple

import numpy as np

_TINY = 1e-300


# --------------------------------------------------------------------------------------------------
# Quadratic-form construction (Section 3, "Structured pruning in dense layers": H = X^T X, G = X^T X W)
# --------------------------------------------------------------------------------------------------
def gram(X: np.ndarray, W: np.ndarray, lam_abs: float = 0.0, lam_rel: float = 0.0):
    """H = X^T X + lam I, G = H W, c0 = Tr(W^T G), lam = lam_abs + lam_rel * mean(diag(X^T X))."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    H = X.T @ X
    lam = float(lam_abs) + float(lam_rel) * float(np.mean(np.diag(H)))
    H = H + lam * np.eye(H.shape[0])
    G = H @ W
    c0 = float(np.sum(W * G))
    return H, G, c0, lam


def objective_direct(X: np.ndarray, W: np.ndarray, What: np.ndarray, lam: float) -> float:
    """The layer-wise reconstruction loss itself (eq. (obj-ver1) without the 1/(2N) factor, plus ridge)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    D = W - np.asarray(What, dtype=np.float64)
    return float(np.sum((X @ D) ** 2) + lam * np.sum(D ** 2))


def gram_target(X: np.ndarray, Y: np.ndarray, W: np.ndarray, lam_abs: float = 0.0, lam_rel: float = 0.0):
    """Sequential-pipeline variant (Appendix B.1, "Pruning strategies"): the layer is asked to reproduce the DENSE
    model's output Y = Xhat W from the pruned model's input X, i.e. obj(What) = ||Y - X What||_F^2 + lam ||W - What||_F^2.
    Expanding gives the same quadratic form with H = X^T X + lam I, G = X^T Y + lam W, c0 = ||Y||_F^2 + lam ||W||_F^2."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    H = X.T @ X
    lam = float(lam_abs) + float(lam_rel) * float(np.mean(np.diag(H)))
    H = H + lam * np.eye(H.shape[0])
    G = X.T @ Y + lam * W
    c0 = float(np.sum(Y * Y) + lam * np.sum(W * W))
    return H, G, c0, lam


def objective_target(X: np.ndarray, Y: np.ndarray, W: np.ndarray, What: np.ndarray, lam: float) -> float:
    """||Y - X What||_F^2 + lam ||W - What||_F^2 from its definition."""
    X = np.asarray(X, dtype=np.float64)
    What = np.asarray(What, dtype=np.float64)
    return float(np.sum((np.asarray(Y, dtype=np.float64) - X @ What) ** 2) + lam * np.sum((np.asarray(W, dtype=np.float64) - What) ** 2))


def unfold(F: np.ndarray, kh: int, kw: int, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Rows of X for a convolutional layer (Section 3, "Structured pruning in convolutional layers"): the feature map
    F (batch, C, Hin, Win), zero-padded by `pad`, is cut into kh x kw patches with the given stride; the patch at
    output position (b, oy, ox) becomes the row b*Hout*Wout + oy*Wout + ox, and its entry for input channel c and
    kernel offset (dy, dx) sits in column c*kh*kw + dy*kw + dx, so that the rows of W that act on channel c are the
    group Q^c of kh*kw consecutive rows."""
    F = np.asarray(F, dtype=np.float64)
    B, C, Hin, Win = F.shape
    Hout = (Hin + 2 * pad - kh) // stride + 1
    Wout = (Win + 2 * pad - kw) // stride + 1
    X = np.zeros((B * Hout * Wout, C * kh * kw))
    for b in range(B):
        for oy in range(Hout):
            for ox in range(Wout):
                row = (b * Hout + oy) * Wout + ox
                for c in range(C):
                    for dy in range(kh):
                        for dx in range(kw):
                            y, x = oy * stride + dy - pad, ox * stride + dx - pad
                            if 0 <= y < Hin and 0 <= x < Win:
                                X[row, (c * kh + dy) * kw + dx] = F[b, c, y, x]
    return X


def objective_quadratic(H: np.ndarray, G: np.ndarray, c0: float, What: np.ndarray) -> float:
    """c0 + 2 L(What) with L from eq. (MIQP)."""
    return float(c0 + np.sum(What * (H @ What)) - 2.0 * np.sum(G * What))


# --------------------------------------------------------------------------------------------------
# Row sets and the optimum for a fixed support (eq. (indexS), eq. (deff2), eq. (optf))
# --------------------------------------------------------------------------------------------------
def rows_of(groups: Sequence[int], q: int) -> np.ndarray:
    """Rows of the contiguous equal-size groups Q^j = {j q, ..., j q + q - 1} (Section 3, MIQP paragraph)."""
    g = np.asarray(list(groups), dtype=np.int64)
    return (g[:, None] * q + np.arange(q, dtype=np.int64)[None, :]).reshape(-1)


def solve_support(H: np.ndarray, G: np.ndarray, c0: float, groups: Sequence[int], q: int):
    """Optimal weights for kept groups: What_K = (H_KK)^-1 G_K, zero elsewhere; obj = c0 - Tr(G_K^T What_K)."""
    rows = rows_of(sorted(groups), q)
    What = np.zeros_like(G)
    if len(rows):
        Lc = np.linalg.cholesky(H[np.ix_(rows, rows)])
        Y = np.linalg.solve(Lc, G[rows])
        What[rows] = np.linalg.solve(Lc.T, Y)
    obj = float(c0 - np.sum(G[rows] * What[rows]))
    return What, obj


def n_choose_k(n: int, k: int) -> int:
    c = 1
    for i in range(1, k + 1):
        c = c * (n - k + i) // i
    return c


def brute_force(H: np.ndarray, G: np.ndarray, c0: float, p: int, q: int, k: int):
    """Global optimum of eq. (struc) by enumerating every support of k kept groups (tiny p only).

    Returns (best_groups, best_obj, all_objs) with all_objs in itertools.combinations order."""
    objs = []
    best, best_obj = None, np.inf
    for comb in itertools.combinations(range(p), k):
        _, o = solve_support(H, G, c0, comb, q)
        objs.append(o)
        if o < best_obj:
            best, best_obj = comb, o
    return list(best), float(best_obj), np.array(objs)


# --------------------------------------------------------------------------------------------------
# Magnitude support (Appendix B.1, "MP": group Frobenius norm, drop the smallest)
# --------------------------------------------------------------------------------------------------
def group_magnitudes(W: np.ndarray, p: int, q: int) -> np.ndarray:
    W = np.asarray(W, dtype=np.float64)
    return np.sqrt(np.sum(W.reshape(p, q * W.shape[1]) ** 2, axis=1))


def magnitude_support(W: np.ndarray, p: int, q: int, k: int) -> List[int]:
    mu = group_magnitudes(W, p, q)
    order = np.argsort(-mu, kind="stable")        # equal norms: lower index first
    return sorted(int(j) for j in order[:k])


# --------------------------------------------------------------------------------------------------
# Search state: what Proposition 4.1 assumes is at hand -- f, the inverse of H on the kept rows, and the
# optimal weights -- for the current kept set.
# --------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class State:
    groups: List[int]          # kept groups, in the row-block order of P / What_K
    P: np.ndarray              # (k q) x (k q) inverse of H on the kept rows
    What_K: np.ndarray         # (k q) x m optimal kept weights
    f: float                   # eq. (optf)

    def copy(self) -> "State":
        return State(list(self.groups), self.P.copy(), self.What_K.copy(), self.f)


def init_state(H: np.ndarray, G: np.ndarray, groups: Sequence[int], q: int) -> State:
    """Fresh state for a kept set: direct inverse and product (Algorithm 1, line 1, for a given start)."""
    groups = list(groups)
    rows = rows_of(groups, q)
    P = np.linalg.inv(H[np.ix_(rows, rows)])
    P = 0.5 * (P + P.T)
    What_K = P @ G[rows]
    f = -0.5 * float(np.sum(G[rows] * What_K))
    return State(groups, P, What_K, f)


def _block(slot: int, q: int) -> np.ndarray:
    return np.arange(slot * q, (slot + 1) * q)


def removal_score(st: State, slot: int, q: int) -> float:
    """obj(K minus g) - obj(K) = Tr(What_r^T C^-1 What_r), C = the g-block of P (Case 1; Lemma A.1)."""
    r = _block(slot, q)
    C = st.P[np.ix_(r, r)]
    Wr = st.What_K[r]
    return float(np.sum(Wr * np.linalg.solve(C, Wr)))


def removal_scores(st: State, p: int, q: int) -> np.ndarray:
    """Length-p array indexed by group id; +inf for groups that are not kept."""
    out = np.full(p, np.inf)
    for slot, g in enumerate(st.groups):
        out[g] = removal_score(st, slot, q)
    return out


def addition_quantities(st: State, H: np.ndarray, G: np.ndarray, j: int, q: int):
    """Case 2 for the single group j: C = (H_rr - H_rK P H_Kr)^-1 and the new group's weights What_r."""
    rows = rows_of(st.groups, q)
    r = rows_of([j], q)
    HKr = H[np.ix_(rows, r)]
    Cinv = H[np.ix_(r, r)] - HKr.T @ st.P @ HKr          # Schur complement of the candidate
    Bm = -st.P @ HKr @ np.linalg.inv(Cinv)               # the paper's B
    C = np.linalg.inv(Cinv)
    Wr = Bm.T @ G[rows] + C @ G[r]                       # B^T G_K + C G_r
    return Cinv, C, Bm, Wr


def addition_score(st: State, H: np.ndarray, G: np.ndarray, j: int, q: int) -> float:
    """obj(K) - obj(K plus j) = Tr(What_r^T C^-1 What_r) with Case 2's C and What_r."""
    Cinv, _, _, Wr = addition_quantities(st, H, G, j, q)
    return float(np.sum(Wr * (Cinv @ Wr)))


def addition_scores(st: State, H: np.ndarray, G: np.ndarray, p: int, q: int) -> np.ndarray:
    """Length-p array indexed by group id; -inf for kept groups.  All candidates at the current state
    (eq. (impact)), evaluated with two matmuls: V = P H_{K,Kc}, Rm = G_Kc - V^T G_K."""
    out = np.full(p, -np.inf)
    kept = set(st.groups)
    cand = [j for j in range(p) if j not in kept]
    if not cand:
        return out
    rows = rows_of(st.groups, q)
    crow = rows_of(cand, q)
    HKc = H[np.ix_(rows, crow)]
    V = st.P @ HKc
    Rm = G[crow] - V.T @ G[rows]
    for t, j in enumerate(cand):
        b = _block(t, q)
        s = H[np.ix_(crow[b], crow[b])] - HKc[:, b].T @ V[:, b]
        Rj = Rm[b]
        out[j] = float(np.sum(Rj * np.linalg.solve(s, Rj)))
    return out


def remove_group(st: State, slot: int, q: int) -> State:
    """Case 1: new inverse A - B C^-1 B^T, new weights What - [B C^-1; E] What_r, f raised."""
    kr = st.P.shape[0]
    r = _block(slot, q)
    keep = np.setdiff1d(np.arange(kr), r)
    A = st.P[np.ix_(keep, keep)]
    Bm = st.P[np.ix_(keep, r)]
    C = st.P[np.ix_(r, r)]
    Wr = st.What_K[r]
    BCinv = Bm @ np.linalg.inv(C)
    Pn = A - BCinv @ Bm.T
    Pn = 0.5 * (Pn + Pn.T)
    Wn = st.What_K[keep] - BCinv @ Wr
    fn = st.f + 0.5 * float(np.sum(Wr * np.linalg.solve(C, Wr)))
    groups = st.groups[:slot] + st.groups[slot + 1:]
    return State(groups, Pn, Wn, fn)


def add_group(st: State, H: np.ndarray, G: np.ndarray, j: int, q: int) -> State:
    """Case 2: bordered inverse [[A, B], [B^T, C]], new weights, f lowered.  The new group is appended."""
    Cinv, C, Bm, Wr = addition_quantities(st, H, G, j, q)
    A = st.P + Bm @ Cinv @ Bm.T
    Pn = np.block([[A, Bm], [Bm.T, C]])
    Pn = 0.5 * (Pn + Pn.T)
    top = st.What_K + (Bm @ Cinv) @ Wr
    Wn = np.vstack([top, Wr])
    fn = st.f - 0.5 * float(np.sum(Wr * (Cinv @ Wr)))
    return State(st.groups + [j], Pn, Wn, fn)


# --------------------------------------------------------------------------------------------------
# Local search (Section 4.2 with t-hat = 2, p-hat = 0, i.e. s1 = s2 = 1: one group out, one group in)
# --------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class SwapRecord:
    g_out: int
    j_in: int
    rem: float          # removal score of g_out at the current state
    add: float          # addition score of j_in at the current state
    delta: float        # exact change of obj for the pair (Case 3)
    gap_rem: float      # relative gap best vs second-best removal score
    gap_add: float      # relative gap best vs second-best addition score
    deficit_rem: float  # (rem[g_out] - min rem) / |min rem|  (0 unless a followed choice was not the argmin)
    deficit_add: float  # (max add - add[j_in]) / |max add|
    accepted: bool
    obj_after: float
    rem_all: Optional[np.ndarray] = None   # with keep_scores: every removal score at the state the iteration started from
    add_all: Optional[np.ndarray] = None   # and every addition score (indexed by group id, +-inf where not applicable)


@dataclasses.dataclass
class SearchResult:
    support: List[int]             # sorted kept groups at the end
    obj_initial: float
    obj_final: float               # tracked through the f updates
    iters: int
    accepted: int
    trace: List[SwapRecord]
    state: State


def _gap_low(vals: np.ndarray) -> float:
    v = np.sort(vals[np.isfinite(vals)])
    if len(v) < 2:
        return np.inf
    return float(abs(v[1] - v[0]) / max(abs(v[0]), _TINY))


def _gap_high(vals: np.ndarray) -> float:
    v = np.sort(vals[np.isfinite(vals)])[::-1]
    if len(v) < 2:
        return np.inf
    return float(abs(v[0] - v[1]) / max(abs(v[0]), _TINY))


def swap_delta(st: State, H: np.ndarray, G: np.ndarray, g: int, j: int, q: int):
    """Exact obj(K - g + j) - obj(K) through Case 3: Case 1 on g, then Case 2's score of j there."""
    slot = st.groups.index(g)
    rem = removal_score(st, slot, q)
    mid = remove_group(st, slot, q)
    add_mid = addition_score(mid, H, G, j, q)
    return rem - add_mid, mid


def local_search(H: np.ndarray, G: np.ndarray, c0: float, groups0: Sequence[int], p: int, q: int,
                 max_swaps: int, rel_tol: float = 0.0, always_accept: bool = False,
                 follow: Optional[Sequence[Tuple[int, int]]] = None, exact_in: bool = False,
                 start: Optional[State] = None, keep_scores: bool = False) -> SearchResult:
    """Swap search from the kept set groups0.

    exact_in: a stronger rule for the entering group than the separable scores of eq. (impact): with the leaving
    group g fixed (lowest removal score), every candidate j is scored at the state reached by removing g
    (Case 1 applied, then eq. (impact) there), which is the exact gain of the pair (g, j); the record's add, gap_add
    and deficit_add then refer to these scores.

    follow: optional list of (g_out, j_in) pairs to apply instead of the oracle's own selection (used to
    validate another implementation's trajectory step by step: the record then holds how far each forced
    choice was from the oracle's best, and the oracle's exact delta for it).  With follow, the loop runs
    len(follow) iterations and applies every pair.

    start: optional State of groups0 that the caller already holds (what init_state(H, G, sorted(groups0), q) returns);
    saves building it again, changes nothing else.  keep_scores: every record also keeps the two score arrays of its
    iteration."""
    if start is not None and list(start.groups) != sorted(groups0):
        raise ValueError("start must be the state of sorted(groups0)")
    st = start.copy() if start is not None else init_state(H, G, sorted(groups0), q)
    obj0 = c0 + 2.0 * st.f
    trace: List[SwapRecord] = []
    accepted = 0
    iters = 0
    n_iter = len(follow) if follow is not None else max_swaps
    for it in range(n_iter):
        if len(st.groups) == 0 or len(st.groups) == p:
            break
        rem = removal_scores(st, p, q)
        if exact_in:
            g = follow[it][0] if follow is not None else int(np.argmin(rem))
            mid_g = remove_group(st, st.groups.index(g), q)
            add = addition_scores(mid_g, H, G, p, q)
            add[g] = -np.inf                      # g itself is a candidate at that state; putting it back is no swap
            j = follow[it][1] if follow is not None else int(np.argmax(add))
        else:
            add = addition_scores(st, H, G, p, q)
            if follow is not None:
                g, j = follow[it]
            else:
                g, j = int(np.argmin(rem)), int(np.argmax(add))
        rmin, amax = float(np.min(rem)), float(np.max(add))
        delta, mid = swap_delta(st, H, G, g, j, q)
        obj = c0 + 2.0 * st.f
        ok = True if (always_accept or follow is not None) else (delta < -rel_tol * obj)
        iters += 1
        rec = SwapRecord(g, j, float(rem[g]), float(add[j]), float(delta), _gap_low(rem), _gap_high(add),
                         float((rem[g] - rmin) / max(abs(rmin), _TINY)),
                         float((amax - add[j]) / max(abs(amax), _TINY)), ok, obj)
        if keep_scores:
            rec.rem_all, rec.add_all = rem, add
        if not ok:
            trace.append(rec)
            break
        st = add_group(mid, H, G, j, q)
        accepted += 1
        rec.obj_after = c0 + 2.0 * st.f
        trace.append(rec)
    return SearchResult(sorted(st.groups), obj0, c0 + 2.0 * st.f, iters, accepted, trace, st)


# --------------------------------------------------------------------------------------------------
# Block moves (Section 4.2 with t-hat = 2 s, p-hat = 0: s1 = s2 = s groups leave and s enter per iteration)
# --------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class BlockRecord:
    out: List[int]         # groups leaving, cheapest removal first
    inn: List[int]         # groups entering, largest gain first
    delta: float           # exact change of obj for the whole move (Case 1 s times, then Case 2 s times)
    gap_rem: float         # relative gap between the costliest removal chosen and the cheapest kept group left
    gap_add: float         # relative gap between the smallest gain chosen and the largest gain left out
    deficit_rem: float     # how far a forced choice is from the oracle's own s-th best (0 for its own choice)
    deficit_add: float
    accepted: bool
    obj_after: float


@dataclasses.dataclass
class BlockResult:
    support: List[int]
    obj_initial: float
    obj_final: float
    iters: int
    accepted: int
    trace: List[BlockRecord]
    state: State


def block_search(H: np.ndarray, G: np.ndarray, c0: float, groups0: Sequence[int], p: int, q: int, max_iters: int,
                 s: int, rel_tol: float = 0.0, always_accept: bool = False,
                 follow: Optional[Sequence[Tuple[Sequence[int], Sequence[int]]]] = None) -> BlockResult:
    """Local search with s groups out and s in per iteration.  All impacts (eq. (impact)) are evaluated at the state
    the iteration starts from; the s kept groups that are cheapest to remove leave, the s outside groups with the
    largest gain enter (lowest index on ties; s is cut to what either side has).  The move is applied only if its
    exact effect lowers obj by more than rel_tol*obj (always_accept: always), otherwise the search stops.
    s = 1 is local_search.  follow: per-iteration (out, inn) lists to apply instead of the oracle's own choice."""
    if s < 1:
        raise ValueError("s must be >= 1")
    st = init_state(H, G, sorted(groups0), q)
    obj0 = c0 + 2.0 * st.f
    trace: List[BlockRecord] = []
    accepted = iters = 0
    n_iter = len(follow) if follow is not None else max_iters
    for it in range(n_iter):
        take = min(s, len(st.groups), p - len(st.groups))
        if take == 0:
            break
        rem = removal_scores(st, p, q)
        add = addition_scores(st, H, G, p, q)
        kept_order = sorted(st.groups, key=lambda g: (rem[g], g))
        kept_set = set(st.groups)
        cand_order = sorted((j for j in range(p) if j not in kept_set), key=lambda j: (-add[j], j))
        own_out, own_in = kept_order[:take], cand_order[:take]
        if follow is not None:
            out, inn = list(follow[it][0]), list(follow[it][1])
            if (len(out) != take or len(inn) != take or len(set(out)) != take or len(set(inn)) != take
                    or any(g not in kept_set for g in out) or any(j in kept_set for j in inn)):
                raise ValueError("forced move must take %d distinct kept groups out and %d distinct others in" % (take, take))
        else:
            out, inn = own_out, own_in
        edge_r, edge_a = float(rem[own_out[-1]]), float(add[own_in[-1]])
        nxt_r = float(rem[kept_order[take]]) if take < len(kept_order) else np.inf
        nxt_a = float(add[cand_order[take]]) if take < len(cand_order) else -np.inf
        gap_r = float(abs(nxt_r - edge_r) / max(abs(edge_r), _TINY)) if np.isfinite(nxt_r) else np.inf
        gap_a = float(abs(edge_a - nxt_a) / max(abs(edge_a), _TINY)) if np.isfinite(nxt_a) else np.inf
        def_r = float((max(float(rem[g]) for g in out) - edge_r) / max(abs(edge_r), _TINY))
        def_a = float((edge_a - min(float(add[j]) for j in inn)) / max(abs(edge_a), _TINY))
        new = st
        for g in out:
            new = remove_group(new, new.groups.index(g), q)
        for j in inn:
            new = add_group(new, H, G, j, q)
        obj = c0 + 2.0 * st.f
        delta = 2.0 * (new.f - st.f)
        ok = True if (always_accept or follow is not None) else (delta < -rel_tol * obj)
        iters += 1
        rec = BlockRecord(list(out), list(inn), float(delta), gap_r, gap_a, def_r, def_a, ok, obj)
        trace.append(rec)
        if not ok:
            break
        st = new
        accepted += 1
        rec.obj_after = c0 + 2.0 * st.f
    return BlockResult(sorted(st.groups), obj0, c0 + 2.0 * st.f, iters, accepted, trace, st)


# --------------------------------------------------------------------------------------------------
# Nested schedule from the dense layer (Algorithm 1 with S_0 empty and t_i = p_i = t-hat: Section 4.2;
# Appendix B.1 uses t-hat = 2 for channels and heads, 10 for the intermediate dimension of FFN layers)
# --------------------------------------------------------------------------------------------------
@dataclasses.dataclass
class GreedyRecord:
    removed: List[int]     # groups pruned in this iteration, cheapest first
    costs: List[float]     # their removal scores at the state the iteration started from
    gap: float             # relative gap between the costliest chosen score and the cheapest one left out
    deficit: float         # (costliest chosen - the oracle's own t-th smallest) / |that|; 0 unless choices were forced
    obj_after: float


@dataclasses.dataclass
class GreedyResult:
    support: List[int]
    obj_final: float       # tracked through the f updates (obj of the dense layer is 0)
    trace: List[GreedyRecord]
    state: State


def greedy_from_dense(H: np.ndarray, G: np.ndarray, c0: float, p: int, q: int, k: int, t_hat: int,
                      follow: Optional[Sequence[Sequence[int]]] = None) -> GreedyResult:
    """Starts from the dense layer (every group kept: P = H^-1, What = H^-1 G) and prunes t_hat groups
    per iteration until k are left (the last iteration takes what remains).  With p-hat = t-hat nothing
    re-enters (s1 = 0), so an iteration only needs the impact of removing each kept group (eq. (impact),
    closed form of Case 1), all evaluated at the state the iteration starts from; the t_hat cheapest go
    (lowest index on ties) and the inverse and the weights follow by Case 1.

    follow: optional list of per-iteration removal lists to apply instead of the oracle's own choice."""
    if t_hat < 1:
        raise ValueError("t_hat must be >= 1")
    st = init_state(H, G, list(range(p)), q)
    trace: List[GreedyRecord] = []
    it = 0
    while len(st.groups) > k:
        take = min(t_hat, len(st.groups) - k)
        rem = removal_scores(st, p, q)
        order = sorted(st.groups, key=lambda g: (rem[g], g))
        own = order[:take]
        chosen = list(follow[it]) if follow is not None else own
        if len(chosen) != take or any(g not in st.groups for g in chosen) or len(set(chosen)) != take:
            raise ValueError("forced removals must be %d distinct kept groups" % take)
        edge = float(rem[own[-1]])
        nxt = float(rem[order[take]]) if take < len(order) else np.inf
        gap = float(abs(nxt - edge) / max(abs(edge), _TINY)) if np.isfinite(nxt) else np.inf
        worst = max(float(rem[g]) for g in chosen)
        deficit = float((worst - edge) / max(abs(edge), _TINY))
        for g in chosen:
            st = remove_group(st, st.groups.index(g), q)
        trace.append(GreedyRecord(list(chosen), [float(rem[g]) for g in chosen], gap, deficit, c0 + 2.0 * st.f))
        it += 1
    return GreedyResult(sorted(st.groups), c0 + 2.0 * st.f, trace, st)


# --------------------------------------------------------------------------------------------------
# Whole path: Gram -> magnitude support -> swap search -> fresh solve on the final support
# --------------------------------------------------------------------------------------------------
def prune_layer(X: np.ndarray, W: np.ndarray, p: int, q: int, k: int, max_swaps: int,
                lam_abs: float = 0.0, lam_rel: float = 0.0, rel_tol: float = 0.0,
                always_accept: bool = False):
    H, G, c0, lam = gram(X, W, lam_abs, lam_rel)
    K0 = magnitude_support(W, p, q, k)
    res = local_search(H, G, c0, K0, p, q, max_swaps, rel_tol, always_accept)
    What, obj = solve_support(H, G, c0, res.support, q)
    return dict(H=H, G=G, c0=c0, lam=lam, support0=K0, search=res, support=res.support, What=What, obj=obj)
