"""Pins for the oracle's acceptance step (CPU only): the invariants the method fixes, a
hand-worked fixture, closed forms (eq. 1 of the paper) and Monte-Carlo exactness."""
import os

import numpy as np
import pytest

import gen
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accept_hand_worked.txt")


def _softmax64(l, T=1.0):
    z = l / T
    z = z - z.max(-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(-1, keepdims=True)


def _rand_dist(rng, shape, conc=1.0):
    return _softmax64(rng.standard_normal(shape) * conc)


def _draw(rng, p, n):
    """n categorical draws from the single distribution p by inverse CDF (test-side input synthesis)."""
    cdf = np.cumsum(p)
    return np.minimum(np.searchsorted(cdf, rng.random(n) * cdf[-1], side="right"), len(p) - 1).astype(np.int32)


# ------------------------------------------------------------------ hand-worked fixture
def _parse_golden():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split("->")
        name, T, prow, qrow, toks, ua, us = lhs.split()
        vec = lambda s: np.array([[float(x) for x in r.split(",")] for r in s.split(";")])
        cases.append(dict(name=name, T=float(T), p=vec(prow), q=vec(qrow),
                          toks=[int(x) for x in toks.split(",")], ua=[float(x) for x in ua.split(",")],
                          us=float(us), want=tuple(int(x) for x in rhs.split())))
    return cases


@pytest.mark.parametrize("case", _parse_golden(), ids=lambda c: c["name"])
@pytest.mark.parametrize("as_tree", [False, True])
def test_hand_worked_cases(case, as_tree):
    p, q = case["p"], case["q"]
    Nq = p.shape[0]
    k = Nq - 1
    assert len(case["toks"]) == k
    logits = (case["T"] * np.log(p))[None]
    toks = np.array([[0] + case["toks"]], np.int32)
    un = np.zeros((1, Nq, 2), np.float32)
    un[0, 1:, 0] = case["ua"]
    un[0, :, 1] = case["us"]
    r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, draft_probs=q[None].astype(np.float32),
                                  uniforms=un, temperature=case["T"],
                                  parents=gen.chain_parents(1, Nq) if as_tree else None)
    assert (int(r.accept_len[0]), int(r.next_token[0])) == case["want"]
    assert r.accept_mask[0].tolist() == [1] * (1 + case["want"][0]) + [0] * (k - case["want"][0])


# ------------------------------------------------------------------ P1 greedy
@pytest.mark.parametrize("as_tree", [False, True])
def test_greedy_is_longest_argmax_prefix(as_tree):
    rng = np.random.default_rng(5)
    B, Nq, V = 200, 6, 50
    logits = rng.standard_normal((B, Nq, V))
    top = logits.argmax(-1)
    toks = np.zeros((B, Nq), np.int32)
    for i in range(1, Nq):
        hit = rng.random(B) < 0.7
        toks[:, i] = np.where(hit, top[:, i - 1], rng.integers(0, V, B))
    r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, temperature=0.0,
                                  parents=gen.chain_parents(B, Nq) if as_tree else None)
    for b in range(B):
        n = 0
        while n < Nq - 1 and toks[b, n + 1] == top[b, n]:
            n += 1
        assert r.accept_len[b] == n
        assert r.next_token[b] == top[b, n]
        assert r.accept_mask[b].tolist() == [1] * (n + 1) + [0] * (Nq - 1 - n)
        assert r.stop_node[b] == n
    assert 0 < r.accept_len.mean() < Nq - 1


def test_greedy_lowest_index_on_exact_tie():
    logits = np.zeros((1, 2, 7))
    logits[0, 0, [2, 5]] = 1.0
    logits[0, 1, [6, 3]] = 2.0
    r = oracle.accept_from_logits(logits=logits, draft_tokens=np.array([[0, 2]], np.int32), temperature=0.0)
    assert r.accept_len[0] == 1 and r.next_token[0] == 3
    r = oracle.accept_from_logits(logits=logits, draft_tokens=np.array([[0, 5]], np.int32), temperature=0.0)
    assert r.accept_len[0] == 0 and r.next_token[0] == 2


# ------------------------------------------------------------------ P1 on branching trees (hand-worked)
GOLDEN_TREE = os.path.join(os.path.dirname(__file__), "golden", "greedy_tree_hand_worked.txt")


def _parse_golden_tree():
    cases = []
    for line in open(GOLDEN_TREE):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split("->")
        name, par, toks, best = lhs.split()
        ints = lambda s: [int(x) for x in s.split(",")]
        alen, nxt, mask, stop = rhs.split()
        cases.append(dict(name=name, par=ints(par), toks=ints(toks), best=ints(best), accept_len=int(alen),
                          next_token=int(nxt), mask=ints(mask), stop=int(stop)))
    return cases


def _logits_with_best(best, V, rng):
    """A row per node whose largest entry is at best[n]; the other entries are a scrambled descending ramp."""
    lg = np.empty((len(best), V))
    for n, t in enumerate(best):
        lg[n] = rng.permutation(np.linspace(-3.0, 1.0, V))
        lg[n, t] = 2.5
    return lg


@pytest.mark.parametrize("case", _parse_golden_tree(), ids=lambda c: c["name"])
def test_greedy_walk_on_hand_worked_branching_trees(case):
    V = 16
    Nq = len(case["par"])
    lg = _logits_with_best(case["best"], V, np.random.default_rng(Nq))
    # two copies of the request in one batch: the second one checks the per-request offsets of parents / tokens
    r = oracle.accept_from_logits(logits=np.stack([lg, lg]), draft_tokens=np.array([case["toks"]] * 2, np.int32),
                                  parents=np.array([case["par"]] * 2, np.int32), temperature=0.0)
    for b in range(2):
        assert int(r.accept_len[b]) == case["accept_len"]
        assert int(r.next_token[b]) == case["next_token"]
        assert r.accept_mask[b].tolist() == case["mask"]
        assert int(r.stop_node[b]) == case["stop"]
    # p_at_draft at T = 0: 1 where the node's token is its PARENT's arg-max, else 0
    want = [0.0] + [1.0 if case["toks"][n] == case["best"][case["par"][n]] else 0.0 for n in range(1, Nq)]
    assert r.p_at_draft[0].tolist() == want


def test_greedy_tree_walk_agrees_with_a_recursive_search_on_random_trees():
    """Independent statement of the same rule: the accepted path is the root plus, recursively, the path from the
    lowest-numbered child carrying the current arg-max.  Random trees with up to 4 children per node and many
    duplicated tokens, so that wrong-parent and duplicate-sibling situations occur all the time."""
    rng = np.random.default_rng(77)
    B, Nq, V = 400, 12, 5
    logits = rng.standard_normal((B, Nq, V))
    top = logits.argmax(-1)
    par = np.full((B, Nq), -1, np.int32)
    for n in range(1, Nq):
        par[:, n] = rng.integers(0, n, B)
    toks = rng.integers(0, V, (B, Nq)).astype(np.int32)
    r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, parents=par, temperature=0.0)

    def path_from(b, n):
        kids = [c for c in range(n + 1, Nq) if par[b, c] == n and toks[b, c] == top[b, n]]
        return [n] + (path_from(b, min(kids)) if kids else [])

    depths = []
    for b in range(B):
        path = path_from(b, 0)
        mask = np.zeros(Nq, np.uint8)
        mask[path] = 1
        assert r.accept_len[b] == len(path) - 1 and r.stop_node[b] == path[-1]
        assert r.next_token[b] == top[b, path[-1]]
        assert np.array_equal(r.accept_mask[b], mask)
        depths.append(len(path) - 1)
    assert max(depths) >= 3 and min(depths) == 0


def test_p_at_draft_and_row_lse_on_a_branching_tree_against_library_softmax():
    """p_at_draft[n] = softmax(l[parent(n)] / T)[tok_n] gathered through non-chain parents (a chain-only gather
    `row n-1` fails here), and row_lse = logsumexp(l / T); at T = 0 the reading is logsumexp of the raw logits."""
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(78)
    B, V = 7, 33
    par = np.array([-1, 0, 0, 1, 0, 2, 2, 4, 1, 7], np.int32)
    Nq = len(par)
    assert (par[1:] != np.arange(Nq - 1)).sum() >= 6
    logits = rng.standard_normal((B, Nq, V)) * 2.0
    toks = rng.integers(0, V, (B, Nq)).astype(np.int32)
    q = _rand_dist(rng, (B, Nq, V)).astype(np.float32)
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    parents = np.broadcast_to(par, (B, Nq)).copy()
    for T in (1.0, 0.6):
        Tf = float(np.float32(T))
        r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, draft_probs=q, uniforms=un, parents=parents,
                                      temperature=T)
        p = softmax(logits / Tf, axis=-1)
        want = p[np.arange(B)[:, None], par[None, 1:], toks[:, 1:]]
        np.testing.assert_allclose(r.p_at_draft[:, 1:], want, rtol=1e-11)
        assert (r.p_at_draft[:, 0] == 0).all()
        np.testing.assert_allclose(r.row_lse, logsumexp(logits / Tf, axis=-1), rtol=1e-13)
    r0 = oracle.accept_from_logits(logits=logits, draft_tokens=toks, parents=parents, temperature=0.0)
    np.testing.assert_allclose(r0.row_lse, logsumexp(logits, axis=-1), rtol=1e-13)
    top = logits.argmax(-1)
    want0 = (toks[:, 1:] == top[np.arange(B)[:, None], par[None, 1:]]).astype(np.float64)
    assert np.array_equal(r0.p_at_draft[:, 1:], want0)
    # chain form at T = 0 as well
    rc = oracle.accept_from_logits(logits=logits, draft_tokens=toks, temperature=0.0)
    np.testing.assert_allclose(rc.row_lse, logsumexp(logits, axis=-1), rtol=1e-13)
    assert np.array_equal(rc.p_at_draft[:, 1:], (toks[:, 1:] == top[:, :-1]).astype(np.float64))


# ------------------------------------------------------------------ P2 q == p
@pytest.mark.parametrize("T", [1.0, 0.7])
def test_q_equal_p_accepts_everything(T):
    rng = np.random.default_rng(6)
    B, Nq, V = 300, 5, 40
    logits = rng.standard_normal((B, Nq, V)) * 2
    p = _softmax64(logits, float(np.float32(T)))
    toks = rng.integers(0, V, (B, Nq)).astype(np.int32)
    un = rng.random((B, Nq, 2)).astype(np.float32)
    un[un >= 1.0] = 0.5
    un[:7, :, 0] = np.float32(1.0 - 2.0 ** -24)  # the largest uniform the generator can emit
    r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, draft_probs=p.astype(np.float32),
                                  uniforms=un, temperature=T)
    assert (r.accept_len == Nq - 1).all() and (r.accept_mask == 1).all()
    # p_at_draft and row_lse against the library softmax
    par = np.arange(-1, Nq - 1)
    want = p[np.arange(B)[:, None], par[None, 1:], toks[:, 1:]]
    np.testing.assert_allclose(r.p_at_draft[:, 1:], want, rtol=1e-12)
    from scipy.special import logsumexp
    np.testing.assert_allclose(r.row_lse, logsumexp(logits / float(np.float32(T)), axis=-1), rtol=1e-13)


# ------------------------------------------------------------------ P9 special cases
def test_k0_is_plain_sampling_and_matches_inverse_cdf():
    rng = np.random.default_rng(8)
    B, V = 5000, 16
    p = _rand_dist(rng, (V,), 1.5)
    logits = np.broadcast_to(np.log(p), (B, 1, V)).copy()
    un = rng.random((B, 1, 2)).astype(np.float32)
    r = oracle.accept_from_logits(logits=logits, draft_tokens=np.zeros((B, 1), np.int32),
                                  draft_probs=np.full((B, 1, V), 1 / V, np.float32), uniforms=un,
                                  temperature=1.0, want_cdf=True)
    assert (r.accept_len == 0).all()
    cdf = np.cumsum(_softmax64(np.log(p)))
    want = np.searchsorted(cdf, un[:, 0, 1].astype(np.float64), side="right")
    # identical except possibly when u sits within rounding of a CDF knot
    safe = np.abs(cdf[None, :] - un[:, 0, 1:2].astype(np.float64)).min(-1) > 1e-9
    assert (r.next_token[safe] == want[safe]).all() and safe.mean() > 0.99
    np.testing.assert_allclose(r.final_cdf[0], cdf, rtol=1e-12)


@pytest.mark.parametrize("as_tree", [False, True])
def test_zero_target_probability_always_rejects_and_resamples_from_p(as_tree):
    rng = np.random.default_rng(9)
    B, V = 20000, 8
    p = _rand_dist(rng, (V,))
    p[3] = 0.0
    p /= p.sum()
    with np.errstate(divide="ignore"):
        logits = np.broadcast_to(np.log(p), (B, 2, V)).copy()
    q = np.zeros((B, 2, V), np.float32)
    q[:, :, 3] = 1.0
    un = rng.random((B, 2, 2)).astype(np.float32)
    un[: B // 2, 1, 0] = 0.0  # u = 0 must still reject because p(d) = 0
    toks = np.full((B, 2), 3, np.int32)
    r = oracle.accept_from_logits(logits=logits, draft_tokens=toks, draft_probs=q, uniforms=un, temperature=1.0,
                                  parents=gen.chain_parents(B, 2) if as_tree else None)
    assert (r.accept_len == 0).all()
    f = np.bincount(r.next_token, minlength=V) / B
    assert f[3] == 0
    assert np.all(np.abs(f - p) <= 4 * np.sqrt(p * (1 - p) / B) + 1e-12)


def test_u_zero_accepts_iff_p_positive():
    p = np.array([[[0.25, 0.75, 0.0], [0.2, 0.3, 0.5]]])
    with np.errstate(divide="ignore"):
        logits = np.log(p)
    q = np.array([[[0.1, 0.1, 0.8], [1 / 3, 1 / 3, 1 / 3]]], np.float32)
    un = np.zeros((1, 2, 2), np.float32)
    r = oracle.accept_from_logits(logits=logits, draft_tokens=np.array([[0, 1]], np.int32), draft_probs=q,
                                  uniforms=un, temperature=1.0)
    assert r.accept_len[0] == 1
    r = oracle.accept_from_logits(logits=logits, draft_tokens=np.array([[0, 2]], np.int32), draft_probs=q,
                                  uniforms=un, temperature=1.0)
    assert r.accept_len[0] == 0


def test_degenerate_residual_falls_back_to_p():
    """p == q exactly and a forced rejection is impossible; but p <= q everywhere with the
    draft token's p(d) = 0 < q(d) leaves residual max(0, p - q) == 0 only if p == q elsewhere.
    Build p = (0.5, 0.5, 0), q = (0.5, 0.5, 0) with d = 2 (q(d) = 0 = p(d)): u*0 < 0 is false =>
    rejected with Z = 0 => next token drawn from p itself."""
    p = np.array([[[0.5, 0.5, 0.0], [0.2, 0.3, 0.5]]])
    with np.errstate(divide="ignore"):
        logits = np.log(p)
    q = np.array([[[0.5, 0.5, 0.0], [1 / 3, 1 / 3, 1 / 3]]], np.float32)
    for us, want in [(0.25, 0), (0.75, 1)]:
        un = np.zeros((1, 2, 2), np.float32)
        un[0, 0, 1] = us
        r = oracle.accept_from_logits(logits=logits, draft_tokens=np.array([[0, 2]], np.int32),
                                      draft_probs=q, uniforms=un, temperature=1.0)
        assert r.accept_len[0] == 0 and r.next_token[0] == want


def test_chain_routine_equals_tree_walk_on_chain_parents():
    w = gen.llama_chain(21, batch=64, num_q=6, num_q_heads=2, num_kv_heads=1, head_dim=8, page_size=4,
                        hidden_size=32, vocab=300, len_lo=8, len_hi=12, draft_noise=1.5)
    args = dict(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                uniforms=w.uniforms, dtype=w.dtype, temperature=1.0, want_cdf=True)
    a = oracle.accept(**args)
    b = oracle.accept(parents=gen.chain_parents(w.batch, w.num_q), **args)
    for f in ("accept_len", "next_token", "accept_mask", "stop_node"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    np.testing.assert_allclose(a.final_cdf, b.final_cdf, rtol=1e-12, atol=1e-15)
    np.testing.assert_array_equal(np.isnan(a.test_margin), np.isnan(b.test_margin))
    assert 0 < a.accept_len.mean() < w.num_q - 1


# ------------------------------------------------------------------ P3 / P5 / P6 Monte-Carlo, chain
def _within(freq, p, n, sig=4.0):
    return np.all(np.abs(freq - p) <= sig * np.sqrt(np.maximum(p * (1 - p), 1e-12) / n) + 1e-9)


@pytest.mark.parametrize("seed,T", [(1, 1.0), (2, 0.8)])
def test_monte_carlo_chain_emits_target_distribution(seed, T):
    rng = np.random.default_rng(seed)
    B, k, V = 250_000, 4, 16
    Nq = k + 1
    Tf = float(np.float32(T))
    lrow = rng.standard_normal((Nq, V)) * 1.5
    p = _softmax64(lrow, Tf)
    q = _softmax64(lrow / Tf + rng.standard_normal((Nq, V)) * 0.8).astype(np.float32)
    toks = np.zeros((B, Nq), np.int32)
    for i in range(1, Nq):
        toks[:, i] = _draw(rng, q[i - 1].astype(np.float64), B)
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    r = oracle.accept_from_logits(logits=np.broadcast_to(lrow, (B, Nq, V)).copy(), draft_tokens=toks,
                                  draft_probs=np.broadcast_to(q, (B, Nq, V)).copy(), uniforms=un,
                                  temperature=T)
    L = r.accept_len
    alpha = np.minimum(p, q.astype(np.float64)).sum(-1)  # acceptance probability of row j
    reach = 1.0
    expect_len = 0.0
    for i in range(Nq):
        sel = L >= i  # trials that reached row i
        n = int(sel.sum())
        assert abs(n / B - reach) <= 4 * np.sqrt(reach * (1 - reach) / B) + 1e-9
        # token emitted after i accepted drafts: d_{i+1} if accepted too, else the corrected/bonus token
        if i < k:
            emitted = np.where(L[sel] >= i + 1, toks[sel, i + 1], r.next_token[sel])
        else:
            emitted = r.next_token[sel]
        f = np.bincount(emitted, minlength=V) / n
        assert _within(f, p[i], n), (i, f, p[i])
        if i < k:
            # P6: rejection probability at row i equals the residual mass 1 - alpha_i
            rej = (L[sel] == i).mean()
            assert abs(rej - (1 - alpha[i])) <= 4 * np.sqrt(alpha[i] * (1 - alpha[i]) / n) + 1e-9
            expect_len += reach * alpha[i]
            reach *= alpha[i]
    # P5: E[accept_len + 1] = sum_i prod_{j<i} alpha_j  (eq. 1 when all alpha_j are equal)
    assert abs(L.mean() - expect_len) <= 4 * L.std() / np.sqrt(B)


def test_expected_length_reduces_to_eq1_for_constant_alpha():
    """Same (p, q) at every row => alpha constant => E[L] = (1 - alpha^(k+1)) / (1 - alpha)."""
    rng = np.random.default_rng(3)
    B, k, V = 200_000, 5, 16
    Nq = k + 1
    l0 = rng.standard_normal(V)
    p = _softmax64(l0)
    q = _softmax64(l0 + rng.standard_normal(V)).astype(np.float32)
    alpha = np.minimum(p, q.astype(np.float64)).sum()
    toks = np.zeros((B, Nq), np.int32)
    for i in range(1, Nq):
        toks[:, i] = _draw(rng, q.astype(np.float64), B)
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    r = oracle.accept_from_logits(logits=np.broadcast_to(l0, (B, Nq, V)).copy(), draft_tokens=toks,
                                  draft_probs=np.broadcast_to(q, (B, Nq, V)).copy(), uniforms=un,
                                  temperature=1.0)
    emitted = r.accept_len + 1.0
    want = (1 - alpha ** (k + 1)) / (1 - alpha)
    assert abs(emitted.mean() - want) <= 4 * emitted.std() / np.sqrt(B)


# ------------------------------------------------------------------ P3 Monte-Carlo, tree
def test_monte_carlo_tree_emits_target_distribution():
    rng = np.random.default_rng(4)
    B, V = 250_000, 16
    #            0   1  2  3  4  5  6  7  8
    par = np.array([-1, 0, 0, 0, 1, 1, 2, 4, 3], np.int32)
    Nq = len(par)
    lrow = rng.standard_normal((Nq, V)) * 1.5
    p = _softmax64(lrow)
    q = _softmax64(lrow + rng.standard_normal((Nq, V)) * 1.2).astype(np.float32)
    toks = np.zeros((B, Nq), np.int32)
    for n in range(1, Nq):
        toks[:, n] = _draw(rng, q[par[n]].astype(np.float64), B)
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    r = oracle.accept_from_logits(logits=np.broadcast_to(lrow, (B, Nq, V)).copy(), draft_tokens=toks,
                                  draft_probs=np.broadcast_to(q, (B, Nq, V)).copy(), uniforms=un,
                                  parents=np.broadcast_to(par, (B, Nq)).copy(), temperature=1.0)
    depth = np.zeros(Nq, int)
    for n in range(1, Nq):
        depth[n] = depth[par[n]] + 1
    mask = r.accept_mask.astype(bool)
    assert mask[:, 0].all()
    assert np.array_equal(mask.sum(1) - 1, r.accept_len)
    assert np.array_equal(depth[r.stop_node], r.accept_len)
    # the token emitted right after node c was reached: the accepted child's token, or next_token
    for c in range(Nq):
        sel = mask[:, c]
        n = int(sel.sum())
        if n < 2000:
            continue
        kids = [m for m in range(Nq) if par[m] == c]
        emitted = r.next_token[sel].copy()
        for m in kids:
            took = mask[sel, m]
            emitted[took] = toks[sel, m][took]
        f = np.bincount(emitted, minlength=V) / n
        assert _within(f, p[c], n), (c, n)
    # more candidates per node => strictly more acceptance than the first-child-only chain
    first_only = 1 - np.minimum(p[0], q[0].astype(np.float64)).sum()
    assert (r.accept_len == 0).mean() < first_only


# ------------------------------------------------------------------ siblings drawn without replacement
def _draw_siblings_without_replacement(rng, q, par, B):
    """Tokens [B, Nq]: the children of a node are drawn in node order, each from the parent's row with the earlier
    siblings' tokens removed and the rest renormalised (inverse-CDF draws, written here independently)."""
    Nq, V = q.shape
    toks = np.zeros((B, Nq), np.int32)
    for n in range(1, Nq):
        rows = np.broadcast_to(q[par[n]].astype(np.float64), (B, V)).copy()
        for m in range(1, n):
            if par[m] == par[n]:
                rows[np.arange(B), toks[:, m]] = 0.0
        rows /= rows.sum(1, keepdims=True)
        cdf = np.cumsum(rows, axis=1)
        u = rng.random(B)
        toks[:, n] = np.minimum((cdf <= u[:, None]).sum(1), V - 1)
    return toks


def test_monte_carlo_tree_without_replacement_emits_target_distribution():
    """Three distinct candidates per node: the emitted token is distributed as the target's p at every node reached
    often enough - and it is NOT when the with-replacement rule is applied to the same drafts (the check has teeth)."""
    rng = np.random.default_rng(14)
    B, V = 250_000, 16
    par = np.array([-1, 0, 0, 0, 1, 1, 2, 4, 3], np.int32)
    Nq = len(par)
    lrow = rng.standard_normal((Nq, V)) * 1.5
    p = _softmax64(lrow)
    q = _softmax64(lrow + rng.standard_normal((Nq, V)) * 1.2).astype(np.float32)
    toks = _draw_siblings_without_replacement(rng, q, par, B)
    for a, b in ((1, 2), (1, 3), (2, 3), (4, 5)):
        assert (toks[:, a] != toks[:, b]).all()
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    kw = dict(logits=np.broadcast_to(lrow, (B, Nq, V)).copy(), draft_tokens=toks,
              draft_probs=np.broadcast_to(q, (B, Nq, V)).copy(), uniforms=un,
              parents=np.broadcast_to(par, (B, Nq)).copy(), temperature=1.0)

    def root_freq(r):
        mask = r.accept_mask.astype(bool)
        emitted = r.next_token.copy()
        for m in (1, 2, 3):
            emitted[mask[:, m]] = toks[mask[:, m], m]
        return np.bincount(emitted, minlength=V) / B

    r = oracle.accept_from_logits(without_replacement=True, **kw)
    mask = r.accept_mask.astype(bool)
    for c in range(Nq):
        sel = mask[:, c]
        n = int(sel.sum())
        if n < 2000:
            continue
        emitted = r.next_token[sel].copy()
        for m in [m for m in range(Nq) if par[m] == c]:
            took = mask[sel, m]
            emitted[took] = toks[sel, m][took]
        assert _within(np.bincount(emitted, minlength=V) / n, p[c], n), (c, n)
    assert _within(root_freq(r), p[0], B)
    assert not _within(root_freq(oracle.accept_from_logits(**kw)), p[0], B)


def test_without_replacement_hand_worked_step():
    """Vocabulary {0, 1, 2}, p = (0.5, 0.3, 0.2), q = (0.2, 0.5, 0.3), two candidates 1 then 2 under the root.
    Candidate 1: p/q = 0.6, rejected by u = 0.7.  Residual max(p - q, 0) = (0.3, 0, 0) -> p' = (1, 0, 0).
    Without replacement the second candidate was drawn from q' = (0.2, 0, 0.3) / 0.5 = (0.4, 0, 0.6):
    p'(2) / q'(2) = 0 -> rejected for any u, and the next token is drawn from max(p' - q', 0) = (0.6, 0, 0) -> token 0.
    A candidate 0 in second place: p'(0) / q'(0) = 1 / 0.4 > 1 -> accepted for every u < 1 (with replacement the
    ratio 1 / 0.2 gives the same decision; the two rules differ in q', checked through test_margin = |p'/q' - u|)."""
    lg = np.log(np.array([0.5, 0.3, 0.2]))[None, None, :].repeat(3, axis=1)
    q = np.array([0.2, 0.5, 0.3], np.float32)[None, None, :].repeat(3, axis=1)
    par = np.array([[-1, 0, 0]], np.int32)
    un = np.array([[[0, 0.3], [0.7, 0.5], [0.9, 0.5]]], np.float32)
    r = oracle.accept_from_logits(logits=lg, draft_tokens=np.array([[0, 1, 2]], np.int32), draft_probs=q, uniforms=un,
                                  parents=par, temperature=1.0, without_replacement=True)
    assert r.accept_len[0] == 0 and r.next_token[0] == 0 and not r.accept_mask[0, 1:].any()
    assert abs(r.test_margin[0, 1] - abs(0.6 - np.float32(0.7))) < 1e-6 and abs(r.test_margin[0, 2] - np.float32(0.9)) < 1e-6
    for wor, ratio in ((True, 1 / 0.4), (False, 1 / 0.2)):
        r = oracle.accept_from_logits(logits=lg, draft_tokens=np.array([[0, 1, 0]], np.int32), draft_probs=q, uniforms=un,
                                      parents=par, temperature=1.0, without_replacement=wor)
        assert r.accept_len[0] == 1 and r.accept_mask[0, 2] == 1 and r.stop_node[0] == 2
        assert abs(r.test_margin[0, 2] - (ratio - np.float32(0.9))) < 1e-5


def test_without_replacement_changes_nothing_on_chains_and_single_children():
    w = gen.llama_chain(71, batch=6, len_lo=8, len_hi=20, vocab=64, hidden_size=32, num_q_heads=2, num_kv_heads=1,
                        head_dim=8, page_size=4, dtype=gen.F32)
    lg = oracle.logits(hidden=w.hidden, lm_head=w.lm_head, dtype=w.dtype)
    kw = dict(logits=lg, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs, uniforms=w.uniforms,
              parents=gen.chain_parents(w.batch, w.num_q), temperature=w.temperature)
    a, b = oracle.accept_from_logits(**kw), oracle.accept_from_logits(without_replacement=True, **kw)
    for f in ("accept_len", "next_token", "accept_mask", "stop_node"):
        assert np.array_equal(getattr(a, f), getattr(b, f))


# ------------------------------------------------------------------ draft model with a smaller vocabulary
def test_monte_carlo_subvocabulary_draft_still_emits_target_distribution():
    """q lives on 6 of the 16 target ids (ids the draft model cannot emit have q = 0).  Speculative
    sampling is exact for any q, so the emitted token is still distributed as p - which fails if the
    compact rows are scattered to the wrong ids, or if mass off the draft vocabulary is dropped from
    the residual."""
    rng = np.random.default_rng(7)
    B, k, V, Vd = 250_000, 3, 16, 6
    Nq = k + 1
    d2t = np.sort(rng.choice(V, size=Vd, replace=False)).astype(np.int32)
    lrow = rng.standard_normal((Nq, V)) * 1.2
    p = _softmax64(lrow)
    q_sub = _softmax64(lrow[:, d2t] + rng.standard_normal((Nq, Vd)) * 0.7).astype(np.float32)
    toks = np.zeros((B, Nq), np.int32)
    for i in range(1, Nq):
        toks[:, i] = d2t[_draw(rng, q_sub[i - 1].astype(np.float64), B)]
    un = gen.workloads._uniform24(rng, (B, Nq, 2))
    r = oracle.accept_from_logits(logits=np.broadcast_to(lrow, (B, Nq, V)).copy(), draft_tokens=toks,
                                  draft_probs=np.broadcast_to(q_sub, (B, Nq, Vd)).copy(), uniforms=un,
                                  temperature=1.0, draft_to_target=d2t)
    L = r.accept_len
    q_dense = np.zeros((Nq, V))
    q_dense[:, d2t] = q_sub
    alpha = np.minimum(p, q_dense).sum(-1)
    reach = 1.0
    for i in range(Nq):
        sel = L >= i
        n = int(sel.sum())
        assert abs(n / B - reach) <= 4 * np.sqrt(reach * (1 - reach) / B) + 1e-9
        emitted = np.where(L[sel] >= i + 1, toks[sel, min(i + 1, k)], r.next_token[sel]) if i < k else r.next_token[sel]
        f = np.bincount(emitted, minlength=V) / n
        assert _within(f, p[i], n), (i, f, p[i])
        if i < k:
            reach *= alpha[i]
    # ids off the draft vocabulary can only ever appear as corrected / bonus tokens
    off = np.setdiff1d(np.arange(V), d2t)
    assert np.isin(r.next_token, off).mean() > 0.2


def test_full_draft_vocabulary_with_identity_map_equals_dense_call():
    w = gen.tiny_chain(5)
    a = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                      uniforms=w.uniforms, dtype=w.dtype, temperature=w.temperature)
    b = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                      uniforms=w.uniforms, dtype=w.dtype, temperature=w.temperature,
                      draft_to_target=np.arange(w.vocab, dtype=np.int32))
    assert np.array_equal(a.accept_len, b.accept_len) and np.array_equal(a.next_token, b.next_token)


def test_subvocabulary_generator_is_consistent():
    w = gen.llama_chain(31, batch=6, len_lo=20, len_hi=40, vocab=1000, hidden_size=64, draft_vocab=250)
    assert w.draft_probs.shape == (6, 5, 250) and w.draft_vocab == 250
    d2t, t2d = w.draft_to_target, w.target_to_draft()
    assert np.all(np.diff(d2t) > 0) and np.array_equal(t2d[d2t], np.arange(250))
    assert (t2d >= 0).sum() == 250 and np.all(t2d[w.draft_tokens[:, 1:]] >= 0)
    assert np.allclose(w.draft_probs.sum(-1), 1.0, atol=1e-4)


def test_one_temperature_per_request_is_the_scalar_oracle_request_by_request():
    """A workload with its own temperature per request (0 = greedy): every request must come out as the scalar
    oracle gives it alone at that temperature; equal temperatures must reproduce the scalar call on the batch."""
    import dataclasses
    temps = np.array([1.0, 0.0, 0.6, 1.7], np.float32)
    w = gen.llama_chain(33, batch=4, len_lo=20, len_hi=50, vocab=400, hidden_size=64, temperatures=temps)
    a = oracle.accept_workload(w)
    for b in range(4):
        wb = dataclasses.replace(w.take_requests([b]), temperatures=None, temperature=float(temps[b]))
        if temps[b] == 0:
            wb = dataclasses.replace(wb, draft_probs=None, uniforms=None)
        one = oracle.accept_workload(wb)
        assert one.accept_len[0] == a.accept_len[b] and one.next_token[0] == a.next_token[b]
        assert np.array_equal(one.accept_mask[0], a.accept_mask[b]) and np.array_equal(one.row_lse[0], a.row_lse[b])
    ws = dataclasses.replace(w, temperatures=None, temperature=0.6)
    wt = dataclasses.replace(w, temperatures=np.full(4, 0.6, np.float32))
    x, y = oracle.accept_workload(ws), oracle.accept_workload(wt)
    for f in ("accept_len", "next_token", "accept_mask", "p_at_draft", "row_lse"):
        assert np.array_equal(getattr(x, f), getattr(y, f)), f
    # the generator draws request b's draft distribution at its own temperature: a colder request is more peaked
    assert w.draft_probs[2].max(axis=-1).mean() > w.draft_probs[3].max(axis=-1).mean()
