"""Pins of the acceptance oracle: exact enumeration of the output law (the property the
paper claims for speculative decoding, Section 5), a hand-worked rational example,
textbook special cases and limits (CPU only)."""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.stats import qmc

import oracle
from oracle import RULE_DETERMINISTIC as DET, RULE_DRAFT_WOR as WOR, RULE_DRAFT_WR as WR, RULE_GREEDY as GREEDY
from synth_inputs import trees

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _logits_of(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def _softmax64(z, temp=1.0):
    z = np.asarray(z, dtype=np.float64) / temp
    e = np.exp(z - z.max())
    return e / e.sum()


# ------------------------------------------------------------------------------
# An enumerator that knows only the formulas of the rule (no oracle code): the exact law of
# the token emitted at a node with k drafted children, for a given ordered sibling list.
# ------------------------------------------------------------------------------
def _cond_law_first_token(p, q, sibs, rule):
    """P(first emitted token = v | ordered sibling tokens), exact."""
    V = len(p)
    law = np.zeros(V)
    reach = 1.0                      # probability that all earlier siblings were rejected
    p = p.copy()
    q = None if q is None else q.copy()
    for x in sibs:
        if rule == DET:
            a = p[x]
        else:
            a = 1.0 if q[x] <= 0 and p[x] > 0 else (0.0 if q[x] <= 0 else min(1.0, p[x] / q[x]))
        law[x] += reach * a
        reach *= (1.0 - a)
        if reach == 0.0:
            return law
        if rule == DET:
            p[x] = 0.0
            p = p / p.sum()
        else:
            r = np.maximum(p - q, 0.0)
            if r.sum() > 0:
                p = r / r.sum()
            if rule == WOR:
                q[x] = 0.0
                if q.sum() > 0:
                    q = q / q.sum()
    return law + reach * p


def _sibling_draws(q, k, rule, V):
    """All ordered sibling lists with their draw probability under the matching sampler."""
    if rule == WR:
        for sibs in itertools.product(range(V), repeat=k):
            yield sibs, float(np.prod([q[x] for x in sibs]))
    else:   # without replacement
        for sibs in itertools.permutations(range(V), k):
            pr, rest = 1.0, 1.0
            for x in sibs:
                pr *= q[x] / rest
                rest -= q[x]
            yield sibs, pr


@pytest.mark.parametrize("rule,k", [(WOR, 1), (WOR, 2), (WOR, 3), (WR, 2), (WR, 3)])
def test_rule_preserves_target_law_exact_enumeration(rule, k):
    """Section 5: speculative decoding preserves the target's sampling law.  Summed over how the
    siblings were drawn and over accept/reject outcomes, the first emitted token follows p."""
    rng = np.random.default_rng(100 + k)
    V = 4
    for _ in range(5):
        p = rng.dirichlet(np.ones(V))
        q = rng.dirichlet(np.ones(V))
        law = np.zeros(V)
        for sibs, pr in _sibling_draws(q, k, rule, V):
            law += pr * _cond_law_first_token(p, q, sibs, rule)
        np.testing.assert_allclose(law, p, rtol=0, atol=1e-12)


def test_mismatched_sibling_sampler_is_not_exact():
    """Why the generator and the rule must agree: the with-replacement rule applied to siblings
    drawn without replacement does NOT reproduce p."""
    rng = np.random.default_rng(7)
    V, k = 4, 2
    p = rng.dirichlet(np.ones(V))
    q = rng.dirichlet(np.ones(V))
    law = np.zeros(V)
    for sibs, pr in _sibling_draws(q, k, WOR, V):
        law += pr * _cond_law_first_token(p, q, sibs, WR)
    assert np.abs(law - p).max() > 1e-4


@pytest.mark.parametrize("k", [1, 2, 3])
def test_deterministic_rule_exact_for_any_fixed_candidates(k):
    rng = np.random.default_rng(200 + k)
    V = 5
    p = rng.dirichlet(np.ones(V))
    for sibs in itertools.permutations(range(V), k):
        np.testing.assert_allclose(_cond_law_first_token(p, None, sibs, DET), p, rtol=0, atol=1e-12)


def _star_tree(k):
    return np.array([-1] + [0] * k, dtype=np.int32)


def _oracle_first_token_law(p, q, sibs, rule, n_log2=17, seed=0):
    """Empirical law of the oracle's first emitted token over a scrambled Sobol set of uniforms."""
    V, k = len(p), len(sibs)
    T = k + 1
    tl = np.tile(_logits_of(p), (T, 1))
    dl = None if q is None else np.tile(_logits_of(q), (T, 1))
    token = np.array([0] + list(sibs), dtype=np.int32)
    pts = qmc.Sobol(d=k + 1, scramble=True, seed=seed).random_base2(n_log2).astype(np.float32)
    pts = np.minimum(pts, np.float32(1.0) - np.float32(2 ** -24))
    un = np.zeros((len(pts), 2 * T), dtype=np.float32)
    un[:, 1:T] = pts[:, :k]
    un[:, T:] = pts[:, k:k + 1]            # whichever node the walk stops at, same final uniform
    res = oracle.tree_accept_many(tl, dl, token, _star_tree(k), un, temperature=1.0, rule=rule)
    first = np.where(res["n_accepted"] > 0, token[res["last_node"]], res["final_token"])
    # children are leaves here, so an accepted child ends the walk with a bonus token drawn at it
    return np.bincount(first, minlength=V) / len(pts), res


@pytest.mark.parametrize("rule", [DET, WOR, WR])
def test_oracle_matches_enumerated_conditional_law(rule):
    """The implementation, driven over a low-discrepancy set of uniforms, reproduces the exact
    conditional law of the first emitted token for fixed siblings; weighted by the draw
    probabilities it reproduces the target law."""
    rng = np.random.default_rng(300 + rule)
    V, k = 4, 2
    p = rng.dirichlet(np.ones(V) * 2)
    q = None if rule == DET else rng.dirichlet(np.ones(V) * 2)
    # float32 logits round the laws slightly: enumerate with the rounded ones
    p_r = _softmax64(_logits_of(p))
    q_r = None if q is None else _softmax64(_logits_of(q))
    total = np.zeros(V)
    draws = list(_sibling_draws(q_r if q_r is not None else np.full(V, 1.0 / V), k, WOR if rule == DET else rule, V))
    for sibs, pr in draws:
        emp, _ = _oracle_first_token_law(p, q, sibs, rule)
        exact = _cond_law_first_token(p_r, q_r, sibs, rule)
        np.testing.assert_allclose(emp, exact, rtol=0, atol=2e-3)
        total += pr * emp
    np.testing.assert_allclose(total, p_r, rtol=0, atol=1e-3)


def test_two_level_pair_law():
    """Root with two children, each with one child: the emitted pair (first, second token)
    follows p_root(a) * p_{node reached}(b) whenever a drafted child was accepted, and the walk
    stops with one token otherwise (deterministic rule, exact for any candidates)."""
    rng = np.random.default_rng(41)
    V = 4
    parent = np.array([-1, 0, 0, 1, 2], dtype=np.int32)
    token = np.array([0, 1, 3, 2, 0], dtype=np.int32)
    laws = rng.dirichlet(np.ones(V) * 2, size=5)
    tl = np.stack([_logits_of(l) for l in laws])
    laws = np.stack([_softmax64(t) for t in tl])
    T = 5
    pts = qmc.Sobol(d=5, scramble=True, seed=3).random_base2(18).astype(np.float32)
    pts = np.minimum(pts, np.float32(1.0) - np.float32(2 ** -24))
    un = np.zeros((len(pts), 2 * T), dtype=np.float32)
    un[:, 1:5] = pts[:, :4]
    un[:, T:] = pts[:, 4:5]
    res = oracle.tree_accept_many(tl, None, token, parent, un, temperature=1.0, rule=DET)
    nacc, last, ftok = res["n_accepted"], res["last_node"], res["final_token"]
    # exact: P(accept child 1) = p0[1]; P(accept child 2) = p0[3] (zero-and-renormalise telescopes)
    assert abs(np.mean((nacc >= 1) & np.isin(last, [1, 3])) - laws[0][1]) < 2e-3
    assert abs(np.mean((nacc >= 1) & np.isin(last, [2, 4])) - laws[0][3]) < 2e-3
    # first token law overall = p_root
    first = np.where(nacc == 0, ftok, np.where(np.isin(last, [1, 3]), 1, 3))
    np.testing.assert_allclose(np.bincount(first, minlength=V) / len(pts), laws[0], rtol=0, atol=2e-3)
    # given the walk reached node 1, the second token follows p_1
    at1 = np.isin(last, [1, 3])
    second = np.where(last[at1] == 3, 2, ftok[at1])
    np.testing.assert_allclose(np.bincount(second, minlength=V) / at1.sum(), laws[1], rtol=0, atol=5e-3)


def test_rational_worked_example():
    with open(os.path.join(GOLDEN, "accept_rational_example.json")) as f:
        g = json.load(f)
    p, q = np.array(g["p"]), np.array(g["q"])
    tl = np.tile(_logits_of(p), (3, 1))
    dl = np.tile(_logits_of(q), (3, 1))
    par1 = np.array([-1, 0], dtype=np.int32)

    def run(tokens, parent, u, rule, draft=True):
        T = len(parent)
        assert len(u) == T + 1          # one uniform per node, then the final-draw uniform
        un = np.zeros(2 * T, dtype=np.float32)
        un[:T] = u[:T]
        un[T:] = u[-1]
        return oracle.tree_accept(tl[:T], dl[:T] if draft else None, tokens, parent, un, temperature=1.0, rule=rule)

    # child = token 2: accepted iff u < 1/3; residual is the point mass on token 0
    for u1, acc in [(0.30, 1), (0.3333, 1), (0.3334, 0), (0.9, 0)]:
        for uf in (0.0, 0.5, 0.999):
            r = run([0, 2], par1, [0.0, u1, uf], WOR)
            assert r["n_accepted"] == acc
            if not acc:
                assert (r["final_token"], r["final_kind"]) == (0, oracle.FINAL_RESIDUAL)
            else:
                assert r["final_kind"] == oracle.FINAL_BONUS and r["last_node"] == 1
    # child = token 0 or 1: ratio >= 1, always accepted
    for tok in (0, 1):
        for u1 in (0.0, 0.5, 0.99999994):
            assert run([0, tok], par1, [0.0, u1, 0.5], WOR)["n_accepted"] == 1
    # deterministic rule: accept iff u < 1/6; else law (3/5, 2/5, 0)
    assert run([0, 2], par1, [0.0, 0.16, 0.5], DET, draft=False)["n_accepted"] == 1
    r = run([0, 2], par1, [0.0, 0.17, 0.59], DET, draft=False)
    assert (r["n_accepted"], r["final_token"], r["final_kind"]) == (0, 0, oracle.FINAL_RESIDUAL)
    r = run([0, 2], par1, [0.0, 0.17, 0.61], DET, draft=False)
    assert (r["n_accepted"], r["final_token"]) == (0, 1)
    # siblings (2, 1) without replacement: both rejected at u = 0.9, 0.0+ ; final token 0
    par2 = np.array([-1, 0, 0], dtype=np.int32)
    r = run([0, 2, 1], par2, [0.0, 0.9, 1e-6, 0.7], WOR)
    assert (r["n_accepted"], r["final_token"], r["final_kind"]) == (0, 0, oracle.FINAL_RESIDUAL)


def test_root_only_tree_is_inverse_cdf_sampling():
    rng = np.random.default_rng(5)
    V = 1000
    z = (rng.standard_normal(V) * 2).astype(np.float32)
    for temp in (1.0, 0.7):
        p = _softmax64(z, temp)
        cdf = np.cumsum(p)
        for u in rng.random(50, dtype=np.float32):
            r = oracle.tree_accept(z[None], None, [3], [-1], np.array([0.0, u], np.float32), temperature=temp, rule=DET)
            assert r["n_accepted"] == 0 and r["final_kind"] == oracle.FINAL_BONUS
            assert r["final_token"] == int(np.searchsorted(cdf, float(u), side="right"))
            assert r["path"][0] == 0 and r["last_node"] == 0


def test_identical_draft_and_target_accept_first_child_chain():
    """q = p: the ratio is 1, every first child is accepted down to a leaf, bonus token."""
    rng = np.random.default_rng(6)
    T, V = 20, 50
    parent = trees.random_tree(rng, T, 5, 3)
    tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
    token = rng.integers(0, V, T).astype(np.int32)
    un = rng.random(2 * T, dtype=np.float32)
    r = oracle.tree_accept(tl, tl.copy(), token, parent, un, temperature=1.0, rule=WOR)
    expect = [0]
    while True:
        ch = [c for c in range(T) if parent[c] == expect[-1]]
        if not ch:
            break
        expect.append(ch[0])
    assert r["path"][:len(expect)].tolist() == expect and r["n_accepted"] == len(expect) - 1
    assert r["final_kind"] == oracle.FINAL_BONUS and r["last_node"] == expect[-1]
    assert np.all(r["path"][len(expect):] == -1)


def test_greedy_is_the_low_temperature_limit():
    rng = np.random.default_rng(8)
    T, V = 30, 40
    for trial in range(20):
        parent = trees.random_tree(rng, T, 6, 4)
        tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
        token = np.zeros(T, np.int32)
        for u in range(T):
            ch = [c for c in range(T) if parent[c] == u]
            order = np.argsort(-(tl[u] + rng.standard_normal(V)))     # noisy top-k proposals
            for c, x in zip(ch, order):
                token[c] = x
        un = rng.random(2 * T, dtype=np.float32) * 0.98 + 0.01
        g = oracle.tree_accept(tl, None, token, parent, None, temperature=0.0, rule=GREEDY)
        cold = oracle.tree_accept(tl, None, token, parent, un, temperature=1e-3, rule=DET)
        assert g["path"].tolist() == cold["path"].tolist()
        assert g["final_token"] == cold["final_token"] == int(np.argmax(tl[g["last_node"]]))
        # greedy: stop node's kind is BONUS iff no drafted child was turned down there
        has_kids = any(parent[c] == g["last_node"] for c in range(T))
        assert g["final_kind"] == (oracle.FINAL_RESIDUAL if has_kids else oracle.FINAL_BONUS)


def test_greedy_ties_take_lowest_index():
    tl = np.zeros((2, 5), np.float32)
    tl[0, [1, 3]] = 2.0
    for tok, acc in [(1, 1), (3, 0)]:
        r = oracle.tree_accept(tl, None, [0, tok], [-1, 0], None, temperature=0.0, rule=GREEDY)
        assert r["n_accepted"] == acc


def test_chain_acceptance_rate_is_one_minus_total_variation():
    """Linear speculation (one child per node): a position is accepted with probability
    sum_v min(p, q) when the drafted token is drawn from q."""
    rng = np.random.default_rng(9)
    V, n = 6, 1 << 16
    p = rng.dirichlet(np.ones(V))
    q = rng.dirichlet(np.ones(V))
    tl = np.tile(_logits_of(p), (2, 1))
    dl = np.tile(_logits_of(q), (2, 1))
    pr, qr = _softmax64(tl[0]), _softmax64(dl[0])
    acc = 0.0
    for x in range(V):
        pts = qmc.Sobol(d=2, scramble=True, seed=x).random_base2(14).astype(np.float32)
        pts = np.minimum(pts, np.float32(1.0) - np.float32(2 ** -24))
        un = np.zeros((len(pts), 4), np.float32)
        un[:, 1] = pts[:, 0]
        un[:, 2:] = pts[:, 1:2]
        res = oracle.tree_accept_many(tl, dl, np.array([0, x], np.int32), np.array([-1, 0], np.int32), un,
                                      temperature=1.0, rule=WOR)
        acc += qr[x] * np.mean(res["n_accepted"] == 1)
    assert abs(acc - np.minimum(pr, qr).sum()) < 1e-3


def test_extreme_uniforms():
    rng = np.random.default_rng(10)
    T, V = 25, 30
    parent = trees.random_tree(rng, T, 5, 3)
    tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
    dl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
    token = rng.integers(0, V, T).astype(np.int32)
    # u = 0: every test 0 * q < p passes (p > 0 everywhere): first-child chain
    r = oracle.tree_accept(tl, dl, token, parent, np.zeros(2 * T, np.float32), temperature=1.0, rule=WOR)
    cur, n = 0, 0
    while True:
        ch = [c for c in range(T) if parent[c] == cur]
        if not ch:
            break
        cur, n = ch[0], n + 1
    assert r["last_node"] == cur and r["n_accepted"] == n
    # u -> 1-: a first child is accepted only if p(x) >= q(x) (up to the last ulp of u)
    one = np.full(2 * T, np.float32(1.0) - np.float32(2 ** -24), np.float32)
    r = oracle.tree_accept(tl, dl, token, parent, one, temperature=1.0, rule=WOR)
    if r["n_accepted"] > 0:
        c = int(r["path"][1])
        first = min(cc for cc in range(T) if parent[cc] == 0)
        if c == first:
            p0, q0 = _softmax64(tl[0]), _softmax64(dl[0])
            assert p0[token[c]] >= q0[token[c]] * float(one[0])


def test_residual_token_support():
    """After rejections the final token comes from the corrected law: under the draft rules it
    has p > q at the stop node (single child), under the deterministic rule it is never a
    rejected candidate."""
    rng = np.random.default_rng(12)
    V = 12
    p = rng.dirichlet(np.ones(V))
    q = rng.dirichlet(np.ones(V))
    tl = np.tile(_logits_of(p), (3, 1))
    dl = np.tile(_logits_of(q), (3, 1))
    pr, qr = _softmax64(tl[0]), _softmax64(dl[0])
    un = rng.random((4000, 6), dtype=np.float32)
    x = int(np.argmax(qr - pr))
    res = oracle.tree_accept_many(tl[:2], dl[:2], np.array([0, x], np.int32), np.array([-1, 0], np.int32),
                                  un[:, :4].copy(), temperature=1.0, rule=WOR)
    rej = res["n_accepted"] == 0
    assert rej.any() and np.all(res["final_kind"][rej] == oracle.FINAL_RESIDUAL)
    assert np.all(pr[res["final_token"][rej]] > qr[res["final_token"][rej]])
    cands = np.array([0, 3, 7], np.int32)
    res = oracle.tree_accept_many(tl, None, cands, np.array([-1, 0, 0], np.int32), un, temperature=1.0, rule=DET)
    rej = res["n_accepted"] == 0
    assert rej.any() and not np.isin(res["final_token"][rej], cands[1:]).any()


def _accept_bits_independently(tl, dl, token, parent, un, temp, rule):
    """Every node's accept bit computed on its own from its parent's rows and its sibling rank
    (numpy, fp64), then a scan over the bits: the data-parallel formulation."""
    T, V = tl.shape
    bits = np.zeros(T, bool)
    stop_law = {}
    for u in range(T):
        p = _softmax64(tl[u], temp)
        q = None if dl is None else _softmax64(dl[u], temp)
        stop_law[(u, 0)] = p.copy()
        nrej = 0
        for c in range(u + 1, T):
            if parent[c] != u:
                continue
            x = token[c]
            bits[c] = (un[c] < p[x]) if rule == DET else (float(un[c]) * q[x] < p[x])
            # chain continues as if c was rejected
            if rule == DET:
                p[x] = 0.0
                p = p / p.sum()
            else:
                r = np.maximum(p - q, 0)
                if r.sum() > 0:
                    p = r / r.sum()
                if rule == WOR:
                    q[x] = 0
                    q = q / q.sum()
            nrej += 1
            stop_law[(u, nrej)] = p.copy()
    cur, path = 0, [0]
    while True:
        nxt, nrej = -1, 0
        for c in range(cur + 1, T):
            if parent[c] == cur:
                if bits[c]:
                    nxt = c
                    break
                nrej += 1
        if nxt < 0:
            break
        cur = nxt
        path.append(cur)
    law = stop_law[(cur, nrej)]
    ftok = int(np.searchsorted(np.cumsum(law), float(un[T + cur]), side="right"))
    return path, min(ftok, V - 1), nrej > 0


@pytest.mark.parametrize("rule", [DET, WOR, WR])
def test_path_independence_of_accept_bits(rule):
    rng = np.random.default_rng(13 + rule)
    T, V = 24, 64
    for trial in range(25):
        parent = trees.random_tree(rng, T, 5, 4)
        tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
        dl = None if rule == DET else (0.8 * tl + 0.6 * rng.standard_normal((T, V)) * 2).astype(np.float32)
        token = rng.integers(0, V, T).astype(np.int32)
        un = rng.random(2 * T, dtype=np.float32)
        r = oracle.tree_accept(tl, dl, token, parent, un, temperature=0.8, rule=rule)
        path, ftok, rejected = _accept_bits_independently(tl, dl, token, parent, un, 0.8, rule)
        assert r["path"][:r["n_accepted"] + 1].tolist() == path
        assert r["final_token"] == ftok
        assert r["final_kind"] == (oracle.FINAL_RESIDUAL if rejected else oracle.FINAL_BONUS)


def test_selected_contemplate_follows_last_node():
    """Section 3.1: the future prediction kept is the one paired with the last accepted node."""
    rng = np.random.default_rng(14)
    T, V = 10, 20
    parent = trees.chain_tree(T)
    tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
    token = np.concatenate([[0], np.argmax(tl[:-1], axis=1)]).astype(np.int32)
    token[6] = (token[6] + 1) % V       # greedy walk stops at node 5
    r = oracle.tree_accept(tl, None, token, parent, None, temperature=0.0, rule=GREEDY,
                           con_anchor=np.arange(T, dtype=np.int32))
    assert r["last_node"] == 5 and r["selected_con"] == 5 and r["n_accepted"] == 5
    r = oracle.tree_accept(tl, None, token, parent, None, temperature=0.0, rule=GREEDY,
                           con_anchor=np.array([0, 0], np.int32))
    assert r["selected_con"] == -1


@pytest.mark.parametrize("kw", [
    dict(parent=[-1, 1]), dict(parent=[0, 0]), dict(token=[0, 99]), dict(token=[0, -1]),
])
def test_bad_inputs_are_rejected(kw):
    tl = np.zeros((2, 5), np.float32)
    args = dict(parent=[-1, 0], token=[0, 1])
    args.update(kw)
    with pytest.raises(oracle.OracleError):
        oracle.tree_accept(tl, None, args["token"], args["parent"], np.zeros(4, np.float32),
                           temperature=1.0, rule=DET)


# ---- the literal sample-and-match reading (Section 2, step 3) ---------------------------------------------
def test_sample_and_match_is_autoregressive_sampling_along_the_tree():
    """With node-indexed uniforms the emitted tokens must be exactly what plain sampling of the target would
    emit: at each visited node the token searchsorted(cumsum(p_node), u[T+node]); the walk follows a child iff it
    carries that token.  Checked with an independent numpy walk."""
    rng = np.random.default_rng(77)
    T, V = 14, 9
    SM = oracle.RULE_SAMPLE_MATCH
    for trial in range(200):
        parent = trees.random_tree(rng, T, 4, 3)
        tl = (rng.standard_normal((T, V)) * 1.5).astype(np.float32)
        token = rng.integers(0, V, size=T).astype(np.int32)
        un = rng.random(2 * T, dtype=np.float32)
        temp = 1.0 if trial % 2 else 0.7
        r = oracle.tree_accept(tl, None, token, parent, un, temperature=temp, rule=SM)
        cur, path = 0, [0]
        while True:
            y = int(np.searchsorted(np.cumsum(_softmax64(tl[cur], temp)), float(un[T + cur]), side="right"))
            kids = [c for c in range(cur + 1, T) if parent[c] == cur]
            hit = [c for c in kids if token[c] == y]
            if not hit:
                break
            cur = hit[0]
            path.append(cur)
        assert list(r["path"][:len(path)]) == path and r["n_accepted"] == len(path) - 1
        assert r["final_token"] == y and r["last_node"] == cur
        assert r["final_kind"] == (oracle.FINAL_RESIDUAL if kids else oracle.FINAL_BONUS)


def test_sample_and_match_first_token_law_is_the_target_law():
    """Over a stratified grid of the root's uniform the first emitted token (the accepted child's token, or the
    final token when nothing is accepted) is distributed as softmax(target[root]) up to the grid resolution."""
    rng = np.random.default_rng(78)
    T, V, n = 5, 6, 4000
    parent = np.array([-1, 0, 0, 0, 1], dtype=np.int32)
    token = np.array([0, 2, 4, 5, 1], dtype=np.int32)
    tl = rng.standard_normal((T, V)).astype(np.float32)
    counts = np.zeros(V)
    for k in range(n):
        un = np.full(2 * T, 0.5, dtype=np.float32)
        un[T + 0] = (k + 0.5) / n
        r = oracle.tree_accept(tl, None, token, parent, un, temperature=1.0, rule=oracle.RULE_SAMPLE_MATCH)
        first = token[r["path"][1]] if r["n_accepted"] >= 1 else r["final_token"]
        counts[first] += 1
    assert np.abs(counts / n - _softmax64(tl[0], 1.0)).max() <= 2.0 / n


@pytest.mark.parametrize("rule", [DET, WOR, WR])
def test_banned_tokens_equal_a_smaller_vocabulary(rule):
    """Logits of -infinity carry no mass: the walk over a vocabulary with banned entries is the walk over the
    vocabulary without them (entries renumbered), for the same uniforms - textbook softmax over the finite
    entries.  Pins what the oracle does with -infinity, which the HIP path is then held to."""
    rng = np.random.default_rng(91)
    V, T = 40, 9
    parent = trees.random_tree(rng, T, 4, 3)
    keep = np.sort(rng.choice(V, size=25, replace=False))            # the entries that stay finite
    new_of = -np.ones(V, dtype=np.int64)
    new_of[keep] = np.arange(len(keep))
    for trial in range(40):
        tl = rng.normal(0, 2, size=(T, V)).astype(np.float32)
        dl = (0.8 * tl + rng.normal(0, 1, size=(T, V))).astype(np.float32)
        tl[:, np.setdiff1d(np.arange(V), keep)] = -np.inf
        dl[:, np.setdiff1d(np.arange(V), keep)] = -np.inf
        token = rng.choice(keep, size=T).astype(np.int32)
        un = rng.random(2 * T, dtype=np.float32)
        draft = None if rule == DET else dl
        full = oracle.tree_accept(tl, draft, token, parent, un, temperature=0.9, rule=rule)
        small = oracle.tree_accept(np.ascontiguousarray(tl[:, keep]), None if draft is None else np.ascontiguousarray(dl[:, keep]),
                                   new_of[token].astype(np.int32), parent, un, temperature=0.9, rule=rule)
        assert np.array_equal(full["path"], small["path"]) and full["final_kind"] == small["final_kind"]
        assert new_of[full["final_token"]] == small["final_token"]
