"""GPU parity: tree_accept (HIP, through the C ABI) against the fp64 CPU oracle on identical
seeded inputs.  Paths, counts, kinds and tokens must be bit-exact; a disagreement is tolerated
only when some comparison along the oracle's walk lies within 1e-6 of its threshold, and such
cases are counted (harness.compare_accept)."""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from synth_inputs import trees
from tests import harness as H

pytestmark = pytest.mark.gpu

RULES = {"greedy": oracle.RULE_GREEDY, "det": oracle.RULE_DETERMINISTIC, "wor": oracle.RULE_DRAFT_WOR,
         "wr": oracle.RULE_DRAFT_WR, "match": oracle.RULE_SAMPLE_MATCH}


def _batch(seed, *, B, T, V, rule, temp, corr=0.9, max_depth=6, max_children=4, std=2.0, C=0, tree=None, boost=0.0):
    rng = np.random.default_rng(seed)
    parents = np.stack([tree if tree is not None else trees.random_tree(rng, T, max_depth, max_children)
                        for _ in range(B)])
    ca = None if C == 0 else rng.integers(0, T, size=(B, C)).astype(np.int32)
    return si.make_accept_inputs(rng, parent=parents, V=V, temperature=temp, rule=rule, logit_std=std,
                                 con_anchor=ca, draft_target_corr=corr, proposal_noise_std=1.0, child_boost=boost)


def _run_and_compare(inp, **kw):
    got = H.run_accept(inp, **kw)
    exact, near = H.compare_accept(inp, got)
    print(f"[accept] B={inp.B} T={inp.T} V={inp.V} rule={inp.rule} temp={inp.temperature}: "
          f"{exact} exact, {near} within 1e-6 of a threshold")
    assert near <= max(1, inp.B // 100)
    return got


@pytest.mark.parametrize("mode", [0, 1])
def test_tiny_workload(mode):
    _run_and_compare(si.accept_case(0, mode))
    _run_and_compare(si.accept_case(0, mode, draft_target_corr=0.9))


@pytest.mark.parametrize("rule", ["det", "wor", "wr"])
@pytest.mark.parametrize("temp", [1.0, 0.7])
def test_many_small_sequences(rule, temp):
    """256 independent sequences per call; vocabulary size not a multiple of 4."""
    inp = _batch(21, B=256, T=24, V=5003, rule=RULES[rule], temp=temp, C=3, boost=7.0)
    got = _run_and_compare(inp)
    # the walks must be non-trivial for the test to mean anything
    assert got["n_accepted"].max() >= 3 and (got["final_kind"] == 1).any() and (got["final_kind"] == 0).any()


def test_greedy_many_sequences_and_ties():
    inp = _batch(22, B=128, T=30, V=777, rule=RULES["greedy"], temp=0.0)
    inp.target_logits[:, :, 5] = inp.target_logits[:, :, 300] = 50.0      # tie: index 5 must win
    inp.token[:, 1] = 5
    got = _run_and_compare(inp)
    assert np.all(got["n_accepted"] >= 1)
    inp.token[:, 1] = 300
    _run_and_compare(inp)


@pytest.mark.parametrize("rule", ["det", "wor", "wr"])
def test_uncorrelated_draft_and_wide_star(rule):
    """Independent draft/target logits (mostly rejections) and a root with 20 children: long
    sibling chains."""
    star = np.array([-1] + [0] * 20 + [1, 1, 2], dtype=np.int32)
    inp = _batch(23, B=32, T=24, V=4096, rule=RULES[rule], temp=1.0, corr=0.0, tree=star)
    got = _run_and_compare(inp)
    assert (got["n_accepted"] == 0).any()


def test_deterministic_rule_more_than_64_rejected_siblings_and_repeated_tokens():
    """A root with 100 children (and a node with 20 further down): the deterministic rule replays the rejections at a
    node from one wave's registers up to 64 of them and from LDS beyond; several siblings propose the same token,
    which is taken out of the law once.  Uncorrelated proposals: most walks reject everything at the root."""
    star = np.array([-1] + [0] * 100 + [1] * 20 + [3, 3], dtype=np.int32)
    inp = _batch(29, B=48, T=len(star), V=2048, rule=RULES["det"], temp=1.0, corr=0.0, tree=star)
    inp.token[:, 10] = inp.token[:, 5]            # repeated proposals among the first 64 ...
    inp.token[:, 90] = inp.token[:, 5]            # ... across the boundary ...
    inp.token[:, 95] = inp.token[:, 80]           # ... and beyond it
    got = _run_and_compare(inp)
    assert (got["n_accepted"] == 0).sum() >= 8 and (got["n_accepted"] >= 1).any()
    # the same tree with likelier children: deeper walks, rejections at the 20-child node as well
    inp2 = _batch(30, B=48, T=len(star), V=2048, rule=RULES["det"], temp=1.0, corr=0.0, tree=star, boost=5.0)
    inp2.token[:, 110] = inp2.token[:, 105]
    _run_and_compare(inp2)


def test_root_only_and_chain_trees():
    for rule in ("greedy", "det", "wor"):
        temp = 0.0 if rule == "greedy" else 1.0
        _run_and_compare(_batch(24, B=16, T=1, V=1000, rule=RULES[rule], temp=temp))
        _run_and_compare(_batch(25, B=16, T=12, V=1000, rule=RULES[rule], temp=temp, tree=trees.chain_tree(12)))


def test_identical_draft_and_target_accepts_first_child_chain():
    inp = _batch(26, B=8, T=40, V=2000, rule=RULES["wor"], temp=1.0, corr=1.0)
    assert np.array_equal(inp.draft_logits, inp.target_logits)
    got = _run_and_compare(inp)
    assert np.all(got["final_kind"] == 0)


def test_more_contemplate_rows_than_the_on_chip_table():
    """200 contemplate rows per sequence (the walk kernel keeps the first 128 anchors on chip and reads the rest from
    memory); the first 150 belong to no node, so the selected row, when there is one, lies beyond the table."""
    inp = _batch(71, B=12, T=10, V=500, rule=RULES["det"], temp=1.0, C=200, max_depth=3, boost=4.0)
    inp.con_anchor[:, :150] = -1
    got = _run_and_compare(inp)
    assert (got["selected_con"] >= 150).sum() >= 3 and np.all((got["selected_con"] == -1) | (got["selected_con"] >= 150))


def test_padded_logit_rows():
    inp = _batch(27, B=4, T=20, V=3001, rule=RULES["wor"], temp=1.0)
    _run_and_compare(inp, row_stride=3008)
    _run_and_compare(inp, row_stride=3003)      # rows not 16-byte aligned: scalar loads


def test_bad_trees_and_tokens_are_flagged():
    import paper_2603_08899_amd as tv
    inp = _batch(28, B=4, T=10, V=500, rule=RULES["det"], temp=1.0)
    inp.parent[1, 4] = 6
    inp.token[2, 3] = 500
    inp.parent[3, 0] = 0
    got = H.run_accept(inp)
    assert got["status"][0] == 0 and got["n_accepted"][0] >= 0
    assert got["status"][1] & tv.TV_STATUS_BAD_PARENT
    assert got["status"][2] & tv.TV_STATUS_BAD_TOKEN
    assert got["status"][3] & tv.TV_STATUS_BAD_PARENT
    for b in (1, 2, 3):
        assert got["n_accepted"][b] == -1 and got["final_token"][b] == -1 and np.all(got["path"][b] == -1)
    ref = H.oracle_accept(inp, 0)
    assert got["final_token"][0] == ref["final_token"] and np.array_equal(got["path"][0], ref["path"])


# ---- the named workloads at full size ------------------------------------------------------------------------
@pytest.mark.parametrize("index,mode,corr,boost", [
    (1, 0, 0.0, 0.0), (1, 0, 0.9, 5.0), (2, 0, 0.0, 0.0), (2, 0, 0.0, 5.0), (2, 1, 0.0, 0.0), (2, 1, 0.0, 5.0),
    (4, 0, 0.0, 0.0), (4, 0, 0.9, 5.0)])
def test_full_vocabulary_single_sequence(index, mode, corr, boost):
    """V = 128256 (Llama-3) and 151936 (Qwen-3), T = 60; plain recipe and the longer-walk variant."""
    got = _run_and_compare(si.accept_case(index, mode, draft_target_corr=corr, child_boost=boost))
    print("accepted", int(got["n_accepted"][0]))


def test_full_vocabulary_batch_of_eight():
    _run_and_compare(si.accept_case(3, 0))
    got = _run_and_compare(si.accept_case(3, 0, child_boost=5.0))
    assert got["n_accepted"].max() >= 2


@pytest.mark.parametrize("rule", ["wor", "wr"])
def test_draft_rules_more_nodes_with_children_than_groups(rule):
    """Full vocabulary (32 workgroups per sibling-chain group, so about sixteen groups are resident) and trees
    with far more nodes that have children than that: a 50-node chain (49 such nodes: four passes of the groups,
    the last one short) and two bushy sequences in one call (the passes run over both).  The accepted path of
    the chain goes deep (draft and target laws nearly equal), so the chain kernel's results for late nodes are used."""
    inp = _batch(64, B=1, T=50, V=128256, rule=RULES[rule], temp=1.0, corr=0.9995, tree=trees.chain_tree(50))
    got = _run_and_compare(inp)
    assert int(got["n_accepted"][0]) >= 10
    _run_and_compare(_batch(62, B=2, T=60, V=128256, rule=RULES[rule], temp=1.0, corr=0.9, boost=4.0, max_depth=12,
                            max_children=2))


@pytest.mark.parametrize("rule", ["det", "wor"])
def test_full_vocabulary_more_sequences_than_resident_groups(rule):
    """20 sequences at V = 128256: the final draw takes a group of 128 workgroups per sequence and only about eight
    groups are resident, so the groups go round the sequences several times (fresh hand-off slots each time)."""
    inp = _batch(81, B=20, T=16, V=128256, rule=RULES[rule], temp=1.0, corr=0.9, boost=4.0, max_depth=5, max_children=3)
    got = _run_and_compare(inp)
    assert len(set(got["final_token"].tolist())) > 10


def test_many_uniform_draws_on_one_full_size_tree():
    """One Llama-3-sized tree, 24 different sets of uniforms (as a batch sharing logits by copy)."""
    base = si.accept_case(1, 0, draft_target_corr=0.9, child_boost=4.0)
    B = 6
    rng = np.random.default_rng(3)
    inp = si.AcceptInputs(
        B=B, T=base.T, V=base.V, C=base.C, temperature=base.temperature, rule=base.rule,
        target_logits=np.repeat(base.target_logits, B, axis=0), draft_logits=np.repeat(base.draft_logits, B, axis=0),
        token=np.repeat(base.token, B, axis=0), parent=np.repeat(base.parent, B, axis=0),
        uniforms=rng.random((B, 2 * base.T), dtype=np.float32), con_anchor=np.repeat(base.con_anchor, B, axis=0))
    got = _run_and_compare(inp)
    assert len(set(got["final_token"].tolist())) > 1


@pytest.mark.parametrize("rule", ["wor", "wr"])
def test_wait_limit_of_one_changes_nothing(rule):
    """With a wait limit of one look the workgroups of a sibling-chain group hardly ever see each other's shares in
    time and compute them themselves: the call must return and give the oracle's result all the same (the waits
    between workgroups are a shortcut, not something the result or the kernel's end depends on)."""
    import paper_2603_08899_amd as tv
    inp = si.accept_case(1, 0, draft_target_corr=0.9, child_boost=5.0)
    import dataclasses
    inp = dataclasses.replace(inp, rule=RULES[rule])
    normal = _run_and_compare(inp)
    old = tv.tv_set_wait_limit(1)
    try:
        got = _run_and_compare(inp)
    finally:
        tv.tv_set_wait_limit(old)
    for k in ("status", "n_accepted", "final_token", "final_kind", "last_node", "selected_con", "path"):
        assert np.array_equal(got[k], normal[k]), k
    small = _batch(61, B=40, T=24, V=9001, rule=RULES[rule], temp=0.7, C=2, boost=7.0)
    old = tv.tv_set_wait_limit(1)
    try:
        _run_and_compare(small)
    finally:
        tv.tv_set_wait_limit(old)


@pytest.mark.parametrize("rule", ["det", "wor", "wr", "match", "greedy"])
def test_minus_infinity_logits_have_no_mass(rule):
    """Banned tokens and a padded vocabulary tail: -infinity logits scattered over the rows, a whole trailing range
    of them, and - for a few children - a drafted token whose target logit is -infinity (never accepted under the
    stochastic rules)."""
    temp = 0.0 if rule == "greedy" else 1.0
    inp = _batch(71, B=24, T=24, V=20011, rule=RULES[rule], temp=temp, C=2, boost=7.0)
    rng = np.random.default_rng(72)
    for m in (inp.target_logits, inp.draft_logits):
        if m is None:
            continue
        m[rng.random(m.shape) < 0.05] = -np.inf
        m[:, :, 17000:] = -np.inf                 # the tail: more than one whole range of the statistics pass
        m[:, 3, :9000] = -np.inf                  # a row whose leading ranges are empty
    for b in range(0, inp.B, 3):                  # a child whose token the target bans
        c = 1 + b % (inp.T - 1)
        inp.target_logits[b, inp.parent[b, c], inp.token[b, c]] = -np.inf
    got = _run_and_compare(inp)
    assert np.all(got["final_token"] >= 0) and np.all(got["final_token"] < 17000)


def test_a_row_without_any_mass_gives_no_token():
    """A row that is -infinity throughout has no law (the oracle's softmax is undefined there, so this checks the
    documented behaviour only): children of that node are rejected, a walk that stops there returns token -1, and
    nothing turns into NaN on the way."""
    inp = _batch(73, B=4, T=12, V=6000, rule=RULES["det"], temp=1.0, boost=7.0)
    inp.target_logits[0, 0, :] = -np.inf          # the root's row: the walk cannot leave the root
    got = H.run_accept(inp)
    assert got["status"][0] == 0 and got["n_accepted"][0] == 0 and got["final_token"][0] == -1
    assert got["last_node"][0] == 0 and got["path"][0][0] == 0
    for b in range(1, 4):
        ref = H.oracle_accept(inp, b)
        assert got["final_token"][b] == ref["final_token"] and np.array_equal(got["path"][b], ref["path"])


# ---- the literal sample-and-match reading -----------------------------------------------------------------------
@pytest.mark.parametrize("temp", [1.0, 0.7])
def test_sample_and_match_many_small_sequences(temp):
    inp = _batch(41, B=256, T=24, V=5003, rule=RULES["match"], temp=temp, C=3, boost=7.0)
    inp.draft_logits = None
    got = _run_and_compare(inp)
    assert got["n_accepted"].max() >= 2 and got["n_accepted"].min() <= 2       # walks of different lengths


def test_sample_and_match_full_vocabulary_and_padded_rows():
    import dataclasses
    base = si.accept_case(2, 1, child_boost=5.0)
    inp = dataclasses.replace(base, rule=RULES["match"])
    got = _run_and_compare(inp)
    print("accepted", int(got["n_accepted"][0]))
    small = _batch(42, B=4, T=20, V=3001, rule=RULES["match"], temp=1.0, boost=6.0)
    small.draft_logits = None
    _run_and_compare(small, row_stride=3003)
    # batch of eight at full size
    b8 = dataclasses.replace(si.accept_case(3, 0, child_boost=5.0), rule=RULES["match"])
    _run_and_compare(b8)


# ---- bf16 logits ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rule", ["greedy", "det", "wor", "wr", "match"])
def test_bf16_logits_many_small_sequences(rule):
    """The logits handed over as bf16; the oracle gets the same bf16 values (exact in fp32/fp64).  bf16 logits
    tie often (8 mantissa bits), which exercises the lowest-index rules."""
    temp = 0.0 if rule == "greedy" else 1.0
    inp = H.logits_rounded_to_bf16(_batch(41, B=128, T=24, V=5003, rule=RULES[rule], temp=temp, C=3, boost=7.0))
    got = _run_and_compare(inp, logits_dtype="bf16")
    assert got["n_accepted"].max() >= 2


def test_bf16_logits_padded_and_unaligned_rows():
    inp = H.logits_rounded_to_bf16(_batch(42, B=4, T=20, V=3001, rule=RULES["wor"], temp=0.7))
    _run_and_compare(inp, row_stride=3008, logits_dtype="bf16")
    _run_and_compare(inp, row_stride=3003, logits_dtype="bf16")     # rows not 8-byte aligned: scalar loads
    _run_and_compare(inp, row_stride=3004, logits_dtype="bf16")     # 8-byte but not 16-byte aligned rows


@pytest.mark.parametrize("index,mode,boost", [(2, 0, 5.0), (2, 1, 5.0), (4, 0, 5.0), (1, 0, 0.0)])
def test_bf16_logits_full_vocabulary(index, mode, boost):
    inp = H.logits_rounded_to_bf16(si.accept_case(index, mode, draft_target_corr=0.9 if index != 2 else 0.0,
                                                  child_boost=boost))
    got = _run_and_compare(inp, logits_dtype="bf16")
    print("accepted", int(got["n_accepted"][0]))


# ---- seeded random draws over everything at once ----------------------------------------------------------------
@pytest.mark.parametrize("seed", range(48))
def test_random_configurations(seed):
    """Rule, temperature, batch size, tree size and shape, vocabulary size (any residue mod 8, below and above one
    4096-entry range), contemplate rows, padded logit rows and the logits' type, all drawn together."""
    rng = np.random.default_rng(7000 + seed)
    rule = str(rng.choice(["greedy", "det", "wor", "wr", "match"]))
    temp = 0.0 if rule == "greedy" else float(rng.choice([0.5, 0.7, 1.0, 1.3]))
    B = int(rng.choice([1, 2, 7, 40]))
    T = int(rng.integers(1, 49))
    V = int(rng.choice([int(rng.integers(2, 200)), int(rng.integers(1000, 9000)), int(rng.integers(9000, 40000))]))
    C = int(rng.integers(0, 4))
    dtype = str(rng.choice(["f32", "bf16"]))
    pad = int(rng.choice([0, 0, 1, 3, 8]))
    inp = _batch(7100 + seed, B=B, T=T, V=V, rule=RULES[rule], temp=temp, C=C, corr=float(rng.choice([0.0, 0.9])),
                 boost=float(rng.choice([0.0, 4.0, 8.0])), max_depth=int(rng.integers(6, 13)),
                 max_children=int(rng.integers(2, 9)))
    if rule in ("greedy", "det", "match"):
        inp.draft_logits = None
    if dtype == "bf16":
        inp = H.logits_rounded_to_bf16(inp)
    print(f"[random] seed {seed}: rule={rule} temp={temp} B={B} T={T} V={V} C={C} {dtype} row_stride={V + pad if pad else 0}",
          flush=True)
    _run_and_compare(inp, row_stride=V + pad if pad else 0, logits_dtype=dtype)
