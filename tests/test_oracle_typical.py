"""Pins for the oracle's sampling-decoding pieces: softmax at a temperature, entropy, the
typical-acceptance inequality (Section III-B, Eq. 1) and the inverse-CDF draw of the next root.

Against: hand-worked cases (tests/golden/typical_cases.json), SciPy's softmax and entropy,
closed forms (uniform and two-point distributions), a brute-force enumeration of root-to-node
paths that tests every prefix directly, the zero-temperature limit (which must reproduce greedy
acceptance), NumPy's searchsorted on the cumulative sum, and structural invariants.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

import workload as wl
from oracle import specdec_oracle as orc

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "typical_cases.json")))


@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: c["name"][:40])
def test_hand_worked_cases(case):
    t = GOLD["tree"]
    parent, depth = np.array(t["parent"]), np.array(t["depth"])
    logits = np.log(np.array(case["weights"], float))
    tok = np.array(case["tok"])
    tau, eps, delta = case["temperature"], case["epsilon"], case["delta"]
    p0 = orc.softmax_t(logits[0], tau)
    assert orc.entropy(p0) == pytest.approx(case["entropy_at_node0"], abs=2e-6)
    assert orc.typical_threshold(p0, eps, delta) == pytest.approx(case["threshold_at_node0"], abs=2e-6)
    ok, chain, _ = orc.typical_accept(tok, logits, parent, depth, tau, eps, delta)
    assert list(ok) == case["ok"] and chain == case["chain"]
    stop = np.zeros(4, bool)
    stop[case["stop"]] = True
    n_acc = orc.fragment_cut([tok[c] for c in chain], stop, case["fallback"])
    assert n_acc == case["n_accept"]
    last = chain[n_acc - 1]
    assert orc.sample_token(orc.softmax_t(logits[last], tau), case["u"]) == case["next_root"]


@pytest.mark.parametrize("tau", [0.2, 0.8, 1.0, 2.5])
def test_softmax_and_entropy_match_scipy(tau):
    rng = np.random.default_rng(11)
    for V in (2, 7, 1000):
        lg = rng.normal(size=V) * 4
        p = orc.softmax_t(lg, tau)
        np.testing.assert_allclose(p, scipy.special.softmax(lg / tau), rtol=1e-12, atol=0)
        assert p.sum() == pytest.approx(1.0, abs=1e-12)
        assert orc.entropy(p) == pytest.approx(scipy.stats.entropy(p), rel=1e-12)


def test_entropy_and_threshold_closed_forms():
    for V in (1, 2, 10, 4096):
        p = np.full(V, 1.0 / V)
        assert orc.entropy(p) == pytest.approx(math.log(V), abs=1e-12)
        # uniform: exp(-H) = 1/V, so the threshold is min(eps, delta / V)
        assert orc.typical_threshold(p, 0.09, 0.3) == pytest.approx(min(0.09, 0.3 / V), rel=1e-12)
    onehot = np.zeros(9)
    onehot[4] = 1.0
    assert orc.entropy(onehot) == 0.0 and orc.typical_threshold(onehot, 0.09, 0.3) == pytest.approx(0.09)
    a = 0.3
    two = np.array([a, 1 - a])
    assert orc.entropy(two) == pytest.approx(-a * math.log(a) - (1 - a) * math.log(1 - a), rel=1e-14)


def _paths(parent):
    out = []
    for j in range(len(parent)):
        p, i = [], j
        while i >= 0:
            p.append(i)
            i = parent[i]
        out.append(p[::-1])
    return out


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_over_paths(seed):
    """Every root-to-node path, every prefix, tested with SciPy's probabilities directly."""
    rng = np.random.default_rng(seed)
    H, k, V, T = 3, 4, 12, 16
    tree = wl.default_tree(T, H, k)
    parent, depth, rank = (np.asarray(a) for a in tree)
    logits = rng.normal(size=(T, V)) * 2
    cand = np.stack([rng.permutation(V)[:k] for _ in range(H)])
    tok = np.array([rng.integers(V)] + [cand[depth[j] - 1][rank[j]] for j in range(1, T)])
    tau, eps, delta = 0.8, 0.25, 0.9
    ok, chain, _ = orc.typical_accept(tok, logits, parent, depth, tau, eps, delta)
    best_len, best_path = 0, None
    for path in _paths(parent):
        good = True
        for a, c in zip(path[:-1], path[1:]):
            p = scipy.special.softmax(logits[a] / tau)
            thr = min(eps, delta * math.exp(-scipy.stats.entropy(p)))
            good = good and p[tok[c]] > thr
        assert bool(ok[path[-1]]) == good
        if good and len(path) > best_len:             # strict: the first (lowest index) longest path wins
            best_len, best_path = len(path), path
    assert chain == best_path


@pytest.mark.parametrize("seed", range(4))
def test_zero_temperature_limit_is_greedy_acceptance(seed):
    """As the temperature goes to 0 the base distribution collapses onto its arg-max: the entropy
    goes to 0, the threshold to min(eps, delta) < 1, and only the arg-max token keeps probability
    ~1. Typical acceptance must then select exactly what greedy acceptance selects."""
    rng = np.random.default_rng(100 + seed)
    H, k, V, T = 4, 5, 50, 32
    parent, depth, rank = (np.asarray(a) for a in wl.default_tree(T, H, k))
    logits = rng.normal(size=(T, V))
    am = orc.argmax_lowest(logits)
    # plant the arg-max continuation on some nodes so that several paths are accepted
    tok = rng.integers(V, size=T)
    for j in range(1, T):
        if rng.random() < 0.6:
            tok[j] = am[parent[j]]
    ok_g, chain_g = orc.greedy_accept(tok, am, parent, depth)
    ok_t, chain_t, _ = orc.typical_accept(tok, logits, parent, depth, 1e-3, 0.3, 0.6)
    assert list(ok_t) == list(ok_g) and chain_t == chain_g


def test_threshold_extremes():
    rng = np.random.default_rng(5)
    H, k, V, T = 3, 4, 20, 16
    parent, depth, rank = (np.asarray(a) for a in wl.default_tree(T, H, k))
    logits = rng.normal(size=(T, V))
    tok = rng.integers(V, size=T)
    ok, chain, _ = orc.typical_accept(tok, logits, parent, depth, 1.0, 0.0, 0.0)      # threshold 0: all pass
    assert ok.all() and depth[chain[-1]] == depth.max() and chain[-1] == int(np.argmax(depth == depth.max()))
    ok, chain, _ = orc.typical_accept(tok, logits, parent, depth, 1.0, 1.0, 1e9)      # threshold 1: none can
    assert list(ok) == [True] + [False] * (T - 1) and chain == [0]
    # prefix closure and chain validity for a mid threshold
    ok, chain, lm = orc.typical_accept(tok, logits, parent, depth, 0.8, 0.05, 0.3)
    for j in range(1, T):
        assert not ok[j] or ok[parent[j]]
        assert (lm[j] > 0) == bool(ok[j]) or not ok[parent[j]]
    assert chain[0] == 0 and all(parent[c] == a for a, c in zip(chain[:-1], chain[1:]))


def test_sample_token_is_the_inverse_cdf():
    rng = np.random.default_rng(9)
    for V in (1, 3, 17, 500):
        p = orc.softmax_t(rng.normal(size=V) * 3, 0.8)
        cdf = np.cumsum(p)
        for u in list(rng.random(200)) + [0.0, 0.5, 1.0 - 2**-40]:
            want = min(int(np.searchsorted(cdf, u, side="right")), V - 1)
            assert orc.sample_token(p, u) == want
    # frequencies on a grid of u reproduce the probabilities
    p = np.array([0.5, 0.0, 0.3, 0.2])
    n = 10000
    draws = np.bincount([orc.sample_token(p, (i + 0.5) / n) for i in range(n)], minlength=4)
    np.testing.assert_allclose(draws / n, p, atol=1.5 / n)
    assert orc.sample_token(p, 0.999999999) == 3 and orc.sample_token(np.array([0.0, 1.0, 0.0]), 0.999) == 1


def test_typical_step_commits_and_draws(tmp_path):
    """spec_step in sampling mode on the tiny model: the step is the greedy step's forward plus
    Eq. 1 and a draw; with epsilon = delta = 0 every drafted token passes, so the kept run is the
    rank-0 path of the tree cut by the stop rule, and the next root is the draw at its last node."""
    shape = wl.preset("tiny").model
    weights = {k: v.double().numpy() for k, v in wl.make_weights(shape).items()}
    prompt = wl.zipf_prompt(shape.vocab, 24)
    st = orc.prefill(weights, shape, prompt, 128)
    tree = wl.default_tree(16, shape.n_medusa, shape.topk)
    stop = wl.stop_set(shape.vocab, 0.2)
    typ = dict(temperature=0.8, epsilon=0.0, delta=0.0, u=0.37)
    n0 = st.kv.n
    rec = orc.spec_step(weights, shape, st, tree, stop, "keep_all", typical=typ)
    depth = np.asarray(tree[1])
    assert rec.ok.all() and rec.n_accept_raw == depth.max() + 1
    assert st.kv.n == n0 + rec.n_accept and 1 <= rec.n_accept <= rec.n_accept_raw
    last = rec.src_slots[-1]
    assert rec.next_root == orc.sample_token(orc.softmax_t(rec.logits[last], 0.8), 0.37)
    assert st.root_tok == rec.next_root
