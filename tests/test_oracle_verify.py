"""Pins for the oracle's tree assembly, greedy acceptance and fragment cut.

Against: hand-worked cases (tests/golden/verify_cases.json), a brute-force enumeration of
root-to-node paths written independently of the parent-pointer scan, and structural
invariants of the rule in Section III-B (prefix-closed acceptance, cut inside the run).
"""
import json
import os

import numpy as np
import pytest

import workload as wl
from oracle import specdec_oracle as orc

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "verify_cases.json")))


@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: c["name"][:40])
def test_hand_worked_cases(case):
    t = GOLD["tree"]
    parent, depth = np.array(t["parent"]), np.array(t["depth"])
    tok, am = np.array(case["tok"]), np.array(case["am"])
    stop = np.zeros(128, bool)
    stop[case["stop"]] = True
    ok, chain = orc.greedy_accept(tok, am, parent, depth)
    assert chain == case["chain"]
    assert orc.fragment_cut([tok[c] for c in chain], stop, case["fallback"]) == case["n_accept"]


def _paths(parent):
    out = []
    for j in range(len(parent)):
        p, i = [], j
        while i >= 0:
            p.append(i)
            i = parent[i]
        out.append(p[::-1])
    return out


def _brute_force(tok, am, parent, stop, fallback):
    """Walk every root-to-node path token by token; keep the longest accepted prefix."""
    best = [0]
    for path in _paths(parent):
        acc = [path[0]]
        for a, b in zip(path[:-1], path[1:]):
            if tok[b] != am[a]:
                break
            acc.append(b)
        if len(acc) > len(best) or (len(acc) == len(best) and acc[-1] < best[-1]):
            best = acc
    toks = [tok[c] for c in best]
    stops = [j for j, t in enumerate(toks) if stop[t]]
    if stops:
        n = stops[-1] + 1
    else:
        n = len(best) if fallback == "keep_all" else 1
    return best, n


@pytest.mark.parametrize("seed", range(40))
def test_acceptance_equals_brute_force_over_paths(seed):
    rng = np.random.default_rng(seed)
    H, k = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    maxT = sum(k ** d for d in range(H + 1))
    T = int(rng.integers(1, min(maxT, 40) + 1))
    parent, depth, rank = wl.default_tree(T, H, k) if seed % 2 else wl.full_tree(min(H, 3), min(k, 3))
    T = len(parent)
    V = 6                                              # tiny vocabulary: matches are frequent
    root = int(rng.integers(V))
    cand = np.stack([rng.permutation(V)[:k] for _ in range(H)]) if seed % 2 else \
        np.stack([rng.permutation(V)[:3] for _ in range(3)])
    tok, pos, anc = orc.tree_inputs(root, cand, parent, depth, rank, n=17)
    am = rng.integers(V, size=T)
    stop = rng.random(V) < 0.3
    fallback = "keep_all" if seed % 3 else "keep_one"
    ok, chain = orc.greedy_accept(tok, am, parent, depth)
    n_acc = orc.fragment_cut([tok[c] for c in chain], stop, fallback)
    want_chain, want_n = _brute_force(tok, am, parent, stop, fallback)
    assert chain == want_chain and n_acc == want_n
    # structure: acceptance is prefix closed; one chain; the cut stays inside the run
    for j in range(1, T):
        if ok[j]:
            assert ok[parent[j]]
    for d in range(1, H + 1):
        assert sum(1 for j in range(T) if ok[j] and depth[j] == d) <= 1
    assert 1 <= n_acc <= len(chain) <= H + 1
    if any(stop[tok[c]] for c in chain):
        assert stop[tok[chain[n_acc - 1]]]
    assert orc.fragment_cut([tok[c] for c in chain], np.ones(V, bool), "keep_one") == len(chain)
    assert orc.fragment_cut([tok[c] for c in chain], np.zeros(V, bool), "keep_one") == 1
    assert orc.fragment_cut([tok[c] for c in chain], np.zeros(V, bool), "keep_all") == len(chain)


def test_tree_inputs_tokens_positions_and_ancestor_mask():
    parent, depth, rank = wl.default_tree(16, 3, 4)
    cand = np.arange(100, 112).reshape(3, 4)
    tok, pos, anc = orc.tree_inputs(7, cand, parent, depth, rank, n=50)
    assert tok[0] == 7 and pos[0] == 50
    for j in range(1, 16):
        assert tok[j] == 100 + 4 * (depth[j] - 1) + rank[j]      # head depth-1, rank r
        assert pos[j] == 50 + depth[j]
        assert anc[j].sum() == depth[j] + 1 and anc[j, j] and anc[j, 0] and anc[j, parent[j]]
        assert not anc[j, j + 1:].any()                          # depth-major => lower triangular
    # the mask is exactly the reflexive-transitive closure of `parent`
    for j, path in enumerate(_paths(parent)):
        assert sorted(np.nonzero(anc[j])[0]) == path
