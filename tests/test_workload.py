"""Sanity of the seeded input generators (inputs only; no method arithmetic to pin)."""
import numpy as np
import pytest

import workload as wl


@pytest.mark.parametrize("T,H,k", [(16, 3, 4), (64, 4, 10), (32, 4, 10), (128, 5, 10), (1, 3, 4)])
def test_default_tree_is_a_valid_tree(T, H, k):
    parent, depth, rank = wl.default_tree(T, H, k)
    assert len(parent) == T and parent[0] == -1 and depth[0] == 0
    seen = set()
    for j in range(1, T):
        assert 0 <= parent[j] < j
        assert depth[j] == depth[parent[j]] + 1 <= H
        assert 0 <= rank[j] < k
        assert (parent[j], rank[j]) not in seen       # siblings have distinct ranks
        seen.add((parent[j], rank[j]))
    assert np.all(np.diff(depth) >= 0)                # depth-major numbering


def test_default_tree_is_deterministic_and_greedy_in_score():
    a = wl.default_tree(64, 4, 10)
    b = wl.default_tree(64, 4, 10)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    parent, depth, rank = a
    # the best-scoring path (all ranks 0) must be present down to full depth
    j = 0
    for d in range(1, 5):
        kids = [c for c in range(64) if parent[c] == j and rank[c] == 0]
        assert len(kids) == 1
        j = kids[0]


def test_full_and_chain_trees():
    parent, depth, rank = wl.full_tree(2, 3)
    assert len(parent) == 1 + 3 + 9
    parent, depth, rank = wl.chain_tree(4, rank=1)
    assert list(parent) == [-1, 0, 1, 2] and list(depth) == [0, 1, 2, 3] and list(rank) == [0, 1, 1, 1]


def test_zipf_prompt_shape_and_skew():
    p = wl.zipf_prompt(1024, 20000)
    assert p.dtype == np.int32 and p.min() >= 0 and p.max() < 1024
    counts = np.bincount(p, minlength=1024)
    assert counts[0] > counts[10] > counts[200]
    # P(id=0) = 1 / sum_r (r+1)^-1.1
    p0 = 1.0 / np.sum(np.arange(1, 1025, dtype=np.float64) ** -1.1)
    assert abs(counts[0] / 20000 - p0) < 0.02
    assert np.array_equal(p, wl.zipf_prompt(1024, 20000))


def test_stop_set_count_and_packing():
    m = wl.stop_set(32016, 0.2)
    assert m.sum() == int(0.2 * 32016)
    words = wl.pack_mask_words(m)
    assert words.dtype == np.uint32 and len(words) == (32016 + 31) // 32
    for t in [0, 1, 31, 32, 33, 32015]:
        assert bool((words[t // 32] >> (t % 32)) & 1) == bool(m[t])


def test_round_to_bf16_matches_torch():
    import torch
    a = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(wl.round_to_bf16(a), torch.from_numpy(a).bfloat16().float().numpy())


def test_weights_shapes_and_seeding():
    shape = wl.preset("tiny").model
    w = wl.make_weights(shape)
    assert w["l0.wqkv"].shape == (3 * 256, 256) and w["l1.w_down"].shape == (256, 688)
    assert w["embed"].shape == (1024, 256) and w["medusa2.w"].shape == (256, 256)
    assert float(w["final_norm"].min()) == 1.0
    w2 = wl.make_weights(shape)
    assert all((w[k] == w2[k]).all() for k in w)
    assert abs(float(w["l0.wo"].std()) - 0.02) < 1e-3


def test_plant_drafts_keeps_candidates_distinct():
    rng = np.random.default_rng(0)
    cand = np.arange(12, dtype=np.int32).reshape(3, 4)
    out = wl.plant_drafts(cand, np.array([1, 100, 101]), (1.0, 1.0, 1.0), rng)
    for d, t in enumerate([1, 100, 101]):
        assert t in out[d] and len(set(out[d])) == 4
