"""The commit of accepted key/value rows alone (sd_kv_commit_rows): a pure copy, so everything is bit-exact.

Reference: what a row of the tree scratch holds is read by committing that one row alone and reading it back in
natural layout; a list of rows committed at once must then give exactly those rows, in list order, at the rows after
the old length, for every layer, head and sequence, whatever the alignment of the old length inside the cache's
32-row blocks and 4-row value groups, and must leave every row before the old length untouched. The rows' values
themselves are checked against the oracle by the lock-step tests (tests/lockstep.py: compare_kv_rows)."""
import dataclasses

import numpy as np
import pytest
import torch

import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()
    return sd


def _rows(kv, shape, b, row0, n):
    return [tuple(t.clone() for t in kv.read_rows(layer, b, row0, n)) for layer in range(shape.n_layers)]


@pytest.mark.parametrize("name,T", [("tiny", 16), ("7b", 64), ("7b-h10", 256)])
def test_commit_stage_moves_rows_bit_exactly(sd, name, T):
    """Lists of 1 to Tp rows: short ones (what a step commits), every row of the scratch (value pieces replaced
    whole), and, with the 256-row scratch at head_dim 128, lists too long for the kernel's copy of the scratch in LDS
    (it then gathers from global memory)."""
    shape = dataclasses.replace(wl.preset(name, 2).model, dtype="bf16")
    Tp = (T + 31) // 32 * 32
    B, cap = (2 if Tp < 256 else 1), 160 + Tp            # (a pass takes at most 256 rows)
    weights = wl.make_weights(shape, device="cuda")
    model = sd.Model(shape, weights, B * Tp)
    kv = sd.KVCache(model, B, cap)
    rng = np.random.default_rng(12)
    lens0 = [37, 50][:B]
    for b, n in enumerate(lens0):
        for layer in range(shape.n_layers):
            k = wl.synthetic_kv_rows(wl.SEEDS["kvfill"], f"k{b}.{layer}", (cap, shape.n_heads, shape.head_dim), "bf16").cuda()
            v = wl.synthetic_kv_rows(wl.SEEDS["kvfill"], f"v{b}.{layer}", (cap, shape.n_heads, shape.head_dim), "bf16").cuda()
            kv.write_rows(layer, b, 0, k, v)           # the whole cache holds known rows, past the lengths too
    kv.set_len(lens0)
    with pytest.raises(sd.SpecDecError) as e:           # nothing has computed tree rows for this batch yet
        sd.kv_commit_rows(model, kv, torch.zeros((B, 1), dtype=torch.int32, device="cuda"),
                          torch.ones(B, dtype=torch.int32, device="cuda"))
    assert e.value.name == "SD_ERR_STATE"
    tree = sd.Tree(*wl.default_tree(T, shape.n_medusa, shape.topk), shape.n_medusa, shape.topk)
    words = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    roots = rng.integers(shape.vocab, size=B).astype(np.int32)
    cand = np.stack([np.stack([rng.permutation(shape.vocab)[: shape.topk] for _ in range(shape.n_medusa)])
                     for _ in range(B)]).astype(np.int32)
    kv.set_draft(roots, cand)
    sd.spec_step(model, kv, tree, words)                 # leaves the tree's K/V rows of both sequences in the scratch
    torch.cuda.synchronize()
    # what every tree row holds: commit it alone, read it back
    ref = [[None] * T for _ in range(B)]
    one = torch.ones(B, dtype=torch.int32, device="cuda")
    for c in range(T):
        kv.set_len(lens0)
        sd.kv_commit_rows(model, kv, torch.full((B, 1), c, dtype=torch.int32, device="cuda"), one)
        assert kv.len() == [n + 1 for n in lens0]
        for b in range(B):
            ref[b][c] = _rows(kv, shape, b, lens0[b], 1)
    assert any(not torch.equal(ref[0][0][0][0], ref[0][c][0][0]) for c in range(1, T))     # the rows do differ
    # lists of rows, at old lengths of every alignment (value groups of 4 rows, blocks of 32)
    cases = [(lens, Tp if i in (1, 5) else min(Tp, 40) if i == 3 else int(rng.integers(1, min(Tp, 24) + 1)))
             for i, lens in enumerate(([37, 50], [40, 63], [64, 31], [1, 127], [95, 98], [48, 16]))]
    # many more old lengths (every alignment in a 16-row half) and list lengths of 1 .. Tp rows
    cases += [([int(x) for x in rng.integers(1, 121, size=2)], int(rng.integers(1, Tp + 1))) for _ in range(80)]
    for lens, W in cases:
        lens = lens[:B]
        slots = rng.integers(T, size=(B, W)).astype(np.int32)
        n_rows = np.array([W, int(rng.integers(0, W + 1))][:B], np.int32)
        kv.set_len(lens)
        before = [_rows(kv, shape, b, max(lens[b] - 9, 0), min(9, lens[b])) for b in range(B)]
        after_keep = [_rows(kv, shape, b, lens[b] + int(n_rows[b]), 5) for b in range(B)]
        sd.kv_commit_rows(model, kv, torch.from_numpy(slots).cuda(), torch.from_numpy(n_rows).cuda())
        assert kv.len() == [lens[b] + int(n_rows[b]) for b in range(B)]
        for b in range(B):
            got = _rows(kv, shape, b, lens[b], int(n_rows[b])) if n_rows[b] else []
            for layer in range(shape.n_layers):
                for j in range(int(n_rows[b])):
                    want_k, want_v = ref[b][slots[b, j]][layer]
                    assert torch.equal(got[layer][0][j], want_k[0]) and torch.equal(got[layer][1][j], want_v[0]), \
                        f"lens {lens}, sequence {b}, layer {layer}, row {j} (tree row {slots[b, j]})"
            now = _rows(kv, shape, b, max(lens[b] - 9, 0), min(9, lens[b]))
            for (k0, v0), (k1, v1) in zip(before[b], now):
                assert torch.equal(k0, k1) and torch.equal(v0, v1), "rows before the old length changed"
            # rows past the new length inside the same 4-row value group may be anything; beyond that group: untouched
            past = _rows(kv, shape, b, lens[b] + int(n_rows[b]), 5)
            for (k0, v0), (k1, v1) in zip(after_keep[b], past):
                assert torch.equal(k0, k1), "key rows past the new length changed"
                assert torch.equal(v0[4:], v1[4:]), "value rows beyond the last written group changed"
    with pytest.raises(sd.SpecDecError) as e:
        sd.kv_commit_rows(model, kv, torch.zeros((B, Tp + 1), dtype=torch.int32, device="cuda"), one)
    assert e.value.name == "SD_ERR_SHAPE"
    kv.set_len([cap - 3, 10][:B])
    with pytest.raises(sd.SpecDecError) as e:
        sd.kv_commit_rows(model, kv, torch.zeros((B, 4), dtype=torch.int32, device="cuda"), one)
    assert e.value.name == "SD_ERR_KV_FULL" and kv.len() == [cap - 3, 10][:B]
