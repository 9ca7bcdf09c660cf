"""The entry point that allocates nothing: sd_verify_tree_typical_static against sd_verify_tree_typical.

Two calls in a row through the C ABI, the second on a smaller input (fewer sequences, a smaller tree), each
compared bit for bit with the existing entry point on the same inputs: the outputs are integers decided by the
same kernels, so they must be identical. The static statistics buffer keeps the first call's contents; the
second call must not see them. Also: the size limit is refused with SD_ERR_SHAPE before anything is enqueued,
and torch's allocator is not called between the two sides' launches (the outputs are made beforehand)."""
import numpy as np
import pytest
import torch

import workload as wl

pytestmark = pytest.mark.gpu

TY = dict(temperature=0.8, epsilon=0.09, delta=0.3)


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()
    return sd


def _case(rng, T, H, k, V, batch):
    parent, depth, rank = wl.default_tree(T, H, k)
    stop = rng.random(V) < 0.3
    scale = rng.choice([0.05, 1.0, 3.0, 8.0], size=(batch * T, 1))
    logits = (rng.standard_normal((batch * T, V)) * scale).astype(np.float32).reshape(batch, T, V)
    tok = rng.integers(V, size=(batch, T)).astype(np.int32)
    for b in range(batch):                                   # likely tokens, so that accepted chains grow
        for j in range(1, T):
            if rng.random() < 0.7:
                tok[b, j] = int(np.argmax(logits[b, parent[j]]))
    return (parent, depth, rank), stop, logits, tok


def test_static_entry_point_matches_the_allocating_one_twice_in_a_row(sd):
    rng = np.random.default_rng(2024)
    seen = []
    for T, H, k, V, batch in [(64, 4, 10, 3000, 48), (16, 3, 4, 257, 5)]:       # the second call is the smaller one
        tree_np, stop, logits, tok = _case(rng, T, H, k, V, batch)
        tree = sd.Tree(*tree_np, H, k)
        words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
        tok_d, logits_d = torch.from_numpy(tok).cuda(), torch.from_numpy(logits).cuda()
        i32 = dict(dtype=torch.int32, device="cuda")
        out = (torch.full((batch,), -7, **i32), torch.full((batch,), -7, **i32),
               torch.full((batch, H + 1), -7, **i32), torch.full((batch, H + 1), -7, **i32))
        want = sd.verify_tree_typical(tree, tok_d, logits_d, words, **TY)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
        sd.verify_tree_typical_static(tree, tok_d, logits_d, words, out, **TY)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
        for got, ref, name in zip(out, want[:4], ("n_accept", "n_accept_raw", "tokens", "src_slots")):
            assert torch.equal(got, ref), f"{name} differs (T={T}, batch={batch})"
        seen.append(sorted(set(out[1].cpu().tolist())))
    assert len(seen[0]) > 2                                   # accepted runs of several lengths were decided


def test_static_entry_point_refuses_sizes_beyond_its_buffer(sd):
    T, H, k, V = 64, 4, 10, 100
    tree = sd.Tree(*wl.default_tree(T, H, k), H, k)
    batch = 4096 // T + 1
    i32 = dict(dtype=torch.int32, device="cuda")
    out = (torch.full((batch,), -7, **i32), torch.full((batch,), -7, **i32),
           torch.full((batch, H + 1), -7, **i32), torch.full((batch, H + 1), -7, **i32))
    tok = torch.zeros((batch, T), **i32)
    logits = torch.zeros((batch, T, V), dtype=torch.float32, device="cuda")
    words = torch.zeros((V + 31) // 32, **i32)
    with pytest.raises(sd.SpecDecError) as e:
        sd.verify_tree_typical_static(tree, tok, logits, words, out, **TY)
    assert e.value.name == "SD_ERR_SHAPE" and "4096" in str(e.value)
    torch.cuda.synchronize()
    assert all(int(t.min()) == -7 and int(t.max()) == -7 for t in out)      # nothing was enqueued
