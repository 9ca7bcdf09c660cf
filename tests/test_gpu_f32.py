"""The float32 device path (dtype "f32": weights, activations and the KV cache in float32) against the oracle.

configs[0] is specified in float32. The comparison is the same lock-step one as for the bf16 path; on top of
the common bounds the float32 path must be far inside them: it differs from the float64 oracle only by float32
rounding of sums of a few hundred to a few thousand terms, so logits, draft-head logits and committed K/V rows are
held to 2e-5 here (measured: 1.3e-6), a thousandth of the bound the bf16 path is given."""
import numpy as np
import pytest
import torch

import workload as wl
from oracle import specdec_oracle as orc
from tests import lockstep
from tests.test_gpu_configs import _run_batch_steps

pytestmark = pytest.mark.gpu

F32_MAX_ABS = 2e-5


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()
    return sd


def _tight(rep):
    assert rep.max_abs <= F32_MAX_ABS and rep.kv_max_abs <= F32_MAX_ABS and rep.head_max_abs <= F32_MAX_ABS, rep


@pytest.mark.parametrize("fallback", ["keep_all", "keep_one"])
def test_tiny_config_in_float32_lockstep(sd, fallback):
    """configs[0] as specified: prefill of 64 tokens (two 32-row chunks), then 32 speculative steps on planted drafts."""
    shape = wl.preset("tiny").model
    assert shape.dtype == "f32"
    weights = wl.make_weights(shape, medusa_bias_std=0.02)
    w64 = lockstep.weights_to_f64(weights)
    model = sd.Model(shape, {k: v.cuda() for k, v in weights.items()}, 32, fallback)
    kv = sd.KVCache(model, 1, 256)
    prompt = wl.zipf_prompt(shape.vocab, 64)
    stop = wl.stop_set(shape.vocab, 0.2)
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(16, shape.n_medusa, shape.topk)
    tree = sd.Tree(*tree_np, shape.n_medusa, shape.topk)
    rep = lockstep.Report()
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [len(prompt)])
    st = orc.prefill(w64, shape, prompt, 256)
    assert kv.len() == [64]
    lockstep.compare_kv_rows(kv, st, shape, 0, 64, rep)
    root, cand = kv.get_draft()
    assert int(root[0]) == st.root_tok
    g = orc.prefill(w64, shape, prompt, 256)
    for _ in range(150):
        orc.greedy_step(w64, shape, g)
    truth = g.emitted
    rng = np.random.default_rng(wl.SEEDS["force"])

    def plant(s):
        e = len(s.emitted)
        return wl.plant_drafts(s.cand, np.array(truth[e + 1: e + 1 + shape.n_medusa]), (0.9, 0.8, 0.7), rng)

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 32, fallback, plant, rep=rep)
    print(f"\n[tiny f32/{fallback}] {rep}")
    assert rep.steps == 32 and max(rep.accepted) >= 3
    assert st.emitted == truth[: len(st.emitted)]
    _tight(rep)
    # plain greedy steps continue the same stream
    for _ in range(3):
        want = orc.greedy_step(w64, shape, st)
        out = sd.greedy_step(model, kv, want_logits=True)
        assert int(out.tokens[0, 0]) == want.tokens[0]
    assert kv.len() == [st.kv.n]


def test_float32_batch_of_three_ragged(sd):
    """Three sequences of different lengths over a synthetic float32 cache: every accepted depth, a forced
    mid-chain cut, a 64-node tree (two 32-row blocks per sequence)."""
    shape = wl.preset("tiny").model
    rep = _run_batch_steps(sd, shape, 3, 64, [45, 70, 33], 128, n_steps=4)
    print(f"\n[tiny f32 batch] {rep}")
    assert rep.mid_cuts >= 1 and len(set(rep.accepted)) >= 3
    _tight(rep)


def test_float32_cache_rows_round_trip_and_commit_stage(sd):
    """Rows written are the rows read back, bit for bit; the commit stage alone copies tree rows bit for bit."""
    shape = wl.preset("tiny").model
    weights = wl.make_weights(shape)
    model = sd.Model(shape, {k: v.cuda() for k, v in weights.items()}, 64)
    kv = sd.KVCache(model, 2, 96)
    k = wl.synthetic_kv_rows(5, "k", (40, shape.n_heads, shape.head_dim), "f32").cuda()
    v = wl.synthetic_kv_rows(5, "v", (40, shape.n_heads, shape.head_dim), "f32").cuda()
    kv.write_rows(1, 1, 7, k, v)
    k2, v2 = kv.read_rows(1, 1, 7, 40)
    assert torch.equal(k, k2) and torch.equal(v, v2)
    k0, _ = kv.read_rows(0, 1, 7, 40)
    assert not k0.any()                                    # other layers untouched (the cache starts as zeros)
    kv.set_len([10, 20])
    tree_np = wl.default_tree(16, shape.n_medusa, shape.topk)
    tree = sd.Tree(*tree_np, shape.n_medusa, shape.topk)
    words = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    kv.set_draft([1, 2], np.zeros((2, shape.n_medusa, shape.topk), np.int32) + np.arange(shape.topk, dtype=np.int32))
    sd.spec_step(model, kv, tree, words)
    lens = kv.len()
    # single-row commits give the reference rows; then the same slots as one call of three rows
    slots = torch.tensor([[3, 0, 9], [5, 5, 1]], dtype=torch.int32, device="cuda")
    ref = []
    for j in range(3):
        kv.set_len(lens)
        sd.kv_commit_rows(model, kv, slots[:, j:j + 1].contiguous(), torch.ones(2, dtype=torch.int32, device="cuda"))
        ref.append([[kv.read_rows(l, b, lens[b], 1) for l in range(shape.n_layers)] for b in range(2)])
    kv.set_len(lens)
    sd.kv_commit_rows(model, kv, slots, torch.tensor([3, 2], dtype=torch.int32, device="cuda"))
    assert kv.len() == [lens[0] + 3, lens[1] + 2]
    for b, n in enumerate([3, 2]):
        for l in range(shape.n_layers):
            kk, vv = kv.read_rows(l, b, lens[b], n)
            for j in range(n):
                assert torch.equal(kk[j], ref[j][b][l][0][0]) and torch.equal(vv[j], ref[j][b][l][1][0])


def test_float32_model_refuses_bfloat16_weights(sd):
    shape = wl.preset("tiny").model
    weights = wl.make_weights(shape)
    with pytest.raises(ValueError):
        sd.Model(shape, {k: v.bfloat16().cuda() for k, v in weights.items()}, 32)


def test_float32_sampling_decoding_lockstep(sd):
    """Typical acceptance and a sampled next root on the float32 path (peaked distributions: temperature 0.04)."""
    from tests.test_gpu_typical import TY, _plant_greedy_continuation, _setup
    shape = wl.preset("tiny").model
    w64, model, kv, stop, words, tree_np, tree, st = _setup(sd, shape, 64, 320, 16, "keep_all")
    rng = np.random.default_rng(wl.SEEDS["force"])
    plant = _plant_greedy_continuation(w64, shape, (0.9, 0.8, 0.7), np.random.default_rng(1))
    rep = lockstep.lockstep_typical(model, kv, tree, tree_np, stop, words, w64, shape, st, 24, "keep_all",
                                    dict(TY, temperature=0.04), rng, cand_fn=plant)
    print(f"\n[tiny f32 typical] {rep}")
    assert rep.steps == 24 and len(set(rep.raw)) > 2
    assert rep.accept_near_ties <= 1 and rep.root_near_ties <= 1
    assert rep.max_abs <= F32_MAX_ABS
