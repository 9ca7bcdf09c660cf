"""GPU parity of the other draft-head schedule: heads on every tree row inside the verifying pass
(H * T rows per sequence through the shared LM head in 256-row chunks, the last kept node's rows
ranked afterwards). The oracle is the same step: what a step computes does not depend on the
schedule, so logits, verdict, committed K/V, head logits and next candidates are held to the
same bars as the default schedule, and the two schedules are compared with each other."""
import numpy as np
import pytest
import torch

import workload as wl
from oracle import specdec_oracle as orc
from tests import lockstep
from tests.test_gpu_configs import _run_batch_steps, _shape
from tests.test_gpu_parity import _bf16_shape, _prefill_both, _setup

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()
    return sd


def test_tiny_shape_lockstep_all_nodes(sd):
    """configs[0] shape: 3 heads x 32 rows = 96 head rows, one chunk of four row blocks."""
    shape = _bf16_shape("tiny")
    _, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 64, 256, 16)
    model.set_draft_schedule("all_nodes")
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, 256, rep, 0.0)
    g = orc.prefill(w64, shape, prompt, 256)
    for _ in range(150):
        orc.greedy_step(w64, shape, g)
    truth = g.emitted
    rng = np.random.default_rng(wl.SEEDS["force"])

    def plant(s):
        e = len(s.emitted)
        return wl.plant_drafts(s.cand, np.array(truth[e + 1: e + 1 + shape.n_medusa]), (0.9, 0.8, 0.7), rng)

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 32, "keep_all", plant, rep=rep)
    print(f"\n[tiny/all_nodes] {rep}")
    assert rep.steps == 32 and max(rep.accepted) >= 3
    assert st.emitted == truth[: len(st.emitted)]


@pytest.mark.parametrize("name,B,T,lens,cap", [
    ("7b", 1, 64, [300], 512),                            # 256 head rows: one full chunk
    ("7b-batch8", 8, 32, [64, 100, 150, 200, 260, 300, 350, 400], 512),   # 1024 head rows
    ("13b", 1, 129, [300], 512),                         # 5 x 160 = 800 rows: three chunks of 256 and one of 32
    ("7b-h10", 1, 200, [200], 512),                      # 10 x 224 = 2240 rows: eight chunks of 256 and one of 192
])
def test_all_nodes_schedule_matches_oracle(sd, name, B, T, lens, cap):
    shape = _shape(name)
    rep = _run_batch_steps(sd, shape, B, T, lens, cap, n_steps=2, schedule="all_nodes")
    print(f"\n[{name} all_nodes] {rep}")
    assert rep.steps == 2


def test_two_schedules_agree(sd):
    """Same model, two caches, eight steps each way from the same prompt: identical emitted tokens
    and verdicts; head logits equal to summation order; candidates equal unless a near-tie."""
    shape = _bf16_shape("7b", 2)
    _, weights, w64, model, kv_a, prompt, stop, words, tree_np, tree = _setup(sd, shape, 100, 256, 64)
    kv_b = sd.KVCache(model, 1, 256)
    toks = torch.from_numpy(prompt).cuda()
    sd.prefill(model, kv_a, toks, [len(prompt)])
    sd.prefill(model, kv_b, toks, [len(prompt)])
    worst = 0.0
    for step in range(8):
        model.set_draft_schedule("after_accept")
        a = sd.spec_step(model, kv_a, tree, words, want_head_logits=True)
        model.set_draft_schedule("all_nodes")
        b = sd.spec_step(model, kv_b, tree, words, want_head_logits=True)
        torch.cuda.synchronize()
        assert torch.equal(a.n_accept, b.n_accept) and torch.equal(a.tokens, b.tokens)
        assert torch.equal(a.src_slots, b.src_slots)
        ha, hb = a.head_logits.double().cpu().numpy(), b.head_logits.double().cpu().numpy()
        worst = max(worst, float(np.abs(ha - hb).max()))
        ra, ca = kv_a.get_draft()
        rb, cb = kv_b.get_draft()
        assert torch.equal(ra, rb)
        ca, cb = ca.cpu().numpy(), cb.cpu().numpy()
        for i in range(shape.n_medusa):
            if not np.array_equal(ca[0, i], cb[0, i]):
                # only a swap of two candidates whose logits are within the summation-order error
                diff = np.nonzero(ca[0, i] != cb[0, i])[0]
                assert np.abs(ha[0, i, ca[0, i, diff]] - ha[0, i, cb[0, i, diff]]).max() <= 1e-3
                kv_b.set_draft(ra.cpu().numpy(), ca)       # keep the two runs on the same candidates
    print(f"\n[schedules] head logits differ by at most {worst:.3g}")
    assert worst <= 1e-3
    assert kv_a.len() == kv_b.len()


def test_unknown_schedule_is_refused(sd):
    shape = _bf16_shape("tiny")
    _, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 8, 64, 16)
    assert sd.lib().sd_set_draft_schedule(model.handle, 7) != 0
    assert b"unknown schedule" in sd.lib().sd_last_error()
    assert sd.lib().sd_set_draft_schedule(None, 0) != 0
