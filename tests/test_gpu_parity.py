"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

import workload as wl
from oracle import specdec_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()                       # fails loudly if the library has not been built
    return sd


def _bf16_shape(name, n_layers=None):
    import dataclasses
    w = wl.preset(name, n_layers)
    return dataclasses.replace(w.model, dtype="bf16")


def _paths(parent):
    out = []
    for j in range(len(parent)):
        p, i = [], j
        while i >= 0:
            p.append(i)
            i = parent[i]
        out.append(p[::-1])
    return out


# ----------------------------------------------------------------------------- verify kernel
@pytest.mark.parametrize("T,H,k,fallback", [(16, 3, 4, "keep_all"), (64, 4, 10, "keep_all"), (64, 4, 10, "keep_one"),
                                            (128, 5, 10, "keep_all"), (1, 3, 4, "keep_one"), (33, 4, 10, "keep_all"),
                                            (100, 15, 2, "keep_one"), (129, 10, 10, "keep_all"),
                                            (256, 10, 10, "keep_all"), (200, 15, 2, "keep_one")])
def test_verify_kernel_bit_exact(sd, T, H, k, fallback):
    """Acceptance + fragment cut alone, many random cases per launch, bit-exact."""
    rng = np.random.default_rng(T * 131 + H)
    parent, depth, rank = wl.default_tree(T, H, k)
    tree = sd.Tree(parent, depth, rank, H, k)
    V, batch = 50, 512
    stop = rng.random(V) < 0.3
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tok = rng.integers(V, size=(batch, T)).astype(np.int32)
    am = rng.integers(V, size=(batch, T)).astype(np.int32)
    # make long accepted chains frequent: copy the parent's arg-max into many nodes
    for b in range(batch):
        for j in range(1, T):
            if rng.random() < 0.7:
                tok[b, j] = am[b, parent[j]]
    n_acc, n_raw, tokens, slots = sd.verify_tree(tree, torch.from_numpy(tok).cuda(), torch.from_numpy(am).cuda(), words,
                                                 V, fallback)
    torch.cuda.synchronize()
    n_acc, n_raw, tokens, slots = (t.cpu().numpy() for t in (n_acc, n_raw, tokens, slots))
    lengths = set()
    for b in range(batch):
        ok, chain = orc.greedy_accept(tok[b], am[b], parent, depth)
        want = orc.fragment_cut([tok[b][c] for c in chain], stop, fallback)
        assert n_raw[b] == len(chain) and n_acc[b] == want
        assert list(slots[b][:want]) == chain[:want] and list(tokens[b][:want]) == [tok[b][c] for c in chain[:want]]
        assert (slots[b][want:] == -1).all() and (tokens[b][want:] == -1).all()
        lengths.add(len(chain))
    if T > 1:
        assert len(lengths) > 1


# ----------------------------------------------------------------------------- cache row access
@pytest.mark.parametrize("name", ["tiny", "7b"])
def test_kv_rows_round_trip(sd, name):
    shape = _bf16_shape(name, 2)
    weights = {k: v.cuda() for k, v in wl.make_weights(shape).items()}
    model = sd.Model(shape, weights, 64)
    kv = sd.KVCache(model, 2, 100)
    g = torch.Generator().manual_seed(5)
    for layer, seq, row0, nrows in [(0, 0, 0, 37), (1, 1, 30, 70), (0, 1, 99, 1)]:
        k = torch.randn((nrows, shape.n_heads, shape.head_dim), generator=g).bfloat16().cuda()
        v = torch.randn((nrows, shape.n_heads, shape.head_dim), generator=g).bfloat16().cuda()
        kv.write_rows(layer, seq, row0, k, v)
        k2, v2 = kv.read_rows(layer, seq, row0, nrows)
        assert torch.equal(k, k2) and torch.equal(v, v2)
    # rows of other (layer, seq) planes were not touched
    k0, v0 = kv.read_rows(1, 0, 0, 100)
    assert float(k0.abs().max()) == 0.0 and float(v0.abs().max()) == 0.0


# ----------------------------------------------------------------------------- full step, lock-step
def _setup(sd, shape, prompt_len, cap, T, fallback="keep_all", max_rows=64, seed=wl.SEEDS["weights"]):
    from tests import lockstep
    weights = wl.make_weights(shape, seed=seed)
    w64 = lockstep.weights_to_f64(weights)
    model = sd.Model(shape, {k: v.cuda() for k, v in weights.items()}, max_rows, fallback)
    kv = sd.KVCache(model, 1, cap)
    prompt = wl.zipf_prompt(shape.vocab, prompt_len)
    stop = wl.stop_set(shape.vocab, 0.2)
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(T, shape.n_medusa, shape.topk)
    tree = sd.Tree(*tree_np, shape.n_medusa, shape.topk)
    return lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree


def _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, cap, rep, kv_tol):
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [len(prompt)])
    st = orc.prefill(w64, shape, prompt, cap)
    assert kv.len() == [len(prompt)]
    lockstep.compare_kv_rows(kv, st, shape, 0, len(prompt), rep, kv_tol)
    root, cand = kv.get_draft()
    return st, int(root[0]), cand[0].cpu().numpy()


@pytest.mark.parametrize("fallback", ["keep_all", "keep_one"])
def test_tiny_shape_lockstep_32_steps(sd, fallback):
    """configs[0] shapes (bf16 storage): prefill 64 tokens, 32 speculative steps, planted drafts."""
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 64, 256, 16, fallback)
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, 256, rep, 0.0)
    # the plain-greedy continuation, for planting drafts
    g = orc.prefill(w64, shape, prompt, 256)
    for _ in range(150):
        orc.greedy_step(w64, shape, g)
    truth = g.emitted
    rng = np.random.default_rng(wl.SEEDS["force"])

    def plant(s):
        e = len(s.emitted)
        return wl.plant_drafts(s.cand, np.array(truth[e + 1: e + 1 + shape.n_medusa]), (0.9, 0.8, 0.7), rng)

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 32, fallback, plant, rep=rep)
    print(f"\n[tiny/{fallback}] {rep}")
    assert rep.steps == 32 and max(rep.accepted) >= 3
    assert st.emitted == truth[: len(st.emitted)]          # lossless, by the oracle's own stream


def test_tiny_shape_against_the_fp32_oracle(sd):
    """configs[0] as specified (fp32 weights, fp32 cache) on the oracle's side, against the bf16 device path
    given the same weights rounded to bf16: the storage rounding itself stays inside the logits bounds
    (2e-2 max-abs, 1e-2 relative). (The float32 device path proper is covered by test_gpu_f32.py.)"""
    import dataclasses
    shape32 = wl.preset("tiny").model
    assert shape32.dtype == "f32"
    from tests import lockstep
    weights = wl.make_weights(shape32)
    assert weights["l0.wqkv"].dtype == torch.float32
    w64 = lockstep.weights_to_f64(weights)
    model = sd.Model(dataclasses.replace(shape32, dtype="bf16"), {k: v.bfloat16().cuda() for k, v in weights.items()}, 64)
    kv = sd.KVCache(model, 1, 256)
    prompt = wl.zipf_prompt(shape32.vocab, 64)
    stop = wl.stop_set(shape32.vocab, 0.2)
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(16, shape32.n_medusa, shape32.topk)
    tree = sd.Tree(*tree_np, shape32.n_medusa, shape32.topk)
    rep = lockstep.Report()
    # the oracle's rows are not rounded here: half a bfloat16 spacing of storage rounding plus the effect of
    # the bf16 weights on the rows themselves, bounded like the logits
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape32, prompt, 256, rep, lockstep.LOGIT_MAX_ABS)
    g = orc.prefill(w64, shape32, prompt, 256)
    for _ in range(150):
        orc.greedy_step(w64, shape32, g)
    truth = g.emitted
    rng = np.random.default_rng(wl.SEEDS["force"])

    def plant(s):
        e = len(s.emitted)
        return wl.plant_drafts(s.cand, np.array(truth[e + 1: e + 1 + shape32.n_medusa]), (0.9, 0.8, 0.7), rng)

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape32, st, 32, "keep_all", plant,
                                 kv_tol=lockstep.LOGIT_MAX_ABS, rep=rep)
    print(f"\n[tiny, fp32 oracle] {rep}")
    assert rep.steps == 32 and max(rep.accepted) >= 3
    assert st.emitted == truth[: len(st.emitted)]


def test_7b_width_two_layers_lockstep(sd):
    """Full 7B width and vocabulary, depth cut to 2 layers: prefill 100 tokens (two ragged
    chunks), then speculative steps on the 64-node tree with random heads and planted drafts."""
    shape = _bf16_shape("7b", 2)
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 100, 160, 64)
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, 160, rep, 0.0)
    assert root == st.root_tok
    g = orc.prefill(w64, shape, prompt, 160)
    for _ in range(24):
        orc.greedy_step(w64, shape, g)
    truth = g.emitted
    rng = np.random.default_rng(wl.SEEDS["force"])

    def plant(s):
        e = len(s.emitted)
        return wl.plant_drafts(s.cand, np.array(truth[e + 1: e + 1 + shape.n_medusa]), (0.9, 0.85, 0.8, 0.75), rng)

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 2, "keep_all", None, 0.0, rep)
    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 4, "keep_all", plant, 0.0, rep)
    print(f"\n[7b-L2] {rep}")
    assert max(rep.accepted) >= 2
    assert st.emitted == truth[: len(st.emitted)]


def test_greedy_step_matches_oracle(sd):
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 40, 128, 16)
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, 128, rep, 0.0)
    for i in range(8):
        kv.set_draft([st.root_tok], np.asarray(st.cand)[None])
        out = sd.greedy_step(model, kv, want_logits=True)
        rec = orc.greedy_step(w64, shape, st)
        torch.cuda.synchronize()
        lockstep.check_logits(out.logits[0].cpu().numpy().astype(np.float64), rec.logits, rep)
        assert int(out.n_accept[0]) == 1 and int(out.tokens[0, 0]) == rec.tokens[0] and int(out.src_slots[0, 0]) == 0
        assert kv.len() == [st.kv.n]
        lockstep.compare_kv_rows(kv, st, shape, st.kv.n - 1, st.kv.n, rep)


def test_errors_leave_state_untouched(sd):
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 20, 20 + shape.n_medusa, 16)
    with pytest.raises(sd.SpecDecError) as e:
        sd.spec_step(model, kv, tree, words)
    assert e.value.name == "SD_ERR_STATE"
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [20])
    with pytest.raises(sd.SpecDecError) as e:                       # 20 + H + 1 > cap
        sd.spec_step(model, kv, tree, words)
    assert e.value.name == "SD_ERR_KV_FULL" and kv.len() == [20]
    with pytest.raises(sd.SpecDecError) as e:
        sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [20])
    assert e.value.name == "SD_ERR_KV_FULL" and kv.len() == [20]


def test_step_that_exactly_fits_the_cache(sd):
    """cap = prompt + H + 1 (not a multiple of the 32-row cache blocks): the step is accepted, matches the
    oracle up to the last cache row, and the one after it is refused without touching anything."""
    shape = _bf16_shape("tiny")
    cap = 21 + shape.n_medusa + 1
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 21, cap, 16)
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, kv, w64, shape, prompt, cap, rep, 0.0)
    truth = orc.prefill(w64, shape, prompt, cap + 8)
    for _ in range(shape.n_medusa + 1):
        orc.greedy_step(w64, shape, truth)

    def plant(s):                                  # the whole chain is right: H + 1 tokens unless a stop cuts it
        c = np.array(s.cand, np.int32).copy()
        for i in range(shape.n_medusa):
            want = truth.emitted[1 + i]
            dup = np.nonzero(c[i] == want)[0]
            if dup.size:
                c[i, dup[0]] = c[i, 0]
            c[i, 0] = want
        return c

    rep = lockstep.lockstep_spec(model, kv, tree, tree_np, stop, words, w64, shape, st, 1, "keep_all", plant, rep=rep)
    assert rep.steps == 1 and rep.raw[0] == shape.n_medusa + 1
    n = kv.len()[0]
    assert n == 21 + rep.accepted[0] <= cap
    with pytest.raises(sd.SpecDecError) as e:
        sd.spec_step(model, kv, tree, words)
    assert e.value.name == "SD_ERR_KV_FULL" and kv.len() == [n]


def test_graph_mode_replays_equal_eager(sd):
    """Graph mode: the captured step, replayed many times with eager work and synchronisations
    in between, gives bit-identical outputs to the eager path (same deterministic kernels)."""
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 40, 256, 16)
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [40])
    root0, cand0 = kv.get_draft()
    root0, cand0 = root0.clone(), cand0.clone()
    rng = np.random.default_rng(3)
    cands = [np.stack([rng.permutation(shape.vocab)[: shape.topk] for _ in range(shape.n_medusa)]).astype(np.int32)
             for _ in range(12)]
    forced = torch.zeros((1, shape.n_medusa, shape.topk), dtype=torch.int32, device="cuda")

    def run(n_steps):
        kv.set_len([40])
        kv.set_draft(root0, cand0)
        res = []
        out = sd.spec_step(model, kv, tree, words, want_logits=True, want_argmax=True, forced_cand=forced)
        for i in range(n_steps):
            forced.copy_(torch.from_numpy(cands[i])[None])
            sd.spec_step(model, kv, tree, words, forced_cand=forced, out=out)
            torch.cuda.synchronize()
            res.append((out.logits.clone(), out.tokens.clone(), out.n_accept.clone(), out.src_slots.clone(), kv.len()))
            _ = (out.logits * 2).sum().item()              # unrelated eager work between replays
        return res

    eager = run(12)
    model.set_graph_mode(True)
    graph = run(12)
    model.set_graph_mode(False)
    for a, b in zip(eager, graph):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2]) and torch.equal(a[3], b[3])
        assert a[4] == b[4]


def test_graph_mode_survives_a_destroyed_and_recreated_cache(sd):
    """Graph keys name a cache by a serial number, not by its handle's address: a cache that is destroyed and
    replaced by one of another capacity (whose handle may get the same address, and whose buffer does here)
    must not replay the first one's graph. Each cache's graph-mode steps equal its own eager steps."""
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 40, 256, 16)
    kv.close()
    buf = torch.empty(sd.lib().sd_kv_bytes(model.cfg, 1, 256) + 16, dtype=torch.uint8, device="cuda")
    forced = torch.zeros((1, shape.n_medusa, shape.topk), dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(5)
    cands = [torch.from_numpy(np.stack([rng.permutation(shape.vocab)[: shape.topk] for _ in range(shape.n_medusa)])
                              .astype(np.int32))[None] for _ in range(4)]
    out = None
    for cap in (256, 96, 160):
        res = {}
        for graphs in (False, True):
            cache = sd.KVCache(model, 1, cap, buf=buf)
            model.set_graph_mode(graphs)
            sd.prefill(model, cache, torch.from_numpy(prompt).cuda(), [40])
            got = []
            for c in cands:
                forced.copy_(c)
                out = sd.spec_step(model, cache, tree, words, want_logits=True, want_argmax=True, forced_cand=forced,
                                   out=out)
                torch.cuda.synchronize()
                got.append((out.logits.clone(), out.tokens.clone(), out.n_accept.clone(), cache.len()))
            res[graphs] = got
            cache.close()
        model.set_graph_mode(False)
        for a, b in zip(res[False], res[True]):
            assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2]) and a[3] == b[3]


def test_cache_buffer_full_of_nans_cannot_reach_the_logits(sd):
    """A caller's cache buffer may hold anything (here: every 16-bit word a bfloat16 NaN). sd_kv_create clears
    it, so the value rows past the committed length inside a partly filled block, which attention multiplies
    by probabilities of exactly zero, are zeros and not NaNs. Prefill 45 rows (a partly filled second block)
    and one step, against the oracle."""
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 45, 128, 16)
    kv.close()
    nbytes = sd.lib().sd_kv_bytes(model.cfg, 1, 128)
    buf = torch.full((nbytes // 2,), 0x7FC0, dtype=torch.int16, device="cuda").view(torch.uint8)
    cache = sd.KVCache(model, 1, 128, buf=buf)
    rep = lockstep.Report()
    st, root, cand = _prefill_both(sd, lockstep, model, cache, w64, shape, prompt, 128, rep, 0.0)
    assert root == st.root_tok
    rep = lockstep.lockstep_spec(model, cache, tree, tree_np, stop, words, w64, shape, st, 2, "keep_all", rep=rep)
    assert rep.steps == 2 and np.isfinite(rep.max_abs)


def test_greedy_step_without_draft_heads(sd):
    """sd_set_greedy_drafts(0): the plain next-token step gives the same token and logits and leaves the
    carried candidates untouched."""
    shape = _bf16_shape("tiny")
    lockstep, weights, w64, model, kv, prompt, stop, words, tree_np, tree = _setup(sd, shape, 40, 128, 16)
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [40])
    root0, cand0 = kv.get_draft()
    root0, cand0 = root0.clone(), cand0.clone()
    a = sd.greedy_step(model, kv, want_logits=True)
    torch.cuda.synchronize()
    root_a, cand_a = [t.clone() for t in kv.get_draft()]
    kv.set_len([40])
    kv.set_draft(root0, cand0)
    model.set_greedy_drafts(False)
    b = sd.greedy_step(model, kv, want_logits=True)
    torch.cuda.synchronize()
    root_b, cand_b = [t.clone() for t in kv.get_draft()]
    model.set_greedy_drafts(True)
    assert torch.equal(a.logits, b.logits) and torch.equal(a.tokens, b.tokens) and torch.equal(root_a, root_b)
    assert torch.equal(cand_b, cand0) and kv.len() == [41]
    assert not torch.equal(cand_a, cand0)                  # with the heads on, the candidates had moved on
