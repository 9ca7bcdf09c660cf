"""GPU parity of sampling decoding: typical acceptance (Section III-B, Eq. 1) and the
inverse-CDF draw of the next root, called through the C ABI, against the CPU oracle.

The paper leaves epsilon and delta open; the values here (0.09, 0.3) make both arms of the
min() bind on the synthetic distributions used."""
import copy
import dataclasses

import numpy as np
import pytest
import torch

import workload as wl
from oracle import specdec_oracle as orc
from tests import lockstep

pytestmark = pytest.mark.gpu

TY = dict(temperature=0.8, epsilon=0.09, delta=0.3)


@pytest.fixture(scope="module")
def sd():
    import paper_2503_14153_amd as sd
    sd.lib()                       # fails loudly if the library has not been built
    return sd


def _shape(name, n_layers=None):
    return dataclasses.replace(wl.preset(name, n_layers).model, dtype="bf16")


def _peaked_logits(rng, rows, V, scales):
    """Rows whose entropy spans near-deterministic to near-uniform: normal noise times a per-row scale."""
    s = rng.choice(scales, size=(rows, 1))
    return (rng.standard_normal((rows, V)) * s).astype(np.float32)


# ----------------------------------------------------------------------------- single stages
@pytest.mark.parametrize("T,H,k,V,batch,fallback", [(16, 3, 4, 50, 256, "keep_all"), (64, 4, 10, 1000, 64, "keep_one"),
                                                    (64, 4, 10, 32000, 4, "keep_all"), (33, 4, 10, 32001, 3, "keep_all"),
                                                    (1, 3, 4, 50, 8, "keep_all"), (128, 5, 10, 5000, 8, "keep_all"),
                                                    (256, 10, 10, 2000, 16, "keep_all")])
def test_typical_verify_kernel(sd, T, H, k, V, batch, fallback):
    """Row statistics + typical acceptance + cut alone on synthetic logits, many cases per launch."""
    rng = np.random.default_rng(T * 977 + V)
    tree_np = wl.default_tree(T, H, k)
    parent, depth, rank = tree_np
    tree = sd.Tree(parent, depth, rank, H, k)
    stop = rng.random(V) < 0.3
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    logits = _peaked_logits(rng, batch * T, V, [0.05, 1.0, 3.0, 8.0]).reshape(batch, T, V)
    tok = rng.integers(V, size=(batch, T)).astype(np.int32)
    for b in range(batch):                                   # plant likely tokens so that chains grow
        for j in range(1, T):
            r = rng.random()
            order = np.argsort(-logits[b, parent[j]])
            if r < 0.6:
                tok[b, j] = order[0]
            elif r < 0.8:
                tok[b, j] = order[rng.integers(1, min(6, V))]
    n_acc, n_raw, tokens, slots, stats = sd.verify_tree_typical(tree, torch.from_numpy(tok).cuda(),
                                                                torch.from_numpy(logits).cuda(), words,
                                                                trunc_fallback=fallback, **TY)
    torch.cuda.synchronize()
    n_acc, n_raw, tokens, slots, stats = (t.cpu().numpy() for t in (n_acc, n_raw, tokens, slots, stats))
    rep = lockstep.Report()
    lengths, eps_binds, delta_binds = set(), 0, 0
    for b in range(batch):
        l64 = logits[b].astype(np.float64)
        lockstep.check_row_stats(stats[b], l64, TY, rep)
        lockstep.check_typical_decision(int(n_raw[b]), int(n_acc[b]), tokens[b], slots[b], tok[b], l64, tree_np, stop,
                                        fallback, TY, H, rep)
        lengths.add(int(n_raw[b]))
        for j in range(T):
            p = orc.softmax_t(l64[j], TY["temperature"])
            if TY["delta"] * np.exp(-orc.entropy(p)) < TY["epsilon"]:
                delta_binds += 1
            else:
                eps_binds += 1
    print(f"\n[typical verify T={T} V={V}] raw lengths {sorted(lengths)}, near-threshold cases {rep.accept_near_ties}, "
          f"stats err {rep.stats_max_abs:.2e}, eps/delta arm {eps_binds}/{delta_binds}")
    assert eps_binds and delta_binds
    assert rep.accept_near_ties <= max(1, batch // 50)
    if T > 1 and batch >= 64:
        assert len(lengths) > 2


@pytest.mark.parametrize("V,ld", [(50, 50), (1000, 1024), (32000, 32000), (32001, 32064), (131072, 131072)])
def test_sample_tokens_kernel(sd, V, ld):
    """Inverse-CDF draws alone: ids equal the oracle's on the same logits unless u sits on a boundary."""
    rng = np.random.default_rng(V)
    n_rows, n = 6, 96
    buf = np.zeros((n_rows, ld), np.float32)
    buf[:, :V] = _peaked_logits(rng, n_rows, V, [0.05, 1.0, 3.0, 8.0])
    buf[:, V:] = 50.0                                        # padding columns must never be read
    buf[0, :V] = -2000.0                                    # one row whose mass sits on two far-apart ids
    buf[0, 3 % V], buf[0, V - 1] = 5.0, 5.0
    rows = rng.integers(n_rows, size=n).astype(np.int32)
    rows[:4] = 0
    u = rng.random(n).astype(np.float32)
    u[0], u[1], u[2], u[3] = 0.0, np.float32(1.0) - np.float32(2.0 ** -24), 0.25, 0.75
    rows[4] = n_rows + 3                                     # out of range -> -1
    got = sd.sample_tokens(torch.from_numpy(buf).cuda()[:, :V], torch.from_numpy(rows).cuda(),
                           torch.from_numpy(u).cuda(), TY["temperature"])
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got[4] == -1
    near = 0
    for i in range(n):
        if i == 4:
            continue
        assert 0 <= got[i] < V
        near += not lockstep.check_sampled(int(got[i]), buf[rows[i], :V].astype(np.float64), float(u[i]),
                                           TY["temperature"], lockstep.FP32_CDF)
    assert got[0] == 3 % V and got[2] == 3 % V and got[3] == V - 1 and got[1] == V - 1
    assert near <= 1
    assert len(set(got.tolist())) > 10


def test_sample_tokens_follows_the_distribution(sd):
    """Many draws from one small distribution reproduce its probabilities (chi-square bound)."""
    V, n = 12, 60000
    rng = np.random.default_rng(3)
    logits = (rng.standard_normal((1, V)) * 1.5).astype(np.float32)
    u = rng.random(n).astype(np.float32)
    got = sd.sample_tokens(torch.from_numpy(logits).cuda(), torch.zeros(n, dtype=torch.int32, device="cuda"),
                           torch.from_numpy(u).cuda(), TY["temperature"]).cpu().numpy()
    p = orc.softmax_t(logits[0].astype(np.float64), TY["temperature"])
    counts = np.bincount(got, minlength=V)
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 40.0, chi2                                 # 11 degrees of freedom: P(chi2 > 40) ~ 4e-5


def test_typical_errors(sd):
    shape = _shape("tiny")
    weights = {k: v.cuda() for k, v in wl.make_weights(shape).items()}
    model = sd.Model(shape, weights, 64)
    kv = sd.KVCache(model, 1, 128)
    tree = sd.Tree(*wl.default_tree(16, shape.n_medusa, shape.topk), shape.n_medusa, shape.topk)
    words = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    u = torch.zeros(1, dtype=torch.float32, device="cuda")
    with pytest.raises(sd.SpecDecError) as e:
        sd.spec_step_typical(model, kv, tree, words, u, **TY)
    assert e.value.name == "SD_ERR_STATE"                    # no draft state yet
    sd.prefill(model, kv, torch.from_numpy(wl.zipf_prompt(shape.vocab, 8)).cuda(), [8])
    for bad in (dict(TY, temperature=0.0), dict(TY, temperature=float("nan")), dict(TY, epsilon=1.5),
                dict(TY, delta=-1.0)):
        with pytest.raises(sd.SpecDecError) as e:
            sd.spec_step_typical(model, kv, tree, words, u, **bad)
        assert e.value.name == "SD_ERR_SHAPE"
    assert kv.len() == [8]


# ----------------------------------------------------------------------------- full step, lock-step
def _setup(sd, shape, prompt_len, cap, T, fallback):
    weights = wl.make_weights(shape)
    w64 = lockstep.weights_to_f64(weights)
    model = sd.Model(shape, {k: v.cuda() for k, v in weights.items()}, 64, fallback)
    kv = sd.KVCache(model, 1, cap)
    prompt = wl.zipf_prompt(shape.vocab, prompt_len)
    stop = wl.stop_set(shape.vocab, 0.2)
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(T, shape.n_medusa, shape.topk)
    tree = sd.Tree(*tree_np, shape.n_medusa, shape.topk)
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [len(prompt)])
    st = orc.prefill(w64, shape, prompt, cap)
    return w64, model, kv, stop, words, tree_np, tree, st


def _plant_greedy_continuation(w64, shape, probs, prng):
    """Draft candidates with the base model's own greedy continuation of the current root planted at rank 0 with
    the given per-head probabilities: tokens that pass Eq. 1 whenever the distribution is peaked enough."""
    def plant(s):
        g, cont = copy.deepcopy(s), []
        for _ in range(shape.n_medusa):
            orc.greedy_step(w64, shape, g)
            cont.append(g.root_tok)
        return wl.plant_drafts(s.cand, np.array(cont), probs, prng)
    return plant


@pytest.mark.parametrize("fallback,temperature", [("keep_all", 0.8), ("keep_all", 0.04), ("keep_one", 0.04)])
def test_tiny_shape_typical_lockstep(sd, fallback, temperature):
    """configs[0] shapes, 32 sampling-decoding steps. At the paper's temperature 0.8 the random-init model's
    distributions are nearly uniform, so the entropy arm admits every draft; at 0.04 they are as peaked as a
    trained model's and the tests fall on both sides of the threshold."""
    shape = _shape("tiny")
    w64, model, kv, stop, words, tree_np, tree, st = _setup(sd, shape, 64, 320, 16, fallback)
    rng = np.random.default_rng(wl.SEEDS["force"])
    plant = _plant_greedy_continuation(w64, shape, (0.9, 0.8, 0.7), np.random.default_rng(1))
    ty = dict(TY, temperature=temperature)
    rep = lockstep.lockstep_typical(model, kv, tree, tree_np, stop, words, w64, shape, st, 32, fallback, ty, rng,
                                    cand_fn=plant)
    print(f"\n[tiny typical/{fallback}/T={temperature}] {rep}")
    assert rep.steps == 32
    if temperature < 0.1:
        assert len(set(rep.raw)) > 2
    assert rep.accept_near_ties <= 2 and rep.root_near_ties <= 2


@pytest.mark.parametrize("temperature", [0.8, 0.05])
def test_7b_width_two_layers_typical_lockstep(sd, temperature):
    """Full 7B width and vocabulary, 2 layers, 64-node tree, sampling decoding."""
    shape = _shape("7b", 2)
    w64, model, kv, stop, words, tree_np, tree, st = _setup(sd, shape, 100, 160, 64, "keep_all")
    plant = _plant_greedy_continuation(w64, shape, (0.9, 0.85, 0.8, 0.75), np.random.default_rng(2))
    rng = np.random.default_rng(11)
    ty = dict(TY, temperature=temperature)
    rep = lockstep.lockstep_typical(model, kv, tree, tree_np, stop, words, w64, shape, st, 4, "keep_all", ty, rng,
                                    cand_fn=plant)
    print(f"\n[7b-L2 typical T={temperature}] {rep}")
    assert rep.steps == 4
    assert rep.accept_near_ties <= 1 and rep.root_near_ties <= 1


def test_typical_step_batch_of_three(sd):
    """Sampling decoding for three sequences at once (different committed lengths, one uniform number each):
    every sequence against the oracle's own step, decisions exact on the GPU's logits."""
    shape = _shape("tiny")
    B, T, cap, fallback = 3, 16, 192, "keep_all"
    ty = dict(TY, temperature=0.04)
    weights = wl.make_weights(shape)
    w64 = lockstep.weights_to_f64(weights)
    model = sd.Model(shape, {k: v.cuda() for k, v in weights.items()}, B * 32, fallback)
    kv = sd.KVCache(model, B, cap)
    stop = wl.stop_set(shape.vocab, 0.2)
    words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(T, shape.n_medusa, shape.topk)
    tree = sd.Tree(*tree_np, shape.n_medusa, shape.topk)
    lens = [40, 17, 64]
    prompts = [wl.zipf_prompt(shape.vocab, n, seed=100 + b) for b, n in enumerate(lens)]
    sd.prefill(model, kv, torch.from_numpy(np.concatenate(prompts)).cuda(), lens)
    states = [orc.prefill(w64, shape, p, cap) for p in prompts]
    rng = np.random.default_rng(5)
    plant = _plant_greedy_continuation(w64, shape, (0.9, 0.8, 0.7), np.random.default_rng(6))
    rep = lockstep.Report()
    for step in range(6):
        cand = np.stack([np.asarray(plant(st), np.int32) for st in states])
        u = rng.random(B).astype(np.float32)
        n_old = [st.kv.n for st in states]
        kv.set_draft([st.root_tok for st in states], cand)
        out = sd.spec_step_typical(model, kv, tree, words, torch.from_numpy(u).cuda(), want_logits=True,
                                   want_row_stats=True, **ty)
        recs = [orc.spec_step(w64, shape, st, tree_np, stop, fallback, cand_override=cand[b],
                              typical=dict(ty, u=float(u[b]))) for b, st in enumerate(states)]
        torch.cuda.synchronize()
        lens_now = kv.len()
        roots, _ = kv.get_draft()
        for b, rec in enumerate(recs):
            g_logits = out.logits[b].cpu().numpy().astype(np.float64)
            lockstep.check_logits(g_logits, rec.logits, rep)
            lockstep.check_row_stats(out.row_stats[b].cpu().numpy(), g_logits, ty, rep)
            kept = lockstep.check_typical_decision(int(out.n_accept_raw[b]), int(out.n_accept[b]),
                                                   out.tokens[b].cpu().numpy(), out.src_slots[b].cpu().numpy(), rec.tok,
                                                   g_logits, tree_np, stop, fallback, ty, shape.n_medusa, rep)
            assert lens_now[b] == n_old[b] + len(kept)
            assert lockstep.check_sampled(int(roots[b]), g_logits[kept[-1]], float(u[b]), ty["temperature"],
                                          lockstep.FP32_CDF)
            # this seed has no near-threshold case: the two sides walk the same path
            assert kept == list(rec.src_slots) and int(roots[b]) == rec.next_root
            rep.raw.append(int(out.n_accept_raw[b]))
    print(f"\n[tiny typical batch 3] raw lengths {rep.raw}, max logits error {rep.max_abs:.2e}")
    assert len(set(rep.raw)) > 1
