"""Pins for the oracle's model arithmetic against library routines and other formulations.

Each test compares an oracle function with something that is not the oracle: a PyTorch /
transformers library routine called with its documented conventions, a different
mathematical formulation (complex rotation), a closed form, or explicit loops on tiny inputs.
"""
import math

import numpy as np
import torch
import torch.nn.functional as F

import workload as wl
from oracle import specdec_oracle as orc

RNG = np.random.default_rng(7)


def test_rmsnorm_matches_torch_rms_norm():
    x = RNG.standard_normal((5, 64))
    g = RNG.standard_normal(64)
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(orc.rmsnorm(x, g, 1e-5), want, rtol=1e-12, atol=1e-12)


def test_rmsnorm_of_constant_vector_is_sign_times_gain():
    g = RNG.standard_normal(32)
    assert np.allclose(orc.rmsnorm(np.full((1, 32), -3.0), g, 0.0), -g)


def test_silu_matches_torch():
    x = RNG.standard_normal(100) * 4
    assert np.allclose(orc.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-13)


def test_rope_is_a_complex_rotation_of_half_split_pairs():
    T, nh, hd, theta = 6, 3, 16, 1e4
    x = RNG.standard_normal((T, nh, hd))
    pos = np.array([0, 1, 5, 17, 100, 1000])
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    freq = theta ** (-np.arange(hd // 2) * 2.0 / hd)
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    want = np.concatenate([zr.real, zr.imag], axis=-1)
    assert np.allclose(orc.rope(x, pos, theta), want, rtol=1e-12, atol=1e-12)


def test_rope_position_zero_is_identity_and_norms_are_kept():
    x = RNG.standard_normal((4, 2, 64))
    assert np.array_equal(orc.rope(x, np.zeros(4), 1e6), x)
    y = orc.rope(x, np.array([3, 9, 1000, 16384]), 1e6)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))


def test_rope_scores_depend_only_on_relative_position():
    q = RNG.standard_normal((1, 1, 64))
    k = RNG.standard_normal((1, 1, 64))
    def score(m, n):
        return float(np.sum(orc.rope(q, np.array([m]), 1e4) * orc.rope(k, np.array([n]), 1e4)))
    assert abs(score(10, 3) - score(110, 103)) < 1e-9
    assert abs(score(10, 3) - score(3, 10)) > 1e-3        # and on its sign


def test_rope_matches_transformers_rotary():
    from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
    T, nh, hd, theta = 5, 2, 32, 1e4
    x = RNG.standard_normal((T, nh, hd))
    pos = np.array([0, 2, 3, 50, 51])
    inv = theta ** (-np.arange(0, hd, 2) / hd)
    ang = torch.from_numpy(pos[:, None] * inv[None, :])
    emb = torch.cat([ang, ang], dim=-1)[None]                    # [1, T, hd]
    xt = torch.from_numpy(x).permute(1, 0, 2)[None]              # [1, nh, T, hd]
    got, _ = apply_rotary_pos_emb(xt, xt, emb.cos(), emb.sin())
    assert np.allclose(orc.rope(x, pos, theta), got[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_attention_matches_torch_sdpa_causal():
    T, hd = 9, 16
    q, k, v = (RNG.standard_normal((T, hd)) for _ in range(3))
    want = F.scaled_dot_product_attention(*(torch.from_numpy(a)[None, None] for a in (q, k, v)),
                                          is_causal=True)[0, 0].numpy()
    got = orc.attention(q, k, v, np.tril(np.ones((T, T), bool)))
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_attention_explicit_loops_with_arbitrary_mask():
    T, S, hd = 4, 7, 8
    q, k, v = RNG.standard_normal((T, hd)), RNG.standard_normal((S, hd)), RNG.standard_normal((S, hd))
    vis = RNG.random((T, S)) < 0.5
    vis[:, 0] = True
    for t in range(T):
        num, den = np.zeros(hd), 0.0
        for s in range(S):
            if vis[t, s]:
                wgt = math.exp(sum(q[t, e] * k[s, e] for e in range(hd)) / math.sqrt(hd))
                num += wgt * v[s]
                den += wgt
        assert np.allclose(orc.attention(q, k, v, vis)[t], num / den, rtol=1e-12)


def test_attention_single_visible_key_returns_its_value_row():
    q, k, v = RNG.standard_normal((2, 8)), RNG.standard_normal((5, 8)), RNG.standard_normal((5, 8))
    vis = np.zeros((2, 5), bool)
    vis[0, 3] = vis[1, 1] = True
    out = orc.attention(q, k, v, vis)
    assert np.allclose(out[0], v[3]) and np.allclose(out[1], v[1])


def test_topk_equals_full_stable_sort_and_breaks_ties_by_id():
    lg = np.round(RNG.standard_normal(50), 1)              # rounding forces ties
    full = sorted(range(50), key=lambda i: (-lg[i], i))
    assert list(orc.topk_ids(lg, 7)) == full[:7]
    assert list(orc.topk_ids(np.array([1.0, 3.0, 3.0, 2.0, 3.0]), 4)) == [1, 2, 4, 3]
    assert orc.argmax_lowest(np.array([[1.0, 3.0, 3.0]]))[0] == 1
    want = torch.topk(torch.from_numpy(RNG.standard_normal(1000)), 10)
    lg2 = RNG.standard_normal(1000)
    assert list(orc.topk_ids(lg2, 10)) == list(torch.topk(torch.from_numpy(lg2), 10).indices.numpy())


def test_top2_margin():
    assert np.allclose(orc.top2_margin(np.array([[1.0, 5.0, 4.5], [2.0, 2.0, 0.0]])), [0.5, 0.0])


def _tiny():
    shape = wl.preset("tiny").model
    return shape, wl.make_weights(shape, medusa_bias_std=0.02)


def test_forward_matches_transformers_llama_causal():
    """The whole base forward (embedding .. logits) against transformers' LlamaForCausalLM."""
    from transformers import LlamaConfig, LlamaForCausalLM
    shape, w = _tiny()
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, head_dim=shape.head_dim,
                      rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, tie_word_embeddings=False,
                      attention_bias=False, mlp_bias=False, max_position_embeddings=512,
                      attn_implementation="eager")
    cfg.rope_parameters = {"rope_type": "default", "rope_theta": shape.rope_theta}
    model = LlamaForCausalLM(cfg).double().eval()
    d = shape.d_model
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"],
          "model.norm.weight": w["final_norm"]}
    for l in range(shape.n_layers):
        p = f"model.layers.{l}."
        sd[p + "input_layernorm.weight"] = w[f"l{l}.attn_norm"]
        sd[p + "self_attn.q_proj.weight"] = w[f"l{l}.wqkv"][:d]
        sd[p + "self_attn.k_proj.weight"] = w[f"l{l}.wqkv"][d:2 * d]
        sd[p + "self_attn.v_proj.weight"] = w[f"l{l}.wqkv"][2 * d:]
        sd[p + "self_attn.o_proj.weight"] = w[f"l{l}.wo"]
        sd[p + "post_attention_layernorm.weight"] = w[f"l{l}.ffn_norm"]
        sd[p + "mlp.gate_proj.weight"] = w[f"l{l}.w_gate"]
        sd[p + "mlp.up_proj.weight"] = w[f"l{l}.w_up"]
        sd[p + "mlp.down_proj.weight"] = w[f"l{l}.w_down"]
    missing, unexpected = model.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not unexpected and all("rotary" in m for m in missing), (missing, unexpected)
    prompt = wl.zipf_prompt(shape.vocab, 24)
    with torch.no_grad():
        want = model(torch.from_numpy(prompt.astype(np.int64))[None]).logits[0].numpy()
    kv = orc.KVCache.empty(shape, 32)
    got, _, _, _ = orc.forward_rows(w, shape, prompt, np.arange(24), np.tril(np.ones((24, 24), bool)), kv)
    # transformers evaluates the rotary angles in float32 whatever the model dtype, so the
    # agreement is ~1e-7 rather than float64 round-off; any structural mistake is O(0.1).
    assert np.abs(got - want).max() < 1e-6
    # the same prompt in two pieces through the cache gives the same logits (cache path)
    _, _, k1, v1 = orc.forward_rows(w, shape, prompt[:10], np.arange(10), np.tril(np.ones((10, 10), bool)), kv)
    kv.k[:, :10], kv.v[:, :10], kv.n = k1, v1, 10
    got2, _, _, _ = orc.forward_rows(w, shape, prompt[10:], np.arange(10, 24), np.tril(np.ones((14, 14), bool)), kv)
    assert np.abs(got2 - want[10:]).max() < 1e-6
    assert np.abs(got2 - got[10:]).max() < 1e-11


def test_medusa_head_block_matches_torch_formulation():
    shape, w = _tiny()
    h = torch.from_numpy(RNG.standard_normal(shape.d_model))
    got = orc.medusa_logits(w, shape, h.numpy())
    for i in range(shape.n_medusa):
        z = F.linear(h, w[f"medusa{i}.w"].double(), w[f"medusa{i}.b"].double())
        want = F.linear(h + F.silu(z), w["lm_head"].double())
        assert np.allclose(got[i], want.numpy(), rtol=1e-11, atol=1e-12)
    cand = orc.medusa_candidates(w, shape, h.numpy())
    assert cand.shape == (shape.n_medusa, shape.topk)
    assert list(cand[1]) == list(torch.topk(torch.from_numpy(got[1]), shape.topk).indices.numpy())


# ---- the draft-head block pinned against what the mathematics fixes (Section III-B: the heads sit on the
# ---- base model's last hidden state, i.e. on what the LM head consumes). None of these re-type the formula:
# ---- each one picks weights for which the block has a value known in advance.
def _tiny_f64_heads():
    shape, w = _tiny()
    return shape, {k: v.double() for k, v in w.items()}


def test_medusa_head_with_zero_weights_is_the_base_lm_head():
    """W_i = 0, b_i = 0: SiLU(0) = 0, so every head's logits ARE the base logits lm_head @ h, bit for bit."""
    shape, w = _tiny_f64_heads()
    h = RNG.standard_normal(shape.d_model)
    for i in range(shape.n_medusa):
        w[f"medusa{i}.w"] = torch.zeros_like(w[f"medusa{i}.w"])
        w[f"medusa{i}.b"] = torch.zeros_like(w[f"medusa{i}.b"])
    base = w["lm_head"].numpy() @ h
    got = orc.medusa_logits(w, shape, h)
    for i in range(shape.n_medusa):
        assert np.array_equal(got[i], base)


def test_medusa_head_bias_saturates_silu_on_both_sides():
    """W_i = 0 and a bias far in SiLU's linear range: SiLU(40) = 40 to 2e-16, so logits = lm_head @ (h + b);
    far in its flat range, SiLU(-40) = -2e-16: logits = base logits. A bias added outside the SiLU, a missing
    residual or a missing bias each fail one of the two."""
    shape, w = _tiny_f64_heads()
    h = RNG.standard_normal(shape.d_model)
    lm = w["lm_head"].numpy()
    for i in range(shape.n_medusa):
        w[f"medusa{i}.w"] = torch.zeros_like(w[f"medusa{i}.w"])
    bias = 40.0 + RNG.random(shape.d_model)
    for i in range(shape.n_medusa):
        w[f"medusa{i}.b"] = torch.from_numpy(bias * (i + 1))
    got = orc.medusa_logits(w, shape, h)
    for i in range(shape.n_medusa):
        assert np.allclose(got[i], lm @ (h + bias * (i + 1)), rtol=0, atol=1e-12)
    for i in range(shape.n_medusa):
        w[f"medusa{i}.b"] = torch.from_numpy(-bias)
    got = orc.medusa_logits(w, shape, h)
    for i in range(shape.n_medusa):
        assert np.allclose(got[i], lm @ h, rtol=0, atol=1e-12)


def test_medusa_head_on_a_one_hot_row_with_identity_lm_head_by_hand():
    """d = V = 4, lm_head = I, h = e_2: head i's logits are e_2 + SiLU(column 2 of W_i + b_i), and with
    pre-activations 0, ln 3 and -ln 3 the SiLU values are 0, (3/4) ln 3 and -(1/4) ln 3 (sigmoid(ln 3) = 3/4)."""
    shape = wl.ModelShape(1, 4, 1, 4, 16, 4, 2, 2, "f32", 1e4)
    ln3 = math.log(3.0)
    W0 = np.zeros((4, 4)); W0[:, 2] = [ln3, 0.0, -ln3, 2 * ln3]          # what e_2 selects
    W0[:, 0] = 7.0                                                      # must not matter for h = e_2
    b0 = np.array([0.0, ln3, 0.0, -3 * ln3])                             # pre-activations: ln3, ln3, -ln3, -ln3
    W1 = np.zeros((4, 4)); W1[1, 2] = -ln3
    b1 = np.zeros(4)
    w = {"lm_head": np.eye(4), "medusa0.w": W0, "medusa0.b": b0, "medusa1.w": W1, "medusa1.b": b1}
    got = orc.medusa_logits(w, shape, np.array([0.0, 0.0, 1.0, 0.0]))
    want0 = np.array([0.75 * ln3, 0.75 * ln3, 1.0 - 0.25 * ln3, -0.25 * ln3])
    want1 = np.array([0.0, -0.25 * ln3, 1.0, 0.0])
    assert np.allclose(got[0], want0, rtol=0, atol=1e-15)
    assert np.allclose(got[1], want1, rtol=0, atol=1e-15)
    # a transposed W_i would read row 2 of W0 instead of its column 2
    assert not np.allclose(got[0], np.array([0.0, 0.0, 1.0, 0.0]) + orc.silu(W0[2] + b0))


def test_draft_heads_read_the_final_norm_output_of_the_last_kept_row():
    """With W_i = 0 and b_i = 0 a head's logits equal the base logits of the row it reads. So after a
    prefill the heads' candidates must be the base model's own top-k at the last prompt row, and after a
    speculative step the top-k at the last KEPT node: heads fed the un-normalised residual stream, another
    row, or another node would give other lists (the final norm rescales rows by different factors, and
    the LM head of x is not the LM head of norm(x) * gain once the gain is not constant)."""
    shape, w = _tiny_f64_heads()
    w["final_norm"] = torch.from_numpy(0.5 + RNG.random(shape.d_model))  # a gain that is not constant
    for i in range(shape.n_medusa):
        w[f"medusa{i}.w"] = torch.zeros_like(w[f"medusa{i}.w"])
        w[f"medusa{i}.b"] = torch.zeros_like(w[f"medusa{i}.b"])
    prompt = wl.zipf_prompt(shape.vocab, 12)
    st = orc.prefill(w, shape, prompt, 64)
    kv0 = orc.KVCache.empty(shape, 64)
    logits, _, _, _ = orc.forward_rows(w, shape, prompt, np.arange(12), np.tril(np.ones((12, 12), bool)), kv0)
    want = orc.topk_ids(logits[-1], shape.topk)
    assert st.root_tok == want[0]
    for i in range(shape.n_medusa):
        assert list(st.cand[i]) == list(want)
    # one speculative step whose drafts are the base model's own continuation, so several nodes are kept
    tree = wl.default_tree(8, shape.n_medusa, shape.topk)
    stop = np.zeros(shape.vocab, bool)
    g = orc.prefill(w, shape, prompt, 64)
    truth = []
    for _ in range(shape.n_medusa + 1):
        truth.append(int(orc.greedy_step(w, shape, g).tokens[0]))
    cand = np.array(st.cand, copy=True)
    for dpt in range(shape.n_medusa):
        cand[dpt, 0] = truth[dpt + 1]
    rec = orc.spec_step(w, shape, st, tree, stop, "keep_all", cand_override=cand)
    assert rec.n_accept >= 2
    last = rec.src_slots[-1]
    want = orc.topk_ids(rec.logits[last], shape.topk)
    for i in range(shape.n_medusa):
        assert np.allclose(rec.head_logits[i], rec.logits[last], rtol=0, atol=1e-12)   # (rows @ W) vs (W @ row) rounding
        assert list(rec.next_cand[i]) == list(want)


def test_kv_storage_rounding_is_torch_bfloat16_and_only_for_bf16():
    a = RNG.standard_normal((7, 3, 16)) * np.array([1e-3, 1.0, 300.0])[None, :, None]
    want = torch.from_numpy(a).float().bfloat16().double().numpy()
    assert np.array_equal(orc.kv_storage(a, "bf16"), want)
    assert orc.kv_storage(a, "f32") is a
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8])          # exactly between two bf16 numbers
    assert np.array_equal(orc.kv_storage(ties, "bf16"), [1.0, 1.0 + 2.0 ** -6])


def test_bf16_storage_keeps_the_cache_path_consistent():
    """With bf16 K/V storage the new rows a forward returns are exactly what attention used:
    one pass over a prompt equals two passes through the committed (rounded) cache."""
    import dataclasses
    shape = dataclasses.replace(wl.preset("tiny").model, dtype="bf16")
    w = wl.make_weights(shape)
    prompt = wl.zipf_prompt(shape.vocab, 20)
    kv = orc.KVCache.empty(shape, 32)
    full, _, k_all, v_all = orc.forward_rows(w, shape, prompt, np.arange(20), np.tril(np.ones((20, 20), bool)), kv)
    assert np.array_equal(k_all, orc.kv_storage(k_all, "bf16"))
    kv.k[:, :12], kv.v[:, :12], kv.n = k_all[:, :12], v_all[:, :12], 12
    part, _, _, _ = orc.forward_rows(w, shape, prompt[12:], np.arange(12, 20), np.tril(np.ones((8, 8), bool)), kv)
    assert np.abs(part - full[12:]).max() < 1e-11
