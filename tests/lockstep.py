"""Lock-step comparison of the HIP path with the CPU oracle (helper for the GPU parity tests).

Both sides get the same committed history and the same draft state at every step; each keeps
its own KV cache. Floating-point outputs are compared within the stated tolerances; integer
outputs must be bit-exact given the same arg-max, and the arg-max itself may differ only where
the oracle's top-2 logit margin is below 1e-2 (counted and reported; the cache and draft state
are then resynchronised from the oracle).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import contextlib

import numpy as np
import torch

import paper_2503_14153_amd as sd
from oracle import specdec_oracle as orc

LOGIT_MAX_ABS = 2e-2      # max-abs error of the base logits
LOGIT_REL = 1e-2          # Frobenius-norm relative error of the base logits
NEAR_TIE = 1e-2           # oracle top-2 margin below which an arg-max flip is tolerated


def weights_to_f64(weights: dict) -> dict:
    """Widen once, so the oracle does not re-convert every matrix at every call."""
    return {k: v.detach().cpu().double().numpy() for k, v in weights.items()}


@dataclass
class Report:
    steps: int = 0
    max_abs: float = 0.0
    max_rel: float = 0.0
    near_tie_flips: int = 0
    cand_near_ties: int = 0
    accepted: list = field(default_factory=list)
    raw: list = field(default_factory=list)
    kv_max_abs: float = 0.0
    kv_flipped: float = 0.0         # largest share of committed K/V entries that differ by one bfloat16 spacing
    head_max_abs: float = 0.0
    accept_near_ties: int = 0       # typical acceptance: decisions that differ at an oracle near-tie
    root_near_ties: int = 0         # sampled next root differs with u near a boundary of the oracle's CDF
    stats_max_abs: float = 0.0


def check_logits(got: np.ndarray, want: np.ndarray, rep: Report, max_abs=LOGIT_MAX_ABS, rel=LOGIT_REL):
    err = float(np.abs(got - want).max())
    r = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    rep.max_abs, rep.max_rel = max(rep.max_abs, err), max(rep.max_rel, r)
    assert err <= max_abs, f"logits max-abs error {err:.4g} > {max_abs}"
    assert r <= rel, f"logits relative error {r:.4g} > {rel}"


def check_cand(got: np.ndarray, want: np.ndarray, head_logits: np.ndarray, rep: Report):
    """Top-k candidates: identical, except where the oracle's logits are within NEAR_TIE."""
    for i in range(want.shape[0]):
        for r in range(want.shape[1]):
            if got[i, r] != want[i, r]:
                gap = abs(head_logits[i, want[i, r]] - head_logits[i, got[i, r]])
                assert gap < NEAR_TIE, f"head {i} rank {r}: got id {got[i, r]}, want {want[i, r]}, gap {gap:.4g}"
                rep.cand_near_ties += 1


def bf16_ulp(a: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 numbers (8 significant bits) at the magnitude of every entry of a."""
    m = np.maximum(np.abs(a), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(m)) - 7)


# The relative error with which an evaluation in float32 reaches a K/V entry before it is rounded to the storage
# format: the HIP path's GEMM operands are two-term bfloat16 expansions (16 mantissa bits, error 2^-17 per activation,
# independent in sign), which over a random-sign contraction leave 2^-17 / sqrt(3) of the result.
KV_PRE_ROUNDING_EPS = 2.0 ** -17 / np.sqrt(3.0)


@contextlib.contextmanager
def perturbed_kv_rounding(eps: float, seed: int = 12345):
    """Inside the block the oracle multiplies every K/V row by (1 + eps * N(0, 1)) BEFORE rounding it to the cache's
    storage format; everything else stays float64. Two such evaluations differ exactly where the rounding decisions
    of a bfloat16 cache differ, which is what separates ANY float32 implementation from the oracle once the depth is
    large: the difference it leaves in the logits is the oracle's own sensitivity, the floor under every tolerance."""
    orig = orc.kv_storage
    rng = np.random.default_rng(seed)
    orc.kv_storage = lambda a, dtype: orig(np.asarray(a) * (1.0 + eps * rng.standard_normal(np.shape(a))), dtype)
    try:
        yield
    finally:
        orc.kv_storage = orig


KV_UNROUNDED = LOGIT_MAX_ABS / 2      # bound on the difference of the two sides' K/V entries BEFORE storage rounding


def kv_rows_close(got: np.ndarray, want: np.ndarray, extra: float = 0.0):
    """Committed K/V rows against the oracle's. Both sides round (nearly) the same real number to bfloat16,
    one from a float32 computation, one from a float64 one. Before rounding the two differ by what the
    arithmetic differs: the entries are sums of the same kind as the logits (a normalised row times
    N(0, 0.02^2) weights) and are bounded like them; they sit earlier in the network (the worst seen over
    some 10^5 entries per step is 8e-3 in a second layer, where a flipped rounding of a first-layer K/V entry
    already feeds in), so KV_UNROUNDED = half the logits bound. Rounding then moves each side by at most half
    a spacing, and where the two
    unrounded values fall on either side of a rounding boundary the stored numbers differ by one whole
    spacing. Bound per entry: one bfloat16 spacing at the larger magnitude + KV_UNROUNDED (+ `extra` when
    the oracle's rows are not rounded at all). Returns (largest difference, share of entries that differ)."""
    diff = np.abs(got - want)
    extra = extra + KV_UNROUNDED
    allowed = bf16_ulp(np.maximum(np.abs(got), np.abs(want))) + extra
    bad = diff > allowed
    assert not bad.any(), (f"{int(bad.sum())} committed K/V entries differ by more than one bfloat16 spacing "
                           f"(+{extra}); worst {float(diff.max()):.4g} where {float(allowed[np.unravel_index(diff.argmax(), diff.shape)]):.4g} is allowed")
    return float(diff.max()), float(np.mean(diff > 0))


def compare_kv_rows(kv: sd.KVCache, st: orc.DecodeState, shape, row0: int, row1: int, rep: Report, extra: float = 0.0,
                    seq: int = 0):
    for layer in range(shape.n_layers):
        k, v = kv.read_rows(layer, seq, row0, row1 - row0)
        dk, fk = kv_rows_close(k.float().cpu().numpy().astype(np.float64), st.kv.k[layer, row0:row1], extra)
        dv, fv = kv_rows_close(v.float().cpu().numpy().astype(np.float64), st.kv.v[layer, row0:row1], extra)
        rep.kv_max_abs = max(rep.kv_max_abs, dk, dv)
        rep.kv_flipped = max(rep.kv_flipped, fk, fv)
        # differing entries are rounding decisions near a boundary (a few per cent at these error levels; another
        # rounding mode on either side, e.g. truncation, would make about half of them differ)
        # (a float32 cache holds unrounded rows: nearly every entry differs from the float64 one in its last bits)
        assert extra > 0 or shape.dtype == "f32" or max(fk, fv) < 0.25, \
            f"layer {layer}: {max(fk, fv):.1%} of the committed K/V entries differ"


def resync_kv_rows(kv: sd.KVCache, st: orc.DecodeState, shape, row0: int, seq: int = 0):
    """Overwrite the GPU cache rows of sequence `seq` from row0 on with the oracle's."""
    n = st.kv.n
    if n > row0:
        for layer in range(shape.n_layers):
            k = torch.from_numpy(st.kv.k[layer, row0:n]).to(kv.model.torch_dtype).cuda().contiguous()
            v = torch.from_numpy(st.kv.v[layer, row0:n]).to(kv.model.torch_dtype).cuda().contiguous()
            kv.write_rows(layer, seq, row0, k, v)


def resync_kv(kv: sd.KVCache, st: orc.DecodeState, shape, row0: int):
    """Batch 1: overwrite the GPU cache rows from row0 on with the oracle's and adopt its length."""
    resync_kv_rows(kv, st, shape, row0)
    kv.set_len([st.kv.n])


def check_step_outputs(out, b: int, rec, tree_np, stop_np, fallback: str, shape, rep: Report,
                       logit_max_abs: float = LOGIT_MAX_ABS):
    """Compare sequence b of one GPU step with the oracle's record of the same step.

    Logits within tolerance; arg-max equal except at oracle near-ties; accepted length, tokens
    and source slots bit-exact against the oracle's rule applied to the arg-max the GPU saw.
    Returns (accepted length, accepted chain) as the GPU must have computed them."""
    parent, depth, rank = tree_np
    check_logits(out.logits[b].cpu().numpy().astype(np.float64), rec.logits, rep, max_abs=logit_max_abs)
    am = out.argmax[b].cpu().numpy()
    flips = np.nonzero(am != rec.am)[0]
    for j in flips:
        assert rec.margin[j] < NEAR_TIE, f"arg-max differs at node {j} with oracle margin {rec.margin[j]:.4g}"
    rep.near_tie_flips += len(flips)
    ok, chain = orc.greedy_accept(rec.tok, am, parent, depth)
    n_acc = orc.fragment_cut([rec.tok[c] for c in chain], stop_np, fallback)
    W = shape.n_medusa + 1
    want_tok = np.full(W, -1, np.int32)
    want_slot = np.full(W, -1, np.int32)
    want_tok[:n_acc] = [rec.tok[c] for c in chain[:n_acc]]
    want_slot[:n_acc] = chain[:n_acc]
    assert int(out.n_accept[b]) == n_acc and int(out.n_accept_raw[b]) == len(chain)
    rep.raw.append(len(chain))
    assert np.array_equal(out.tokens[b].cpu().numpy(), want_tok)
    assert np.array_equal(out.src_slots[b].cpu().numpy(), want_slot)
    return n_acc, chain


def lockstep_spec(model: sd.Model, kv: sd.KVCache, tree: sd.Tree, tree_np, stop_np: np.ndarray,
                  stop_words: torch.Tensor, w64: dict, shape, st: orc.DecodeState, n_steps: int, fallback: str,
                  cand_fn=None, kv_tol: float = 0.0, rep: Report | None = None) -> Report:
    """Run n_steps speculative steps on both sides (batch 1). `cand_fn(st)` may edit the draft.
    kv_tol: allowance on top of one bfloat16 spacing for the committed rows (see kv_rows_close)."""
    rep = rep or Report()
    parent, depth, rank = tree_np
    for _ in range(n_steps):
        cand = np.asarray(st.cand if cand_fn is None else cand_fn(st), dtype=np.int32)
        n_old = st.kv.n
        kv.set_draft([st.root_tok], cand[None])
        out = sd.spec_step(model, kv, tree, stop_words, want_logits=True, want_argmax=True, want_head_logits=True)
        rec = orc.spec_step(w64, shape, st, tree_np, stop_np, fallback, cand_override=cand)
        torch.cuda.synchronize()
        n_acc, chain = check_step_outputs(out, 0, rec, tree_np, stop_np, fallback, shape, rep)
        assert kv.len() == [n_old + n_acc]
        rep.accepted.append(n_acc)
        am = out.argmax[0].cpu().numpy()
        same_path = n_acc == rec.n_accept and chain[:n_acc] == list(rec.src_slots)
        # the token that starts the next step is the device's own arg-max at the node it kept last,
        # whichever way a near-tie fell
        root, gcand = kv.get_draft()
        assert int(root[0]) == int(am[chain[n_acc - 1]])
        if same_path:
            compare_kv_rows(kv, st, shape, n_old, n_old + n_acc, rep, kv_tol)
            last = rec.src_slots[-1]
            if am[last] == rec.am[last]:
                assert int(root[0]) == rec.next_root
            hl = out.head_logits[0].cpu().numpy().astype(np.float64)
            herr = float(np.abs(hl - rec.head_logits).max())
            rep.head_max_abs = max(rep.head_max_abs, herr)
            assert herr <= 2 * LOGIT_MAX_ABS, f"draft-head logits differ by {herr:.4g}"
            check_cand(gcand[0].cpu().numpy(), rec.next_cand, rec.head_logits, rep)
        else:
            resync_kv(kv, st, shape, n_old)
        rep.steps += 1
    return rep


# ----------------------------------------------------------------------------- sampling decoding
FP32_LOG_MARGIN = 2e-4    # |log p - log threshold| below which fp32 sums may decide the other way
FP32_CDF = 2e-5           # distance of u from a CDF boundary below which fp32 sums may pick a neighbour


def check_row_stats(stats: np.ndarray, logits64: np.ndarray, ty: dict, rep: Report):
    """{max, Z, H, c} of every row against their definitions evaluated in fp64 on the same logits."""
    for j in range(logits64.shape[0]):
        x = (logits64[j] - logits64[j].max()) / ty["temperature"]
        Z = np.exp(x).sum()
        p = np.exp(x) / Z
        H = orc.entropy(p)
        with np.errstate(divide="ignore"):
            c = min(np.log(ty["epsilon"]), np.log(ty["delta"]) - H) + np.log(Z)
        want = np.array([logits64[j].max(), Z, H, c])
        err = np.abs(stats[j].astype(np.float64) - want)
        err[1] /= Z                                             # Z: relative
        if not np.isfinite(c):
            assert stats[j, 3] == want[3]
            err[3] = 0.0
        rep.stats_max_abs = max(rep.stats_max_abs, float(err.max()))
        assert err[0] == 0.0 and err.max() < 1e-4, f"row {j}: stats {stats[j]} vs {want}"


def typical_outputs_from_logits(tok, logits64, tree_np, stop_np, fallback, ty):
    parent, depth, rank = tree_np
    ok, chain, log_margin = orc.typical_accept(tok, logits64, parent, depth, ty["temperature"], ty["epsilon"],
                                               ty["delta"])
    n_acc = orc.fragment_cut([tok[c] for c in chain], stop_np, fallback)
    return ok, chain, log_margin, n_acc


def check_typical_decision(got_n_raw, got_n_acc, got_tokens, got_slots, tok, logits64, tree_np, stop_np, fallback, ty,
                           H, rep: Report, tol=FP32_LOG_MARGIN):
    """The GPU's acceptance outputs against the oracle's rule on the very logits the GPU used.

    Bit-exact unless some node's own test lies within `tol` of its threshold (then the outputs
    must equal the oracle's for one of the ways those few tests can fall). Returns the chain."""
    parent, depth, rank = tree_np
    ok, chain, lm, n_acc = typical_outputs_from_logits(tok, logits64, tree_np, stop_np, fallback, ty)
    W = H + 1

    def pack(chain, n_acc):
        t, s = np.full(W, -1, np.int32), np.full(W, -1, np.int32)
        t[:n_acc] = [tok[c] for c in chain[:n_acc]]
        s[:n_acc] = chain[:n_acc]
        return len(chain), n_acc, t, s

    def same(w):
        return (got_n_raw == w[0] and got_n_acc == w[1] and np.array_equal(got_tokens, w[2])
                and np.array_equal(got_slots, w[3]))

    if same(pack(chain, n_acc)):
        return chain[:n_acc]
    close = [j for j in range(1, len(parent)) if abs(lm[j]) < tol]
    assert close and len(close) <= 8, f"typical acceptance differs with no test near its threshold (got n_raw " \
                                      f"{got_n_raw}, want {len(chain)})"
    T = len(parent)
    p_tok = np.array([np.inf] + [lm[j] for j in range(1, T)])
    for bits in range(1, 1 << len(close)):
        match = p_tok > 0
        for i, j in enumerate(close):
            if (bits >> i) & 1:
                match[j] = not match[j]
        okf = np.zeros(T, bool)
        okf[0] = True
        for j in range(1, T):
            okf[j] = okf[parent[j]] and match[j]
        best = 0
        for j in range(T):
            if okf[j] and depth[j] > depth[best]:
                best = j
        ch, i = [], best
        while i >= 0:
            ch.append(i)
            i = parent[i]
        ch = ch[::-1]
        na = orc.fragment_cut([tok[c] for c in ch], stop_np, fallback)
        if same(pack(ch, na)):
            rep.accept_near_ties += 1
            return ch[:na]
    raise AssertionError("typical acceptance differs beyond what the near-threshold tests explain")


def check_sampled(got: int, logits_row64: np.ndarray, u: float, temperature: float, tol: float) -> bool:
    """True if `got` is the inverse-CDF draw at u, or u is within tol of got's CDF interval."""
    p = orc.softmax_t(logits_row64, temperature)
    if got == orc.sample_token(p, u):
        return True
    F = np.cumsum(p)
    lo = F[got - 1] if got > 0 else 0.0
    assert lo - tol <= u < F[got] + tol, f"sampled id {got}: u={u} outside [{lo}, {F[got]}) by more than {tol}"
    return False


def lockstep_typical(model: sd.Model, kv: sd.KVCache, tree: sd.Tree, tree_np, stop_np: np.ndarray,
                     stop_words: torch.Tensor, w64: dict, shape, st: orc.DecodeState, n_steps: int, fallback: str,
                     ty: dict, rng: np.random.Generator, cand_fn=None, kv_tol: float = 0.0,
                     rep: Report | None = None) -> Report:
    """Sampling decoding on both sides (batch 1): typical acceptance and a sampled next root.

    Two comparisons per step. (1) The GPU's decisions against the oracle's rule applied, in
    fp64, to the GPU's own logits: exact up to fp32 summation (FP32_* margins). (2) The GPU
    step against the oracle's step on its own fp64 logits: logits within tolerance, decisions
    equal unless the oracle's margin is below what this step's measured logit differences can move."""
    rep = rep or Report()
    tau = ty["temperature"]
    for _ in range(n_steps):
        cand = np.asarray(st.cand if cand_fn is None else cand_fn(st), dtype=np.int32)
        n_old = st.kv.n
        u = float(np.float32(rng.random()))
        kv.set_draft([st.root_tok], cand[None])
        out = sd.spec_step_typical(model, kv, tree, stop_words, torch.tensor([u], dtype=torch.float32, device="cuda"),
                                   temperature=tau, epsilon=ty["epsilon"], delta=ty["delta"], want_logits=True,
                                   want_argmax=True, want_head_logits=True, want_row_stats=True)
        rec = orc.spec_step(w64, shape, st, tree_np, stop_np, fallback, cand_override=cand, typical=dict(ty, u=u))
        torch.cuda.synchronize()
        g_logits = out.logits[0].cpu().numpy().astype(np.float64)
        check_logits(g_logits, rec.logits, rep)
        # how far this step's logit differences can move a log-probability (the token's logit and log Z each by
        # err / tau), the log-threshold (through the entropy, by about as much again), and a cumulative probability
        err = float(np.abs(g_logits - rec.logits).max())
        logit_margin = 4 * err / tau + FP32_LOG_MARGIN
        cdf_margin = float(np.expm1(2 * err / tau)) + FP32_CDF
        check_row_stats(out.row_stats[0].cpu().numpy(), g_logits, ty, rep)
        n_raw, n_acc = int(out.n_accept_raw[0]), int(out.n_accept[0])
        kept = check_typical_decision(n_raw, n_acc, out.tokens[0].cpu().numpy(), out.src_slots[0].cpu().numpy(),
                                      rec.tok, g_logits, tree_np, stop_np, fallback, ty, shape.n_medusa, rep)
        assert kv.len() == [n_old + n_acc]
        rep.accepted.append(n_acc)
        rep.raw.append(n_raw)
        root, gcand = kv.get_draft()
        root = int(root[0])
        if not check_sampled(root, g_logits[kept[-1]], u, tau, FP32_CDF):
            rep.root_near_ties += 1
        same_path = n_acc == rec.n_accept and kept == list(rec.src_slots)
        if same_path:
            compare_kv_rows(kv, st, shape, n_old, n_old + n_acc, rep, kv_tol)
            if not check_sampled(root, rec.logits[kept[-1]], u, tau, cdf_margin):
                rep.root_near_ties += 1
            hl = out.head_logits[0].cpu().numpy().astype(np.float64)
            herr = float(np.abs(hl - rec.head_logits).max())
            rep.head_max_abs = max(rep.head_max_abs, herr)
            assert herr <= 2 * LOGIT_MAX_ABS, f"draft-head logits differ by {herr:.4g}"
            check_cand(gcand[0].cpu().numpy(), rec.next_cand, rec.head_logits, rep)
        else:
            # the two sides took different paths: only legitimate at an oracle near-tie
            lm = rec.log_margin
            assert np.any(np.abs(lm[1:]) < logit_margin), "paths differ with every oracle margin clear of its threshold"
            rep.accept_near_ties += 1
            resync_kv(kv, st, shape, n_old)
        rep.steps += 1
    return rep
