"""CPU oracle for the syntax-aligned speculative-decoding step (NumPy, float64).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it. It shares no code with the HIP path and never
imports it. It is deliberately plain: one function per step of the method, no blocking, no
fusion, no caching tricks, float64 everywhere, NumPy matmul as the only library primitive.

What it computes follows the paper's decoding description (Section III-B):
  * at position t the base model predicts token t+1 and draft head i predicts token t+i+1;
  * the candidates of a step are the top-k tokens of the base model and of every head;
  * a drafted token is accepted only if it, and every token before it, passes the acceptance
    test; under greedy decoding (one of the two decoding modes of Section IV-A) the test is
    "equals the base model's arg-max given the tokens before it"; under sampling decoding it is
    the typical-acceptance inequality (Section III-B, Eq. 1): the base model's probability of the
    token must exceed min(epsilon, delta * exp(-entropy of the base distribution));
  * the accepted run is then cut back to the end of its last complete syntactic fragment
    (the paper marks fragment ends with a [FRAG] token; here any id in a stop set);
  * the step emits the longest accepted, cut-back prefix over all candidates.
The base model is the Llama-style decoder the paper names (CodeLlama-7b, Section III-B):
RMSNorm, rotary position embedding, multi-head attention, SwiGLU feed-forward. The paper
says nothing about tree attention or the KV cache; verifying all candidates in one forward
pass over a token tree is the Medusa technique the paper builds on, and the invariants that
pin this file (tests/test_oracle_*.py) are exactly that it must not change the result.

Parity pins: every function below is pinned by CPU tests against something other than itself
(library routines, brute force over paths, plain greedy decoding, hand-worked cases); see the
test files named tests/test_oracle_*.py. The seeded input generators (package `workload`)
are inputs, not method arithmetic: parity unpinned for them beyond fixed seeds.

Conventions (readings of points the paper leaves open):
  * every weight matrix is [out_features, in_features]; y = W x;
  * rotary embedding pairs dimension i with i + head_dim/2, angle pos * theta^(-2i/head_dim);
  * attention scale 1/sqrt(head_dim); invisible keys are excluded from the softmax;
  * arg-max ties go to the lowest token id; top-k is by descending logit, ties to lower id;
  * a draft head is h_i = h + SiLU(W_i h + b_i) on the final-norm output h, followed by the
    base model's own LM head;
  * a tree node's token depends only on (depth, rank): tok = cand[depth-1][rank];
  * the cut keeps the stop token itself; when the accepted run holds no stop token the
    whole run is kept ("keep_all") or only its first token ("keep_one");
  * sampling decoding (Section IV-A: temperature 0.8): probabilities are softmax(logits /
    temperature); the root token of a step is always accepted (it was drawn from the base model
    itself at the previous step); among several accepted paths the deepest wins, the lowest node
    index on equal depth; the next root is drawn from the base distribution at the last kept
    node by inverting its cumulative distribution over ascending token ids at a uniform number
    that is an INPUT of the step (the oracle draws nothing itself);
  * precision: the paper loads its models in float16 (Section IV-A) and says nothing else.
    Here a model's `dtype` names a STORAGE format, not an arithmetic: for "bf16" the weights,
    the embeddings and every key/value row exist only as bfloat16 numbers (a K/V row is
    rounded once, when it is produced, and that rounded row is what attention reads in the
    same step and what is committed to the cache); everything computed in between is exact
    up to float64 rounding. For "f32" nothing is rounded.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------- model pieces
def _w(weights, name) -> np.ndarray:
    """Fetch a weight as float64 (weights may hold float32 / widened-bf16 arrays)."""
    a = weights[name]
    if hasattr(a, "detach"):           # a torch CPU tensor: widen without touching values
        a = a.detach().to("cpu").double().numpy()
    return np.asarray(a, dtype=F64)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate x[T, n_heads, head_dim] to positions pos[T] (half-split pairing)."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = F64(theta) ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def kv_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round key/value rows to the cache's storage format (bfloat16: nearest, ties to even)."""
    if dtype != "bf16":
        return a
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape).astype(F64)


def attention(q: np.ndarray, keys: np.ndarray, vals: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """Softmax attention of queries q[T, hd] over keys/vals[S, hd]; visible[T, S] is boolean."""
    hd = q.shape[-1]
    s = (q @ keys.T) / np.sqrt(F64(hd))
    s = np.where(visible, s, -np.inf)
    s = s - np.max(s, axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / np.sum(p, axis=-1, keepdims=True)
    return p @ vals


@dataclass
class KVCache:
    """Committed keys (already rotated) and values: [n_layers, cap, n_heads, head_dim]."""
    k: np.ndarray
    v: np.ndarray
    n: int = 0

    @classmethod
    def empty(cls, shape, cap: int) -> "KVCache":
        dims = (shape.n_layers, cap, shape.n_heads, shape.head_dim)
        return cls(np.zeros(dims, F64), np.zeros(dims, F64), 0)

    def copy(self) -> "KVCache":
        return KVCache(self.k.copy(), self.v.copy(), self.n)


def forward_rows(weights, shape, tok, pos, visible, kv: KVCache):
    """Base-model forward of T new rows on top of the committed cache.

    tok[T] token ids, pos[T] positions, visible[T, T]: row j may attend new row i. Every new
    row also attends all committed rows 0..kv.n-1. The cache is not modified.
    Returns (logits[T, V], h[T, d] = final-norm output, k_new, v_new[L, T, n_heads, hd]).
    """
    T = len(tok)
    nh, hd, d = shape.n_heads, shape.head_dim, shape.d_model
    n = kv.n
    x = _w(weights, "embed")[np.asarray(tok)]
    k_new = np.zeros((shape.n_layers, T, nh, hd), F64)
    v_new = np.zeros((shape.n_layers, T, nh, hd), F64)
    vis_all = np.concatenate([np.ones((T, n), bool), np.asarray(visible, bool)], axis=1)
    for l in range(shape.n_layers):
        a = rmsnorm(x, _w(weights, f"l{l}.attn_norm"), shape.rms_eps)
        qkv = a @ _w(weights, f"l{l}.wqkv").T
        q = rope(qkv[:, :d].reshape(T, nh, hd), pos, shape.rope_theta)
        k = kv_storage(rope(qkv[:, d:2 * d].reshape(T, nh, hd), pos, shape.rope_theta), shape.dtype)
        v = kv_storage(qkv[:, 2 * d:].reshape(T, nh, hd), shape.dtype)
        k_new[l], v_new[l] = k, v
        o = np.zeros((T, nh, hd), F64)
        for h in range(nh):
            keys = np.concatenate([kv.k[l, :n, h], k[:, h]], axis=0)
            vals = np.concatenate([kv.v[l, :n, h], v[:, h]], axis=0)
            o[:, h] = attention(q[:, h], keys, vals, vis_all)
        x = x + o.reshape(T, d) @ _w(weights, f"l{l}.wo").T
        f = rmsnorm(x, _w(weights, f"l{l}.ffn_norm"), shape.rms_eps)
        gate = f @ _w(weights, f"l{l}.w_gate").T
        up = f @ _w(weights, f"l{l}.w_up").T
        x = x + (silu(gate) * up) @ _w(weights, f"l{l}.w_down").T
    h = rmsnorm(x, _w(weights, "final_norm"), shape.rms_eps)
    logits = h @ _w(weights, "lm_head").T
    return logits, h, k_new, v_new


def argmax_lowest(logits: np.ndarray) -> np.ndarray:
    """Row-wise arg-max; np.argmax returns the first (= lowest id) maximum."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def top2_margin(logits: np.ndarray) -> np.ndarray:
    """Row-wise gap between the largest and second-largest logit (for near-tie accounting)."""
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def topk_ids(logits: np.ndarray, k: int) -> np.ndarray:
    """The k ids with the largest logits, descending; equal logits -> lower id first."""
    ids = np.arange(logits.shape[-1])
    order = np.lexsort((ids, -logits))
    return order[:k].astype(np.int32)


def medusa_logits(weights, shape, h_row: np.ndarray) -> np.ndarray:
    """Draft heads on one final-norm row h[d]: logits[H, V] (head i drafts token t+i+2)."""
    lm = _w(weights, "lm_head")
    out = np.zeros((shape.n_medusa, shape.vocab), F64)
    for i in range(shape.n_medusa):
        z = _w(weights, f"medusa{i}.w") @ h_row + _w(weights, f"medusa{i}.b")
        out[i] = lm @ (h_row + silu(z))
    return out


def medusa_candidates(weights, shape, h_row: np.ndarray) -> np.ndarray:
    lg = medusa_logits(weights, shape, h_row)
    return np.stack([topk_ids(lg[i], shape.topk) for i in range(shape.n_medusa)])


# ----------------------------------------------------------------------------- tree pieces
def tree_inputs(root_tok: int, cand: np.ndarray, parent, depth, rank, n: int):
    """Assemble the token tree of one step.

    Node 0 carries the base model's token for position n (the root); node j >= 1 carries
    head (depth[j]-1)'s candidate of rank rank[j]; its position is n + depth[j]; it may
    attend its ancestors and itself.
    """
    T = len(parent)
    tok = np.zeros(T, np.int32)
    pos = np.zeros(T, np.int32)
    anc = np.zeros((T, T), bool)
    for j in range(T):
        tok[j] = root_tok if j == 0 else cand[depth[j] - 1][rank[j]]
        pos[j] = n + depth[j]
        i = j
        while i >= 0:
            anc[j, i] = True
            i = parent[i]
    return tok, pos, anc


def greedy_accept(tok, am, parent, depth):
    """Prefix-closed greedy acceptance over the tree.

    The root is the base model's own token and is always accepted. A drafted node is
    accepted iff its parent is accepted and its token equals the base arg-max at the parent.
    Returns (ok[T], chain) where chain is the root-to-deepest accepted path (deepest accepted
    node; lowest node index on equal depth).
    """
    T = len(parent)
    ok = np.zeros(T, bool)
    ok[0] = True
    for j in range(1, T):
        ok[j] = ok[parent[j]] and tok[j] == am[parent[j]]
    best = 0
    for j in range(T):
        if ok[j] and depth[j] > depth[best]:
            best = j
    chain = []
    i = best
    while i >= 0:
        chain.append(i)
        i = parent[i]
    return ok, chain[::-1]


def fragment_cut(chain_tokens, stop: np.ndarray, fallback: str = "keep_all") -> int:
    """Length kept after cutting an accepted run back to its last complete fragment.

    The run is kept up to and including its last token that lies in the stop set. A run
    without any stop token is kept whole ("keep_all") or reduced to its first token
    ("keep_one"). The result is always in [1, len(run)].
    """
    last = -1
    for j, t in enumerate(chain_tokens):
        if stop[t]:
            last = j
    if last >= 0:
        return last + 1
    return len(chain_tokens) if fallback == "keep_all" else 1


def softmax_t(logits: np.ndarray, temperature: float) -> np.ndarray:
    """softmax(logits / temperature) of one row, in float64."""
    x = np.asarray(logits, F64) / F64(temperature)
    e = np.exp(x - x.max())
    return e / e.sum()


def entropy(p: np.ndarray) -> float:
    """Shannon entropy (natural log) of a probability vector; 0 log 0 = 0."""
    q = p[p > 0]
    return float(-(q * np.log(q)).sum())


def typical_threshold(p: np.ndarray, epsilon: float, delta: float) -> float:
    """Right-hand side of the typical-acceptance inequality (Section III-B, Eq. 1)."""
    return float(min(F64(epsilon), F64(delta) * np.exp(-entropy(p))))


def typical_accept(tok, logits, parent, depth, temperature: float, epsilon: float, delta: float):
    """Prefix-closed typical acceptance over the tree (Section III-B, Eq. 1).

    The root is always accepted. A drafted node is accepted iff its parent is accepted and the
    base model's probability of its token, given the tokens up to its parent, exceeds
    min(epsilon, delta * exp(-H)) with H the entropy of that same distribution. Returns
    (ok[T], chain, log_margin[T]) where chain is the root-to-deepest accepted path (lowest node
    index on equal depth) and log_margin[j] = log p - log threshold of node j's own test.
    """
    T = len(parent)
    ok = np.zeros(T, bool)
    ok[0] = True
    log_margin = np.full(T, np.inf)
    for j in range(1, T):
        p = softmax_t(logits[parent[j]], temperature)
        thr = typical_threshold(p, epsilon, delta)
        pj = p[tok[j]]
        with np.errstate(divide="ignore"):
            log_margin[j] = np.log(pj) - np.log(thr) if thr > 0 else np.inf
        ok[j] = ok[parent[j]] and pj > thr
    best = 0
    for j in range(T):
        if ok[j] and depth[j] > depth[best]:
            best = j
    chain = []
    i = best
    while i >= 0:
        chain.append(i)
        i = parent[i]
    return ok, chain[::-1], log_margin


def sample_token(p: np.ndarray, u: float) -> int:
    """Inverse-CDF draw: the smallest token id whose cumulative probability exceeds u in [0, 1)."""
    acc = F64(0.0)
    last_positive = 0
    for v in range(len(p)):
        if p[v] > 0:
            last_positive = v
        acc += p[v]
        if acc > u:
            return v
    return last_positive            # u at or above the rounded total: the last token that has mass


# ----------------------------------------------------------------------------- decoding state
@dataclass
class DecodeState:
    """What one sequence carries between steps."""
    kv: KVCache
    root_tok: int = 0                      # base arg-max at the last committed position
    cand: np.ndarray | None = None         # [H, k] draft candidates from that same position
    emitted: list = field(default_factory=list)


@dataclass
class StepRecord:
    tok: np.ndarray
    pos: np.ndarray
    logits: np.ndarray
    am: np.ndarray
    ok: np.ndarray
    chain: list
    n_accept_raw: int
    n_accept: int
    tokens: np.ndarray
    src_slots: np.ndarray
    margin: np.ndarray
    next_root: int
    next_cand: np.ndarray
    head_logits: np.ndarray
    log_margin: np.ndarray | None = None   # typical acceptance: log p - log threshold per node


def prefill(weights, shape, prompt, cap: int) -> DecodeState:
    """Run the prompt causally, commit its K/V, and draft from its last position."""
    P = len(prompt)
    kv = KVCache.empty(shape, cap)
    causal = np.tril(np.ones((P, P), bool))
    logits, h, k_new, v_new = forward_rows(weights, shape, prompt, np.arange(P), causal, kv)
    kv.k[:, :P], kv.v[:, :P] = k_new, v_new
    kv.n = P
    st = DecodeState(kv)
    st.root_tok = int(argmax_lowest(logits[-1:])[0])
    st.cand = medusa_candidates(weights, shape, h[-1])
    return st


def spec_step(weights, shape, st: DecodeState, tree, stop: np.ndarray,
              fallback: str = "keep_all", cand_override=None, typical=None) -> StepRecord:
    """One speculative step: draft tree -> one verifying forward -> accept -> cut -> commit.

    `tree` = (parent, depth, rank). `cand_override` replaces the carried draft candidates
    (used to plant known continuations). `typical` = None for greedy acceptance, or a dict
    {temperature, epsilon, delta, u} for sampling decoding: typical acceptance (Eq. 1) and the
    next root drawn at the uniform number u. Updates `st` in place and returns the record.
    """
    parent, depth, rank = tree
    cand = st.cand if cand_override is None else np.asarray(cand_override)
    n = st.kv.n
    if n + shape.n_medusa + 1 > st.kv.k.shape[1]:
        raise OverflowError("KV cache full")
    tok, pos, anc = tree_inputs(st.root_tok, cand, parent, depth, rank, n)
    logits, h, k_new, v_new = forward_rows(weights, shape, tok, pos, anc, st.kv)
    am = argmax_lowest(logits)
    log_margin = None
    if typical is None:
        ok, chain = greedy_accept(tok, am, parent, depth)
    else:
        ok, chain, log_margin = typical_accept(tok, logits, parent, depth, typical["temperature"],
                                               typical["epsilon"], typical["delta"])
    n_raw = len(chain)
    n_acc = fragment_cut([tok[c] for c in chain], stop, fallback)
    kept = chain[:n_acc]
    for j, c in enumerate(kept):          # compaction: node c's row lands at position n + j
        st.kv.k[:, n + j] = k_new[:, c]
        st.kv.v[:, n + j] = v_new[:, c]
    st.kv.n = n + n_acc
    last = kept[-1]
    if typical is None:
        next_root = int(am[last])
    else:
        next_root = sample_token(softmax_t(logits[last], typical["temperature"]), typical["u"])
    head_lg = medusa_logits(weights, shape, h[last])
    rec = StepRecord(
        tok=tok, pos=pos, logits=logits, am=am, ok=ok, chain=chain,
        n_accept_raw=n_raw, n_accept=n_acc,
        tokens=np.array([tok[c] for c in kept], np.int32),
        src_slots=np.array(kept, np.int32),
        margin=top2_margin(logits),
        next_root=next_root,
        log_margin=log_margin,
        next_cand=np.stack([topk_ids(head_lg[i], shape.topk) for i in range(shape.n_medusa)]),
        head_logits=head_lg,
    )
    st.emitted.extend(int(t) for t in rec.tokens)
    st.root_tok, st.cand = rec.next_root, rec.next_cand
    return rec


def greedy_step(weights, shape, st: DecodeState) -> StepRecord:
    """Plain next-token decoding: a step whose tree is the root alone."""
    root_only = (np.array([-1], np.int32), np.array([0], np.int32), np.array([0], np.int32))
    no_stop = np.zeros(shape.vocab, bool)
    return spec_step(weights, shape, st, root_only, no_stop, "keep_all")
