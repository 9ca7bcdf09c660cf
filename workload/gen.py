"""Seeded generators for every input of the speculative-decoding step.

Nothing here computes any part of the method (no forward pass, no acceptance, no tree
assembly from candidates): these functions only draw the numbers and shapes that the method
consumes. They stand in for inputs the paper uses but which are not available: trained
CodeLlama-7b weights and draft heads (Section IV-A), the 575 Verilog speed prompts
(Section IV-B) and the set of syntactically significant token ids (Section III-C).
"""
from __future__ import annotations

import heapq
import math
import zlib

import numpy as np
import torch

from .configs import ModelShape

# One seed per input family, so inputs can be regenerated independently.
SEEDS = {"weights": 1234, "prompt": 1, "stop": 2, "kvfill": 3, "force": 4, "kvlen": 5, "labels": 6}


# --------------------------------------------------------------------------- numeric helpers
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _torch_gen(seed: int, name: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + zlib.crc32(name.encode())) % (2**63 - 1))
    return g


def _normal(seed, name, shape, std, dtype, device) -> torch.Tensor:
    g = _torch_gen(seed, name, device)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, std, generator=g)
    return t.to(dtype)


# --------------------------------------------------------------------------- weights
def weight_names(m: ModelShape):
    names = ["embed", "lm_head", "final_norm"]
    for l in range(m.n_layers):
        names += [f"l{l}.attn_norm", f"l{l}.wqkv", f"l{l}.wo",
                  f"l{l}.ffn_norm", f"l{l}.w_gate", f"l{l}.w_up", f"l{l}.w_down"]
    for i in range(m.n_medusa):
        names += [f"medusa{i}.w", f"medusa{i}.b"]
    return names


def weight_shape(m: ModelShape, name: str):
    d, F, V = m.d_model, m.d_ffn, m.vocab
    base = name.split(".")[-1]
    if name in ("embed", "lm_head"):
        return (V, d)
    if base in ("final_norm", "attn_norm", "ffn_norm", "b"):
        return (d,)
    return {"wqkv": (3 * d, d), "wo": (d, d), "w_gate": (F, d), "w_up": (F, d),
            "w_down": (d, F), "w": (d, d)}[base]


def make_weights(m: ModelShape, seed: int = SEEDS["weights"], device="cpu",
                 medusa_bias_std: float = 0.0, std: float = 0.02) -> dict[str, torch.Tensor]:
    """Random-initialised weights, every matrix stored [out_features, in_features].

    Matrices ~ N(0, std^2); RMSNorm gains are 1; draft-head biases are 0 unless
    `medusa_bias_std` > 0. `wqkv` stacks the q, k and v projections along the output axis.
    For dtype "bf16" the values are rounded to bfloat16 once, here, so every consumer reads
    identical numbers.
    """
    dt = torch.bfloat16 if m.dtype == "bf16" else torch.float32
    w = {}
    for name in weight_names(m):
        shape = weight_shape(m, name)
        base = name.split(".")[-1]
        if base in ("final_norm", "attn_norm", "ffn_norm"):
            w[name] = torch.ones(shape, dtype=dt, device=device)
        elif base == "b":
            if medusa_bias_std > 0:
                w[name] = _normal(seed, name, shape, medusa_bias_std, dt, device)
            else:
                w[name] = torch.zeros(shape, dtype=dt, device=device)
        else:
            w[name] = _normal(seed, name, shape, std, dt, device)
    return w


def synthetic_kv_rows(seed: int, tag: str, shape, dtype: str, device="cpu",
                      std: float = 0.5) -> torch.Tensor:
    """I.i.d. N(0, std^2) rows that stand in for already-rotated cached keys / values."""
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return _normal(seed, "kv." + tag, shape, std, dt, device)


# --------------------------------------------------------------------------- integer inputs
def zipf_prompt(vocab: int, length: int, seed: int = SEEDS["prompt"], s: float = 1.1) -> np.ndarray:
    """Token ids with P(id = r) proportional to (r+1)^-s, by inverse CDF in float64."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    p = (np.arange(1, vocab + 1, dtype=np.float64)) ** (-s)
    cdf = np.cumsum(p)
    cdf /= cdf[-1]
    u = rng.random(length)
    return np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)


def frag_filled_labels(batch: int, seq: int, vocab: int, frag_id: int, pad_id: int, mean_fragment: float = 4.0,
                       min_fill: float = 0.5, seed: int = SEEDS["labels"]) -> np.ndarray:
    """Base-model label rows [batch, seq]: Zipf token ids with `frag_id` inserted after fragments whose lengths are
    geometric with the given mean (identifiers, keywords and operators are a few tokens each); every sequence holds
    between min_fill*seq and seq such entries and is filled up with `pad_id`. Ids equal to frag_id / pad_id never
    occur as ordinary tokens."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = np.full((batch, seq), pad_id, dtype=np.int32)
    for b in range(batch):
        n = int(rng.integers(int(min_fill * seq), seq + 1))
        toks = zipf_prompt(vocab, n, seed=seed * 1000 + b)
        toks = np.where((toks == frag_id) | (toks == pad_id), 0, toks)
        row, i = [], 0
        while len(row) < n:
            L = int(rng.geometric(1.0 / mean_fragment))
            row.extend(toks[i: i + L].tolist())
            row.append(frag_id)
            i += L
        out[b, :n] = row[:n]
    return out


def stop_set(vocab: int, frac: float = 0.2, seed: int = SEEDS["stop"]) -> np.ndarray:
    """Boolean [vocab]: exactly floor(frac*vocab) ids flagged as syntactically significant."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    mask = np.zeros(vocab, dtype=bool)
    mask[rng.permutation(vocab)[: int(math.floor(frac * vocab))]] = True
    return mask


def pack_mask_words(mask: np.ndarray) -> np.ndarray:
    """Boolean [V] -> uint32 words, bit (id % 32) of word (id // 32)."""
    V = mask.shape[0]
    padded = np.zeros(((V + 31) // 32) * 32, dtype=np.uint8)
    padded[:V] = mask
    return np.packbits(padded.reshape(-1, 32), axis=1, bitorder="little").view("<u4").reshape(-1).copy()


# --------------------------------------------------------------------------- tree shapes
def default_tree(T: int, H: int, k: int):
    """Fixed candidate-tree shape with T nodes (root included), depth <= H, rank < k.

    Best-first growth: a node reached through head ranks (r_1..r_d) scores
    prod_j 0.6 * 0.5^{r_j}; the T-1 best-scoring nodes are kept (ties: smaller depth, then
    lexicographically smaller rank tuple). A node's ancestors always outscore it, so the
    kept set is a tree. Nodes are numbered depth-major, so parent[j] < j.
    Returns int32 arrays (parent, depth, rank); parent[0] = -1, rank[0] = 0.
    """
    def score(t):
        return -(len(t) * math.log(0.6) + sum(t) * math.log(0.5))

    heap = [(score((r,)), 1, (r,)) for r in range(k)] if H >= 1 else []
    heapq.heapify(heap)
    kept = [()]
    while len(kept) < T:
        if not heap:
            raise ValueError(f"a tree with depth<={H}, rank<{k} has fewer than {T} nodes")
        _, d, t = heapq.heappop(heap)
        kept.append(t)
        if d < H:
            for r in range(k):
                heapq.heappush(heap, (score(t + (r,)), d + 1, t + (r,)))
    kept.sort(key=lambda t: (len(t), t))
    index = {t: i for i, t in enumerate(kept)}
    parent = np.array([-1] + [index[t[:-1]] for t in kept[1:]], dtype=np.int32)
    depth = np.array([len(t) for t in kept], dtype=np.int32)
    rank = np.array([0] + [t[-1] for t in kept[1:]], dtype=np.int32)
    return parent, depth, rank


def chain_tree(T: int, rank: int = 0):
    """A single path root -> ... of T nodes, every draft node taking head rank `rank`."""
    parent = np.arange(-1, T - 1, dtype=np.int32)
    depth = np.arange(T, dtype=np.int32)
    r = np.full(T, rank, dtype=np.int32)
    r[0] = 0
    return parent, depth, r


def full_tree(H: int, k: int):
    """The complete k-ary tree of depth H (every rank combination), depth-major."""
    tuples = [()]
    level = [()]
    for _ in range(H):
        level = [t + (r,) for t in level for r in range(k)]
        tuples += level
    index = {t: i for i, t in enumerate(tuples)}
    parent = np.array([-1] + [index[t[:-1]] for t in tuples[1:]], dtype=np.int32)
    depth = np.array([len(t) for t in tuples], dtype=np.int32)
    rank = np.array([0] + [t[-1] for t in tuples[1:]], dtype=np.int32)
    return parent, depth, rank


# --------------------------------------------------------------------------- planted drafts
def plant_drafts(cand: np.ndarray, truth: np.ndarray, p_depth, rng: np.random.Generator,
                 rank_probs=(0.6, 0.25, 0.15)) -> np.ndarray:
    """Overwrite some draft candidates with the known continuation.

    `cand` is [H, k] (head i's candidates, best first); `truth[d-1]` is the token that plain
    greedy decoding emits d positions after the root token. With probability p_depth[d-1]
    head d-1's list gets truth[d-1] at a rank drawn from `rank_probs`; planting stops at the
    first depth that is not planted, so what is planted is a prefix of the continuation.
    Candidates of one head stay distinct. This only edits an *input* of the step; whether
    and how far the planted tokens are accepted is for the method to decide.
    """
    out = np.array(cand, dtype=np.int32, copy=True)
    H, k = out.shape
    ranks = np.arange(len(rank_probs))
    for d in range(min(H, len(truth))):
        if rng.random() >= p_depth[d]:
            break
        r = int(rng.choice(ranks, p=np.asarray(rank_probs) / np.sum(rank_probs)))
        r = min(r, k - 1)
        t = int(truth[d])
        dup = np.nonzero(out[d] == t)[0]
        if dup.size:
            out[d, dup[0]] = out[d, r]
        out[d, r] = t
    return out
