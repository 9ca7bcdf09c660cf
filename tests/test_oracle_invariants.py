"""Pins for the oracle's step loop: properties the method must have whatever the inputs.

  * lossless greedy: the token stream of speculative steps equals plain next-token greedy
    decoding from the same prompt (the paper builds on Medusa-1's lossless acceleration,
    Section II-B; any prefix of a greedy-verified run is greedy output, so the fragment cut
    of Section III-B keeps this);
  * verifying a tree in one pass equals running every root-to-node path by itself;
  * a single-chain tree is sequential decoding;
  * the cache after compaction equals the cache of sequential decoding.
"""
import numpy as np
import pytest

import workload as wl
from oracle import specdec_oracle as orc

W = wl.preset("tiny")
SHAPE = W.model
WEIGHTS = wl.make_weights(SHAPE)
PROMPT = wl.zipf_prompt(SHAPE.vocab, 24)
STOP = wl.stop_set(SHAPE.vocab, 0.2)


@pytest.fixture(scope="module")
def greedy_run():
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, 128)
    recs = [orc.greedy_step(WEIGHTS, SHAPE, st) for _ in range(60)]
    return st, recs


def test_plain_greedy_is_argmax_of_a_fresh_full_forward(greedy_run):
    """Plain greedy through the cache == recomputing the whole sequence from scratch."""
    st, _ = greedy_run
    seq = list(PROMPT)
    for _ in range(6):
        kv = orc.KVCache.empty(SHAPE, 1)
        P = len(seq)
        lg, _, _, _ = orc.forward_rows(WEIGHTS, SHAPE, np.array(seq), np.arange(P), np.tril(np.ones((P, P), bool)), kv)
        seq.append(int(np.argmax(lg[-1])))
    assert seq[len(PROMPT):] == st.emitted[:6]


@pytest.mark.parametrize("fallback", ["keep_all", "keep_one"])
@pytest.mark.parametrize("tree_kind", ["default16", "full", "chain"])
def test_lossless_with_random_heads(greedy_run, fallback, tree_kind):
    truth = greedy_run[0].emitted
    tree = {"default16": wl.default_tree(16, 3, 4), "full": wl.full_tree(2, 4),
            "chain": wl.chain_tree(4)}[tree_kind]
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, 128)
    for _ in range(8):
        orc.spec_step(WEIGHTS, SHAPE, st, tree, STOP, fallback)
    assert st.emitted == truth[: len(st.emitted)]


@pytest.mark.parametrize("fallback,stop_frac", [("keep_all", 0.2), ("keep_one", 0.2), ("keep_all", 0.0),
                                                ("keep_one", 1.0), ("keep_all", 0.6)])
def test_lossless_with_planted_drafts_and_cache_equals_sequential(greedy_run, fallback, stop_frac):
    g_state, g_recs = greedy_run
    truth = g_state.emitted
    stop = wl.stop_set(SHAPE.vocab, stop_frac)
    tree = wl.default_tree(16, 3, 4)
    parent, depth, rank = tree
    paths = {}
    for j in range(16):
        t, i = [], j
        while i > 0:
            t.append(int(rank[i]))
            i = parent[i]
        paths[tuple(t[::-1])] = j
    rng = np.random.default_rng(11)
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, 128)
    raw_lengths, cut_lengths = [], []
    for _ in range(12):
        e = len(st.emitted)
        assert st.root_tok == truth[e]
        cont = np.array(truth[e + 1: e + 1 + SHAPE.n_medusa])
        cand = wl.plant_drafts(st.cand, cont, (0.9, 0.8, 0.7), rng)
        # closed form for the raw accepted length: follow the planted ranks while the tree has them
        m, ranks = 0, ()
        for d in range(SHAPE.n_medusa):
            r = np.nonzero(cand[d] == cont[d])[0]
            if r.size == 0 or ranks + (int(r[0]),) not in paths:
                break
            ranks += (int(r[0]),)
            m += 1
        rec = orc.spec_step(WEIGHTS, SHAPE, st, tree, stop, fallback, cand_override=cand)
        assert rec.n_accept_raw == m + 1
        assert rec.src_slots[-1] == paths[ranks[: rec.n_accept - 1]]
        raw_lengths.append(rec.n_accept_raw)
        cut_lengths.append(rec.n_accept)
        assert st.emitted == truth[: len(st.emitted)]
        # committed cache == cache of plain sequential decoding of the same tokens
        n = st.kv.n
        assert n == len(PROMPT) + len(st.emitted)
        assert np.abs(st.kv.k[:, :n] - g_state.kv.k[:, :n]).max() < 1e-10
        assert np.abs(st.kv.v[:, :n] - g_state.kv.v[:, :n]).max() < 1e-10
    assert max(raw_lengths) >= 3                       # the planted drafts really were accepted
    if stop_frac == 1.0:
        assert cut_lengths == raw_lengths              # every token is a stop token: no cut
    if stop_frac == 0.0 and fallback == "keep_all":
        assert cut_lengths == raw_lengths
    if stop_frac == 0.2:
        assert any(c < r for c, r in zip(cut_lengths, raw_lengths)) or fallback == "keep_all"


def test_tree_pass_equals_separate_per_path_forwards():
    """Brute force: each root-to-node path run alone as a causal chain gives the node's logits."""
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, 64)
    parent, depth, rank = wl.default_tree(16, 3, 4)
    tok, pos, anc = orc.tree_inputs(st.root_tok, st.cand, parent, depth, rank, st.kv.n)
    logits, h, k_new, v_new = orc.forward_rows(WEIGHTS, SHAPE, tok, pos, anc, st.kv)
    for j in range(16):
        path, i = [], j
        while i >= 0:
            path.append(i)
            i = parent[i]
        path = path[::-1]
        seq = np.concatenate([PROMPT, tok[path]])
        P = len(seq)
        lg, _, k_all, v_all = orc.forward_rows(WEIGHTS, SHAPE, seq, np.arange(P), np.tril(np.ones((P, P), bool)),
                                               orc.KVCache.empty(SHAPE, 1))
        assert np.abs(lg[-1] - logits[j]).max() < 1e-10
        assert np.abs(k_all[:, -1] - k_new[:, j]).max() < 1e-10


def test_chain_tree_equals_sequential_steps(greedy_run):
    g_state, g_recs = greedy_run
    truth = g_state.emitted
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, 64)
    chain = wl.chain_tree(4)
    cand = np.array(st.cand)
    for d in range(3):
        dup = np.nonzero(cand[d] == truth[d + 1])[0]
        if dup.size:
            cand[d, dup[0]] = cand[d, 0]
        cand[d, 0] = truth[d + 1]
    rec = orc.spec_step(WEIGHTS, SHAPE, st, chain, np.zeros(SHAPE.vocab, bool), "keep_all", cand_override=cand)
    for j in range(4):                                  # row j's logits == the j-th sequential step's
        assert np.abs(rec.logits[j] - g_recs[j].logits[0]).max() < 1e-10
    assert rec.n_accept == 4 and list(rec.tokens) == truth[:4]


def test_kv_overflow_is_refused_without_side_effects():
    st = orc.prefill(WEIGHTS, SHAPE, PROMPT, len(PROMPT) + SHAPE.n_medusa)
    before = st.kv.n
    with pytest.raises(OverflowError):
        orc.spec_step(WEIGHTS, SHAPE, st, wl.default_tree(16, 3, 4), STOP)
    assert st.kv.n == before and st.emitted == []
