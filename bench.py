#!/usr/bin/env python3
"""Benchmark of the speculative-decoding step on one MI355X.

A "step" is one pass of the whole hot path (tree assembly, embedding, 32 decoder layers with
tree-masked attention over the KV cache, LM head, greedy acceptance with the fragment cut, KV
commit, draft heads + top-k) for one sequence with a 64-node candidate tree, on the
CodeLlama-7b-shaped synthetic workload. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

Timed loop = what a decoding loop does: launch a step, read back the committed length and the
emitted tokens, choose the next step's planted draft candidates. Inputs (weights, cache,
candidate table, stop mask) are resident in HBM before the timed region starts.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def kernel_source_hash(names) -> str:
    """SHA-256 over the code of the named HIP sources (in sorted order): `//` comments, trailing blanks and empty
    lines do not count, so that rewording a comment does not orphan the counters taken with the same code."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in sorted(names):
        h.update(name.encode())
        with open(os.path.join(ROOT, "paper_2503_14153_amd", "csrc", name), "r") as f:
            for line in f:
                code = re.sub(r"//.*$", "", line).rstrip()
                if code:
                    h.update(code.encode())
                    h.update(b"\n")
    return h.hexdigest()


def counted_traffic(profile: str, key: str):
    """HBM-side bytes per launch (read + written) of one kernel, as two rocprofv3 --pmc runs counted them
    (FETCH_SIZE, WRITE_SIZE, scaled by what the same counters read for sd_calib's 1 GiB copy kernel). The
    counter summaries under profiles/ carry the figure on a line `<key>: <bytes>` together with the sources of the
    kernel (`kernel_sources: a.hip b.h ...`) and their hash at the time (`kernel_source_sha256: ...`); a summary
    taken with other sources is not this build's traffic, and the bench line then says null rather than repeat a
    stale number."""
    path = os.path.join(ROOT, "profiles", profile)
    try:
        with open(path) as f:
            lines = [ln.strip() for ln in f]
    except OSError:
        return None
    fields = dict(ln.split(": ", 1) for ln in lines if ": " in ln and " " not in ln.split(": ", 1)[0])
    try:
        if fields["kernel_source_sha256"] != kernel_source_hash(fields["kernel_sources"].split()):
            return None
        return float(fields[key])
    except (KeyError, OSError, ValueError):
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="7b", choices=["7b", "7b-long", "7b-batch8", "13b", "7b-h10", "tiny", "labels", "kv-commit"],
                    help="labels = the training-side label construction alone (not the headline step); "
                         "7b-batch8 = eight ragged sequences, the model's own drafts, step time only")
    ap.add_argument("--draft-schedule", default="after_accept", choices=["after_accept", "all_nodes"],
                    help="all_nodes = draft heads on every tree row inside the verifying pass (measured slower here)")
    ap.add_argument("--layers", type=int, default=None, help="cut the depth (debugging only; result is labelled)")
    ap.add_argument("--draft", default="planted", choices=["planted", "random"])
    ap.add_argument("--decoding", default="greedy", choices=["greedy", "sampling"],
                    help="sampling = typical acceptance and a sampled next root at temperature 0.8 (the paper's "
                         "second decoding setting); drafts are then the model's own heads'")
    ap.add_argument("--sync-every", type=int, default=16,
                    help="steps launched between host synchronisations (1 = wait for every step before the next)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=32)
    ap.add_argument("--fused", action="store_true", help="run the optional persistent layer kernel instead of one launch per stage (measured slower; off by default)")
    ap.add_argument("--graph", action="store_true", help="replay captured HIP graphs instead of launching every kernel (measured: no gain, the step is not host-bound)")
    return ap.parse_args()


def weight_bytes(m, lm_head_reads: int = 2) -> float:
    d, F, V, L, H = m.d_model, m.d_ffn, m.vocab, m.n_layers, m.n_medusa
    # every projection once + LM head twice (tree rows, then the draft-head rows) + draft heads; with the
    # heads on every tree row the LM head is read once per 128-row chunk of head rows instead
    return 2.0 * (L * (4 * d * d + 3 * d * F) + lm_head_reads * V * d + H * d * d)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus {args.gpus} is not "
              f"supported, run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import workload as wl
    import paper_2503_14153_amd as sd

    sd.lib()
    torch.cuda.set_device(0)
    if args.workload == "labels":
        return bench_labels(args, torch, wl, sd)
    if args.workload == "kv-commit":
        return bench_kv_commit(args, torch, wl, sd)
    W = wl.preset(args.workload, args.layers)
    if W.batch > 1:
        return bench_batch(args, torch, wl, sd, W)
    shape = W.model                  # "tiny" is specified in float32 and runs on the float32 path; the others are bf16
    T, H, k = W.tree_nodes, shape.n_medusa, shape.topk
    prompt_len = W.prompt_len

    # ---------------------------------------------------------------- inputs, resident in HBM
    weights = wl.make_weights(shape, device="cuda")
    cpu_keep = None
    if not args.no_cpu_baseline:
        names = ["embed", "lm_head", "final_norm"] + [f"medusa{i}.{x}" for i in range(H) for x in "wb"]
        names += [n for n in weights if n.split(".")[0] in tuple(f"l{i}" for i in range(8))]
        cpu_keep = {n: weights[n].cpu() for n in names}
    model = sd.Model(shape, weights, max_rows=256)       # 256: prompt chunks of 256 rows
    del weights
    torch.cuda.empty_cache()
    kv = sd.KVCache(model, 1, W.kv_cap)
    prompt = wl.zipf_prompt(shape.vocab, prompt_len)
    stop = wl.stop_set(shape.vocab, W.stop_frac)
    stop_words = torch.from_numpy(wl.pack_mask_words(stop).view(np.int32)).cuda()
    tree_np = wl.default_tree(T, H, k)
    tree = sd.Tree(*tree_np, H, k)

    t0 = time.perf_counter()
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), [prompt_len])
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    root0, cand0 = kv.get_draft()
    root0, cand0 = root0.clone(), cand0.clone()

    # ---------------------------------------------------------------- plain greedy on the same GPU
    max_emit = W.kv_cap - prompt_len - (H + 1) - 1
    n_truth = min(max_emit, (max(args.steps + args.warmup, args.sync_every + 2) + 1) * (H + 1) + H + 2)
    model.set_fused(args.fused)
    gout = [sd.greedy_step(model, kv) for _ in range(4)]            # warm-up
    torch.cuda.synchronize()
    n_timed = min(64, (n_truth - 4) // 2)

    def timed_greedy(n):                           # same launch discipline as the speculative loop below
        t0 = time.perf_counter()
        for i in range(n):
            gout.append(sd.greedy_step(model, kv))
            if (i + 1) % max(1, args.sync_every) == 0 or i + 1 == n:
                kv.len()
        return time.perf_counter() - t0

    # plain next-token decoding has no draft heads (the paper's NTP baseline): timed without them; with them (what a
    # speculative step can follow at once) for comparison. The emitted tokens are the same either way.
    model.set_greedy_drafts(False)
    greedy_s = timed_greedy(n_timed)
    model.set_greedy_drafts(True)
    greedy_heads_s = timed_greedy(n_timed)
    for _ in range(n_truth - 4 - 2 * n_timed):
        gout.append(sd.greedy_step(model, kv))
    torch.cuda.synchronize()
    truth = torch.stack([o.tokens[0, 0] for o in gout]).cpu().numpy()
    del gout

    # ---------------------------------------------------------------- planted-draft table
    rng = np.random.default_rng(wl.SEEDS["force"])
    p_depth = tuple(round(max(0.5, 0.9 - 0.05 * i), 2) for i in range(H))
    n_table = len(truth) - H
    table = np.zeros((n_table, H, k), np.int32)
    for e in range(n_table):
        filler = (truth[e + 1: e + 1 + H, None] + 1 + np.arange(k)[None, :]) % shape.vocab   # never the true token
        table[e] = wl.plant_drafts(filler, truth[e + 1: e + 1 + H], p_depth, rng) if args.draft == "planted" else filler
    table_dev = torch.from_numpy(table).cuda()

    def reset():
        kv.set_len([prompt_len])
        kv.set_draft(root0, cand0)

    out = sd.StepOutput(
        torch.empty(1, dtype=torch.int32, device="cuda"), torch.empty((1, H + 1), dtype=torch.int32, device="cuda"),
        torch.empty((1, H + 1), dtype=torch.int32, device="cuda"), torch.empty(1, dtype=torch.int32, device="cuda"))
    forced = torch.zeros((1, H, k), dtype=torch.int32, device="cuda")     # fixed buffer: graphs replay on it
    model.set_graph_mode(args.graph)
    model.set_fused(args.fused)
    model.set_draft_schedule(args.draft_schedule)
    state = {"e": 0, "emitted": 0, "diverged": 0, "resets": 0, "i": 0}
    typical = dict(temperature=0.8, epsilon=0.09, delta=0.3)
    n_u = args.steps + args.warmup + args.profile_steps
    u_dev = torch.from_numpy(np.random.default_rng(wl.SEEDS["force"] + 1).random(n_u).astype(np.float32)).cuda()

    # The loop does not wait for a step before launching the next: the planted candidates of step i are picked on
    # the device from the number of tokens emitted so far (a device counter), and the emitted tokens are logged on
    # the device. Every `sync_every` steps the host synchronises, reads the committed length back (which also
    # refreshes the library's bound on it), checks the logged tokens against the plain-greedy stream and decides
    # whether the cache or the planted table could run out within the next window.
    SYNC = max(1, args.sync_every)
    e_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    tok_log = torch.zeros((SYNC, H + 1), dtype=torch.int32, device="cuda")
    nacc_log = torch.zeros(SYNC, dtype=torch.int32, device="cuda")
    # step j of a window writes its verdict straight into row j of the logs (no copies between the steps)
    slot_log = torch.zeros((SYNC, H + 1), dtype=torch.int32, device="cuda")
    raw_log = torch.zeros(SYNC, dtype=torch.int32, device="cuda")
    outs = [sd.StepOutput(nacc_log[j: j + 1], tok_log[j: j + 1], slot_log[j: j + 1], raw_log[j: j + 1]) for j in range(SYNC)]
    room = min(n_table, W.kv_cap - 1 - prompt_len) - (H + 1)          # e may not exceed this when a step starts
    assert room > SYNC * (H + 1), "sync window too long for this cache"

    def restart():
        reset()
        e_dev.zero_()
        state["e"] = 0

    def close_window(n_in_window):
        """Synchronise, account for the window's steps, restart where needed."""
        if n_in_window == 0:
            return
        torch.cuda.synchronize()
        n_now = kv.len()[0]
        nacc = nacc_log[:n_in_window].cpu().numpy()
        e = state["e"]
        if args.decoding == "greedy":
            toks = tok_log[:n_in_window].cpu().numpy()
            for j in range(n_in_window):
                if not np.array_equal(toks[j, :nacc[j]], truth[e: e + nacc[j]]):
                    state["diverged"] += 1          # an arg-max flipped between the two GPU runs
                    restart()
                    return
                e += int(nacc[j])
                state["emitted"] += int(nacc[j])
        else:                                       # nothing to compare a sampled stream with
            e += int(nacc.sum())
            state["emitted"] += int(nacc.sum())
        assert n_now == prompt_len + e, "device length and logged acceptances disagree"
        state["e"] = e
        if e + SYNC * (H + 1) > room:
            restart()
            state["resets"] += 1

    def run_steps(n):
        done = 0
        while done < n:
            w = min(SYNC, n - done)
            for j in range(w):
                if args.decoding == "sampling":
                    i = state["i"]
                    sd.spec_step_typical(model, kv, tree, stop_words, u_dev[i: i + 1], out=outs[j], **typical)
                    state["i"] = i + 1
                else:
                    torch.index_select(table_dev, 0, e_dev, out=forced)
                    sd.spec_step(model, kv, tree, stop_words, forced_cand=forced, out=outs[j])
                    e_dev.add_(outs[j].n_accept)
            close_window(w)
            done += w

    restart()
    run_steps(args.warmup)
    torch.cuda.synchronize()
    state["emitted"] = 0
    t0 = time.perf_counter()
    run_steps(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    emitted = state["emitted"]
    ms_per_step = elapsed / args.steps * 1e3

    # ---------------------------------------------------------------- per-kernel timing (HIP events)
    model.profile_begin(200000)
    run_steps(args.profile_steps)
    prof = model.profile_end()
    g = prof["gemm"]
    gemm_avg_us = g["ms"] / max(g["launches"], 1) * 1e3
    gemm_gbs = g["bytes"] / max(g["ms"], 1e-9) / 1e6
    a = prof["attn"]
    attn_gbs = a["bytes"] / max(a["ms"], 1e-9) / 1e6

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    # ---------------------------------------------------------------- sampling: replay check
    # there is no reference stream under sampling; the self-check is that a replay from the same state with
    # the same uniform numbers emits the same tokens (run outside the timed region)
    replay_mismatches = None
    if args.decoding == "sampling":
        def sampled_stream(n):
            reset()
            toks = []
            for i in range(n):
                sd.spec_step_typical(model, kv, tree, stop_words, u_dev[i: i + 1], out=out, **typical)
                n_acc = int(out.n_accept.cpu()[0])
                toks.append(out.tokens.cpu()[0, :n_acc].tolist())
            return toks
        n_rep = min(32, n_u)
        first, second = sampled_stream(n_rep), sampled_stream(n_rep)
        replay_mismatches = sum(a != b for a, b in zip(first, second))

    cpu = None
    if cpu_keep is not None:
        cpu = cpu_baseline(wl, shape, cpu_keep, T, tree_np, stop, n_cache=prompt_len,
                           typical=dict(typical, u=0.5) if args.decoding == "sampling" else None)

    kv_bytes = (prompt_len + state["e"] / 2) * 2.0 * shape.d_model * 2 * shape.n_layers
    lm_reads = 2 if args.draft_schedule == "after_accept" else 1 + -(-H * ((T + 31) // 32 * 32) // 128)
    step_bytes = weight_bytes(shape, lm_reads) + kv_bytes
    res = {
        "metric": "verified_tree_tokens_per_s", "value": args.steps * T / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{W.name}: {shape.n_layers}-layer d={shape.d_model} Llama-shaped decoder, "
                               f"{H} draft heads top-{k}, {T}-node tree, batch 1, Zipf prompt {prompt_len}, "
                               f"KV cap {W.kv_cap}, 20% stop ids",
                   "draft_schedule": args.draft_schedule,
                   "decoding": args.decoding, "typical_acceptance": typical if args.decoding == "sampling" else None,
                   "draft_mode": args.draft if args.decoding == "greedy" else "own heads",
                   "planted_accuracy_by_depth": list(p_depth) if (args.draft == "planted" and args.decoding == "greedy") else None},
        "accepted_tokens_per_s": emitted / elapsed, "mean_accepted_len": emitted / args.steps,
        "greedy_tokens_per_s": n_timed / greedy_s, "speedup_vs_greedy": (emitted / elapsed) / (n_timed / greedy_s),
        "greedy_with_draft_heads_tokens_per_s": n_timed / greedy_heads_s,
        "prefill_tokens_per_s": prompt_len / prefill_s,
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
        "diverged_resets": state["diverged"], "sampling_replay_mismatches": replay_mismatches, "hip_graphs": args.graph,
        "sync_every": SYNC,
        "roofline": {"kernel": "k_gemm_sk (weight-streaming MFMA GEMM, all projections)", "bound": "hbm",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": counted_traffic("k_gemm_sk_7b_pmc_traffic.txt", "k_gemm_sk_traffic_bytes_per_launch")
                     if (args.workload == "7b" and args.layers is None and not args.fused) else None,
                     "avg_launch_us": gemm_avg_us,
                     "launches_per_step": g["launches"] / args.profile_steps,
                     "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1)},
        "attention": {"kernel": "k_tree_attn", "achieved_GBs": attn_gbs, "frac_hbm": attn_gbs / HBM_PEAK_GBS,
                      "avg_launch_us": a["ms"] / max(a["launches"], 1) * 1e3},
        "cpu_baseline": cpu,
    }
    if shape.dtype == "f32":
        # the float32 path: plain vector-ALU kernels, launch-bound at this size; no per-kernel events are taken
        Tp = (T + 31) // 32 * 32
        flops = 2.0 * Tp * weight_bytes(shape, 1) / 2.0
        res["roofline"] = {"kernel": "k_f32_linear (whole step; float32 vector-ALU path, launch-bound at this size)",
                           "bound": "alu", "achieved": flops / (ms_per_step * 1e-3) / 1e12, "peak": 157.3,
                           "unit": "TFLOP/s", "frac": flops / (ms_per_step * 1e-3) / 1e12 / 157.3, "traffic": None}
        res["attention"] = None
    print(json.dumps(res))


def bench_batch(args, torch, wl, sd, W):
    """A batch of ragged sequences (configs[3] shape): real prefill of Zipf prompts with lengths drawn in
    [1024, 4096], then speculative steps on the model's own (random-head) drafts. Step time and the per-kernel
    figures only: there is no planted stream, so acceptance is that of untrained heads."""
    shape = dataclasses.replace(W.model, dtype="bf16")
    B, T, H, k = W.batch, W.tree_nodes, shape.n_medusa, shape.topk
    Tp = (T + 31) // 32 * 32
    model = sd.Model(shape, wl.make_weights(shape, device="cuda"), max_rows=B * Tp)
    torch.cuda.empty_cache()
    kv = sd.KVCache(model, B, W.kv_cap)
    rng = np.random.Generator(np.random.Philox(key=wl.SEEDS["kvlen"]))
    lens = [int(x) for x in rng.integers(1024, 4097, size=B)]
    prompt = np.concatenate([wl.zipf_prompt(shape.vocab, n, seed=wl.SEEDS["prompt"] + b) for b, n in enumerate(lens)])
    stop_words = torch.from_numpy(wl.pack_mask_words(wl.stop_set(shape.vocab, W.stop_frac)).view(np.int32)).cuda()
    tree = sd.Tree(*wl.default_tree(T, H, k), H, k)
    t0 = time.perf_counter()
    sd.prefill(model, kv, torch.from_numpy(prompt).cuda(), lens)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    root0, cand0 = (t.clone() for t in kv.get_draft())
    out = sd.StepOutput(
        torch.empty(B, dtype=torch.int32, device="cuda"), torch.empty((B, H + 1), dtype=torch.int32, device="cuda"),
        torch.empty((B, H + 1), dtype=torch.int32, device="cuda"), torch.empty(B, dtype=torch.int32, device="cuda"))
    model.set_graph_mode(args.graph)
    model.set_fused(args.fused)
    model.set_draft_schedule(args.draft_schedule)
    room = (W.kv_cap - 1 - max(lens)) // (H + 1)           # steps before the longest sequence could fill its cache
    state = {"left": room, "emitted": 0}

    def run_steps(n):
        for _ in range(n):
            if state["left"] <= 0:
                kv.set_len(lens)
                kv.set_draft(root0, cand0)
                state["left"] = room
            sd.spec_step(model, kv, tree, stop_words, out=out)
            state["emitted"] += sum(kv.len())              # synchronises the stream
            state["left"] -= 1

    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    model.profile_begin(200000)
    run_steps(args.profile_steps)
    prof = model.profile_end()
    g, a = prof["gemm"], prof["attn"]
    gemm_gbs = g["bytes"] / max(g["ms"], 1e-9) / 1e6
    print(json.dumps({
        "metric": "verified_tree_tokens_per_s", "value": args.steps * B * T / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{W.name}: {shape.n_layers}-layer d={shape.d_model} Llama-shaped decoder, {H} draft "
                               f"heads top-{k}, {T}-node trees, batch {B}, Zipf prompts of {lens} tokens, KV cap "
                               f"{W.kv_cap}, 20% stop ids",
                   "draft_schedule": args.draft_schedule, "decoding": "greedy", "draft_mode": "own heads"},
        "prefill_tokens_per_s": sum(lens) / prefill_s, "hip_graphs": args.graph,
        "roofline": {"kernel": "k_gemm_sk (weight-streaming MFMA GEMM, all projections)", "bound": "hbm",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": None, "avg_launch_us": g["ms"] / max(g["launches"], 1) * 1e3,
                     "launches_per_step": g["launches"] / args.profile_steps,
                     "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1)},
        "attention": {"kernel": "k_tree_attn", "achieved_GBs": a["bytes"] / max(a["ms"], 1e-9) / 1e6,
                      "avg_launch_us": a["ms"] / max(a["launches"], 1) * 1e3},
        "cpu_baseline": None}))


def bench_kv_commit(args, torch, wl, sd):
    """The commit of accepted K/V rows (the last stage of a step) under stress: the batched 7B shape (8 sequences
    of 32-node trees, 32 layers, lengths in [1024, 4096]) with every sequence accepting H + 1 = 5 tree rows, and a
    long list (all 32 tree rows of every sequence). In a step the stage moves at most 2.6 MB per sequence and is
    bound by its launch; here it is timed alone, launch after launch, with HIP events on the launch stream.
    Algorithmic bytes = rows * (K and V) * d * 2 bytes * layers, read once and written once."""
    W = wl.preset("7b-batch8", args.layers)
    shape = dataclasses.replace(W.model, dtype="bf16")
    B, T, H, k = W.batch, W.tree_nodes, shape.n_medusa, shape.topk
    Tp = (T + 31) // 32 * 32
    model = sd.Model(shape, wl.make_weights(shape, device="cuda"), max_rows=B * Tp)
    torch.cuda.empty_cache()
    kv = sd.KVCache(model, B, W.kv_cap)
    rng = np.random.Generator(np.random.Philox(key=wl.SEEDS["kvlen"]))
    lens = [int(x) for x in rng.integers(1024, 4097 - 64, size=B)]
    kv.set_len(lens)
    roots = rng.integers(shape.vocab, size=B).astype(np.int32)
    cand = np.stack([np.stack([rng.permutation(shape.vocab)[:k] for _ in range(H)]) for _ in range(B)]).astype(np.int32)
    kv.set_draft(roots, cand)
    tree_np = wl.default_tree(T, H, k)
    tree = sd.Tree(*tree_np, H, k)
    words = torch.zeros((shape.vocab + 31) // 32, dtype=torch.int32, device="cuda")
    sd.spec_step(model, kv, tree, words)                  # fills the tree scratch of all sequences and layers
    torch.cuda.synchronize()
    results = {}
    for label, width in (("accepted_chain", H + 1), ("all_tree_rows", Tp)):
        # a root path of the tree for the short list (what a step commits), every row for the long one
        if width == H + 1:
            j = int(np.argmax(tree_np[1]))
            path = []
            while j >= 0:
                path.append(j)
                j = int(tree_np[0][j])
            slots_row = (path[::-1] + [0] * width)[:width]
        else:
            slots_row = list(range(width))
        slots = torch.tensor([slots_row] * B, dtype=torch.int32, device="cuda")
        n_rows = torch.full((B,), width, dtype=torch.int32, device="cuda")
        per_window = max(1, (W.kv_cap - max(lens)) // width - 1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        total_ms, launches = 0.0, 0
        for it in range(args.warmup + args.steps):
            kv.set_len(lens)                              # synchronises; outside the timed launches
            e0.record()
            for _ in range(per_window):
                sd.kv_commit_rows(model, kv, slots, n_rows)
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                total_ms += e0.elapsed_time(e1)
                launches += per_window
        us = total_ms / launches * 1e3 / 2                # two launches per call: the length bookkeeping and the copy
        nbytes = 2.0 * B * width * 2 * shape.d_model * 2 * shape.n_layers
        results[label] = {"rows_per_sequence": width, "us_per_call": total_ms / launches * 1e3,
                          "algorithmic_bytes": nbytes, "achieved_GBs": nbytes / (total_ms / launches * 1e-3) / 1e9}
        del us
    best = results["all_tree_rows"]
    print(json.dumps({
        "metric": "kv_commit_GBps", "value": best["achieved_GBs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": best["us_per_call"] / 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"kv-commit stress: {shape.n_layers}-layer d={shape.d_model} cache, batch {B}, lengths {lens}, "
                               f"{Tp}-row tree scratch; per call the length bookkeeping kernel and the copy kernel"},
        "variants": results,
        "roofline": {"kernel": "k_kv_commit (stress variant, not the step)", "bound": "hbm", "achieved": best["achieved_GBs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": best["achieved_GBs"] / HBM_PEAK_GBS, "traffic": None,
                     "avg_launch_us": best["us_per_call"], "algorithmic_bytes_per_launch": best["algorithmic_bytes"]},
        "cpu_baseline": None}))


def bench_labels(args, torch, wl, sd):
    """Syntax-enriched label construction (Section III-C) for one training batch: 256 sequences of the paper's
    8192-token limit, ten heads. A "step" is one launch; timed with HIP events on the launch stream."""
    B, S, H, V = 256, 8192, 10, 32000
    frag, pad, ign = V + 1, V + 2, -100
    l0_np = np.tile(wl.frag_filled_labels(16, S, V, frag, pad), (B // 16, 1))
    l0 = torch.from_numpy(l0_np).cuda()
    out = torch.empty((B, H + 1, S), dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        sd.build_labels(l0, H, frag, pad, ign, out=out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()                                       # the binding launches on torch's current stream
    for _ in range(args.steps):
        sd.build_labels(l0, H, frag, pad, ign, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    nbytes = B * S * 4.0 * (H + 2)                    # one read of L_0, one write of the matrix
    gbs = nbytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import labels_oracle as lab
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 10.0:
            lab.syntax_enriched_labels(l0_np[n % 16], H, frag, pad, ign)
            n += 1
        dt = time.perf_counter() - t0
        cpu = {"value": n * S / dt, "unit": "positions/s", "cores": 1, "kind": "oracle",
               "sample": f"{n} sequences of {S} positions with {H} heads, one at a time, {dt:.1f} s"}
    print(json.dumps({
        "metric": "label_positions_per_s", "value": B * S / (ms * 1e-3), "unit": "positions/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"labels: {B} sequences x {S} positions, {H} heads, geometric fragments of mean 4 tokens"},
        "roofline": {"kernel": "k_build_labels", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": counted_traffic("k_build_labels_256x8192_kernel_trace_and_traffic.txt", "k_build_labels_traffic_bytes_per_launch"), "avg_launch_us": ms * 1e3,
                     "algorithmic_bytes_per_launch": nbytes},
        "cpu_baseline": cpu}))


def cpu_baseline(wl, shape, cpu_keep, T, tree_np, stop, n_cache, typical=None):
    """Time the oracle's speculative step on the host, on a bounded sample of the workload."""
    from threadpoolctl import threadpool_info
    from oracle import specdec_oracle as orc

    w64 = {n: t.double().numpy() for n, t in cpu_keep.items()}
    depth_hi = min(8, shape.n_layers)
    depth_lo = max(1, depth_hi // 2)

    def one_step(L):
        sh = shape.with_layers(L)
        kv = orc.KVCache.empty(sh, n_cache + shape.n_medusa + 2)
        for l in range(L):
            dims = (n_cache, shape.n_heads, shape.head_dim)
            kv.k[l, :n_cache] = wl.synthetic_kv_rows(wl.SEEDS["kvfill"], f"k{l}", dims, "bf16").double().numpy()
            kv.v[l, :n_cache] = wl.synthetic_kv_rows(wl.SEEDS["kvfill"], f"v{l}", dims, "bf16").double().numpy()
        kv.n = n_cache
        cand = (np.arange(shape.n_medusa * shape.topk, dtype=np.int32).reshape(shape.n_medusa, shape.topk) * 7 + 3) % shape.vocab
        st = orc.DecodeState(kv, root_tok=11, cand=cand)
        t0 = time.perf_counter()
        orc.spec_step(w64, sh, st, tree_np, stop, typical=typical)
        return time.perf_counter() - t0

    one_step(1)                                      # warm-up: BLAS threads, page faults
    reps = 21
    t_lo = sorted(one_step(depth_lo) for _ in range(reps))[reps // 2]
    t_hi = sorted(one_step(depth_hi) for _ in range(reps))[reps // 2]
    if depth_hi > depth_lo:
        per_layer = max((t_hi - t_lo) / (depth_hi - depth_lo), 1e-9)
        rest = max(t_lo - depth_lo * per_layer, 0.0)
    else:
        per_layer, rest = t_hi / depth_hi, 0.0
    full = rest + shape.n_layers * per_layer
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": T / full, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"one speculative step ({T}-node tree over a {n_cache}-row synthetic cache) timed at {depth_lo} "
                      f"and {depth_hi} of the {shape.n_layers} layers (full width, LM head and draft heads included, "
                      f"median of {reps}); per-layer time {per_layer:.3f} s, rest {rest:.3f} s, extrapolated to "
                      f"{shape.n_layers} layers: {full:.2f} s/step",
            "seconds_measured": reps * (t_lo + t_hi)}


if __name__ == "__main__":
    main()
