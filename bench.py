#!/usr/bin/env python3
"""Benchmark of the speculative-decoding hot path on one MI355X.

One "step" is one draft + verify + accept cycle (all hot-path stages) at batch 1, T = 0, on a
synthetic random-init LLaMA2-7B-shaped model (bf16, prompt 512, dynamic tree depth 6 / top-k 10 /
60 verified tokens).  Prints ONE JSON line: tokens/s over exactly --steps cycles; `roofline`: the verify
step against the HBM peak ((weights + KV read + KV write) / verify time, HIP events on the library's stream),
with the weight-streaming GEMM launches of the verify as its `kernel` sub-object (timed with HIP event pairs
in a separate instrumented pass); `shapes`: the same measurements at the other benchmark shapes (LLaMA3-70B,
LLaMA2-13B, LLaMA3-8B); and the CPU oracle timed on a bounded sample of the headline workload.  Two separately
labelled objects measure the training-side kernels against the matrix-core peak: `hca_attention` (Sec. 3.2)
and `topk_loss` (Sec. 3.1).
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
OTHER_SHAPES = ("llama3-70b", "llama2-13b", "llama3-8b")     # timed after the headline workload, largest first


def measured_traffic(workload_name):
    """HBM bytes (fetch + write) measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by a plain-copy
    calibration, read from the `key = value` lines at the end of profiles/traffic_gemm_stream_<workload>.txt:
    (bytes per verify step over all its kernels, bytes per GEMM launch); None where no such file or line exists."""
    import re
    path = os.path.join(ROOT, "profiles", "traffic_gemm_stream_" + workload_name.replace("-", "_") + ".txt")
    vals = {}
    try:
        for line in open(path):
            m = re.match(r"^(\w+)\s*=\s*([0-9.eE+-]+)\s*$", line)
            if m:
                vals[m.group(1)] = float(m.group(2))
    except OSError:
        pass
    return vals.get("verify_step_hbm_bytes"), vals.get("gemm_launch_hbm_bytes")


# Mean acceptance length the paper reports for its trained drafts (Table 1, mean over its three benchmarks), per model
# and temperature.  Used only for a labelled projection: random-init drafts never match the target.
PAPER_TAU = {("llama2-7b", 0): 5.15, ("llama2-7b", 1): 4.92, ("llama2-13b", 0): 5.58, ("llama2-13b", 1): 5.42,
             ("llama3-8b", 0): 5.08, ("llama3-8b", 1): 4.80, ("llama3-70b", 0): 5.21, ("llama3-70b", 1): 5.16}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="llama2-7b", help="workload name (see workload.CONFIGS)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of target layers (0 = the config's)")
    ap.add_argument("--forced-accept", type=int, default=4,
                    help="draft tokens accepted per cycle in the teacher-forced extra pass (0 = skip the pass)")
    ap.add_argument("--tree", default="", help="override the draft tree as depth,topk,total (default: the config's 6,10,60)")
    ap.add_argument("--static-tree", default="", help="draft a static shape instead of the dynamic tree: chainN (N draft tokens in a "
                    "row) or tree26 (4/8/8/4/1 nodes per depth); add ':sampled' for sampled children (needs a T > 0 config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hca", action="store_true", help="skip the training-attention measurement (separate object in the JSON line)")
    ap.add_argument("--no-loss", action="store_true", help="skip the distillation-loss measurement (separate object in the JSON line)")
    ap.add_argument("--no-roofline-pass", action="store_true", help="skip the instrumented passes (for profilers)")
    ap.add_argument("--no-other-shapes", action="store_true",
                    help="time only the --config workload (default: the other benchmark shapes follow, in `shapes`)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy four times (known traffic, to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def run_cycles(eng, n_cycles, out=None, stamps=None):
    emitted = 0
    for _ in range(n_cycles):
        t = eng.draft_tree()
        eng.verify(t)
        toks = eng.accept(t)                  # returns host integers: the cycle's device work has finished here
        if stamps is not None:
            stamps.append(time.perf_counter())
        emitted += len(toks)
        if out is not None:
            out.extend(toks)
    return emitted


def run_forced_cycles(eng, n_cycles, stream, pos, accept_per_cycle):
    """Cycles on teacher-forced trees: the known continuation (from plain decoding) is grafted into every drafted tree
    so that `accept_per_cycle` draft tokens are accepted; returns (tokens emitted, new position, all matched)."""
    import workload as wl
    emitted, ok = 0, True
    for _ in range(n_cycles):
        t = eng.draft_tree()
        wl.graft_continuation(t.token, t.parent, t.depth, t.n_nodes, stream[pos:pos + accept_per_cycle])
        eng.verify(t)
        toks = eng.accept(t)
        ok &= toks == stream[pos:pos + len(toks)]
        pos += len(toks)
        emitted += len(toks)
    return emitted, pos, ok


def blas_threads():
    """Threads numpy's matmul uses: the OpenMP/BLAS setting when there is one, else the visible CPUs."""
    for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        v = os.environ.get(var, "")
        if v.isdigit() and int(v) > 0:
            return min(int(v), os.cpu_count() or int(v))
    return os.cpu_count()


def cpu_baseline(sh, layers_timed=2):
    """The oracle as it stands, on the host cores: one draft+verify+accept cycle of a depth-truncated model
    (same widths, same prompt length), plus one decoder layer over the tree rows to extrapolate to full depth."""
    import numpy as np
    import workload as wl
    import oracle
    from oracle.llama import as_dtype
    tsh = sh.with_(n_layers=layers_timed)
    w = as_dtype(wl.make_weights(tsh), np.float32)
    prompt = wl.make_prompt(tsh)
    st, _ = oracle.prefill(w, tsh, prompt, len(prompt) + 512, dtype=np.float32)
    # whole cycles until about ten seconds of CPU work have been timed
    draft_s = verify_s = 0.0
    cycles = emitted_total = 0
    while cycles < 48 and draft_s + verify_s < 10.0:
        t0 = time.perf_counter()
        st.cycle = cycles + 1
        tree = oracle.draft_tree(st, tsh.tree_depth, tsh.tree_topk, tsh.tree_total)
        t1 = time.perf_counter()
        logits, feats = oracle.verify_tree(st, tree)
        acc, bonus = oracle.accept_greedy(tree, logits)
        emitted = oracle.commit(st, tree, feats, acc, bonus)
        t2 = time.perf_counter()
        draft_s += t1 - t0
        verify_s += t2 - t1
        cycles += 1
        emitted_total += len(emitted)
    # more layers over the rows of the last tree, to extrapolate linearly in depth
    n = st.n - len(emitted)                                   # the verified rows still sit at slots n + j
    rows = tree.n_nodes
    h = np.random.default_rng(0).standard_normal((rows, tsh.d_model)).astype(np.float32)
    vis = [list(range(n)) + [n + a for a in tree.path(j)] for j in range(rows)]
    reps = 8
    t3 = time.perf_counter()
    for _ in range(reps):
        oracle.decoder_layer(h, w, "layers.0.", tsh, 0, st.tcache, (n + tree.depth).astype(np.int64),
                             [n + j for j in range(rows)], vis)
    t4 = time.perf_counter()
    layer_s = (t4 - t3) / reps
    cycle_s = (draft_s + verify_s) / cycles
    full_cycle = cycle_s + (sh.n_layers - layers_timed) * layer_s
    return {
        "value": emitted_total / cycles / full_cycle, "unit": "tokens/s", "cores": blas_threads(), "kind": "oracle",
        "sample": f"{cycles} cycles on a {layers_timed}-layer truncation at full width ({draft_s + verify_s:.1f} s: draft "
                  f"{draft_s / cycles:.2f} s and verify {verify_s / cycles:.2f} s per cycle), extrapolated to {sh.n_layers} layers "
                  f"with a timed decoder layer ({layer_s:.3f} s, mean of {reps}); numpy fp32",
        "measured_truncated_cycle_s": cycle_s,
    }


MFMA_BF16_PEAK_TFLOPS = 2500.0


def hca_attention_bench(sh, with_cpu, launches=50):
    """Training attention of harmonized context alignment (Sec. 3.2) at the training launch the appendix (Training
    Overhead) describes: batch 2, three aligning steps, 2048 positions, the draft layer's head layout.  Algorithmic
    flop = 4 * head_dim per (query, visible key) pair; timed with events on the stream the kernel is launched on,
    `launches` launches per event pair."""
    import numpy as np
    import torch
    import workload as wl
    import paper_2408_15766_amd as P
    n_streams, batch, seq = 3, 2, 2048
    hq, hkv, hd = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    q, ks, vs = wl.make_hca_streams(sh.seed, n_streams, batch, seq, hq, hkv, hd, drift=0.3)
    dev = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    dq, dks, dvs = dev(q), [dev(k) for k in ks], [dev(v) for v in vs]
    out = torch.empty_like(dq)
    for _ in range(5):
        P.spec_hca_attention(dq, dks, dvs, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        P.spec_hca_attention(dq, dks, dvs, out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / launches
    flop = 4.0 * hd * hq * batch * (seq * (seq + 1) / 2)
    res = {"workload": f"{sh.name} draft layer: batch {batch} x {seq} positions, {n_streams} streams, {hq} query / {hkv} kv heads of {hd}",
           "dtype": "bf16", "ms_per_launch": ms, "launches": launches,
           "roofline": {"bound": "mfma", "achieved": flop / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": flop / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                        "kernel": "hca_attention_kernel", "algorithmic_flop_per_launch": flop}}
    if with_cpu:
        from oracle import hca
        heads = sorted({0, hq // 3, 2 * hq // 3, hq - 1})
        f64 = lambda x: x[0].astype(np.float64)
        t0 = time.perf_counter()
        want = hca.hca_attention(f64(q), [f64(k) for k in ks], [f64(v) for v in vs], heads=heads)
        dt = time.perf_counter() - t0
        got = out[0].float().cpu().numpy()[:, heads]
        res["cpu_baseline"] = {"value": flop * len(heads) / (hq * batch) / dt / 1e12, "unit": "TFLOP/s", "cores": blas_threads(),
                               "kind": "oracle", "sample": f"{len(heads)} of {hq * batch} (batch, head) pairs, numpy fp64, {dt:.2f} s"}
        res["max_abs_diff_vs_oracle_sample"] = float(np.abs(got - want[:, heads]).max())
    return res


def topk_loss_bench(sh, with_cpu, launches=5):
    """Top-K distillation loss through the LM head (Sec. 3.1, Eq. 1; K = 10) for the positions of one training batch
    (batch 2 x 2048, appendix Training Overhead): two LM-head GEMMs of 4096 rows (target and draft features) plus the
    loss kernels.  Algorithmic flop = 2 * (2 * rows) * vocab * d (the loss arithmetic itself is not counted)."""
    import numpy as np
    import torch
    import workload as wl
    import paper_2408_15766_amd as P
    rows, d, vocab, k = 2 * 2048, sh.d_model, sh.vocab, 10
    host = vocab * d <= 2e8                                   # larger heads are drawn on the device; no CPU sample then
    if host:
        ft, fd, w = wl.make_distill_inputs(sh.seed, rows, d, vocab, "bf16")
        dft, dfd, dw = (torch.from_numpy(x).cuda().to(torch.bfloat16) for x in (ft, fd, w))
    else:
        g = torch.Generator(device="cuda").manual_seed(sh.seed)
        dft = torch.randn((rows, d), device="cuda", generator=g).to(torch.bfloat16)
        dfd = (dft.float() + 0.5 * torch.randn((rows, d), device="cuda", generator=g)).to(torch.bfloat16)
        dw = (torch.randn((vocab, d), device="cuda", generator=g) * (3.0 / d ** 0.5)).to(torch.bfloat16)
    head = P.spec_pack_weight(dw)
    del dw
    scratch = torch.empty(P.spec_topk_loss_scratch_bytes(rows, vocab, k), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        topk, ce, tot = P.spec_topk_loss(dft, dfd, head, k, scratch)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        P.spec_topk_loss(dft, dfd, head, k, scratch)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / launches
    flop = 2.0 * (2 * rows) * vocab * d
    res = {"workload": f"{sh.name} LM head: {rows} positions (batch 2 x 2048), d {d}, vocabulary {vocab}, K {k}",
           "dtype": "bf16", "ms_per_call": ms, "calls": launches, "mean_topk_loss": float(tot[0]) / rows, "mean_cross_entropy": float(tot[1]) / rows,
           "roofline": {"bound": "mfma", "achieved": flop / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": flop / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                        "kernel": "gemm_tiled_kernel (LM head, 512-row chunks) + loss_slice_kernel + loss_merge_kernel",
                        "algorithmic_flop_per_call": flop}}
    if with_cpu and host:
        from oracle import distill
        sample = np.arange(0, rows, rows // 16)
        t0 = time.perf_counter()
        want, want_ce = distill.head_losses(ft[sample].astype(np.float64), fd[sample].astype(np.float64), w.astype(np.float64), k)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": flop * len(sample) / rows / dt / 1e12, "unit": "TFLOP/s", "cores": blas_threads(), "kind": "oracle",
                               "sample": f"{len(sample)} of {rows} positions, numpy fp64, {dt:.2f} s"}
        res["max_abs_diff_vs_oracle_sample"] = float(np.abs(topk.cpu().numpy()[sample] - want).max())
    return res


def static_shape(name):
    """(parent, rank) arrays of a named static tree shape (see spec_set_static_tree)."""
    if name.startswith("chain"):
        n = int(name[5:])
        return [-1] + list(range(n)), [0] * (n + 1)
    if name == "tree26":
        return ([-1, 0, 0, 0, 0, 1, 1, 1, 2, 2, 3, 3, 4, 5, 5, 5, 6, 6, 8, 8, 10, 13, 13, 14, 16, 21],
                [0, 0, 1, 2, 3, 0, 1, 2, 0, 1, 0, 1, 0, 0, 1, 2, 0, 1, 0, 1, 0, 0, 1, 0, 0, 0])
    raise SystemExit(f"bench.py: unknown static tree {name!r}")


def measure_shape(sh, weights, steps, warmup, forced_accept_arg, static_tree="", roofline_pass=True, label_overridden=False):
    """All decode-path measurements of one workload on resident weights -> dict (see main for the field meanings)."""
    import torch
    import workload as wl
    import paper_2408_15766_amd as P
    prompt = wl.make_prompt(sh)
    total_cycles = warmup + steps
    max_seq = sh.prompt_len + (sh.tree_depth + 1) * (total_cycles + 1) + sh.tree_total + 32
    static_name, _, static_mode = static_tree.partition(":")

    def engine():
        e = P.Engine(sh, weights, max_seq=max_seq)
        if static_name:
            e.set_static_tree(*static_shape(static_name), sampled=static_mode == "sampled")
        return e

    # ---- pass A: the timed region ------------------------------------------------------------
    eng = engine()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.prefill(prompt)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0                      # not part of `value`: once per request, first call (cold)
    run_cycles(eng, warmup)
    # The interpreter's cyclic collector walks every object torch created at import (tens of ms per full
    # collection); park those in the permanent generation so a collection cannot land inside the timed loop.
    gc.collect()
    gc.freeze()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stamps = [t0]
    emitted = run_cycles(eng, steps, stamps=stamps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    eng.close()
    per_cycle = sorted((b - a_) * 1e3 for a_, b in zip(stamps, stamps[1:]))
    pick = lambda f: per_cycle[min(len(per_cycle) - 1, int(f * len(per_cycle)))]
    ms_per_step = dt / steps * 1e3

    # plain autoregressive decoding through the same kernels (tree = the root alone): the 1.00x reference.
    # The teacher-forced pass (T = 0 only, where the emitted tokens are a function of the weights alone) needs its stream.
    forced_accept = max(0, min(sh.tree_depth, forced_accept_arg)) if sh.temperature == 0 and sh.tree_total > 1 and not static_name else 0
    plain_extra = (total_cycles * (forced_accept + 1) + 1 - total_cycles) if forced_accept else 0
    plain = P.Engine(sh, weights, max_seq=max_seq, tree=(1, 1, 1))
    stream = [plain.prefill(prompt)]
    run_cycles(plain, warmup, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pe = run_cycles(plain, steps, stream)
    torch.cuda.synchronize()
    plain_dt = time.perf_counter() - t0
    run_cycles(plain, plain_extra, stream)                    # untimed: the continuation the forced mode grafts
    plain.close()

    by = wl.algorithmic_bytes(sh)
    n_mid = sh.prompt_len + warmup + steps // 2
    kv_read = n_mid * by["kv_bytes_per_token"]
    kv_write = sh.tree_total * by["kv_bytes_per_token"]
    verify_bytes = by["verify_weights"] + kv_read + kv_write
    out = {
        "workload": f"{sh.name} shape, random init N(0,0.02), prompt {sh.prompt_len} uniform tokens, "
                    + (f"static tree {static_tree}" if static_name else f"tree depth {sh.tree_depth} top-k {sh.tree_topk} total {sh.tree_total}")
                    + f", T={sh.temperature:g}, batch 1",
        "tokens_per_s": emitted / dt, "steps": steps, "warmup": warmup,
        "ms_per_cycle": ms_per_step,
        "cycle_ms_p10_median_p90": [pick(0.1), pick(0.5), pick(0.9)],
        "mean_accepted_length": emitted / steps,
        "plain_decode_tokens_per_s": pe / plain_dt,
        "plain_decode_ms_per_token": plain_dt / steps * 1e3,
        "plain_decode_hbm_frac": (by["verify_weights"] + kv_read + by["kv_bytes_per_token"]) / (plain_dt / steps) / 1e9 / HBM_PEAK_GBPS,
        "prefill_ms": prefill_s * 1e3, "prefill_tokens_per_s": sh.prompt_len / prefill_s,
    }
    tau = PAPER_TAU.get((sh.name, 0 if sh.temperature == 0 else 1))
    if tau and not (label_overridden or static_name):
        out["projection_at_paper_tau"] = {
            "what": "PROJECTION, not a measurement: the paper's mean acceptance length (Table 1) divided by this run's "
                    "measured cycle time; the measured cycles themselves accept about one token",
            "tau": tau, "tokens_per_s": tau / (ms_per_step * 1e-3),
            "speedup_over_plain_decode_same_kernels": tau / (ms_per_step * 1e-3) / (pe / plain_dt)}

    # ---- teacher-forced trees: the same cycles at a paper-like acceptance length (separately labelled) ----
    if forced_accept:
        eng = P.Engine(sh, weights, max_seq=max_seq)
        first = eng.prefill(prompt)
        _, pos, ok0 = run_forced_cycles(eng, warmup, stream, 1, forced_accept)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fe, pos, ok1 = run_forced_cycles(eng, steps, stream, pos, forced_accept)
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        eng.close()
        out["teacher_forced"] = {
            "what": "every drafted tree has the known greedy continuation grafted in on the host (random-init drafts never "
                    "match the target), so the accept, compaction and hand-off stages run at a paper-like acceptance length; "
                    "the host-side tree edit is inside the timed loop",
            "mean_accepted_length": fe / steps, "tokens_per_s": fe / fdt, "ms_per_cycle": fdt / steps * 1e3,
            "speedup_over_plain_decode_same_kernels": (fe / fdt) / (pe / plain_dt),
            "tokens_equal_plain_decoding": bool(first == stream[0] and ok0 and ok1)}
        out["tokens_equal_plain_decoding"] = out["teacher_forced"]["tokens_equal_plain_decoding"]

    # ---- instrumented passes with HIP events on the library's stream --------------------------
    # level 1: one event pair around each call (draft, verify, accept) of the graph-replayed run;
    # level 2: one pair around every GEMM launch, kernels launched individually (perturbs the pipeline: its own pass).
    if roofline_pass:
        step_traffic, launch_traffic = (None, None) if (label_overridden or static_name) else measured_traffic(sh.name)
        for level in (1, 2):
            eng = engine()
            eng.prefill(prompt)
            run_cycles(eng, warmup)
            P.spec_set_profile(eng.ctx, level)
            run_cycles(eng, steps)
            ms, cnt = P.spec_get_profile(eng.ctx)
            eng.close()
            if level == 1:
                draft_ms, verify_ms, accept_ms = (ms[i] / max(cnt[i], 1) for i in range(3))
                gbps = verify_bytes / (verify_ms * 1e-3) / 1e9
                out.update({"draft_ms": draft_ms, "verify_ms": verify_ms, "accept_ms": accept_ms,
                            "verify_hbm_gbps": gbps, "verify_hbm_frac": gbps / HBM_PEAK_GBPS,
                            "draft_hbm_frac": sh.tree_depth * by["draft_forward"] / (draft_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS if sh.tree_total > 1 and not static_name else None})
                out["roofline"] = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                                   "traffic": step_traffic,
                                   "what": "the verify step (one replayed target forward over the tree's rows): algorithmic bytes = "
                                           "weights + KV read + KV write, time = HIP events around the step on the library's stream",
                                   "algorithmic_bytes_per_step": verify_bytes, "step_ms": verify_ms}
            else:
                n_launch = cnt[4] / steps                        # GEMM launches per verify
                pair_ms = ms[6] / max(cnt[6], 1)                 # what an empty event pair measures
                raw_ms = ms[4] / max(cnt[4], 1)
                avg_ms = raw_ms - pair_ms
                bytes_per_launch = by["verify_weights"] / n_launch
                achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
                out["roofline"]["kernel"] = {
                    "name": "gemm_stream_kernel (the verify step's weight-streaming launches)", "bound": "hbm", "achieved": achieved,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": launch_traffic,
                    "launches_per_step": n_launch, "avg_launch_ms": avg_ms, "event_interval_ms": raw_ms, "empty_event_pair_ms": pair_ms,
                    "algorithmic_bytes_per_launch": bytes_per_launch}
                out["roofline"]["kernel_frac"] = achieved / HBM_PEAK_GBPS
                out["roofline"]["kernel_avg_launch_ms"] = avg_ms
    return out


def load_weights(sh):
    import workload as wl
    import paper_2408_15766_amd as P
    return P.pack_weights(wl.iter_device_weights(sh, "cuda"))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (batch-1 decode has no data-parallel units); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import workload as wl

    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read_per_launch": src.numel() * 4, "bytes_written_per_launch": src.numel() * 4}))
        return
    sh = wl.BY_NAME[a.config]
    overridden = bool(a.layers or a.tree)
    if a.layers:
        sh = sh.with_(n_layers=a.layers, name=f"{sh.name}-{a.layers}layer")
    if a.tree:
        d_, k_, n_ = (int(x) for x in a.tree.split(","))
        sh = sh.with_(tree_depth=d_, tree_topk=k_, tree_total=n_)
    torch.cuda.set_device(0)
    weights = load_weights(sh)
    m = measure_shape(sh, weights, a.steps, a.warmup, a.forced_accept, a.static_tree, not a.no_roofline_pass, overridden)
    out = {
        "metric": f"tokens/s (bs=1, T={sh.temperature:g})", "value": m.pop("tokens_per_s"), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": m["ms_per_cycle"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": sh.dtype, "data": "synthetic", "config": {"workload": m.pop("workload")},
    }
    m.pop("steps"); m.pop("warmup")
    out.update(m)

    if not a.no_hca:
        out["hca_attention"] = hca_attention_bench(wl.BY_NAME[a.config], not a.no_cpu_baseline)
    del weights
    gc.collect()
    torch.cuda.empty_cache()
    if not a.no_loss:
        out["topk_loss"] = topk_loss_bench(wl.BY_NAME[a.config], not a.no_cpu_baseline)
        gc.collect()
        torch.cuda.empty_cache()

    # ---- the other benchmark shapes, each with its own resident weights, same measurements, fewer cycles ----
    if not (a.no_other_shapes or overridden or a.static_tree or a.config != "llama2-7b"):
        out["shapes"] = {}
        for name in OTHER_SHAPES:
            osh = wl.BY_NAME[name]
            w = load_weights(osh)
            out["shapes"][name] = measure_shape(osh, w, min(a.steps, 16), min(a.warmup, 3), a.forced_accept, "", not a.no_roofline_pass)
            del w
            gc.collect()
            torch.cuda.empty_cache()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl.BY_NAME[a.config])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
