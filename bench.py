#!/usr/bin/env python3
"""Benchmark of the selective-KV-recompute hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch that is already resident in HBM:
cc_rope_shift -> cc_select -> cc_gather_rows (+ cc_qkv_project) -> cc_sparse_prefill.
Prints ONE JSON line: recomputed tokens/s for the whole path, the roofline of the kernel that
dominates the step (plus every stage's own figure), and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E
PEAK_FP32_VALU_TFLOPS = 157.3
# Back-to-back v_mfma_f32_32x32x16_bf16 on all 1024 SIMDs, two wavefronts per SIMD, four independent
# accumulators each, random bf16 operands in vector registers, nothing else in the loop, sustains this
# on the box over several milliseconds (1490 with one wavefront per SIMD; the clock the chip holds
# under matrix load depends on the operand data: constant operands run ~25 % faster).  Quoted beside
# the vendor peak, never instead of it.
MEASURED_MFMA_BF16_TFLOPS = 1700.0
# Tracked rocprofv3 summary of the default workload: its "HBM traffic per launch" table (FETCH_SIZE / WRITE_SIZE
# scaled by a copy of known size) is where roofline.traffic comes from - it is not measured in this run.
TRAFFIC_PROFILE = os.path.join("profiles", "hot_path_kernels_config3_8b_continuous_batch.md")
TRAFFIC_WORKLOAD = 3
KERNELS_OF_CALL = {"cc_rope_shift": ("rope_shift_kernel",), "cc_select": ("score_v2_kernel", "topn_kernel", "sparse_qk_kernel<G=4,SCORE"),
                   "cc_sparse_prefill": ("attn_v2_kernel", "rope_scatter_kernel", "sparse_qk_kernel<G=4,ATTN")}


def profiled_traffic_bytes(call: str):
    """HBM bytes per launch (read + written) of the kernels of one library call, summed from the tracked
    profile summary's traffic table; None if the file or the rows are missing."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    if not os.path.exists(path) or call not in KERNELS_OF_CALL:
        return None
    total, found, in_table = 0.0, False, False
    for line in open(path):
        if line.startswith("## HBM traffic per launch"):
            in_table = True
            continue
        if in_table and line.startswith("## "):
            break
        if in_table and line.startswith("|") and "---" not in line and "FETCH_SIZE raw" not in line:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 5 and any(k in cells[0] for k in KERNELS_OF_CALL[call]):
                try:
                    total += (float(cells[2]) + float(cells[4])) * 2 ** 20
                    found = True
                except ValueError:
                    pass
    return total if found else None


def algorithmic_work(w, cow: bool = True):
    """Algorithmic flops / bytes of each stage for workload w (only causally visible keys count).
    cow: values stay in the chunk store, so the shift moves keys only."""
    import workload as W
    sp = w.spec
    hq, hkv, d = sp.n_q_heads, sp.n_kv_heads, sp.head_dim
    e = 2 if sp.dtype == "bf16" else 4
    seg = w.segments
    chunk = seg[seg[:, W.SEG_KIND] == W.KIND_CHUNK]
    n_chunk_tok = int(chunk[:, W.SEG_NTOK].sum())
    # score: every token of every chunk that has a prior chunk, against keys 0..p
    score_pairs = 0
    for s in chunk:
        st, n = int(s[W.SEG_START]), int(s[W.SEG_NTOK])
        if st > 0:
            score_pairs += n * st + n * (n + 1) // 2
    return {
        "n_chunk_tok": n_chunk_tok,
        "shift_bytes": n_chunk_tok * hkv * d * e * 2 * (1 if cow else 2),      # K read+write (and V read+write)
        "score_flops": 2.0 * d * hq * score_pairs,
        "recomputed_tokens": w.n_q_tot,
    }


def attention_flops(w, q_pos: np.ndarray) -> float:
    sp = w.spec
    return 4.0 * sp.head_dim * sp.n_q_heads * float((q_pos.astype(np.int64) + 1).sum())


def time_stages(batch, steps: int):
    """Average ms of each library call over `steps` steps (HIP events on the calls' stream)."""
    import torch
    if batch.projected or not batch.fused_gather:
        names = ["rope_shift", "select", "gather", "sparse_prefill"]
        fns = [batch.rope_shift, batch.select, batch.gather, batch.sparse_prefill]
    else:           # per-token q / k_new / v_new are read through cc_select's row list: no gather call
        names = ["rope_shift", "select", "sparse_prefill"]
        fns = [batch.rope_shift, batch.select, batch.sparse_prefill_fused]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        ev[i][0].record()
        for j, f in enumerate(fns):
            f()
            ev[i][j + 1].record()
    torch.cuda.synchronize()
    return {n: float(np.mean([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(steps)]))
            for j, n in enumerate(names)}


def _gpu_request_state(w, batch, r):
    """What the GPU left for request r after a step: chosen index sets per chunk, attention output, and the
    logical K / V of the request as its pages now hold them."""
    import workload as W
    from oracle import cachecraft_oracle as O
    sel = batch.sel_idx.cpu().numpy()
    segs = [w.segments[i] for i in range(int(w.req_seg_off[r]), int(w.req_seg_off[r + 1]))]
    sets = [np.asarray(sel[int(sg[W.SEG_SEL]): int(sg[W.SEG_SEL]) + int(sg[W.SEG_NSEL])], dtype=np.int64)
            for sg in segs if sg[W.SEG_KIND] == W.KIND_CHUNK]
    q0, q1 = int(w.cu_q[r]), int(w.cu_q[r + 1])
    out = batch.out[q0:q1].float().cpu().numpy()
    import torch
    mine = np.unique(np.concatenate([np.asarray(w.req_tab[int(sg[W.SEG_TAB]): int(sg[W.SEG_TAB]) + (int(sg[W.SEG_NTOK]) + 15) // 16],
                                               dtype=np.int64) for sg in segs]))
    idx = torch.as_tensor(mine, device=batch.k_req.device)
    k_pages = batch.k_req.index_select(0, idx).float().cpu().numpy()      # only this request's pages travel to the host
    v_pages = batch.values_pool().index_select(0, idx).float().cpu().numpy()
    n_ctx = int(segs[-1][W.SEG_START] + segs[-1][W.SEG_NTOK])
    hkv, d = w.spec.n_kv_heads, w.spec.head_dim
    k = np.zeros((n_ctx, hkv, d)); v = np.zeros((n_ctx, hkv, d))
    for sg in segs:
        st, n, tab = int(sg[W.SEG_START]), int(sg[W.SEG_NTOK]), int(sg[W.SEG_TAB])
        blk = np.searchsorted(mine, np.asarray(w.req_tab[tab: tab + (n + 15) // 16], dtype=np.int64))
        k[st:st + n] = O.read_k_pages(k_pages, blk, n)
        v[st:st + n] = O.read_v_pages(v_pages, blk, n)
    return sets, out, k, v


def cpu_baseline(w, batch=None, budget_s: float = 20.0):
    """The fp64 oracle as it stands, on a bounded sample: whole requests, in order, until about
    `budget_s` seconds of CPU work are spent (at least one request).  With `batch` (the device batch the
    timed steps ran on) the same requests also give the parity block: the GPU's index sets against the
    oracle's (differences outside the 1e-4 tie band count), and its attention output and fixed K / V
    against the oracle run on the GPU's own sets (untimed)."""
    from oracle import cachecraft_oracle as O
    spent = 0.0
    tokens = 0
    done = 0
    tie_gap = 1e-4
    err2 = {"out": 0.0, "k": 0.0, "v": 0.0}
    ref2 = {"out": 0.0, "k": 0.0, "v": 0.0}
    set_mismatch, set_diff_in_band = 0, 0
    for r in range(w.n_requests):
        t0 = time.perf_counter()
        res = O.run_request(w, r)
        spent += time.perf_counter() - t0
        tokens += int(w.cu_q[r + 1] - w.cu_q[r])
        done += 1
        if batch is not None:
            sets, out, k, v = _gpu_request_state(w, batch, r)
            same = True
            for g, o, sc in zip(sets, res.selected, res.scores):
                diff = np.setxor1d(g, o)
                if len(diff):
                    same = False
                    nth = np.sort(sc)[::-1][len(o) - 1]
                    outside = int((np.abs(sc[diff] - nth) > tie_gap).sum())
                    set_mismatch += outside
                    set_diff_in_band += len(diff) - outside
            if not same:                  # ties broken differently: the oracle attends over the GPU's own sets
                k_sh, v_c, _ = O.shifted_context(w, r)
                k_ctx, v_ctx, _, _, o_out, _ = O.fix_and_attend(w, r, k_sh, v_c, sets)
            else:
                k_ctx, v_ctx, o_out = res.k_ctx, res.v_ctx, res.out
            for name, got, ref in (("out", out, o_out), ("k", k, k_ctx), ("v", v, v_ctx)):
                err2[name] += float(((got - ref) ** 2).sum()); ref2[name] += float((ref ** 2).sum())
        if spent > budget_s:
            break
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        cores = os.cpu_count() or 1
    base = {"value": tokens / spent, "unit": "recomputed tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {done} of {w.n_requests} requests, all stages (shift, score, select, fix, attend), "
                      f"{tokens} recomputed tokens in {spent:.1f} s"}
    parity = None
    if batch is not None:
        rel = lambda n: float(np.sqrt(err2[n] / ref2[n])) if ref2[n] > 0 else 0.0
        parity = {"requests": done, "out_rel_l2": rel("out"), "k_rel_l2": rel("k"), "v_rel_l2": rel("v"),
                  "set_mismatches_outside_tie_band": set_mismatch, "set_differences_inside_tie_band": set_diff_in_band,
                  "bar": {"rel_l2": 1e-2 if w.spec.dtype == "bf16" else 1e-5, "tie_gap": tie_gap}}
    return base, parity


def measured_copy_gbs(mib: int = 512, iters: int = 5) -> float:
    """Read + write rate of torch's device-to-device copy of `mib` MiB (median of `iters`)."""
    import torch
    a = torch.empty(mib * 1024 * 1024, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    b.copy_(a)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        b.copy_(a)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(iters)]))
    return 2.0 * mib * 1024 * 1024 / (ms * 1e-3) / 1e9


def time_layerwise_preload(batch, step_ms: float, n_layers: int = 6) -> dict:
    """n_layers passes of the hot path, each on a chunk store that first has to come from pinned host
    memory (the same bytes every layer): copy-then-compute one layer after the other, against the
    library's preloader (copy stream + events, depth from Eq. (12)) running the copies ahead."""
    import torch
    import paper_2502_15734_amd as P
    k_dev, v_dev = batch.k_store, batch.v_store
    k_host, v_host = k_dev.cpu().pin_memory(), v_dev.cpu().pin_memory()
    nbytes = 2 * k_host.numel() * k_host.element_size()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k_dev.copy_(k_host, non_blocking=True); v_dev.copy_(v_host, non_blocking=True)
    torch.cuda.synchronize()
    ev0.record()
    k_dev.copy_(k_host, non_blocking=True); v_dev.copy_(v_host, non_blocking=True)
    ev1.record(); torch.cuda.synchronize()
    load_ms = ev0.elapsed_time(ev1)
    # one after the other
    t0 = time.perf_counter()
    for _ in range(n_layers):
        k_dev.copy_(k_host, non_blocking=True); v_dev.copy_(v_host, non_blocking=True)
        batch.step()
    torch.cuda.synchronize()
    serial_ms = (time.perf_counter() - t0) * 1e3
    # preloaded: K and V of a layer travel as one unit into one slot of a ring
    depth = P.preload_depth(n_layers, step_ms, load_ms)
    n_slots = min(depth + 1, n_layers)
    slots = [(torch.empty_like(k_dev), torch.empty_like(v_dev)) for _ in range(n_slots)]
    pre_k = P.Preloader(n_layers, depth, n_slots); pre_v = P.Preloader(n_layers, depth, n_slots)
    for l in range(n_layers):
        pre_k.set_layer(l, k_host, slots[l % n_slots][0]); pre_v.set_layer(l, v_host, slots[l % n_slots][1])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for l in range(n_layers):
        pre_k.acquire(l); pre_v.acquire(l)
        batch.k_store, batch.v_store = slots[l % n_slots]
        batch.step()
        pre_k.release(l); pre_v.release(l)
    torch.cuda.synchronize()
    pipelined_ms = (time.perf_counter() - t0) * 1e3
    batch.k_store, batch.v_store = k_dev, v_dev
    pre_k.close(); pre_v.close()
    return {"layers": n_layers, "depth": depth, "slots": n_slots, "bytes_per_layer": nbytes,
            "load_ms_per_layer": load_ms, "host_to_device_GBps": nbytes / (load_ms * 1e-3) / 1e9,
            "step_ms": step_ms, "serial_ms": serial_ms, "pipelined_ms": pipelined_ms}


def time_extra_calls(batch, w, work, steps: int, ms_per_step: float, sparse_prefill_ms: float) -> dict:
    """Entry points that are not part of the timed step, on the batch the step just ran on."""
    import torch

    def timed(fn, n):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record()
        for i in range(n):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(n)]))

    batch.gather()         # the calls below take the compact query rows
    # selection from given scores (the scores cc_select just wrote, so the selection is unchanged)
    from_scores_ms = timed(batch.select_from_scores, steps)
    # attention of the question to every chunk: a pass of its own after cc_sparse_prefill ...
    question_mass_ms = timed(batch.question_mass, steps)
    # ... and as a by-product of cc_sparse_prefill's attention kernel
    prefill_mass_ms = timed(batch.sparse_prefill_mass, steps)
    # inter / intra sums between all segments, over the rows of the last cc_sparse_prefill
    chunk_attention_ms = timed(batch.chunk_attention, max(1, min(steps, 5)))
    # ... and the same sums as a by-product of cc_sparse_prefill's attention kernel
    prefill_pairs_ms = timed(batch.sparse_prefill_pairs, steps)
    preload = time_layerwise_preload(batch, ms_per_step)
    layer_loop = time_layer_loop(w)
    dense = time_decoder_dense(batch, w)
    decoder = time_decoder_loop(w)
    return {"cc_select_from_scores": {"ms": from_scores_ms, "chunk_tokens": work["n_chunk_tok"]},
            "cc_question_mass": {"ms": question_mass_ms, "segments": int(len(w.segments))},
            "cc_sparse_prefill_mass": {"ms": prefill_mass_ms, "over_cc_sparse_prefill_ms": prefill_mass_ms - sparse_prefill_ms},
            "cc_chunk_attention": {"ms": chunk_attention_ms, "segment_pairs": int(batch.pair_off[-1])},
            "cc_sparse_prefill_pairs": {"ms": prefill_pairs_ms, "over_cc_sparse_prefill_ms": prefill_pairs_ms - sparse_prefill_ms},
            "layerwise_preload": preload, "layer_loop": layer_loop, "decoder_layer_dense": dense, "decoder_loop": decoder}


def time_decoder_dense(batch, w) -> dict:
    """The dense operators that take the recomputed rows through the rest of a decoder layer, at the
    model shape the workload's head geometry belongs to (8B: hidden 4096, feed-forward 14336; 70B:
    8192 / 28672), on as many rows as the step recomputes.  Random inputs and weights."""
    import torch
    sp = w.spec
    hq, d = sp.n_q_heads, sp.head_dim
    hidden, ffn = (8192, 28672) if hq * d >= 8192 else (4096, 14336)
    n = batch.n_q_tot
    if n == 0 or sp.dtype != "bf16":
        return {}
    g = torch.Generator(device="cuda").manual_seed(1)
    rnd = lambda *shape, s=1.0: (torch.randn(*shape, device="cuda", generator=g) * s).to(torch.bfloat16)
    h, o = rnd(n, hidden), rnd(n, hq * d, s=0.5)
    gain = (1.0 + 0.1 * torch.randn(hidden, device="cuda", generator=g)).to(torch.bfloat16)
    w_o, w_gate = rnd(hidden, hq * d, s=(hq * d) ** -0.5), rnd(ffn, hidden, s=hidden ** -0.5)
    w_up, w_down = rnd(ffn, hidden, s=hidden ** -0.5), rnd(hidden, ffn, s=ffn ** -0.5)
    h1, x = torch.empty_like(h), torch.empty_like(h)
    act = torch.empty((n, ffn), dtype=torch.bfloat16, device="cuda")
    ctx = batch.ctx
    calls = [("cc_rms_norm", lambda: ctx.rms_norm(h1, gain, 1e-5, x), None, 2.0 * n * hidden * 2),
             ("cc_linear(output projection + residual)", lambda: ctx.linear(o, w_o, h1, residual=h), 2.0 * n * hidden * hq * d, None),
             ("cc_gated_linear", lambda: ctx.gated_linear(x, w_gate, w_up, act), 2.0 * n * hidden * 2 * ffn, None),
             ("cc_linear(down projection + residual)", lambda: ctx.linear(act, w_down, h, residual=h1), 2.0 * n * ffn * hidden, None)]
    out = {"rows": n, "hidden": hidden, "ffn": ffn, "calls": {}}
    total = 0.0
    for name, fn, flops, nbytes in calls:
        fn(); fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        ev[0].record()
        for i in range(5):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
        total += ms
        rec = {"ms": ms}
        if flops is not None:
            rec.update(TFLOPs=flops / ms / 1e9, frac_of_peak=flops / ms / 1e9 / PEAK_MFMA_BF16_TFLOPS)
        else:
            rec.update(GBps=nbytes / ms / 1e6, frac_of_peak=nbytes / ms / 1e6 / PEAK_HBM_GBS)
        out["calls"][name] = rec
    out["ms"] = total
    return out


def time_decoder_loop(w, n_layers: int = 2) -> dict:
    """Whole decoder layers for the recomputed rows of a workload that carries hidden states (config 5):
    norm, QKV projection, partial prefill, output projection, feed-forward; feed-forward width 3.5 x hidden."""
    import workload as W
    from paper_2502_15734_amd.layers import DecoderLoop
    if w.hidden is None or w.spec.dtype != "bf16":
        return {}
    hidden = int(w.hidden.shape[1])
    ffn = hidden * 7 // 2
    weights = [W.layer_weights(w.spec, hidden, ffn, layer=l) for l in range(n_layers)]
    loop = DecoderLoop(w, weights)
    loop.run()                                            # warm-up
    recs = loop.run()
    loop.close()
    return {"hidden": hidden, "ffn": ffn, "layers": [{"layer": r["layer"], "rows": r["rows"], "ms": r["ms"]} for r in recs]}


def time_layer_loop(w, n_layers: int = 4, window: int = 2) -> dict:
    """The loop over layers with Algorithm 1 deciding the focused chunks (identical synthetic layers, so
    every request settles at layer `window`): rows recomputed and time per layer before and after."""
    from paper_2502_15734_amd.layers import LayerLoop
    loop = LayerLoop(w, n_layers, window, preload=False)
    recs = loop.run()
    loop.close()
    return {"window": window, "layers": [{"layer": r["layer"], "rows": r["rows"], "ms": r["ms"]} for r in recs],
            "requests_settled": sum(1 for s in recs[-1]["stop_layer"] if s is not None)}


def stage_figures(w, batch, stage_ms):
    """Per library call: ms, achieved algorithmic rate, fraction of the published peak."""
    work = algorithmic_work(w, batch.cow)
    q_pos = batch.q_pos.cpu().numpy()[: w.n_q_tot]
    attn_flops = attention_flops(w, q_pos)
    proj_flops = 0.0
    if w.hidden is not None:
        sp = w.spec
        proj_flops = 2.0 * w.hidden.shape[1] * (sp.n_q_heads + 2 * sp.n_kv_heads) * sp.head_dim * w.n_q_tot
    stages = {
        "cc_rope_shift": {"bound": "hbm", "ms": stage_ms["rope_shift"], "unit": "GB/s", "peak": PEAK_HBM_GBS,
                          "achieved": work["shift_bytes"] / (stage_ms["rope_shift"] * 1e-3) / 1e9},
        "cc_select": {"bound": "mfma", "ms": stage_ms["select"], "unit": "TFLOP/s", "peak": PEAK_MFMA_BF16_TFLOPS,
                      "achieved": work["score_flops"] / (stage_ms["select"] * 1e-3) / 1e12},
        "cc_sparse_prefill": {"bound": "mfma", "ms": stage_ms["sparse_prefill"], "unit": "TFLOP/s",
                              "peak": PEAK_MFMA_BF16_TFLOPS,
                              "achieved": attn_flops / (stage_ms["sparse_prefill"] * 1e-3) / 1e12},
    }
    if "gather" in stage_ms:
        row_bytes = (w.spec.n_q_heads + 2 * w.spec.n_kv_heads) * w.spec.head_dim * (2 if w.spec.dtype == "bf16" else 4)
        stages["cc_gather_rows(+cc_qkv_project)"] = {
            "bound": "mfma" if proj_flops else "hbm", "ms": stage_ms["gather"],
            "unit": "TFLOP/s" if proj_flops else "GB/s", "peak": PEAK_MFMA_BF16_TFLOPS if proj_flops else PEAK_HBM_GBS,
            "achieved": (proj_flops / (stage_ms["gather"] * 1e-3) / 1e12) if proj_flops else
                        (2.0 * w.n_q_tot * row_bytes / (stage_ms["gather"] * 1e-3) / 1e9)}
    if w.spec.dtype != "bf16":          # the fp32 workload runs on the plain kernels: vector ALU, not MFMA
        for k in ("cc_select", "cc_sparse_prefill"):
            stages[k].update(bound="alu", peak=PEAK_FP32_VALU_TFLOPS)
    for st in stages.values():
        st["frac"] = st["achieved"] / st["peak"]
    return stages, work


def run_workload(wid: int, steps: int, warmup: int):
    """Build workload `wid` on the device, run `warmup` + `steps` whole steps, then time every call of the step."""
    import torch
    import workload as W
    from paper_2502_15734_amd.pipeline import DeviceBatch
    w = W.config(wid)
    batch = DeviceBatch(w)
    for _ in range(warmup):
        batch.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        batch.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stage_ms = time_stages(batch, steps)
    stages, work = stage_figures(w, batch, stage_ms)
    return w, batch, work, dt / steps * 1e3, stage_ms, stages


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, help="benchmark config 1..5 (default 3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-calls", action="store_true",
                    help="skip the timings of entry points outside the step (used for profiles of the step's kernels)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of the other workloads (configs 2, 4, 5) reported under per_config")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 512 MiB device copy (identity cc_gather_rows) so that a "
                         "rocprofv3 --pmc run of this command has a kernel of known HBM traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workload as W
    import paper_2502_15734_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    P.load_library()

    if args.calibrate_copy:
        from paper_2502_15734_amd.binding import CC_BF16, Context
        rows, row_bytes = 1 << 15, 1 << 14                      # 32768 rows x 16 KiB = 512 MiB
        src = torch.empty((rows, row_bytes), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        idx = torch.arange(rows, dtype=torch.int32, device="cuda")
        Context(32, 8, 128, 5.0e5, CC_BF16).gather_rows(src, idx, dst)
        torch.cuda.synchronize()
        del src, dst, idx

    w, batch, work, ms_per_step, stage_ms, stages = run_workload(args.workload, args.steps, args.warmup)
    tokens_per_s = work["recomputed_tokens"] / (ms_per_step * 1e-3)
    extra = None if args.no_extra_calls else time_extra_calls(batch, w, work, args.steps, ms_per_step,
                                                               stage_ms["sparse_prefill"])
    if extra is not None:                  # the extra calls ran on the batch: restore the state a step leaves
        batch.step()
        torch.cuda.synchronize()
    # what a plain device-to-device copy of 512 MiB reaches on this machine, beside the HBM peak
    copy_gbs = measured_copy_gbs()
    stages["cc_rope_shift"]["measured_copy_GBps"] = copy_gbs
    stages["cc_rope_shift"]["frac_of_measured_copy"] = stages["cc_rope_shift"]["achieved"] / copy_gbs
    dominant = max(stages, key=lambda k: stages[k]["ms"])
    dom = stages[dominant]
    kernel_of = {"cc_select": "score_v2_kernel (+ top-N, plan, second pass: ~2 % of the call)",
                 "cc_sparse_prefill": "attn_v2_kernel (+ rope_scatter, plan, second pass: ~5 % of the call)",
                 "cc_rope_shift": "rope_shift_kernel", "cc_gather_rows(+cc_qkv_project)": "qkv_project / gather_rows"}
    traffic = profiled_traffic_bytes(dominant) if args.workload == TRAFFIC_WORKLOAD else None
    roofline = {"kernel": kernel_of[dominant], "call": dominant, "bound": dom["bound"], "achieved": dom["achieved"],
                "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic,
                "traffic_source": (TRAFFIC_PROFILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                   "scaled by a copy of known size; not measured in this run)") if traffic is not None else None,
                "avg_ms": dom["ms"]}
    if dom["bound"] == "mfma":
        roofline["frac_of_measured_mfma_rate"] = dom["achieved"] / MEASURED_MFMA_BF16_TFLOPS

    # the other workloads the benchmark spec names, a few steps each (config 1 is the tiny fp32 case of the tests)
    per_config = None
    if not args.no_per_config:
        per_config = {}
        for wid, n_steps in ((2, 20), (4, 5), (5, 3)):
            if wid == args.workload:
                continue
            w2, b2, work2, ms2, _, stages2 = run_workload(wid, n_steps, 2)
            per_config[W.CONFIG_NAMES[wid]] = {
                "steps": n_steps, "ms_per_step": ms2, "recomputed_tokens": work2["recomputed_tokens"],
                "tokens_per_s": work2["recomputed_tokens"] / (ms2 * 1e-3), "dtype": w2.spec.dtype,
                "stages": {k: {kk: v[kk] for kk in ("ms", "bound", "achieved", "unit", "peak", "frac")} for k, v in stages2.items()}}
            del w2, b2
            torch.cuda.empty_cache()

    result = {
        "metric": "recomputed tokens/sec in selective chunk prefill",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.spec.dtype, "data": "synthetic",
        "config": {"workload": W.CONFIG_NAMES[args.workload]},
        "roofline": roofline,
        "stages": stages,
        "workload_size": {"requests": w.n_requests, "prompt_tokens": w.n_tok, "recomputed_tokens": w.n_q_tot},
        "sparse_prefill_tokens_per_s": w.n_q_tot / (stage_ms["sparse_prefill"] * 1e-3),
        "per_config": per_config,
        # not part of the step: the other entry points of the library, timed on the same batch
        "extra_calls": extra,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["parity"] = cpu_baseline(w, batch, args.cpu_budget)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
