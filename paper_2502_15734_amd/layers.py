"""Loops over layers built from the library's calls (Sec. 3.4).

LayerLoop (attention only): per layer the chunk store arrives through the layer-wise preloader,
cached keys are re-positioned, the chosen tokens are recomputed and attended, the question's
attention to every chunk feeds Algorithm 1, and once a request's focused chunks are settled the
other chunks of that request are no longer recomputed.  The batch holds ONE layer's per-token
tensors; a caller that has a different set per layer installs it through the loop's layer_inputs
hook.

DecoderLoop (whole layers): the hidden states of the chosen rows pass through normalisation,
projections, the partial prefill and the feed-forward network of every layer.

Argument marshalling and call order only; every step runs in libcachecraft.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

from .binding import CC_IMPL_AUTO, FocusTracker, Preloader, preload_depth
from .pipeline import DeviceBatch


class DecoderLoop:
    """The hidden states of the chosen rows through whole decoder layers (Sec. 2.1, Sec. 3.4.3): per
    layer cc_rms_norm -> cc_qkv_project -> cc_sparse_prefill over the re-positioned chunk-caches ->
    cc_linear (output projection + residual) -> cc_rms_norm -> cc_gated_linear -> cc_linear (down
    projection + residual).  The rows are chosen once, before the first layer, from the workload's
    per-token queries (cc_select); every layer sees the same synthetic chunk store.
    weights: one workload.LayerWeights per layer.
    window: if given, the question's attention to every chunk (a by-product of the attention call)
    feeds Algorithm 1 in every layer; once a request's focused chunks are settled, the rows of its
    other chunks leave the list (Sec. 3.2.2) and the surviving rows' hidden states are compacted."""

    def __init__(self, w, weights: Sequence, window: Optional[int] = None, impl: int = CC_IMPL_AUTO,
                 device: str = "cuda", preload: bool = False, depth: int = 1):
        """preload: every layer's chunk store comes from pinned host memory through the layer-wise
        preloader (Algorithm 2), `depth` layers ahead of the one being computed."""
        assert w.hidden is not None, "the workload must carry hidden states"
        self.w, self.window = w, window
        self.batch = DeviceBatch(w, device=device, impl=impl)
        b = self.batch
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device).to(b.dt)
        self.weights = [{k: up(getattr(lw, k)) for k in ("gain_attn", "gain_ffn", "w_qkv", "w_o", "w_gate", "w_up", "w_down")}
                        for lw in weights]
        self.eps = [float(lw.eps) for lw in weights]
        n, hidden, ffn = max(1, b.n_q_tot), w.hidden.shape[1], weights[0].w_gate.shape[0]
        mk = lambda cols: torch.empty((n, cols), dtype=b.dt, device=device)
        self.h, self.h1, self.x, self.act, self.h_alt = mk(hidden), mk(hidden), mk(hidden), mk(ffn), mk(hidden)
        seg = w.segments
        self.chunk_segs = [[s for s in range(int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])) if seg[s][1] == 0]
                           for r in range(w.n_requests)]
        self.trackers = [FocusTracker(max(1, len(c)), window) for c in self.chunk_segs] if window else []
        self.budget = np.array(seg[:, 5], dtype=np.int64)
        self.stop_layer: List[Optional[int]] = [None] * w.n_requests
        self.focused: List[Optional[List[int]]] = [None] * w.n_requests
        self.keep_idx = torch.zeros(n, dtype=torch.int32, device=device)
        self.pre = None
        if preload:
            n_layers = len(weights)
            self.k_host, self.v_host = b.k_store.cpu().pin_memory(), b.v_store.cpu().pin_memory()
            n_slots = min(depth + 1, n_layers)
            self.slots = [(torch.empty_like(b.k_store), torch.empty_like(b.v_store)) for _ in range(n_slots)]
            self.pre = (Preloader(n_layers, depth, n_slots), Preloader(n_layers, depth, n_slots))
            for l in range(n_layers):
                self.pre[0].set_layer(l, self.k_host, self.slots[l % n_slots][0])
                self.pre[1].set_layer(l, self.v_host, self.slots[l % n_slots][1])

    def _shift(self, l):
        """Layer l's chunk-caches (waiting for the preloader's copy if there is one), re-positioned."""
        b = self.batch
        if self.pre is not None:
            self.pre[0].acquire(l); self.pre[1].acquire(l)
            b.k_store, b.v_store = self.slots[l % len(self.slots)]
        b.rope_shift()
        if self.pre is not None:                               # the key slot is free once the shift has read it;
            self.pre[0].release(l)                             # the values are read by the attention, unless copied
            if not b.cow:
                self.pre[1].release(l)

    def _drop_rows(self, new_budget):
        """New budgets: rebuild the row list (same scores, same order) and compact the hidden states."""
        b = self.batch
        old = np.array(getattr(b, "_seg_host", self.w.segments), copy=True)
        b.set_budget(new_budget)
        new = b._seg_host
        keep = np.concatenate([np.arange(int(o[7]), int(o[7]) + int(nw[5])) for o, nw in zip(old, new)] or
                              [np.zeros(0)]).astype(np.int32)
        assert len(keep) == b.n_q_tot
        if b.n_q_tot:
            self.keep_idx[: len(keep)].copy_(torch.from_numpy(keep))
            b.ctx.gather_rows(self.h, self.keep_idx[: len(keep)], self.h_alt[: len(keep)])
            self.h, self.h_alt = self.h_alt, self.h
            b.select_from_scores()

    def run(self, keep: bool = False):
        """Returns one record per layer (ms, rows; with keep also h_in, out, lse, h1, h2 as numpy arrays)."""
        b = self.batch
        self._shift(0)
        b.select()
        records = []
        for l, lw in enumerate(self.weights):
            n = b.n_q_tot
            if n == 0:
                break
            t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
            t0.record()
            h, h1, x, act = self.h[:n], self.h1[:n], self.x[:n], self.act[:n]
            o2 = b.out[:n].view(n, -1)
            if l == 0:
                b.ctx.gather_rows(b.hidden, b.q_row[:n], h)
            else:
                self._shift(l)
            rec = {"layer": l + 1, "rows": n}
            if keep:
                rec["h_in"] = h.float().cpu().numpy()
                rec["cu_q"] = np.array(getattr(b, "cu_q_host", self.w.cu_q), copy=True)
            b.ctx.rms_norm(h, lw["gain_attn"], self.eps[l], x)
            b.ctx.qkv_project(x, lw["w_qkv"], b.q_c[:n], b.k_c[:n], b.v_c[:n])
            if self.window:
                mass = b.sparse_prefill_mass()
            else:
                b.sparse_prefill()
            if self.pre is not None and b.cow:
                self.pre[1].release(l)
            b.ctx.linear(o2, lw["w_o"], h1, residual=h)
            b.ctx.rms_norm(h1, lw["gain_ffn"], self.eps[l], x)
            b.ctx.gated_linear(x, lw["w_gate"], lw["w_up"], act)
            b.ctx.linear(act, lw["w_down"], h, residual=h1)
            t1.record()
            rec["_events"] = (t0, t1)
            if keep:
                torch.cuda.synchronize()
                rec.update(out=b.out[:n].float().cpu().numpy(), lse=b.lse[:n].cpu().numpy(),
                           h1=h1.float().cpu().numpy(), h2=h.float().cpu().numpy())
            if self.window:
                m = mass.cpu().numpy()                     # (synchronises; Algorithm 1 runs on the host)
                rec["mass"] = m[: len(self.w.segments)].copy()
                changed = False
                for r, segs in enumerate(self.chunk_segs):
                    if self.stop_layer[r] is not None or not segs:
                        continue
                    stop, focused = self.trackers[r].update([float(m[s]) for s in segs])
                    if stop:
                        self.stop_layer[r], self.focused[r] = l + 1, focused
                        for i, sgi in enumerate(segs):
                            if i not in focused and self.budget[sgi]:
                                self.budget[sgi] = 0
                                changed = True
                rec["stop_layer"] = list(self.stop_layer)
                rec["focused"] = [None if f is None else list(f) for f in self.focused]
                if changed and l + 1 < len(self.weights):
                    self._drop_rows(self.budget)
            records.append(rec)
        torch.cuda.synchronize()
        for rec in records:
            t0, t1 = rec.pop("_events")
            rec["ms"] = t0.elapsed_time(t1)
        return records

    def close(self):
        for t in self.trackers:
            t.close()
        self.trackers = []
        if self.pre is not None:
            for p in self.pre:
                p.close()
            self.pre = None


class LayerLoop:
    def __init__(self, w, n_layers: int, window: int,
                 layer_inputs: Optional[Callable[[int, DeviceBatch], None]] = None,
                 impl: int = CC_IMPL_AUTO, preload: bool = True, depth: Optional[int] = None,
                 device: str = "cuda"):
        """layer_inputs(l, batch), if given, runs before layer l's attention on the stream the loop
        uses; it may overwrite batch.q / batch.k_new / batch.v_new (or batch.hidden) in place with
        layer l's tensors.  The attention reads them per token through the row list: the loop
        makes no compact copies unless the workload is projected from hidden states."""
        self.w, self.n_layers, self.window, self.layer_inputs = w, n_layers, window, layer_inputs
        self.batch = DeviceBatch(w, device=device, impl=impl)
        b = self.batch
        seg = w.segments
        self.chunk_segs = [[s for s in range(int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])) if seg[s][1] == 0]
                           for r in range(w.n_requests)]
        self.trackers = [FocusTracker(max(1, len(c)), window) for c in self.chunk_segs]
        self.budget = np.array(seg[:, 5], dtype=np.int64)
        self.stop_layer: List[Optional[int]] = [None] * w.n_requests
        self.focused: List[Optional[List[int]]] = [None] * w.n_requests
        self.mass_host = torch.zeros(max(1, len(seg)), dtype=torch.float32).pin_memory()
        self.mass_ready = torch.cuda.Event()
        self.pre = None
        if preload:
            self.k_host, self.v_host = b.k_store.cpu().pin_memory(), b.v_store.cpu().pin_memory()
            self.depth = depth if depth is not None else 1
            n_slots = min(self.depth + 1, n_layers)
            self.slots = [(torch.empty_like(b.k_store), torch.empty_like(b.v_store)) for _ in range(n_slots)]
            self.pre = (Preloader(n_layers, self.depth, n_slots), Preloader(n_layers, self.depth, n_slots))
            for l in range(n_layers):
                self.pre[0].set_layer(l, self.k_host, self.slots[l % n_slots][0])
                self.pre[1].set_layer(l, self.v_host, self.slots[l % n_slots][1])

    def run(self, scores: Optional[np.ndarray] = None, keep_outputs: bool = False):
        """scores: per-token scores to select from (the ordered list a chunk's metadata keeps); by
        default layer 0 computes them with cc_select and the later layers reuse them.
        Returns one record per layer: rows recomputed, per-request focused sets decided so far."""
        b, w = self.batch, self.w
        if scores is not None:
            b.scores.copy_(torch.from_numpy(np.ascontiguousarray(scores, dtype=np.float32)))
        records = []
        for l in range(self.n_layers):
            t_start = torch.cuda.Event(enable_timing=True); t_end = torch.cuda.Event(enable_timing=True)
            t_start.record()
            if self.pre is not None:
                self.pre[0].acquire(l); self.pre[1].acquire(l)
                b.k_store, b.v_store = self.slots[l % len(self.slots)]
            b.rope_shift()
            if l == 0 and scores is None:
                b.select()
            else:
                b.select_from_scores()
            if self.layer_inputs is not None:
                self.layer_inputs(l, b)
            if b.projected:
                b.gather()
            mass = b.sparse_prefill_mass(fused=not b.projected)   # attention + the question's masses in one call
            self.mass_host.copy_(mass, non_blocking=True)
            self.mass_ready.record()
            if self.pre is not None:
                self.pre[0].release(l); self.pre[1].release(l)
            t_end.record()
            rec = {"layer": l + 1, "rows": b.n_q_tot, "_events": (t_start, t_end)}
            if keep_outputs:
                torch.cuda.synchronize()
                rec["out"] = b.out[: b.n_q_tot].float().cpu().numpy()
                rec["lse"] = b.lse[: b.n_q_tot].cpu().numpy()
                rec["sel_idx"] = b.sel_idx[: b.n_q_tot].cpu().numpy()
                rec["cu_q"] = np.array(getattr(b, "cu_q_host", w.cu_q), copy=True)
            # Algorithm 1 on this layer's masses; a settled request drops its unfocused chunks
            self.mass_ready.synchronize()
            m = self.mass_host.numpy()
            rec["mass"] = m[: len(w.segments)].copy()
            changed = False
            for r, segs in enumerate(self.chunk_segs):
                if self.stop_layer[r] is not None or not segs:
                    continue
                stop, focused = self.trackers[r].update([float(m[s]) for s in segs])
                if stop:
                    self.stop_layer[r], self.focused[r] = l + 1, focused
                    for i, sgi in enumerate(segs):
                        if i not in focused:
                            self.budget[sgi] = 0
                            changed = True
            rec["stop_layer"] = list(self.stop_layer)
            rec["focused"] = [None if f is None else list(f) for f in self.focused]
            if changed and l + 1 < self.n_layers:
                b.set_budget(self.budget)
            records.append(rec)
        torch.cuda.synchronize()
        for rec in records:
            t_start, t_end = rec.pop("_events")
            rec["ms"] = t_start.elapsed_time(t_end)
        return records

    def close(self):
        for t in self.trackers:
            t.close()
        if self.pre is not None:
            for p in self.pre:
                p.close()
            self.pre = None
