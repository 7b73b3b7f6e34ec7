"""Device-side staging of one batch and the call sequence of the hot path.

Marshalling only: uploads a workload (numpy arrays from workload.generate) into torch device
tensors, allocates outputs and workspaces once, and issues the library calls in order:

    cc_rope_shift -> cc_select -> cc_gather_rows (+ cc_qkv_project) -> cc_sparse_prefill

All arithmetic happens inside libcachecraft's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from .binding import CC_BF16, CC_F32, CC_IMPL_AUTO, Context


def _dev(a: np.ndarray, dtype=None, device="cuda") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return t if dtype is None else t.to(dtype)


class DeviceBatch:
    def __init__(self, w, device: str = "cuda", impl: int = CC_IMPL_AUTO, poison: bool = False,
                 miss_segments=(), fused_gather: bool = True, cow: bool = True):
        """cow: values of cached chunks stay in the store (cc_rope_shift only records where they are);
        cc_sparse_prefill copies a page's values into the request's pool when it recomputes one of its
        tokens and reads all the others from the store (cc_shared_values).
        miss_segments: global indices of chunk segments that have NO chunk-cache in this batch: they
        are not shifted from the store; K, V of all their tokens are written into the request's pages
        (fill_miss) before the other chunks are scored."""
        sp = w.spec
        self.w = w
        self.fused_gather = fused_gather
        self.cow = cow
        self.device = device
        self.dt = torch.bfloat16 if sp.dtype == "bf16" else torch.float32
        self.ctx = Context(sp.n_q_heads, sp.n_kv_heads, sp.head_dim, sp.rope_theta,
                           CC_BF16 if sp.dtype == "bf16" else CC_F32)
        self.ctx.set_impl(impl)
        hq, hkv, d = sp.n_q_heads, sp.n_kv_heads, sp.head_dim
        dt = self.dt
        # shared chunk store (read-only) and request-owned pages
        self.k_store = _dev(w.k_store, dt, device)
        self.v_store = _dev(w.v_store, dt, device)
        nb = max(1, w.n_req_blocks)
        fill = float("nan") if poison else 0.0
        self.k_req = torch.full((nb, hkv, 16, d), fill, dtype=dt, device=device)
        self.v_req = torch.full((nb, hkv, d, 16), fill, dtype=dt, device=device)
        # stored block that still holds the values of a request page (-1: the request's own block does)
        self.v_map = torch.full((nb,), -1, dtype=torch.int32, device=device)
        # metadata
        self.store_tab = _dev(w.store_tab, None, device)
        self.req_tab = _dev(w.req_tab, None, device)
        miss_tabs = {int(w.segments[s][4]) for s in miss_segments}
        shift_descs = np.ascontiguousarray([d for d in w.shift_descs if int(d[1]) not in miss_tabs],
                                           dtype=w.shift_descs.dtype).reshape(-1, w.shift_descs.shape[1])
        self.shift_descs = _dev(shift_descs, None, device)
        rows, pos, slot = [], [], []
        for s in miss_segments:
            _, kind, start, n, tab, _, tok, _ = (int(v) for v in w.segments[s])
            assert kind == 0, "only chunk segments can be misses"
            t = np.arange(n)
            rows.append(tok + t); pos.append(start + t)
            slot.append(w.req_tab[tab + t // 16].astype(np.int64) * 16 + t % 16)
        cat = lambda xs: np.concatenate(xs).astype(np.int32) if xs else np.zeros(0, dtype=np.int32)
        self.miss_rows, self.miss_pos, self.miss_slot = (_dev(cat(a), None, device) for a in (rows, pos, slot))
        self.segments = _dev(w.segments, None, device)
        self.req_seg_off = _dev(w.req_seg_off, None, device)
        self.cu_q = _dev(w.cu_q, None, device)
        self.n_instances = int(shift_descs.shape[0])
        self.max_shift_tokens = int(shift_descs[:, 2].max()) if self.n_instances else 0
        self.max_seg_tokens = w.max_seg_tokens
        self.n_requests = w.n_requests
        self.n_tok, self.n_q_tot = w.n_tok, w.n_q_tot
        self.max_q_per_req = int(np.diff(w.cu_q).max()) if self.n_requests else 0
        # per-token inputs
        self.q = _dev(w.q, dt, device)
        self.projected = w.hidden is not None
        if self.projected:
            self.hidden = _dev(w.hidden, dt, device)
            self.w_qkv = _dev(w.w_qkv, dt, device)
            self.x_c = torch.empty((max(1, self.n_q_tot), w.hidden.shape[1]), dtype=dt, device=device)
        else:
            self.k_new = _dev(w.k_new, dt, device)
            self.v_new = _dev(w.v_new, dt, device)
        # outputs
        nq = max(1, self.n_q_tot)
        i32 = dict(dtype=torch.int32, device=device)
        self.sel_idx = torch.zeros(nq, **i32)
        self.q_row = torch.zeros(nq, **i32)
        self.q_pos = torch.zeros(nq, **i32)
        self.slot_map = torch.zeros(nq, **i32)
        self.scores = torch.zeros(max(1, self.n_tok), dtype=torch.float32, device=device)
        self.q_c = torch.empty((nq, hq, d), dtype=dt, device=device)
        self.k_c = torch.empty((nq, hkv, d), dtype=dt, device=device)
        self.v_c = torch.empty((nq, hkv, d), dtype=dt, device=device)
        self.out = torch.zeros((nq, hq, d), dtype=dt, device=device)
        self.lse = torch.zeros((nq, hq), dtype=torch.float32, device=device)
        self.ws_select = torch.empty(max(256, self.ctx.select_workspace_bytes(self.n_tok, len(w.segments))),
                                     dtype=torch.uint8, device=device)
        self.ws_prefill = torch.empty(max(256, self.ctx.sparse_prefill_workspace_bytes(self.n_tok, len(w.segments))),
                                      dtype=torch.uint8, device=device)

    # ---- the calls, in path order ------------------------------------------------------------
    def rope_shift(self, with_v: bool = True):
        copy_v = with_v and not self.cow
        self.ctx.rope_shift(self.k_store, self.v_store if copy_v else None, self.k_req,
                            self.v_req if copy_v else None, self.store_tab, self.req_tab,
                            self.shift_descs, self.n_instances, self.max_shift_tokens,
                            v_map=self.v_map if (with_v and self.cow) else None)

    @property
    def shared(self):
        """Argument `shared` of the prefill calls."""
        return (self.v_store, self.v_map) if self.cow else None

    def values_pool(self):
        """The request's value pages as the attention sees them (stored blocks resolved): a copy."""
        v = self.v_req.clone()
        if self.cow:
            idx = torch.nonzero(self.v_map >= 0).flatten()
            v[idx] = self.v_store[self.v_map[idx].long()]
        return v

    def fill_miss(self):
        """K, V of every token of the chunks without a cache, into the request's pages."""
        n = int(self.miss_rows.shape[0])
        if n == 0:
            return
        if not hasattr(self, "k_miss"):
            hkv, d = self.w.spec.n_kv_heads, self.w.spec.head_dim
            self.k_miss = torch.empty((n, hkv, d), dtype=self.dt, device=self.device)
            self.v_miss = torch.empty((n, hkv, d), dtype=self.dt, device=self.device)
        self.ctx.gather_rows(self.k_new, self.miss_rows, self.k_miss)
        self.ctx.gather_rows(self.v_new, self.miss_rows, self.v_miss)
        self.ctx.scatter_kv(self.k_miss, self.v_miss, self.miss_pos, self.miss_slot, self.k_req, self.v_req)

    def _rows(self, t):
        """The first n_q_tot rows of a per-query buffer (the buffers are sized for the largest budget)."""
        return t[: max(1, self.n_q_tot)] if self.n_q_tot < t.shape[0] else t

    def select(self):
        r = self._rows
        self.ctx.select(self.q, self.k_req, self.req_tab, self.segments, self.req_seg_off,
                        self.n_requests, self.max_seg_tokens, r(self.sel_idx), r(self.q_row), r(self.q_pos),
                        r(self.slot_map), self.scores, self.ws_select)

    def select_from_scores(self, scores=None):
        """Selection from given per-token scores (default: the scores cc_select wrote)."""
        r = self._rows
        self.ctx.select_from_scores(self.scores if scores is None else scores, self.req_tab, self.segments,
                                    r(self.sel_idx), r(self.q_row), r(self.q_pos), r(self.slot_map), self.ws_select)

    def set_budget(self, n_select):
        """New token budgets N per segment (numpy int array over all segments; question segments keep
        their length): rewrites n_select / sel_off of the segment table and the row offsets cu_q."""
        seg = np.array(self.w.segments, dtype=np.int32, copy=True) if not hasattr(self, "_seg_host") else self._seg_host
        n_select = np.asarray(n_select, dtype=np.int64)
        is_q = seg[:, 1] != 0
        nsel = np.where(is_q, seg[:, 3], np.minimum(n_select, seg[:, 3])).astype(np.int64)
        seg[:, 5] = nsel
        seg[:, 7] = np.concatenate([[0], np.cumsum(nsel)[:-1]])
        cu_q = np.concatenate([seg[self.w.req_seg_off[:-1], 7], [int(nsel.sum())]]).astype(np.int32)
        assert int(nsel.sum()) <= self.q_c.shape[0], "budget exceeds the buffers this batch was built with"
        self._seg_host = seg
        self.segments.copy_(torch.from_numpy(seg))
        self.cu_q.copy_(torch.from_numpy(cu_q))
        self.n_q_tot = int(nsel.sum())
        self.max_q_per_req = int(np.diff(cu_q).max()) if self.n_requests else 0
        self.cu_q_host = cu_q

    def gather(self):
        """Compact the chosen tokens' rows (and project them when the workload has hidden states)."""
        if self.n_q_tot == 0:
            return
        r = self._rows
        if self.projected:
            self.ctx.gather_rows(self.hidden, r(self.q_row), r(self.x_c))
            self.ctx.qkv_project(r(self.x_c), self.w_qkv, r(self.q_c), r(self.k_c), r(self.v_c))
        else:
            self.ctx.gather_rows(self.q, r(self.q_row), r(self.q_c))
            self.ctx.gather_rows(self.k_new, r(self.q_row), r(self.k_c))
            self.ctx.gather_rows(self.v_new, r(self.q_row), r(self.v_c))

    def sparse_prefill_fused(self):
        """cc_sparse_prefill straight on the per-token tensors, through cc_select's q_row list (no gather)."""
        if self.n_q_tot == 0:
            return
        assert not self.projected
        r = self._rows
        self.ctx.sparse_prefill(self.q, self.k_new, self.v_new, self.q_pos, self.slot_map, self.cu_q,
                                self.max_q_per_req, self.k_req, self.v_req, self.req_tab,
                                self.segments, self.req_seg_off, self.n_requests, self.n_tok, r(self.out), self.lse,
                                self.ws_prefill, src_rows=r(self.q_row), shared=self.shared)

    def sparse_prefill(self):
        if self.n_q_tot == 0:
            return
        r = self._rows
        self.ctx.sparse_prefill(r(self.q_c), r(self.k_c), r(self.v_c), self.q_pos, self.slot_map, self.cu_q,
                                self.max_q_per_req, self.k_req, self.v_req, self.req_tab,
                                self.segments, self.req_seg_off, self.n_requests, self.n_tok, r(self.out), self.lse,
                                self.ws_prefill, shared=self.shared)

    def _mass_buffers(self):
        n_segs = int(self.segments.shape[0])
        if not hasattr(self, "seg_mass"):
            seg = self.w.segments
            self.max_question_rows = int(seg[seg[:, 1] == 1, 3].max()) if (seg[:, 1] == 1).any() else 0
            self.seg_mass = torch.zeros(max(1, n_segs), dtype=torch.float32, device=self.device)
            nbytes = self.ctx.question_mass_workspace_bytes(self.n_tok, n_segs, self.max_question_rows)
            self.ws_mass = torch.empty(max(256, nbytes), dtype=torch.uint8, device=self.device)
        return n_segs

    def _qkv_args(self, fused):
        """(q, k_new, v_new, src_rows) of a prefill call: compact rows, or the per-token tensors read
        through cc_select's row list."""
        r = self._rows
        if fused:
            assert not self.projected, "a projected workload has no per-token q, k, v"
            return self.q, self.k_new, self.v_new, r(self.q_row)
        return r(self.q_c), r(self.k_c), r(self.v_c), None

    def sparse_prefill_mass(self, fused: bool = False):
        """sparse_prefill and the question's masses per segment in one call (by-product where possible).
        fused: read q, k_new, v_new per token through the row list instead of the gathered copies."""
        n_segs = self._mass_buffers()
        if self.n_q_tot == 0:
            self.seg_mass.zero_()
            return self.seg_mass
        if not hasattr(self, "ws_prefill_mass"):
            self.max_segs_per_req = int(np.diff(self.w.req_seg_off).max())
            nbytes = self.ctx.sparse_prefill_mass_workspace_bytes(self.n_tok, n_segs, self.n_requests,
                                                                  self.max_question_rows, self.max_segs_per_req)
            self.ws_prefill_mass = torch.empty(max(256, nbytes), dtype=torch.uint8, device=self.device)
        r = self._rows
        q, k_new, v_new, src_rows = self._qkv_args(fused)
        self.ctx.sparse_prefill_mass(q, k_new, v_new, self.q_pos, self.slot_map, self.cu_q,
                                     self.max_q_per_req, min(self.max_question_rows, self.max_q_per_req), self.k_req,
                                     self.v_req, self.req_tab, self.segments, self.req_seg_off, self.n_requests,
                                     self.max_segs_per_req, self.n_tok, r(self.out), self.lse, self.seg_mass,
                                     self.ws_prefill_mass, src_rows=src_rows, shared=self.shared)
        return self.seg_mass

    def question_mass(self):
        """inter(C_i, U) per segment, from the last sparse_prefill's lse (float32 [n_segs])."""
        self._mass_buffers()
        self.ctx.question_mass(self._rows(self.q_c), self.q_pos, self.cu_q, self.max_question_rows, self.k_req, self.v_req,
                               self.req_tab, self.segments, self.req_seg_off, self.n_requests, self.n_tok,
                               self.lse, self.seg_mass, self.ws_mass)
        return self.seg_mass

    def _pair_buffers(self, n_segs):
        if not hasattr(self, "pair_mass"):
            n_r = np.diff(self.w.req_seg_off).astype(np.int64)
            self.pair_off = np.concatenate([[0], np.cumsum(n_r * (n_r + 1) // 2)])
            self.pair_mass = torch.zeros(max(1, int(self.pair_off[-1])), dtype=torch.float32, device=self.device)
            self.self_mass = torch.zeros(max(1, n_segs), dtype=torch.float32, device=self.device)

    def chunk_attention(self):
        """Segment-to-segment attention sums of the last sparse_prefill's rows: (pair_mass, self_mass,
        pair_off) with pair_off[r] the first pair of request r (pair (t, s) sits at t (t + 1) / 2 + s)."""
        n_segs = int(self.segments.shape[0])
        self._pair_buffers(n_segs)
        if not hasattr(self, "ws_pairs"):
            nbytes = self.ctx.chunk_attention_workspace_bytes(self.n_tok, n_segs, self.q_c.shape[0], self.max_q_per_req)
            self.ws_pairs = torch.empty(max(256, nbytes), dtype=torch.uint8, device=self.device)
        self.ctx.chunk_attention(self._rows(self.q_c), self.q_pos, self.slot_map, self.cu_q, self.max_q_per_req, self.k_req,
                                 self.v_req, self.req_tab, self.segments, self.req_seg_off, self.n_requests,
                                 self.n_tok, self.lse, self.pair_mass, self.self_mass, self.ws_pairs)
        return self.pair_mass, self.self_mass, self.pair_off

    def sparse_prefill_pairs(self, fused: bool = False):
        """sparse_prefill and chunk_attention's sums (and the question's masses) in one call."""
        n_segs = self._mass_buffers()
        self._pair_buffers(n_segs)
        if not hasattr(self, "ws_prefill_pairs"):
            self.max_segs_per_req = int(np.diff(self.w.req_seg_off).max())
            nbytes = self.ctx.sparse_prefill_pairs_workspace_bytes(self.n_tok, n_segs, self.q_c.shape[0],
                                                                   self.max_q_per_req, self.max_segs_per_req)
            self.ws_prefill_pairs = torch.empty(max(256, nbytes), dtype=torch.uint8, device=self.device)
        if self.n_q_tot == 0:
            self.pair_mass.zero_(); self.self_mass.zero_(); self.seg_mass.zero_()
            return self.pair_mass, self.self_mass, self.pair_off
        r = self._rows
        q, k_new, v_new, src_rows = self._qkv_args(fused)
        self.ctx.sparse_prefill_pairs(q, k_new, v_new, self.q_pos, self.slot_map, self.cu_q,
                                      self.max_q_per_req, self.k_req, self.v_req, self.req_tab, self.segments,
                                      self.req_seg_off, self.n_requests, self.max_segs_per_req, self.n_tok,
                                      r(self.out), self.lse, self.seg_mass, self.pair_mass, self.self_mass,
                                      self.ws_prefill_pairs, src_rows=src_rows, shared=self.shared)
        return self.pair_mass, self.self_mass, self.pair_off

    def step(self):
        """One pass of the whole hot path over the batch."""
        self.rope_shift()
        self.fill_miss()
        self.select()
        if self.projected or not self.fused_gather:
            self.gather()
            self.sparse_prefill()
        else:                      # q, k_new, v_new are given per token: read them through the row list
            self.sparse_prefill_fused()

    # ---- test helper: impose a selection computed elsewhere ------------------------------------
    def set_selection(self, sel_idx: np.ndarray, q_row: np.ndarray, q_pos: np.ndarray, slot_map: np.ndarray):
        for dst, src in ((self.sel_idx, sel_idx), (self.q_row, q_row), (self.q_pos, q_pos), (self.slot_map, slot_map)):
            if self.n_q_tot:
                dst.copy_(torch.from_numpy(np.ascontiguousarray(src, dtype=np.int32)))
