"""cc_sparse_prefill_static (the entry point that allocates nothing: its key-tile plan goes into a
device array inside the library) against cc_sparse_prefill, through the C ABI: same out, lse and
fixed K/V bit for bit, on two calls in a row, the second on a smaller batch."""
from __future__ import annotations

import numpy as np
import pytest

import workload as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run_both(w):
    import paper_2502_15734_amd as P
    from paper_2502_15734_amd.pipeline import DeviceBatch
    b = DeviceBatch(w, poison=True)
    b.rope_shift(); b.select()
    r = b._rows
    # reference: the existing entry point with a caller-owned workspace
    b.sparse_prefill_fused()
    torch.cuda.synchronize()
    ref = (b.out.clone(), b.lse.clone(), b.k_req.clone(), b.v_req.clone(), b.v_map.clone())
    # the same batch again (pages restored by the shift), through the entry point without a workspace
    b.out.fill_(float("nan")); b.lse.fill_(float("nan"))
    b.rope_shift()
    lib, ctx = P.load_library(), b.ctx
    p = lambda t: None if t is None else t.data_ptr()
    from paper_2502_15734_amd.binding import _shared
    rc = lib.cc_sparse_prefill_static(
        ctx._h, p(b.q), p(b.k_new), p(b.v_new), p(r(b.q_row)), p(b.q_pos), p(b.slot_map), p(b.cu_q), b.n_q_tot,
        b.max_q_per_req, p(b.k_req), p(b.v_req), b.k_req.shape[0], p(b.req_tab), p(b.segments), b.segments.shape[0],
        p(b.req_seg_off), b.n_requests, b.n_tok, _shared(b.shared), p(r(b.out)), p(b.lse),
        torch.cuda.current_stream().cuda_stream)
    assert rc == 0, lib.cc_last_error(ctx._h)
    torch.cuda.synchronize()
    got = (b.out, b.lse, b.k_req, b.v_req, b.v_map)
    for name, g, e in zip(("out", "lse", "k pages", "v pages", "value map"), got, ref):
        assert torch.equal(torch.nan_to_num(g.float(), nan=-7.0), torch.nan_to_num(e.float(), nan=-7.0)), \
            f"{w.spec.name}: {name} differs between cc_sparse_prefill_static and cc_sparse_prefill"


def test_static_scratch_matches_workspace_call_twice():
    import paper_2502_15734_amd as P
    P.load_library()
    # a batch of several requests and ragged tiles (wide MFMA kernel + redo pass), then a smaller one
    # (narrow kernels; its plan overwrites only the head of what the first call left in the scratch)
    _run_both(W.config(3, 0.25))
    _run_both(W.config(2, 0.25))


def test_static_scratch_rejects_oversized_plan():
    import paper_2502_15734_amd as P
    lib = P.load_library()
    w = W.config(2, 0.25)
    from paper_2502_15734_amd.pipeline import DeviceBatch
    b = DeviceBatch(w)
    p = lambda t: t.data_ptr()
    rc = lib.cc_sparse_prefill_static(
        b.ctx._h, p(b.q), p(b.k_new), p(b.v_new), None, p(b.q_pos), p(b.slot_map), p(b.cu_q), 8, 8, p(b.k_req),
        p(b.v_req), b.k_req.shape[0], p(b.req_tab), p(b.segments), b.segments.shape[0], p(b.req_seg_off),
        b.n_requests, 50_000_000, None, p(b.out), p(b.lse), None)
    assert rc == -3 and b"scratch" in lib.cc_last_error(b.ctx._h)
