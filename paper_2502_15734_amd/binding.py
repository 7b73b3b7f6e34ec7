"""ctypes binding of libcachecraft's C ABI (include/cc.h).  Same names, tensors in, tensors out.

The library is loaded from this package directory (built in-tree by build.py); a missing library
is a hard error -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

CC_F32, CC_BF16 = 0, 1
CC_IMPL_AUTO, CC_IMPL_SCALAR, CC_IMPL_MFMA_NARROW, CC_IMPL_MFMA_WIDE = 0, 1, 2, 3
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None


class CacheCraftError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libcachecraft status {status}: {message}")
        self.status = status


class _Reuse(C.Structure):
    _fields_ = [("beta", C.c_double), ("gamma", C.c_double), ("beta_adj", C.c_double), ("cfo", C.c_double),
                ("n_recompute", C.c_int32), ("reserved", C.c_int32)]


class _Config(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("rope_theta", C.c_double)]


def library_path() -> str:
    """The in-tree library; CACHECRAFT_LIBRARY names another build of it (kernel experiments)."""
    return os.environ.get("CACHECRAFT_LIBRARY") or os.path.join(_HERE, "libcachecraft.so")


def load_library() -> C.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2502_15734_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.cc_create.argtypes = [C.POINTER(vp), C.POINTER(_Config)]
    lib.cc_create.restype = C.c_int
    lib.cc_destroy.argtypes = [vp]
    lib.cc_destroy.restype = None
    lib.cc_status_string.argtypes = [C.c_int]
    lib.cc_status_string.restype = C.c_char_p
    lib.cc_last_error.argtypes = [vp]
    lib.cc_last_error.restype = C.c_char_p
    lib.cc_set_impl.argtypes = [vp, C.c_int]
    lib.cc_set_impl.restype = C.c_int
    lib.cc_rope_shift.argtypes = [vp, vp, vp, i32, vp, vp, i32, vp, vp, vp, i32, i32, vp, vp]
    lib.cc_rope_place.argtypes = [vp, vp, vp, i32, vp, vp, i32, vp, vp, vp, i32, i32, vp, vp]
    lib.cc_rope_place.restype = C.c_int
    lib.cc_rope_shift.restype = C.c_int
    lib.cc_select_workspace_bytes.argtypes = [vp, i32, i32]
    lib.cc_select_workspace_bytes.restype = sz
    lib.cc_select.argtypes = [vp, vp, i32, vp, i32, vp, vp, i32, vp, i32, i32,
                              vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.cc_select.restype = C.c_int
    lib.cc_select_from_scores.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.cc_select_from_scores.restype = C.c_int
    lib.cc_gather_rows.argtypes = [vp, vp, i32, vp, i32, sz, vp, vp]
    lib.cc_gather_rows.restype = C.c_int
    lib.cc_qkv_project.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.cc_qkv_project.restype = C.c_int
    lib.cc_sparse_prefill_workspace_bytes.argtypes = [vp, i32, i32]
    lib.cc_sparse_prefill_workspace_bytes.restype = sz
    lib.cc_sparse_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp, i32,
                                      vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.cc_sparse_prefill.restype = C.c_int
    lib.cc_sparse_prefill_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp, i32,
                                             vp, i32, i32, vp, vp, vp, vp]
    lib.cc_sparse_prefill_static.restype = C.c_int
    lib.cc_rms_norm.argtypes = [vp, vp, vp, C.c_float, i32, i32, vp, vp]
    lib.cc_rms_norm.restype = C.c_int
    lib.cc_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.cc_linear.restype = C.c_int
    lib.cc_gated_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.cc_gated_linear.restype = C.c_int
    lib.cc_sparse_prefill_mass_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    lib.cc_sparse_prefill_mass_workspace_bytes.restype = sz
    lib.cc_sparse_prefill_mass.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, i32, vp, vp, i32,
                                           vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.cc_sparse_prefill_mass.restype = C.c_int
    lib.cc_sparse_prefill_pairs_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    lib.cc_sparse_prefill_pairs_workspace_bytes.restype = sz
    lib.cc_sparse_prefill_pairs.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp, i32,
                                            vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cc_sparse_prefill_pairs.restype = C.c_int
    lib.cc_check_query_list_workspace_bytes.argtypes = [vp, i32]
    lib.cc_check_query_list_workspace_bytes.restype = sz
    lib.cc_check_query_list.argtypes = [vp, vp, i32, i32, vp, vp, sz, vp]
    lib.cc_check_query_list.restype = C.c_int
    lib.cc_scatter_kv.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, vp]
    lib.cc_scatter_kv.restype = C.c_int
    lib.cc_question_mass_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.cc_question_mass_workspace_bytes.restype = sz
    lib.cc_question_mass.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp, i32, vp, i32, i32,
                                     vp, vp, vp, sz, vp]
    lib.cc_question_mass.restype = C.c_int
    lib.cc_chunk_attention_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.cc_chunk_attention_workspace_bytes.restype = sz
    lib.cc_chunk_attention.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp, vp, i32, vp, i32, i32, i32,
                                       vp, vp, vp, vp, sz, vp]
    lib.cc_chunk_attention.restype = C.c_int
    dp = C.POINTER(C.c_double)
    lib.cc_chunk_ab.argtypes = [dp, C.POINTER(i32), i32, C.c_double, i32, dp, dp]
    lib.cc_chunk_ab.restype = C.c_int
    lib.cc_chunk_cci.argtypes = [dp, dp, i32, dp]
    lib.cc_chunk_cci.restype = C.c_int
    lib.cc_chunk_reuse.argtypes = [C.POINTER(C.c_int64), dp, i32, C.POINTER(C.c_int64), i32, C.c_double, C.c_double,
                                   i32, C.POINTER(_Reuse)]
    lib.cc_chunk_reuse.restype = C.c_int
    lib.cc_preload_depth.argtypes = [i32, C.c_double, C.c_double]
    lib.cc_preload_depth.restype = i32
    lib.cc_preloader_create.argtypes = [C.POINTER(vp), i32, i32, i32]
    lib.cc_preloader_create.restype = C.c_int
    lib.cc_preloader_destroy.argtypes = [vp]
    lib.cc_preloader_destroy.restype = None
    lib.cc_preloader_set_layer.argtypes = [vp, i32, vp, vp, sz]
    lib.cc_preloader_set_layer.restype = C.c_int
    lib.cc_preloader_acquire.argtypes = [vp, i32, vp]
    lib.cc_preloader_acquire.restype = C.c_int
    lib.cc_preloader_release.argtypes = [vp, i32, vp]
    lib.cc_preloader_release.restype = C.c_int
    lib.cc_preloader_issued.argtypes = [vp, C.POINTER(i32), i32]
    lib.cc_preloader_issued.restype = i32
    lib.cc_focus_create.argtypes = [C.POINTER(vp), i32, i32]
    lib.cc_focus_create.restype = C.c_int
    lib.cc_focus_destroy.argtypes = [vp]
    lib.cc_focus_destroy.restype = None
    lib.cc_focus_update.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32), C.POINTER(i32)]
    lib.cc_focus_update.restype = C.c_int
    lib.cc_focus_layer.argtypes = [vp]
    lib.cc_focus_layer.restype = i32
    _LIB = lib
    return lib


class SharedValues(C.Structure):
    """cc_shared_values: values that stay in the chunk store until a token of their page is recomputed."""
    _fields_ = [("v_shared", C.c_void_p), ("n_shared_blocks", C.c_int32), ("v_map", C.c_void_p)]


def _shared(shared):
    """(v_shared pool, v_map) or None -> pointer to a cc_shared_values (kept alive by the caller's frame)."""
    if shared is None:
        return None
    v_shared, v_map = shared
    return C.byref(SharedValues(_ptr(v_shared), v_shared.shape[0], _ptr(v_map)))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("libcachecraft takes contiguous tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Context:
    """cc_ctx handle.  Methods mirror the C entry points one to one."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float,
                 dtype: int, block_size: int = 16):
        self._lib = load_library()
        self._h = C.c_void_p()
        cfg = _Config(n_q_heads, n_kv_heads, head_dim, block_size, dtype, 0, rope_theta)
        st = self._lib.cc_create(C.byref(self._h), C.byref(cfg))
        if st != 0:
            raise CacheCraftError(st, self._lib.cc_status_string(st).decode())
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.dtype = dtype

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.cc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != 0:
            raise CacheCraftError(st, self._lib.cc_last_error(self._h).decode())

    def set_impl(self, impl: int):
        self._check(self._lib.cc_set_impl(self._h, impl))

    # -- cc_rope_shift ---------------------------------------------------------------------
    def rope_shift(self, k_src, v_src, k_dst, v_dst, src_tab, dst_tab, descs, n_instances, max_tokens, v_map=None):
        """v_map: if given (v_src and v_dst None), values stay in the store and the map records where."""
        self._check(self._lib.cc_rope_shift(
            self._h, _ptr(k_src), _ptr(v_src), k_src.shape[0], _ptr(k_dst), _ptr(v_dst), k_dst.shape[0],
            _ptr(src_tab), _ptr(dst_tab), _ptr(descs), n_instances, max_tokens, _ptr(v_map), _stream()))

    def rope_place(self, k_src, v_src, k_dst, v_dst, src_tab, dst_tab, descs, n_instances, max_tokens, v_map=None):
        """cc_rope_shift for a store of unrotated keys: descs' delta_pos is the new position of token 0."""
        self._check(self._lib.cc_rope_place(
            self._h, _ptr(k_src), _ptr(v_src), k_src.shape[0], _ptr(k_dst), _ptr(v_dst), k_dst.shape[0],
            _ptr(src_tab), _ptr(dst_tab), _ptr(descs), n_instances, max_tokens, _ptr(v_map), _stream()))

    # -- cc_select ---------------------------------------------------------------------------
    def select_workspace_bytes(self, n_tok: int, n_segs: int) -> int:
        return int(self._lib.cc_select_workspace_bytes(self._h, n_tok, n_segs))

    def select(self, q, k_pool, block_tab, segs, req_seg_off, n_requests, max_seg_tokens,
               sel_idx, q_row, q_pos, slot_map, scores, workspace):
        self._check(self._lib.cc_select(
            self._h, _ptr(q), q.shape[0], _ptr(k_pool), k_pool.shape[0], _ptr(block_tab), _ptr(segs),
            segs.shape[0], _ptr(req_seg_off), n_requests, max_seg_tokens, _ptr(sel_idx), _ptr(q_row),
            _ptr(q_pos), _ptr(slot_map), sel_idx.shape[0], _ptr(scores), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream()))

    # -- cc_select_from_scores ---------------------------------------------------------------
    def select_from_scores(self, scores, block_tab, segs, sel_idx, q_row, q_pos, slot_map, workspace):
        self._check(self._lib.cc_select_from_scores(
            self._h, _ptr(scores), scores.shape[0], _ptr(block_tab), _ptr(segs), segs.shape[0],
            _ptr(sel_idx), _ptr(q_row), _ptr(q_pos), _ptr(slot_map), sel_idx.shape[0], _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream()))

    # -- cc_gather_rows ----------------------------------------------------------------------
    def gather_rows(self, src, row_idx, dst):
        row_bytes = src[0].numel() * src.element_size()
        self._check(self._lib.cc_gather_rows(self._h, _ptr(src), src.shape[0], _ptr(row_idx),
                                             row_idx.shape[0], row_bytes, _ptr(dst), _stream()))

    # -- cc_qkv_project ----------------------------------------------------------------------
    def qkv_project(self, x, w_qkv, q, k, v):
        self._check(self._lib.cc_qkv_project(self._h, _ptr(x), _ptr(w_qkv), x.shape[0], x.shape[1],
                                             _ptr(q), _ptr(k), _ptr(v), _stream()))

    # -- cc_sparse_prefill -------------------------------------------------------------------
    def sparse_prefill_workspace_bytes(self, n_ctx_tokens: int, n_segs: int) -> int:
        return int(self._lib.cc_sparse_prefill_workspace_bytes(self._h, n_ctx_tokens, n_segs))

    def sparse_prefill(self, q, k_new, v_new, q_pos, slot_map, cu_q, max_q_per_req, k_pool, v_pool,
                       block_tab, segs, req_seg_off, n_requests, n_ctx_tokens, out, lse, workspace, src_rows=None,
                       shared=None):
        """src_rows: row of q / k_new / v_new each list row reads (None: they are compact, row j = list row j).
        shared: (v_shared pool, v_map) for values that stay in the chunk store (cc_shared_values), or None."""
        n_q_tot = q.shape[0] if src_rows is None else src_rows.shape[0]
        self._check(self._lib.cc_sparse_prefill(
            self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(src_rows), _ptr(q_pos), _ptr(slot_map), _ptr(cu_q),
            n_q_tot, max_q_per_req, _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], _ptr(block_tab),
            _ptr(segs), segs.shape[0], _ptr(req_seg_off), n_requests, n_ctx_tokens, _shared(shared), _ptr(out), _ptr(lse),
            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))

    def sparse_prefill_static(self, q, k_new, v_new, q_pos, slot_map, cu_q, max_q_per_req, k_pool, v_pool,
                              block_tab, segs, req_seg_off, n_requests, n_ctx_tokens, out, lse, src_rows=None,
                              shared=None):
        """cc_sparse_prefill without a workspace: the plan goes into the library's built-in scratch array."""
        n_q_tot = q.shape[0] if src_rows is None else src_rows.shape[0]
        self._check(self._lib.cc_sparse_prefill_static(
            self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(src_rows), _ptr(q_pos), _ptr(slot_map), _ptr(cu_q),
            n_q_tot, max_q_per_req, _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], _ptr(block_tab),
            _ptr(segs), segs.shape[0], _ptr(req_seg_off), n_requests, n_ctx_tokens, _shared(shared), _ptr(out),
            _ptr(lse), _stream()))

    # -- the rest of a decoder layer for the chosen rows ---------------------------------------------
    def rms_norm(self, x, gain, eps, y):
        self._check(self._lib.cc_rms_norm(self._h, _ptr(x), _ptr(gain), float(eps), x.shape[0], x.shape[1], _ptr(y),
                                          _stream()))

    def linear(self, x, w, y, residual=None):
        """y = x w^T (+ residual); w [out_features, in_features]."""
        self._check(self._lib.cc_linear(self._h, _ptr(x), _ptr(w), _ptr(residual), x.shape[0], w.shape[1], w.shape[0],
                                        _ptr(y), _stream()))

    def gated_linear(self, x, w_gate, w_up, y):
        """y = silu(x w_gate^T) * (x w_up^T)."""
        self._check(self._lib.cc_gated_linear(self._h, _ptr(x), _ptr(w_gate), _ptr(w_up), x.shape[0], w_gate.shape[1],
                                              w_gate.shape[0], _ptr(y), _stream()))

    def sparse_prefill_mass_workspace_bytes(self, n_ctx_tokens, n_segs, n_requests, max_question_rows, max_segs_per_req):
        return int(self._lib.cc_sparse_prefill_mass_workspace_bytes(self._h, n_ctx_tokens, n_segs, n_requests,
                                                                    max_question_rows, max_segs_per_req))

    def sparse_prefill_mass(self, q, k_new, v_new, q_pos, slot_map, cu_q, max_q_per_req, max_question_rows, k_pool,
                            v_pool, block_tab, segs, req_seg_off, n_requests, max_segs_per_req, n_ctx_tokens, out,
                            lse, seg_mass, workspace, src_rows=None, shared=None):
        n_q_tot = q.shape[0] if src_rows is None else src_rows.shape[0]
        self._check(self._lib.cc_sparse_prefill_mass(
            self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(src_rows), _ptr(q_pos), _ptr(slot_map), _ptr(cu_q),
            n_q_tot, max_q_per_req, max_question_rows, _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], _ptr(block_tab),
            _ptr(segs), segs.shape[0], _ptr(req_seg_off), n_requests, max_segs_per_req, n_ctx_tokens, _shared(shared),
            _ptr(out), _ptr(lse), _ptr(seg_mass), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))

    def sparse_prefill_pairs_workspace_bytes(self, n_ctx_tokens, n_segs, n_q_tot, max_q_per_req, max_segs_per_req):
        return int(self._lib.cc_sparse_prefill_pairs_workspace_bytes(self._h, n_ctx_tokens, n_segs, n_q_tot,
                                                                     max_q_per_req, max_segs_per_req))

    def sparse_prefill_pairs(self, q, k_new, v_new, q_pos, slot_map, cu_q, max_q_per_req, k_pool, v_pool, block_tab,
                             segs, req_seg_off, n_requests, max_segs_per_req, n_ctx_tokens, out, lse, seg_mass,
                             pair_mass, self_mass, workspace, src_rows=None, shared=None):
        n_q_tot = q.shape[0] if src_rows is None else src_rows.shape[0]
        self._check(self._lib.cc_sparse_prefill_pairs(
            self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(src_rows), _ptr(q_pos), _ptr(slot_map), _ptr(cu_q),
            n_q_tot, max_q_per_req, _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], _ptr(block_tab), _ptr(segs), segs.shape[0],
            _ptr(req_seg_off), n_requests, max_segs_per_req, n_ctx_tokens, pair_mass.shape[0], _shared(shared),
            _ptr(out), _ptr(lse),
            _ptr(seg_mass), _ptr(pair_mass), _ptr(self_mass), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream()))

    def check_query_list(self, slot_map, n_blocks) -> int:
        """Number of runs of adjacent list rows that name a block an earlier run named (0 = the order the
        scatter relies on).  Synchronises to read the count."""
        nbytes = int(self._lib.cc_check_query_list_workspace_bytes(self._h, n_blocks))
        ws = torch.empty(nbytes, dtype=torch.uint8, device=slot_map.device)
        count = torch.zeros(1, dtype=torch.int32, device=slot_map.device)
        self._check(self._lib.cc_check_query_list(self._h, _ptr(slot_map), slot_map.shape[0], n_blocks, _ptr(count),
                                                  _ptr(ws), nbytes, _stream()))
        return int(count.item())

    def scatter_kv(self, k_new, v_new, q_pos, slot_map, k_pool, v_pool):
        self._check(self._lib.cc_scatter_kv(self._h, _ptr(k_new), _ptr(v_new), _ptr(q_pos), _ptr(slot_map),
                                            k_new.shape[0], _ptr(k_pool), _ptr(v_pool), k_pool.shape[0], _stream()))

    # -- cc_chunk_attention --------------------------------------------------------------------
    def chunk_attention_workspace_bytes(self, n_ctx_tokens: int, n_segs: int, n_q_tot: int, max_q_per_req: int) -> int:
        return int(self._lib.cc_chunk_attention_workspace_bytes(self._h, n_ctx_tokens, n_segs, n_q_tot, max_q_per_req))

    def chunk_attention(self, q, q_pos, slot_map, cu_q, max_q_per_req, k_pool, v_pool, block_tab, segs,
                        req_seg_off, n_requests, n_ctx_tokens, lse, pair_mass, self_mass, workspace):
        self._check(self._lib.cc_chunk_attention(
            self._h, _ptr(q), _ptr(q_pos), _ptr(slot_map), _ptr(cu_q), q.shape[0], max_q_per_req, _ptr(k_pool),
            _ptr(v_pool), k_pool.shape[0], _ptr(block_tab), _ptr(segs), segs.shape[0], _ptr(req_seg_off),
            n_requests, n_ctx_tokens, pair_mass.shape[0], _ptr(lse), _ptr(pair_mass), _ptr(self_mass),
            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))

    # -- cc_question_mass ----------------------------------------------------------------------
    def question_mass_workspace_bytes(self, n_ctx_tokens: int, n_segs: int, max_question_rows: int) -> int:
        return int(self._lib.cc_question_mass_workspace_bytes(self._h, n_ctx_tokens, n_segs, max_question_rows))

    def question_mass(self, q, q_pos, cu_q, max_question_rows, k_pool, v_pool, block_tab, segs, req_seg_off,
                      n_requests, n_ctx_tokens, lse, seg_mass, workspace):
        self._check(self._lib.cc_question_mass(
            self._h, _ptr(q), _ptr(q_pos), _ptr(cu_q), q.shape[0], max_question_rows, _ptr(k_pool), _ptr(v_pool),
            k_pool.shape[0], _ptr(block_tab), _ptr(segs), segs.shape[0], _ptr(req_seg_off), n_requests,
            n_ctx_tokens, _ptr(lse), _ptr(seg_mass), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream()))


# ---- host-only reuse scores (Sec. 3.1, 3.3) ------------------------------------------------------
def _host_status(st: int, what: str):
    if st != 0:
        raise CacheCraftError(st, what)


def chunk_ab(inter, prefix_len, intra: float, chunk_len: int):
    """One layer's (a, b) of a chunk from its inter sums, its prefix chunks' lengths and its intra sum."""
    n = len(inter)
    a, b = C.c_double(), C.c_double()
    _host_status(load_library().cc_chunk_ab((C.c_double * max(1, n))(*[float(v) for v in inter]),
                                            (C.c_int32 * max(1, n))(*[int(v) for v in prefix_len]), n,
                                            float(intra), int(chunk_len), C.byref(a), C.byref(b)), "cc_chunk_ab")
    return a.value, b.value


def chunk_cci(a_layers, b_layers) -> float:
    n = len(a_layers)
    out = C.c_double()
    _host_status(load_library().cc_chunk_cci((C.c_double * max(1, n))(*[float(v) for v in a_layers]),
                                             (C.c_double * max(1, n))(*[float(v) for v in b_layers]), n,
                                             C.byref(out)), "cc_chunk_cci")
    return out.value


def chunk_reuse(old_prefix, old_inter, new_prefix, cci: float, alpha: float, chunk_len: int) -> dict:
    """beta, gamma, beta', CFO and the token budget of a chunk-cache wanted behind a new prefix."""
    n_old, n_new = len(old_prefix), len(new_prefix)
    out = _Reuse()
    _host_status(load_library().cc_chunk_reuse(
        (C.c_int64 * max(1, n_old))(*[int(v) for v in old_prefix]),
        (C.c_double * max(1, n_old))(*[float(v) for v in old_inter]), n_old,
        (C.c_int64 * max(1, n_new))(*[int(v) for v in new_prefix]), n_new, float(cci), float(alpha),
        int(chunk_len), C.byref(out)), "cc_chunk_reuse")
    return {"beta": out.beta, "gamma": out.gamma, "beta_adj": out.beta_adj, "cfo": out.cfo,
            "n_recompute": int(out.n_recompute)}


def preload_depth(n_layers: int, t_prefill: float, t_load: float) -> int:
    """L_p of Eq. (12) / Algorithm 2, line 1."""
    d = int(load_library().cc_preload_depth(n_layers, float(t_prefill), float(t_load)))
    if d < 0:
        raise CacheCraftError(d, "cc_preload_depth")
    return d


class Preloader:
    """Layer-wise preloading (Algorithm 2): pinned host tensors -> slots of a device read buffer."""

    def __init__(self, n_layers: int, depth: int, n_slots: int):
        self._lib = load_library()
        h = C.c_void_p()
        _host_status(self._lib.cc_preloader_create(C.byref(h), n_layers, depth, n_slots), "cc_preloader_create")
        self._h, self.n_layers = h, n_layers
        self._keep = []

    def set_layer(self, layer: int, host_src: torch.Tensor, dev_dst: torch.Tensor):
        assert host_src.is_pinned() and dev_dst.is_cuda and host_src.is_contiguous() and dev_dst.is_contiguous()
        nbytes = host_src.numel() * host_src.element_size()
        assert nbytes <= dev_dst.numel() * dev_dst.element_size()
        self._keep.append((host_src, dev_dst))
        _host_status(self._lib.cc_preloader_set_layer(self._h, layer, host_src.data_ptr(), dev_dst.data_ptr(), nbytes),
                     "cc_preloader_set_layer")

    def acquire(self, layer: int):
        _host_status(self._lib.cc_preloader_acquire(self._h, layer, _stream()), "cc_preloader_acquire")

    def release(self, layer: int):
        _host_status(self._lib.cc_preloader_release(self._h, layer, _stream()), "cc_preloader_release")

    def issued(self):
        buf = (C.c_int32 * self.n_layers)()
        n = self._lib.cc_preloader_issued(self._h, buf, self.n_layers)
        return [int(buf[i]) for i in range(n)]

    def close(self):
        if self._h:
            self._lib.cc_preloader_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class FocusTracker:
    """Algorithm 1 for one request (host only): feed one layer's inter(C_i, U) per call."""

    def __init__(self, n_chunks: int, window: int):
        self._lib = load_library()
        h = C.c_void_p()
        st = self._lib.cc_focus_create(C.byref(h), n_chunks, window)
        if st != 0:
            raise CacheCraftError(st, "cc_focus_create")
        self._h, self.n_chunks = h, n_chunks

    def update(self, inter):
        """Returns (stop, focused chunk indices of this layer)."""
        arr = (C.c_float * self.n_chunks)(*[float(v) for v in inter])
        flags = (C.c_int32 * self.n_chunks)()
        n = C.c_int32(0)
        st = self._lib.cc_focus_update(self._h, arr, flags, C.byref(n))
        if st < 0:
            raise CacheCraftError(st, "cc_focus_update")
        return bool(st), [i for i in range(self.n_chunks) if flags[i]]

    @property
    def layer(self) -> int:
        return int(self._lib.cc_focus_layer(self._h))

    def close(self):
        if self._h:
            self._lib.cc_focus_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
