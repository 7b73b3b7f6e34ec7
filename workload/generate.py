"""Seeded synthetic RAG-prompt workloads for the selective-KV-recompute path.

This module only *draws and lays out inputs*: random tensors, chunk/request
structure, page tables.  It contains none of the method's arithmetic (no
rotation, no attention, no scoring) so that both the CPU oracle and the HIP
path can consume exactly the same inputs without sharing any computation.

Shapes follow the prompt structure S = C_1 .. C_k U (chunks then question,
Sec. 2.2), the per-layer chunk-cache (K_C, V_C) of Sec. 3, and the storage
scheme of Sec. 4: every chunk maps to a list of 16-token blocks and is padded
to a whole number of blocks.

Page layouts (one attention layer):
  K pool  [n_blocks, Hkv, 16, d]   token-major rows of d
  V pool  [n_blocks, Hkv, d, 16]   dimension-major rows of 16 token slots

All bf16 tensors are drawn in fp32 and rounded once to the nearest bf16
(ties to even); they are kept as fp32 arrays holding bf16-representable
values so the oracle can upcast them exactly.
"""
from __future__ import annotations

import math
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

BLOCK = 16  # tokens per KV block (Sec. 4, chunk storage management)

# column indices of the int32 descriptor tables (mirrors include/cc.h)
SHIFT_SRC_TAB, SHIFT_DST_TAB, SHIFT_NTOK, SHIFT_DELTA = range(4)
(SEG_REQ, SEG_KIND, SEG_START, SEG_NTOK, SEG_TAB, SEG_NSEL, SEG_TOK, SEG_SEL) = range(8)
KIND_CHUNK, KIND_QUESTION = 0, 1


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def n_select_for(frac: float, n_tokens: int) -> int:
    """Integer token budget N = ceil(f * |C|), guarded against fp noise in f*|C|."""
    return int(min(n_tokens, max(0, math.ceil(frac * n_tokens - 1e-9))))


@dataclass
class RequestSpec:
    chunks: List[int]            # ids into the shared chunk store, in new prompt order
    fracs: List[float]           # recompute fraction per chunk instance
    question: int                # question length m


@dataclass
class Spec:
    name: str
    dtype: str                   # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    store_lens: List[int]        # token length of every chunk in the shared store
    store_offsets: List[int]     # position each stored chunk was cached at
    requests: List[RequestSpec]
    value_scale: float
    seed: int
    hidden: int = 0              # >0: also draw hidden states + W_qkv (projection workload)
    shuffle_blocks: bool = True  # scatter physical block ids (exercises the page indirection)


@dataclass
class Workload:
    spec: Spec
    # shared chunk store (read-only for the whole path)
    k_store: np.ndarray          # [n_store_blocks, Hkv, 16, d]
    v_store: np.ndarray          # [n_store_blocks, Hkv, d, 16]
    store_tab: np.ndarray        # int32, block ids of every stored chunk, concatenated
    store_tab_off: np.ndarray    # int32 [n_store_chunks+1]
    # request-owned pages
    n_req_blocks: int            # size of the request pool (blocks)
    req_tab: np.ndarray          # int32, block ids of every segment, concatenated
    shift_descs: np.ndarray      # int32 [n_instances, 4]
    segments: np.ndarray         # int32 [n_segs, 8]
    req_seg_off: np.ndarray      # int32 [B+1]
    cu_q: np.ndarray             # int32 [B+1]  offsets into the compact query list
    # per-token tensors for every prompt token (rows in segment order)
    q: np.ndarray                # [n_tok, Hq, d]   pre-rotation queries
    k_new: np.ndarray            # [n_tok, Hkv, d]  pre-rotation recomputed keys
    v_new: np.ndarray            # [n_tok, Hkv, d]  recomputed values
    hidden: Optional[np.ndarray] = None   # [n_tok, hidden]
    w_qkv: Optional[np.ndarray] = None    # [(Hq+2Hkv)*d, hidden]  (out_features x in_features)
    extras: Dict[str, object] = field(default_factory=dict)

    @property
    def n_tok(self) -> int:
        return int(self.q.shape[0])

    @property
    def n_requests(self) -> int:
        return int(self.req_seg_off.shape[0] - 1)

    @property
    def n_q_tot(self) -> int:
        return int(self.cu_q[-1])

    @property
    def max_seg_tokens(self) -> int:
        return int(self.segments[:, SEG_NTOK].max()) if len(self.segments) else 0

    def context_len(self, r: int) -> int:
        s0, s1 = self.req_seg_off[r], self.req_seg_off[r + 1]
        last = self.segments[s1 - 1]
        return int(last[SEG_START] + last[SEG_NTOK]) if s1 > s0 else 0


_DRAW_ROWS = 1 << 22          # elements per independently seeded slab


def _draw(seed: np.random.SeedSequence, shape, scale: float, dtype: str) -> np.ndarray:
    """N(0,1)*scale of the given shape.  The flat array is cut into slabs, each with its own child
    seed, so that slabs can be filled by a thread pool and the result does not depend on the
    number of threads."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    n_slabs = max(1, (n + _DRAW_ROWS - 1) // _DRAW_ROWS)
    children = seed.spawn(n_slabs)

    def fill(i):
        a, b = i * _DRAW_ROWS, min(n, (i + 1) * _DRAW_ROWS)
        g = np.random.Generator(np.random.PCG64(children[i]))
        x = g.standard_normal(size=b - a, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out[a:b] = round_to_bf16(x) if dtype == "bf16" else x

    if n_slabs == 1:
        fill(0)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, range(n_slabs)))
    return out.reshape(shape)


def build(spec: Spec) -> Workload:
    """Lay a spec out as pools, page tables, descriptors and per-token tensors."""
    ss = np.random.SeedSequence(spec.seed)
    s_k, s_v, s_q, s_kn, s_vn, s_struct, s_x, s_w = ss.spawn(8)
    Hq, Hkv, d = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    rs = np.random.Generator(np.random.PCG64(s_struct))

    # ---- shared store: one block list per stored chunk --------------------
    store_pages = [(n + BLOCK - 1) // BLOCK for n in spec.store_lens]
    n_store_blocks = int(sum(store_pages))
    ids = np.arange(n_store_blocks, dtype=np.int32)
    if spec.shuffle_blocks:
        rs.shuffle(ids)
    store_tab_off = np.zeros(len(store_pages) + 1, dtype=np.int32)
    store_tab_off[1:] = np.cumsum(store_pages)
    store_tab = ids
    k_store = _draw(s_k, (n_store_blocks, Hkv, BLOCK, d), spec.value_scale, spec.dtype)
    v_store = _draw(s_v, (n_store_blocks, Hkv, d, BLOCK), spec.value_scale, spec.dtype)

    # ---- requests: segments, request-owned pages, descriptors -------------
    segs, descs, req_seg_off, cu_q = [], [], [0], [0]
    tab_cursor = tok_cursor = sel_cursor = 0
    for r, rq in enumerate(spec.requests):
        pos = 0
        for cid, f in zip(rq.chunks, rq.fracs):
            n = spec.store_lens[cid]
            nsel = n_select_for(f, n)
            segs.append([r, KIND_CHUNK, pos, n, tab_cursor, nsel, tok_cursor, sel_cursor])
            descs.append([int(store_tab_off[cid]), tab_cursor, n, pos - spec.store_offsets[cid]])
            tab_cursor += (n + BLOCK - 1) // BLOCK
            tok_cursor += n
            sel_cursor += nsel
            pos += n
        m = rq.question
        if m > 0:
            segs.append([r, KIND_QUESTION, pos, m, tab_cursor, m, tok_cursor, sel_cursor])
            tab_cursor += (m + BLOCK - 1) // BLOCK
            tok_cursor += m
            sel_cursor += m
        req_seg_off.append(len(segs))
        cu_q.append(sel_cursor)
    n_req_blocks = tab_cursor
    req_ids = np.arange(n_req_blocks, dtype=np.int32)
    if spec.shuffle_blocks:
        rs.shuffle(req_ids)
    n_tok = tok_cursor

    q = _draw(s_q, (n_tok, Hq, d), spec.value_scale, spec.dtype)
    k_new = _draw(s_kn, (n_tok, Hkv, d), spec.value_scale, spec.dtype)
    v_new = _draw(s_vn, (n_tok, Hkv, d), spec.value_scale, spec.dtype)
    hidden = w_qkv = None
    if spec.hidden:
        hidden = _draw(s_x, (n_tok, spec.hidden), 1.0, spec.dtype)
        w_qkv = _draw(s_w, ((Hq + 2 * Hkv) * d, spec.hidden), 0.02, spec.dtype)

    return Workload(
        spec=spec, k_store=k_store, v_store=v_store,
        store_tab=store_tab, store_tab_off=store_tab_off,
        n_req_blocks=n_req_blocks, req_tab=req_ids,
        shift_descs=np.asarray(descs, dtype=np.int32).reshape(-1, 4),
        segments=np.asarray(segs, dtype=np.int32).reshape(-1, 8),
        req_seg_off=np.asarray(req_seg_off, dtype=np.int32),
        cu_q=np.asarray(cu_q, dtype=np.int32),
        q=q, k_new=k_new, v_new=v_new, hidden=hidden, w_qkv=w_qkv)


@dataclass
class LayerWeights:
    """Random weights of one decoder layer (row = output feature), drawn so that activations stay O(1)."""
    gain_attn: np.ndarray        # [hidden]
    gain_ffn: np.ndarray         # [hidden]
    w_qkv: np.ndarray            # [(Hq+2Hkv)*d, hidden]
    w_o: np.ndarray              # [hidden, Hq*d]
    w_gate: np.ndarray           # [ffn, hidden]
    w_up: np.ndarray             # [ffn, hidden]
    w_down: np.ndarray           # [hidden, ffn]
    eps: float


def layer_weights(spec: Spec, hidden: int, ffn: int, layer: int = 0, qkv_scale: float = 0.02) -> LayerWeights:
    """Weights of decoder layer `layer` for the given head geometry (seeded by spec.seed and layer)."""
    Hq, Hkv, d = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    ss = np.random.SeedSequence([spec.seed, 7919, layer]).spawn(7)
    one = lambda a: round_to_bf16(np.float32(1.0) + a) if spec.dtype == "bf16" else (np.float32(1.0) + a).astype(np.float32)
    return LayerWeights(
        gain_attn=one(_draw(ss[0], (hidden,), 0.1, "f32")),
        gain_ffn=one(_draw(ss[1], (hidden,), 0.1, "f32")),
        w_qkv=_draw(ss[2], ((Hq + 2 * Hkv) * d, hidden), qkv_scale, spec.dtype),
        w_o=_draw(ss[3], (hidden, Hq * d), 1.0 / math.sqrt(Hq * d), spec.dtype),
        w_gate=_draw(ss[4], (ffn, hidden), 1.0 / math.sqrt(hidden), spec.dtype),
        w_up=_draw(ss[5], (ffn, hidden), 1.0 / math.sqrt(hidden), spec.dtype),
        w_down=_draw(ss[6], (hidden, ffn), 1.0 / math.sqrt(ffn), spec.dtype),
        eps=1.0e-5)


# ---------------------------------------------------------------------------
# The five benchmark configurations, and scaled-down relatives for tests.
# ---------------------------------------------------------------------------
BASE_SEED = 20250215
CONFIG_NAMES = {
    1: "tiny_fp32_3x64+16",
    2: "llama3_8b_layer_5x512+64",
    3: "llama3_8b_continuous_batch_32req",
    4: "llama3_70b_layer_8req_10x1024+128",
    5: "llama3_8b_32k_4req_32x1000+256_qkvproj",
}


def _permuted_request(rs, n_chunks: int, frac: float, question: int) -> RequestSpec:
    order = [int(i) for i in rs.permutation(n_chunks)]
    return RequestSpec(chunks=order, fracs=[frac] * n_chunks, question=question)


def config_spec(cid: int, scale: float = 1.0) -> Spec:
    """Spec of benchmark config `cid` (1..5).  `scale` < 1 shrinks token counts
    and request counts (same head geometry) for parity tests the oracle can finish."""
    seed = BASE_SEED + cid
    rs = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 7])))
    sc = lambda n, lo=1: max(lo, int(round(n * scale)))
    if cid == 1:
        return Spec(CONFIG_NAMES[1], "f32", 4, 2, 64, 1.0e4, [64] * 3, [0] * 3,
                    [RequestSpec([0, 1, 2], [0.2] * 3, 16)], 1.0, seed)
    if cid == 2:
        n = sc(512, 16)
        return Spec(CONFIG_NAMES[2], "bf16", 32, 8, 128, 5.0e5, [n] * 5, [0] * 5,
                    [_permuted_request(rs, 5, 0.15, sc(64, 4))], 1.0 / math.sqrt(128), seed)
    if cid == 3:
        n_store = sc(200, 12)
        lens = [int(x) for x in rs.integers(sc(256, 8), sc(1024, 24) + 1, size=n_store)]
        w = np.arange(1, n_store + 1, dtype=np.float64) ** -1.1
        w /= w.sum()
        reqs = []
        for _ in range(sc(32, 2)):
            k = int(rs.integers(5, 11))
            k = min(k, n_store)
            chunks = [int(c) for c in rs.choice(n_store, size=k, replace=False, p=w)]
            rs.shuffle(chunks)
            fr = [float(f) for f in rs.uniform(0.05, 0.40, size=k)]
            reqs.append(RequestSpec(chunks, fr, int(rs.integers(sc(32, 2), sc(128, 6) + 1))))
        return Spec(CONFIG_NAMES[3], "bf16", 32, 8, 128, 5.0e5, lens, [0] * n_store, reqs,
                    1.0 / math.sqrt(128), seed)
    if cid == 4:
        B, n = sc(8, 1), sc(1024, 16)
        lens, reqs = [n] * (10 * B), []
        for r in range(B):
            order = [10 * r + int(i) for i in rs.permutation(10)]
            reqs.append(RequestSpec(order, [0.10] * 10, sc(128, 4)))
        return Spec(CONFIG_NAMES[4], "bf16", 64, 8, 128, 5.0e5, lens, [0] * len(lens), reqs,
                    1.0 / math.sqrt(128), seed)
    if cid == 5:
        B, n, k = sc(4, 1), sc(1000, 24), 32 if scale >= 1.0 else max(3, int(round(32 * scale)))
        lens, offs, reqs = [n] * (k * B), [], []
        for r in range(B):
            order = [int(i) for i in rs.permutation(k)]
            new_off = {c: i * n for i, c in enumerate(order)}
            for c in range(k):
                o = int(rs.integers(0, sc(31000, 64) + 1))
                if o == new_off[c]:
                    o += 1
                offs.append(o)
            reqs.append(RequestSpec([k * r + c for c in order], [0.10] * k, sc(256, 8)))
        return Spec(CONFIG_NAMES[5], "bf16", 32, 8, 128, 5.0e5, lens, offs, reqs,
                    1.0 / math.sqrt(128), seed, hidden=4096 if scale >= 1.0 else 256)
    raise ValueError(f"unknown config {cid}")


def config(cid: int, scale: float = 1.0) -> Workload:
    return build(config_spec(cid, scale))


def custom(name: str, dtype: str, Hq: int, Hkv: int, d: int, theta: float,
           chunk_lens: Sequence[int], cached_offsets: Sequence[int],
           requests: Sequence[RequestSpec], value_scale: float, seed: int,
           hidden: int = 0, shuffle_blocks: bool = True) -> Workload:
    return build(Spec(name, dtype, Hq, Hkv, d, theta, list(chunk_lens), list(cached_offsets),
                      list(requests), value_scale, seed, hidden, shuffle_blocks))
