"""Test-side glue: compares the HIP path (through the C ABI binding) with the CPU oracle."""
from __future__ import annotations

import numpy as np

import workload as W
from oracle import cachecraft_oracle as O

TOL = {"bf16": 1e-2, "f32": 1e-5}      # relative L2 bars (attention output, shifted K, fixed K/V)
TIE_GAP = 1e-4                          # index sets: exact except ties within this score gap


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    return float(np.linalg.norm((got - ref).ravel()) / (den if den > 0 else 1.0))


def chunk_segments(w, r):
    s0, s1 = int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])
    return [w.segments[i] for i in range(s0, s1) if w.segments[i][W.SEG_KIND] == W.KIND_CHUNK]


def all_segments(w, r):
    return [w.segments[i] for i in range(int(w.req_seg_off[r]), int(w.req_seg_off[r + 1]))]


def request_context_from_pools(w, r, k_pool: np.ndarray, v_pool: np.ndarray):
    """Logical [n_ctx, Hkv, d] K and V of request r as the device pools hold them."""
    segs = all_segments(w, r)
    n_ctx = int(segs[-1][W.SEG_START] + segs[-1][W.SEG_NTOK]) if segs else 0
    hkv, d = w.spec.n_kv_heads, w.spec.head_dim
    k = np.zeros((n_ctx, hkv, d)); v = np.zeros((n_ctx, hkv, d))
    for sg in segs:
        s, n, tab = int(sg[W.SEG_START]), int(sg[W.SEG_NTOK]), int(sg[W.SEG_TAB])
        blocks = w.req_tab[tab: tab + (n + 15) // 16]
        k[s:s + n] = O.read_k_pages(k_pool, blocks, n)
        v[s:s + n] = O.read_v_pages(v_pool, blocks, n)
    return k, v


def selection_arrays(w, selected_by_req):
    """sel_idx / q_row / q_pos / slot_map of a given selection, laid out like cc_select's outputs."""
    nq = w.n_q_tot
    sel_idx = np.zeros(nq, np.int32); q_row = np.zeros(nq, np.int32)
    q_pos = np.zeros(nq, np.int32); slot = np.zeros(nq, np.int32)
    for r in range(w.n_requests):
        ci = 0
        for sg in all_segments(w, r):
            n, tab, off = int(sg[W.SEG_NTOK]), int(sg[W.SEG_TAB]), int(sg[W.SEG_SEL])
            if sg[W.SEG_KIND] == W.KIND_CHUNK:
                idx = np.asarray(selected_by_req[r][ci], dtype=np.int64); ci += 1
            else:
                idx = np.arange(n, dtype=np.int64)
            m = len(idx)
            sel_idx[off:off + m] = idx
            q_row[off:off + m] = sg[W.SEG_TOK] + idx
            q_pos[off:off + m] = sg[W.SEG_START] + idx
            slot[off:off + m] = w.req_tab[tab + idx // 16] * 16 + idx % 16
    return sel_idx, q_row, q_pos, slot


def gpu_selection(w, sel_idx_gpu: np.ndarray):
    """Per request, per chunk segment: the index set cc_select wrote."""
    out = []
    for r in range(w.n_requests):
        out.append([np.asarray(sel_idx_gpu[int(sg[W.SEG_SEL]): int(sg[W.SEG_SEL]) + int(sg[W.SEG_NSEL])], dtype=np.int64)
                    for sg in chunk_segments(w, r)])
    return out


def assert_selection_matches(w, r, gpu_sets, oracle_scores, oracle_sets):
    """Sets equal in size, ascending, and equal up to ties: every index in the symmetric difference
    must have an oracle score within TIE_GAP of the oracle's N-th largest score of that chunk."""
    for c, sg in enumerate(chunk_segments(w, r)):
        g, o, sc = gpu_sets[c], oracle_sets[c], oracle_scores[c]
        n_sel = int(sg[W.SEG_NSEL])
        assert len(g) == len(o) == n_sel, (r, c, len(g), len(o), n_sel)
        assert np.all(np.diff(g) > 0), f"request {r} chunk {c}: indices not strictly ascending"
        assert n_sel == 0 or (g.min() >= 0 and g.max() < int(sg[W.SEG_NTOK]))
        diff = np.setxor1d(g, o)
        if len(diff):
            nth = np.sort(sc)[::-1][n_sel - 1]
            worst = np.abs(sc[diff] - nth).max()
            assert worst <= TIE_GAP, f"request {r} chunk {c}: {len(diff)} indices differ, score gap {worst:.3e}"
