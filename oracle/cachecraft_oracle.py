"""CPU oracle for selective KV recomputation over reused chunk-caches (Cache-Craft).

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy; written from the paper's
definitions, one step at a time, with no blocking, fusion or paging tricks.
It shares no code with the HIP library and must never be imported by the
product path: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may call it.

What is computed, for one attention layer and a batch of prompts
S = C_1 .. C_k U (Sec. 2.2):

  shift   re-position every cached chunk's keys: the rotary embedding of a key
          cached at position s and now placed at position p is turned by the
          angle (p - s) * inv_freq (Sec. 3.4.3 "Handling Partial Prefill",
          Sec. 4 "RPE Management").  Values are position-free and unchanged.
  score   for each token of a chunk, its attention mass on all *prior* chunks:
          sum over j < i of inter(C_j, t) with a_kl the rows of the causal
          softmax of Eq. (1) (Eq. (2), the block matrix below Eq. (3), Eq. (10)).
  select  the N tokens of each chunk with the largest score (Eq. (10)),
          N given per chunk as an integer.
  fix     recomputed K (rotated to its new position) and V of the selected
          tokens and of the question tokens replace the stale rows (Sec. 3.4.3).
  attend  causal attention of only those tokens against the whole merged K, V
          (Sec. 2.1 per-token form of Eq. (1); Sec. 4 "Selective Token
          Recomputation").

Readings taken where the paper leaves a choice (each is a reading, not a fact
of the paper): rotate-half pairing (x = first half of the head, y = second
half: Sec. 4 names the two halves of a head as the rotated components); frequencies
theta^(-2i/d); logits scaled by 1/sqrt(d) and masked entries excluded from the
softmax; queries of the later chunk attend keys of the earlier chunk; the
softmax denominator runs over every key up to and including the token itself;
a token's score is the mean over query heads; ties go to the lower index;
padding slots of a partly filled block are never keys; grouped-query mapping
kv_head = q_head // (Hq / Hkv).

Two further steps follow the question-to-chunk attention of Sec. 3.2.2:

  question mass   inter(C_i, U): attention weight from the question's tokens to
          the tokens of chunk C_i, the a_kl of Eq. (1) summed as in Eq. (2), with the
          question as the later "chunk".  Reading: mean over query heads (as for the
          token scores), summed over the question's tokens.
  focused chunks  Algorithm 1, in the indexing its lines 5-9 print: gaps
          diff_i = sorted_i - sorted_{i+1} for i = 1..k-1, p_i = diff_i / sum(diff),
          h_i = -sum_{j<=i} p_j log p_j, i* = argmax over i = 1..k-2 of h_{i+1} - h_i,
          F = the top i* chunks.  (Line 7's lower limit j = 0 is taken to be a slip
          for j = 1: p has no element 0.)  0 log 0 = 0; first maximum among equals;
          chunks with equal cumulative score keep prompt order; with k < 3 the range
          of i is empty and with all gaps zero p is undefined -- every chunk is then
          kept.  The stop rule compares the last w sets once l >= w.

And the reuse scores of Sec. 3.1 / 3.3, from the same attention weights:

  inter / intra   Eq. (2) and Eq. (3) between the segments of a prompt; a, b, CCI (sigmoid
          of abar / bbar); prefix overlap beta; order penalty gamma = D / C(m, 2), the normalised
          Kendall tau distance between the old and the new order of the common prefix chunks;
          beta' = beta (1 - gamma); CFO = alpha CCI (1 - beta'); N = ceil(CFO |C|).
          Readings: Eq. (3)'s "k < l" is taken as: a token's weights on strictly earlier tokens
          of its own chunk (the weight on itself is left out); head aggregation is the mean, as
          everywhere; beta = 1 when the old inter sum is zero (nothing was depended on),
          gamma = 0 with fewer than two common chunks; abar = 0 gives ratio 0, bbar = 0 < abar an
          infinite ratio; CFO is clipped to [0, 1]; the ceiling carries the same 1e-9 guard as the
          workload generator's token budget.

The rest of a layer, for the recomputed rows only (Sec. 2.1: the next hidden state comes from the
token's own hidden state plus the feed-forward network applied to its attention output; Sec. 3.4.3:
the attention output goes through the FFN to give the layer's output):

  layer   the pre-normalised decoder layer of the models the paper runs (Llama-3):
          x = rms_norm(h) -> Q, K, V -> attention -> h1 = h + o W_o^T ->
          h2 = h1 + (silu(y W_gate^T) * (y W_up^T)) W_down^T with y = rms_norm(h1).
          Reading: the paper writes the layer only in outline; the concrete operators are those
          of the evaluated models (root-mean-square normalisation with a learned gain and eps
          inside the root, gated SiLU feed-forward, no biases).  Only rows whose hidden state is
          recomputed pass through it; every other token's K and V come from its chunk-cache.

Parity pins (tests/test_oracle_pins.py): every function below is pinned by
closed forms, invariants, limiting cases or brute force -- none is unpinned.
The scoring *definition* (mean over heads, scores in the new context) is pinned
to the reading above, which the paper does not fix.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

BLOCK = 16


# --------------------------------------------------------------------------
# rotary position embedding
# --------------------------------------------------------------------------
def inv_freq(d: int, theta: float) -> np.ndarray:
    """Rotation frequency of pair i: theta^(-2i/d), i = 0 .. d/2-1."""
    i = np.arange(d // 2, dtype=np.float64)
    return np.float64(theta) ** (-2.0 * i / d)


def rotate(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Turn every (x_i, y_i) = (v[i], v[i+d/2]) pair of the last axis by pos * inv_freq_i.

    x: [n, H, d] fp64; pos: [n] (any integer, negative allowed).
    Forward rotation: x' = x cos(phi) - y sin(phi), y' = y cos(phi) + x sin(phi)  (Sec. 4).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    h = d // 2
    phi = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq(d, theta)[None, :]   # [n, d/2]
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    a, b = x[..., :h], x[..., h:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


# --------------------------------------------------------------------------
# reading / writing the paged pools (only at the two ends of the oracle)
# --------------------------------------------------------------------------
def read_k_pages(k_pool: np.ndarray, blocks: Sequence[int], n_tokens: int) -> np.ndarray:
    """K pool [nb, Hkv, 16, d] -> logical [n_tokens, Hkv, d] (padding slots dropped)."""
    pages = np.asarray(k_pool)[np.asarray(blocks, dtype=np.int64)]          # [p, Hkv, 16, d]
    p, hkv, _, d = pages.shape
    return pages.transpose(0, 2, 1, 3).reshape(p * BLOCK, hkv, d)[:n_tokens].astype(np.float64)


def read_v_pages(v_pool: np.ndarray, blocks: Sequence[int], n_tokens: int) -> np.ndarray:
    """V pool [nb, Hkv, d, 16] -> logical [n_tokens, Hkv, d]."""
    pages = np.asarray(v_pool)[np.asarray(blocks, dtype=np.int64)]          # [p, Hkv, d, 16]
    p, hkv, d, _ = pages.shape
    return pages.transpose(0, 3, 1, 2).reshape(p * BLOCK, hkv, d)[:n_tokens].astype(np.float64)


# --------------------------------------------------------------------------
# the steps
# --------------------------------------------------------------------------
def shift_keys(k: np.ndarray, delta: int, theta: float) -> np.ndarray:
    """Keys of one chunk [n, Hkv, d] cached at position s, re-placed at s + delta."""
    n = k.shape[0]
    return rotate(k, np.full(n, delta, dtype=np.int64), theta)


def place_keys(k: np.ndarray, start: int, theta: float) -> np.ndarray:
    """Keys stored without rotation, put at positions start .. start + n - 1 (Sec. 4 "RPE
    Management": the run-time rotation with the new prompt's positions)."""
    pos = start + np.arange(k.shape[0], dtype=np.int64)
    return rotate(k, pos, theta)


def prior_mass(q_rot: np.ndarray, k_ctx: np.ndarray, pos: np.ndarray, chunk_start: int) -> np.ndarray:
    """Per-head attention mass of each query on keys before `chunk_start`.

    q_rot [n, Hq, d]: rotated queries at positions pos [n];
    k_ctx [>= max(pos)+1, Hkv, d]: keys of the context in logical order.
    Returns [n, Hq]: sum_{l < chunk_start} a_{p,l}, a = softmax over l <= p of q.k_l / sqrt(d).
    """
    n, hq, d = q_rot.shape
    hkv = k_ctx.shape[1]
    g = hq // hkv
    out = np.zeros((n, hq), dtype=np.float64)
    n_keys = int(pos.max()) + 1 if n else 0
    key_idx = np.arange(n_keys)
    for h in range(hq):
        logits = q_rot[:, h, :] @ k_ctx[:n_keys, h // g, :].T / np.sqrt(np.float64(d))   # [n, n_keys]
        visible = key_idx[None, :] <= pos[:, None]
        logits = np.where(visible, logits, -np.inf)
        m = logits.max(axis=1, keepdims=True)
        e = np.exp(logits - m)
        a = e / e.sum(axis=1, keepdims=True)
        out[:, h] = a[:, :chunk_start].sum(axis=1)
    return out


def top_n(scores: np.ndarray, n_sel: int) -> np.ndarray:
    """Indices of the n_sel largest scores, lower index first among equals; ascending."""
    order = np.lexsort((np.arange(len(scores)), -np.asarray(scores, dtype=np.float64)))
    return np.sort(order[:n_sel]).astype(np.int64)


def causal_attention_rows(q_rot: np.ndarray, pos: np.ndarray, k_ctx: np.ndarray, v_ctx: np.ndarray):
    """out_j = softmax(q_j K_{:j}^T / sqrt(d)) V_{:j} for the given rows only.

    q_rot [n, Hq, d] (already rotated), pos [n]; k_ctx, v_ctx [n_ctx, Hkv, d] logical order.
    Returns out [n, Hq, d] and lse [n, Hq] (natural log of the softmax denominator).
    """
    n, hq, d = q_rot.shape
    g = hq // k_ctx.shape[1]
    out = np.zeros((n, hq, d), dtype=np.float64)
    lse = np.zeros((n, hq), dtype=np.float64)
    for j in range(n):
        p = int(pos[j])
        for h in range(hq):
            s = k_ctx[: p + 1, h // g, :] @ q_rot[j, h, :] / np.sqrt(np.float64(d))
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[j, h, :] = (e / z) @ v_ctx[: p + 1, h // g, :]
            lse[j, h] = m + np.log(z)
    return out, lse


def causal_attention_rows_dense(q_rot: np.ndarray, pos: np.ndarray, k_ctx: np.ndarray, v_ctx: np.ndarray):
    """causal_attention_rows for many rows at once: per head one logit matrix [n, max(pos)+1] with the
    keys behind each row's position set to -inf, a row-wise softmax, and one product with V.  The same
    definition (Eq. (1) per token, scale 1/sqrt(d)) written with matrices instead of a loop over rows;
    used where thousands of rows of a long prompt are checked.
    """
    n, hq, d = q_rot.shape
    g = hq // k_ctx.shape[1]
    out = np.zeros((n, hq, d), dtype=np.float64)
    lse = np.zeros((n, hq), dtype=np.float64)
    if n == 0:
        return out, lse
    n_keys = int(pos.max()) + 1
    hidden = np.arange(n_keys)[None, :] > np.asarray(pos)[:, None]
    for h in range(hq):
        s = q_rot[:, h, :] @ k_ctx[:n_keys, h // g, :].T / np.sqrt(np.float64(d))
        s[hidden] = -np.inf
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        out[:, h, :] = (e / z) @ v_ctx[:n_keys, h // g, :]
        lse[:, h] = (m + np.log(z))[:, 0]
    return out, lse


# --------------------------------------------------------------------------
# whole path on a workload (the structure produced by workload.generate.build)
# --------------------------------------------------------------------------
@dataclass
class RequestResult:
    k_shifted: np.ndarray        # [n_ctx, Hkv, d] after shift, before fix (question rows = 0)
    k_ctx: np.ndarray            # [n_ctx, Hkv, d] after fix
    v_ctx: np.ndarray            # [n_ctx, Hkv, d] after fix
    scores: List[np.ndarray]     # per chunk segment, [n_c]
    selected: List[np.ndarray]   # per chunk segment, ascending indices within the chunk
    q_pos: np.ndarray            # [n_q] logical positions of the compact query list
    q_row: np.ndarray            # [n_q] rows of q / k_new / v_new
    out: np.ndarray              # [n_q, Hq, d]
    lse: np.ndarray              # [n_q, Hq]


def _segments_of(w, r):
    s0, s1 = int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])
    return [tuple(int(v) for v in w.segments[i]) for i in range(s0, s1)]


def shifted_context(w, r: int, miss_segments: Sequence[int] = ()):
    """Steps gather + shift for request r: logical K (shifted), V, context length.

    miss_segments: indices (within the request) of chunks that have no chunk-cache (C_miss,
    Sec. 3.4.1): their K and V are the freshly computed ones of all their tokens (K rotated to
    the new positions), present before anything is scored."""
    theta = w.spec.rope_theta
    segs = _segments_of(w, r)
    n_ctx = segs[-1][2] + segs[-1][3] if segs else 0
    hkv, d = w.spec.n_kv_heads, w.spec.head_dim
    k = np.zeros((n_ctx, hkv, d), dtype=np.float64)
    v = np.zeros((n_ctx, hkv, d), dtype=np.float64)
    by_dst = {int(dsc[1]): dsc for dsc in w.shift_descs}
    for si, (_, kind, start, n, tab, _, tok, _) in enumerate(segs):
        if kind != 0:
            continue
        if si in miss_segments:
            pos = start + np.arange(n, dtype=np.int64)
            k[start:start + n] = rotate(np.asarray(w.k_new[tok:tok + n], dtype=np.float64), pos, theta)
            v[start:start + n] = np.asarray(w.v_new[tok:tok + n], dtype=np.float64)
            continue
        src_tab, _, n_tok, delta = (int(x) for x in by_dst[tab])
        assert n_tok == n
        blocks = w.store_tab[src_tab: src_tab + (n + BLOCK - 1) // BLOCK]
        k[start:start + n] = shift_keys(read_k_pages(w.k_store, blocks, n), delta, theta)
        v[start:start + n] = read_v_pages(w.v_store, blocks, n)
    return k, v, n_ctx


def score_request(w, r: int, k_shifted: np.ndarray, only_segments: Optional[Sequence[int]] = None):
    """Step score: per chunk segment of request r, mean-over-heads prior-chunk mass of each token."""
    theta = w.spec.rope_theta
    scores = []
    for si, (_, kind, start, n, _, _, tok, _) in enumerate(_segments_of(w, r)):
        if kind != 0:
            continue
        if only_segments is not None and si not in only_segments:
            scores.append(None)
            continue
        if start == 0:
            scores.append(np.zeros(n, dtype=np.float64))     # first chunk: no prior chunk
            continue
        pos = start + np.arange(n, dtype=np.int64)
        q_rot = rotate(np.asarray(w.q[tok:tok + n], dtype=np.float64), pos, theta)
        scores.append(prior_mass(q_rot, k_shifted, pos, start).mean(axis=1))
    return scores


def query_list(w, r: int, selected: Sequence[np.ndarray]):
    """Compact query list of request r: selected tokens chunk by chunk, then the question."""
    q_pos, q_row, ci = [], [], 0
    for (_, kind, start, n, _, _, tok, _) in _segments_of(w, r):
        idx = np.arange(n, dtype=np.int64) if kind != 0 else np.asarray(selected[ci], dtype=np.int64)
        ci += kind == 0
        q_pos.append(start + idx)
        q_row.append(tok + idx)
    cat = lambda xs: np.concatenate(xs) if xs else np.zeros(0, dtype=np.int64)
    return cat(q_pos), cat(q_row)


def fix_and_attend(w, r: int, k_shifted, v_cached, selected, k_new=None, v_new=None, q=None,
                   only_queries: Optional[np.ndarray] = None, dense: bool = False):
    """Steps fix + attend for request r given the chosen token sets (dense: the matrix form of the
    attention, for many rows of a long prompt)."""
    theta = w.spec.rope_theta
    k_new = w.k_new if k_new is None else k_new
    v_new = w.v_new if v_new is None else v_new
    q = w.q if q is None else q
    q_pos, q_row = query_list(w, r, selected)
    k_ctx, v_ctx = k_shifted.copy(), v_cached.copy()
    if len(q_pos):
        k_ctx[q_pos] = rotate(np.asarray(k_new[q_row], dtype=np.float64), q_pos, theta)
        v_ctx[q_pos] = np.asarray(v_new[q_row], dtype=np.float64)
    which = np.arange(len(q_pos)) if only_queries is None else np.asarray(only_queries, dtype=np.int64)
    q_rot = rotate(np.asarray(q[q_row[which]], dtype=np.float64), q_pos[which], theta)
    attend = causal_attention_rows_dense if dense else causal_attention_rows
    out, lse = attend(q_rot, q_pos[which], k_ctx, v_ctx)
    return k_ctx, v_ctx, q_pos, q_row, out, lse


def run_request(w, r: int, selected_override: Optional[Sequence[np.ndarray]] = None,
                k_new=None, v_new=None, q=None, miss_segments: Sequence[int] = ()) -> RequestResult:
    k_sh, v_c, _ = shifted_context(w, r, miss_segments)
    scores = score_request(w, r, k_sh)
    chunk_segs = [s for s in _segments_of(w, r) if s[1] == 0]
    selected = [top_n(sc, seg[5]) for sc, seg in zip(scores, chunk_segs)]
    if selected_override is not None:
        selected = [np.asarray(s, dtype=np.int64) for s in selected_override]
    k_ctx, v_ctx, q_pos, q_row, out, lse = fix_and_attend(w, r, k_sh, v_c, selected, k_new, v_new, q)
    return RequestResult(k_sh, k_ctx, v_ctx, scores, selected, q_pos, q_row, out, lse)


def run(w, selected_override: Optional[Dict[int, Sequence[np.ndarray]]] = None) -> List[RequestResult]:
    """Whole path over every request of the batch (requests are independent)."""
    return [run_request(w, r, None if selected_override is None else selected_override.get(r))
            for r in range(w.n_requests)]


# --------------------------------------------------------------------------
# question-to-chunk attention and the focused chunks (Sec. 3.2.2, Algorithm 1)
# --------------------------------------------------------------------------
def segment_mass_rows(q_rot: np.ndarray, pos: np.ndarray, k_ctx: np.ndarray, bounds: Sequence[int]) -> np.ndarray:
    """Attention weight each given row puts on each segment.

    q_rot [n, Hq, d] rotated queries at positions pos [n]; k_ctx [n_ctx, Hkv, d] logical order;
    bounds [n_seg + 1] logical start of every segment and the end of the last one.
    Returns [n, Hq, n_seg]: sum over keys l of segment s, l <= pos, of the softmax weight a_l
    (softmax over all keys l <= pos, scaled by 1/sqrt(d): Eq. (1) per token).
    """
    n, hq, d = q_rot.shape
    g = hq // k_ctx.shape[1]
    n_seg = len(bounds) - 1
    mass = np.zeros((n, hq, n_seg), dtype=np.float64)
    for j in range(n):
        p = int(pos[j])
        for h in range(hq):
            s = k_ctx[: p + 1, h // g, :] @ q_rot[j, h, :] / np.sqrt(np.float64(d))
            a = np.exp(s - s.max())
            a /= a.sum()
            for i in range(n_seg):
                lo, hi = int(bounds[i]), min(int(bounds[i + 1]), p + 1)
                if hi > lo:
                    mass[j, h, i] = a[lo:hi].sum()
    return mass


def question_chunk_mass(w, r: int, k_ctx: np.ndarray, q=None) -> np.ndarray:
    """inter(C_i, U) for every segment of request r (the question segment's entry is the weight
    the question keeps on itself): sum over question tokens of the mean over heads of the weight
    on the segment's keys.  k_ctx is the request's K after the fix."""
    theta = w.spec.rope_theta
    q = w.q if q is None else q
    segs = _segments_of(w, r)
    bounds = [sg[2] for sg in segs] + [segs[-1][2] + segs[-1][3]]
    total = np.zeros(len(segs), dtype=np.float64)
    for (_, kind, start, n, _, _, tok, _) in segs:
        if kind == 0:
            continue
        pos = start + np.arange(n, dtype=np.int64)
        q_rot = rotate(np.asarray(q[tok:tok + n], dtype=np.float64), pos, theta)
        total += segment_mass_rows(q_rot, pos, k_ctx, bounds).mean(axis=1).sum(axis=0)
    return total


def segment_attention_matrix(w, r: int, k_ctx: np.ndarray, q_pos: np.ndarray, q_row: np.ndarray, q=None):
    """inter / intra sums between the segments of request r over the given rows (positions q_pos,
    rows q_row of q): M[t, s] = sum over rows in segment t of the head-mean weight on the keys of
    segment s (s <= t), and self_w[t] = the same for each row's own key alone.
    inter(C_s, C_t) = M[t, s] for s < t (Eq. (2)); intra(C_t) = M[t, t] - self_w[t] (Eq. (3))."""
    theta = w.spec.rope_theta
    q = w.q if q is None else q
    segs = _segments_of(w, r)
    bounds = [sg[2] for sg in segs] + [segs[-1][2] + segs[-1][3]]
    n_seg = len(segs)
    m = np.zeros((n_seg, n_seg), dtype=np.float64)
    self_w = np.zeros(n_seg, dtype=np.float64)
    if len(q_pos) == 0:
        return m, self_w
    q_rot = rotate(np.asarray(q[q_row], dtype=np.float64), q_pos, theta)
    mass = segment_mass_rows(q_rot, q_pos, k_ctx, bounds).mean(axis=1)          # [n, n_seg]
    hq, d = q_rot.shape[1], q_rot.shape[2]
    g = hq // k_ctx.shape[1]
    _, lse = causal_attention_rows(q_rot, q_pos, k_ctx, np.zeros_like(k_ctx))
    for j, p in enumerate(q_pos):
        t = max(i for i in range(n_seg) if bounds[i] <= p)
        m[t] += mass[j]
        own = [np.exp(k_ctx[p, h // g, :] @ q_rot[j, h, :] / np.sqrt(np.float64(d)) - lse[j, h]) for h in range(hq)]
        self_w[t] += np.mean(own)
    return m, self_w


def chunk_ab(inter: Sequence[float], prefix_len: Sequence[int], intra: float, chunk_len: int):
    """a(C_i) = sum_j inter(C_j, C_i) / (|C_i| |C_j|), b(C_i) = intra(C_i) / |C_i|^2 (Sec. 3.1)."""
    a = sum(float(x) / (chunk_len * int(n)) for x, n in zip(inter, prefix_len))
    return a, float(intra) / (chunk_len * chunk_len)


def cci(a_layers: Sequence[float], b_layers: Sequence[float]) -> float:
    """CCI = sigmoid(abar / bbar) with the layer means of a and b (Sec. 3.1)."""
    abar, bbar = float(np.mean(a_layers)), float(np.mean(b_layers))
    ratio = 0.0 if abar == 0.0 else (np.inf if bbar == 0.0 else abar / bbar)
    return float(1.0 / (1.0 + np.exp(-ratio)))


def prefix_overlap(old_prefix: Sequence[int], old_inter: Sequence[float], new_prefix: Sequence[int]) -> float:
    """beta(C_i | S_new): share of the old inter-attention that came from chunks still in the prefix."""
    total = float(sum(old_inter))
    if total == 0.0:
        return 1.0
    return float(sum(x for c, x in zip(old_prefix, old_inter) if c in set(new_prefix))) / total


def order_penalty(old_prefix: Sequence[int], new_prefix: Sequence[int]) -> float:
    """gamma: discordant pairs between the old and new order of the common chunks, over C(m, 2)."""
    common = [c for c in old_prefix if c in set(new_prefix)]
    m = len(common)
    if m < 2:
        return 0.0
    rank_new = {c: i for i, c in enumerate(new_prefix)}
    d = sum(1 for i in range(m) for j in range(i + 1, m) if rank_new[common[i]] > rank_new[common[j]])
    return d / (m * (m - 1) / 2.0)


def cache_fix_overhead(cci_value: float, beta: float, gamma: float, alpha: float, chunk_len: int):
    """beta' = beta (1 - gamma); CFO = alpha CCI (1 - beta') in [0, 1]; N = ceil(CFO |C|) (Sec. 3.3, 3.2.1)."""
    beta_adj = beta * (1.0 - gamma)
    cfo = min(1.0, max(0.0, alpha * cci_value * (1.0 - beta_adj)))
    n = int(min(chunk_len, max(0, np.ceil(cfo * chunk_len - 1e-9))))
    return beta_adj, cfo, n


def predict_focused(inter_layers: Sequence[Sequence[float]], window: int):
    """Algorithm 1.  inter_layers[l][i] = inter_{l+1}(C_i, U) for chunks i < k.

    Returns (F_star, L_star, F_all): the focused set (sorted chunk indices) and the 1-based layer
    at which it was fixed (None, None if the stop rule never fires), and the set chosen at every
    layer processed.
    """
    k = len(inter_layers[0])
    cinter = np.zeros(k, dtype=np.float64)
    f_all = []
    for l, inter in enumerate(inter_layers, start=1):
        cinter += np.asarray(inter, dtype=np.float64)
        order = sorted(range(k), key=lambda i: (-cinter[i], i))
        sorted_cinter = cinter[order]
        chosen = list(order)
        if k >= 3:
            diff = sorted_cinter[:-1] - sorted_cinter[1:]              # diff_1 .. diff_{k-1}
            if diff.sum() > 0:
                p = diff / diff.sum()
                plogp = np.where(p > 0, p * np.log(np.where(p > 0, p, 1.0)), 0.0)
                h = -np.cumsum(plogp)                                  # h_1 .. h_{k-1}
                jumps = h[1:] - h[:-1]                                 # h_{i+1} - h_i, i = 1 .. k-2
                i_star = int(np.argmax(jumps)) + 1                     # 1-based
                chosen = order[:i_star]
        f = sorted(chosen)
        f_all.append(f)
        if l >= window and all(prev == f for prev in f_all[l - window:l]):
            return f, l, f_all
    return None, None, f_all


# --------------------------------------------------------------------------
# layer-wise preloading (Sec. 3.4.2, Eq. (12), Algorithm 2)
# --------------------------------------------------------------------------
def preload_depth(n_layers: int, t_prefill: float, t_load: float) -> int:
    """L_p = max(1, (L - 1)(1 - T_prefill / T_load) + 1), taken up to the next integer (the loop of
    Algorithm 2 needs a layer count) and at most L; 1 when loading is not slower than compute."""
    if t_load <= 0 or t_prefill >= t_load:
        return 1
    lp = (n_layers - 1) * (1.0 - t_prefill / t_load) + 1.0
    return int(max(1, min(n_layers, np.ceil(lp - 1e-9))))


def preload_schedule(n_layers: int, depth: int):
    """Algorithm 2 as printed: before layer i is computed, layers i .. min(i + L_p, L) are preloaded
    (those not preloaded before).  Returns, for every layer i (0-based), the layers newly asked for
    just before it."""
    done, steps = set(), []
    for i in range(n_layers):
        new = [j for j in range(i, min(i + depth, n_layers - 1) + 1) if j not in done]
        done.update(new)
        steps.append(new)
    return steps


def layer_loop(w, r: int, n_layers: int, window: int, q_scales: Sequence[float], scores=None):
    """The per-layer loop of Sec. 3.4 for request r on one layer's tensors reused for every layer
    (queries of layer l scaled by q_scales[l]): tokens are chosen from one fixed score list (the
    request's scores in the new context unless given), each layer recomputes and attends them, the
    question's attention to the chunks feeds Algorithm 1, and from the layer after the focused set
    settles the other chunks are not recomputed any more (their budget drops to 0).
    Returns one dict per layer: selected sets, q_pos, out, lse, masses, focused set, stop layer."""
    k_sh, v_c, _ = shifted_context(w, r)
    segs = _segments_of(w, r)
    chunk_ids = [i for i, sg in enumerate(segs) if sg[1] == 0]
    if scores is None:
        scores = score_request(w, r, k_sh)
    budget = [segs[i][5] for i in chunk_ids]
    inter_hist, stop_layer, focused, out = [], None, None, []
    for l in range(n_layers):
        selected = [top_n(sc, n) for sc, n in zip(scores, budget)]
        q = np.asarray(w.q, dtype=np.float64) * float(q_scales[l])
        k_ctx, v_ctx, q_pos, q_row, o, lse = fix_and_attend(w, r, k_sh, v_c, selected, q=q)
        mass = question_chunk_mass(w, r, k_ctx, q=q)
        rec = dict(selected=selected, q_pos=q_pos, out=o, lse=lse, mass=mass)
        if stop_layer is None and chunk_ids:
            inter_hist.append([mass[i] for i in chunk_ids])
            f, l_star, _ = predict_focused(inter_hist, window)
            if f is not None:
                stop_layer, focused = l_star, f
                budget = [b if c in f else 0 for c, b in enumerate(budget)]
        rec["stop_layer"], rec["focused"] = stop_layer, focused
        out.append(rec)
    return out


def qkv_project(hidden_rows: np.ndarray, w_qkv: np.ndarray, hq: int, hkv: int, d: int):
    """Q, K, V of the given token rows: X W^T with W [(Hq+2Hkv)d, hidden] (one row per output
    feature: q heads, then k heads, then v heads), split by heads (Sec. 3.4.3: computed only for
    the recomputation and question tokens).  Returns q [n,Hq,d], k [n,Hkv,d], v [n,Hkv,d]."""
    y = np.asarray(hidden_rows, dtype=np.float64) @ np.asarray(w_qkv, dtype=np.float64).T
    n = y.shape[0]
    q = y[:, : hq * d].reshape(n, hq, d)
    k = y[:, hq * d: (hq + hkv) * d].reshape(n, hkv, d)
    v = y[:, (hq + hkv) * d:].reshape(n, hkv, d)
    return q, k, v


# --------------------------------------------------------------------------
# the rest of the layer, for the recomputed rows (Sec. 2.1, Sec. 3.4.3)
# --------------------------------------------------------------------------
def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """x W^T with W [out_features, in_features]."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def silu(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def gated_ffn_in(y: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray) -> np.ndarray:
    """silu(y W_gate^T) * (y W_up^T): the input of the down projection."""
    return silu(linear(y, w_gate)) * linear(y, w_up)


def layer_tail(h_rows: np.ndarray, attn_out: np.ndarray, w_o, gain_ffn, w_gate, w_up, w_down, eps: float):
    """Hidden state after the layer, for rows with hidden state h_rows [n, hidden] and attention
    output attn_out [n, Hq, d]: h1 = h + o W_o^T, h2 = h1 + FFN(rms_norm(h1)).  Returns (h1, h2)."""
    n = h_rows.shape[0]
    h1 = np.asarray(h_rows, dtype=np.float64) + linear(np.asarray(attn_out, dtype=np.float64).reshape(n, -1), w_o)
    h2 = h1 + linear(gated_ffn_in(rms_norm(h1, gain_ffn, eps), w_gate, w_up), w_down)
    return h1, h2


def recompute_layers(w, r: int, selected, weights: Sequence, h_in: Optional[Sequence[np.ndarray]] = None,
                     window: Optional[int] = None):
    """The chosen rows of request r through len(weights) decoder layers (every layer sees the same
    synthetic chunk store): per layer x = rms_norm(h) -> Q, K, V of those rows -> fix + attend over
    the re-positioned caches -> layer_tail.  The first layer's h are the rows of w.hidden; h_in[l],
    if given, replaces the running state at the start of layer l (so that one layer can be checked
    at a time).  With a window, the question's attention to the chunks in every layer feeds
    Algorithm 1 and, from the layer after the focused set settles, the other chunks' rows are
    dropped (Sec. 3.2.2): their hidden states are not carried further.
    Returns per layer a dict with selected, q_pos, h_in, x, out, lse, h1, h2 (+ mass, stop_layer, focused)."""
    hq, hkv, d = w.spec.n_q_heads, w.spec.n_kv_heads, w.spec.head_dim
    selected = [np.asarray(s_) for s_ in selected]
    q_pos, q_row = query_list(w, r, selected)
    k_sh, v_c, _ = shifted_context(w, r)
    segs = _segments_of(w, r)
    chunk_ids = [i for i, sg in enumerate(segs) if sg[1] == 0]
    h = np.asarray(w.hidden[q_row], dtype=np.float64)
    inter_hist, stop_layer, focused = [], None, None
    layers = []
    for l, lw in enumerate(weights):
        if h_in is not None and h_in[l] is not None:
            h = np.asarray(h_in[l], dtype=np.float64)
        x = rms_norm(h, lw.gain_attn, lw.eps)
        qf, kf, vf = qkv_project(x, lw.w_qkv, hq, hkv, d)
        full = lambda a: _rows_at(a, q_row, w.n_tok)
        k_ctx, _, _, _, out, lse = fix_and_attend(w, r, k_sh, v_c, selected, k_new=full(kf), v_new=full(vf), q=full(qf))
        h1, h2 = layer_tail(h, out, lw.w_o, lw.gain_ffn, lw.w_gate, lw.w_up, lw.w_down, lw.eps)
        rec = {"selected": selected, "q_pos": q_pos, "h_in": h, "x": x, "out": out, "lse": lse, "h1": h1, "h2": h2}
        h = h2
        if window is not None:
            mass = question_chunk_mass(w, r, k_ctx, q=full(qf))
            rec["mass"] = mass
            if stop_layer is None and chunk_ids:
                inter_hist.append([mass[i] for i in chunk_ids])
                f, l_star, _ = predict_focused(inter_hist, window)
                if f is not None:
                    stop_layer, focused = l_star, f
                    # rows of the chunks that are not focused leave the list; the others keep their order
                    keep = np.ones(len(q_pos), dtype=bool)
                    for c, i in enumerate(chunk_ids):
                        if c not in f:
                            keep &= ~((q_pos >= segs[i][2]) & (q_pos < segs[i][2] + segs[i][3]))
                    selected = [sel if c in f else np.zeros(0, dtype=np.int64) for c, sel in enumerate(selected)]
                    h = h[keep]
                    q_pos, q_row = query_list(w, r, selected)
            rec["stop_layer"], rec["focused"] = stop_layer, focused
        layers.append(rec)
    return layers


def _rows_at(a: np.ndarray, rows: np.ndarray, n_tok: int) -> np.ndarray:
    """A per-token tensor [n_tok, ...] that holds a's rows at the given token rows (zero elsewhere)."""
    t = np.zeros((n_tok,) + a.shape[1:], dtype=np.float64)
    t[rows] = a
    return t
