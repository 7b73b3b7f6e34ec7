"""Pins for the CPU oracle: closed forms, invariants, limiting cases, library routines, brute force.

Each test fixes the oracle to something other than itself, so that a dropped term, a wrong
sign or index, or a transposed operand anywhere in oracle/cachecraft_oracle.py fails here.
The paper prints no worked numeric example of this path, so the pins are mathematical:
the textbook rotary embedding (cited in Sec. 2.1), the per-token causal attention of Sec. 2.1,
the block structure of inter/intra attention (Eq. (2), Eq. (3) and the matrix below them),
and the selection rule of Eq. (10).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import workload as W
from oracle import cachecraft_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- independent helpers
def rope_complex(x, pos, theta):
    """Textbook rotary embedding written with complex numbers: (x_i + i y_i) * exp(i pos w_i)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    h = d // 2
    w = np.array([theta ** (-(2.0 * i) / d) for i in range(h)])
    z = (x[..., :h] + 1j * x[..., h:]) * np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None, None] * w)
    return np.concatenate([z.real, z.imag], axis=-1)


def dense_causal_gqa(q_rot, k_rot, v, lib=True):
    """Full causal GQA attention over a whole prompt, via torch's library routine (fp64, CPU)."""
    n, hq, d = q_rot.shape
    hkv = k_rot.shape[1]
    g = hq // hkv
    qt = torch.from_numpy(q_rot).permute(1, 0, 2)[None]                 # [1,Hq,n,d]
    kt = torch.from_numpy(np.repeat(k_rot, g, axis=1)).permute(1, 0, 2)[None]
    vt = torch.from_numpy(np.repeat(v, g, axis=1)).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)
    return o[0].permute(1, 0, 2).numpy()


def attention_matrix(q_rot, k_rot):
    """Dense [Hq, n, n] causal softmax weights of Eq. (1), for block-sum checks."""
    n, hq, d = q_rot.shape
    g = hq // k_rot.shape[1]
    a = np.zeros((hq, n, n))
    for h in range(hq):
        s = q_rot[:, h] @ k_rot[:, h // g].T / math.sqrt(d)
        s[np.triu_indices(n, 1)] = -np.inf
        a[h] = torch.softmax(torch.from_numpy(s), dim=-1).numpy()
    return a


def small_workload(fracs=(0.25, 0.25, 0.25), lens=(20, 33, 16), question=5, offsets=(0, 0, 0),
                   order=(0, 1, 2), dtype="f32", Hq=4, Hkv=2, d=16, theta=1.0e4, scale=1.0, seed=11):
    req = W.RequestSpec(list(order), list(fracs), question)
    return W.custom("pin", dtype, Hq, Hkv, d, theta, lens, offsets, [req], scale, seed)


# ----------------------------------------------------------------------------- rotation (shift)
def test_rotate_matches_textbook_complex_form():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 3, 32))
    pos = np.array([0, 1, 5, 17, 1000, 31999, -40])
    np.testing.assert_allclose(O.rotate(x, pos, 5.0e5), rope_complex(x, pos, 5.0e5), rtol=0, atol=1e-12)


def test_rotate_one_hot_closed_form():
    d, theta, p = 64, 1.0e4, 37
    for i in (0, 1, 13, 31):
        k = np.zeros((1, 1, d)); k[0, 0, i] = 1.0
        r = O.rotate(k, np.array([p]), theta)[0, 0]
        phi = p * theta ** (-2.0 * i / d)
        expect = np.zeros(d); expect[i] = math.cos(phi); expect[i + d // 2] = math.sin(phi)
        np.testing.assert_allclose(r, expect, atol=1e-15)
        k = np.zeros((1, 1, d)); k[0, 0, i + d // 2] = 1.0         # y component: (-sin, cos)
        r = O.rotate(k, np.array([p]), theta)[0, 0]
        expect = np.zeros(d); expect[i] = -math.sin(phi); expect[i + d // 2] = math.cos(phi)
        np.testing.assert_allclose(r, expect, atol=1e-15)


def test_shift_composes_and_inverts():
    rng = np.random.default_rng(1)
    k = rng.standard_normal((9, 2, 128))
    a, b = 1536, -411
    ab = O.shift_keys(O.shift_keys(k, a, 5.0e5), b, 5.0e5)
    np.testing.assert_allclose(ab, O.shift_keys(k, a + b, 5.0e5), atol=1e-12)
    np.testing.assert_allclose(O.shift_keys(O.shift_keys(k, a, 5.0e5), -a, 5.0e5), k, atol=1e-12)
    assert np.array_equal(O.shift_keys(k, 0, 5.0e5), k)             # zero shift is bit-exact


def test_place_unrotated_keys_is_the_rotation_at_absolute_positions():
    rng = np.random.default_rng(21)
    k = rng.standard_normal((37, 2, 16))
    for start in (0, 5, 1000):
        got = O.place_keys(k, start, 1.0e4)
        np.testing.assert_allclose(got, rope_complex(k, start + np.arange(37), 1.0e4), atol=1e-12)
    # a store rotated at cached positions c + t and shifted by new - c lands where the unrotated store is placed
    cached = O.place_keys(k, 40, 1.0e4)
    np.testing.assert_allclose(O.shift_keys(cached, 123 - 40, 1.0e4), O.place_keys(k, 123, 1.0e4), atol=1e-11)
    # position 0 of an unrotated key is the key itself
    np.testing.assert_array_equal(O.place_keys(k, 0, 1.0e4)[0], k[0])


def test_shift_preserves_pair_norms():
    rng = np.random.default_rng(2)
    k = rng.standard_normal((5, 2, 64))
    s = O.shift_keys(k, 777, 1.0e4)
    n0 = k[..., :32] ** 2 + k[..., 32:] ** 2
    n1 = s[..., :32] ** 2 + s[..., 32:] ** 2
    np.testing.assert_allclose(n1, n0, rtol=1e-13)


def test_rotation_gives_relative_position_logits():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, 64)); k = rng.standard_normal((1, 1, 64))
    base = None
    for p, s in ((10, 3), (107, 100), (5007, 5000)):
        v = float(O.rotate(q, np.array([p]), 1.0e4)[0, 0] @ O.rotate(k, np.array([s]), 1.0e4)[0, 0])
        base = v if base is None else base
        assert abs(v - base) < 1e-10
    # and it does depend on the distance
    v2 = float(O.rotate(q, np.array([10]), 1.0e4)[0, 0] @ O.rotate(k, np.array([4]), 1.0e4)[0, 0])
    assert abs(v2 - base) > 1e-3


# ----------------------------------------------------------------------------- paged pool readers
def test_page_readers_follow_the_two_layouts():
    hkv, d = 2, 8
    kp = np.arange(3 * hkv * 16 * d, dtype=np.float64).reshape(3, hkv, 16, d)
    vp = np.arange(3 * hkv * d * 16, dtype=np.float64).reshape(3, hkv, d, 16)
    k = O.read_k_pages(kp, [2, 0], 21)
    v = O.read_v_pages(vp, [2, 0], 21)
    assert k.shape == v.shape == (21, hkv, d)
    for t, (blk, slot) in {0: (2, 0), 15: (2, 15), 16: (0, 0), 20: (0, 4)}.items():
        for h in range(hkv):
            for c in range(d):
                assert k[t, h, c] == kp[blk, h, slot, c]
                assert v[t, h, c] == vp[blk, h, c, slot]


# ----------------------------------------------------------------------------- scoring
def test_score_uniform_softmax_closed_form():
    w = small_workload()
    w.q[:] = 0.0                                                     # all logits equal -> uniform rows
    k_sh, _, _ = O.shifted_context(w, 0)
    sc = O.score_request(w, 0, k_sh)
    assert np.array_equal(sc[0], np.zeros(20))                       # first chunk has no prior chunk
    for c, (start, n) in enumerate(((20, 33), (53, 16)), start=1):
        t = np.arange(n)
        np.testing.assert_allclose(sc[c], start / (start + t + 1.0), rtol=1e-13)


def test_score_bruteforce_and_complement():
    w = small_workload(lens=(6, 9, 7), question=3, d=8)
    k_sh, _, _ = O.shifted_context(w, 0)
    sc = O.score_request(w, 0, k_sh)
    hq, hkv, d, theta = 4, 2, 8, 1.0e4
    starts = (0, 6, 15)
    for c, n in enumerate((6, 9, 7)):
        for t in range(n):
            p = starts[c] + t
            tot = 0.0
            for h in range(hq):
                qv = rope_complex(w.q[p][None].astype(np.float64), [p], theta)[0, h]
                logit = [sum(qv[e] * k_sh[l, h // 2, e] for e in range(d)) / math.sqrt(d) for l in range(p + 1)]
                mx = max(logit)
                ex = [math.exp(v - mx) for v in logit]
                prior = sum(ex[: starts[c]]) / sum(ex)
                own = sum(ex[starts[c]:]) / sum(ex)
                assert abs(prior + own - 1.0) < 1e-14
                tot += prior
            assert 0.0 <= sc[c][t] <= 1.0
            assert abs(sc[c][t] - tot / hq) < 1e-13


def test_score_block_sums_equal_inter_attention():
    # sum over the tokens of C_i of the per-token mass == sum_{j<i} inter(C_j, C_i)  (Eq. (2), block matrix)
    w = small_workload(lens=(12, 10, 14), question=4)
    k_sh, _, n_ctx = O.shifted_context(w, 0)
    pos = np.arange(40)                                              # chunk tokens only (question keys come later)
    q_rot = rope_complex(w.q[:36].astype(np.float64), pos[:36], 1.0e4)
    a = attention_matrix(q_rot, k_sh[:36])                           # [Hq, 36, 36]
    sc = O.score_request(w, 0, k_sh)
    bounds = [(0, 12), (12, 22), (22, 36)]
    for i, (s0, s1) in enumerate(bounds):
        inter_sum = sum(a[:, s0:s1, b0:b1].sum(axis=(1, 2)) for (b0, b1) in bounds[:i]) if i else np.zeros(4)
        np.testing.assert_allclose(sc[i].sum(), np.mean(inter_sum), atol=1e-12)


def test_score_goes_to_one_with_a_dominant_prior_key():
    w = small_workload(lens=(8, 8, 8), question=2, d=16, theta=1.0e4)
    k_sh, _, _ = O.shifted_context(w, 0)
    # make key 3 (in chunk 0) line up with every query of chunk 2 at huge magnitude, un-rotated frame
    pos = 16 + np.arange(8)
    q_rot = O.rotate(w.q[16:24].astype(np.float64), pos, 1.0e4)
    k_sh[3] = 0.0
    k_sh[3, :, :] = 200.0 * np.sign(q_rot[4, 0, :])                  # aligns with token 4, head 0
    m = O.prior_mass(q_rot, k_sh, pos, 16)
    assert m[4, 0] > 1.0 - 1e-9


# ----------------------------------------------------------------------------- selection
def test_top_n_against_full_sort_and_edges():
    rng = np.random.default_rng(5)
    for n, k in ((1, 1), (17, 5), (64, 13), (100, 0), (100, 100)):
        s = rng.random(n)
        got = O.top_n(s, k)
        expect = sorted(sorted(range(n), key=lambda i: (-s[i], i))[:k])
        assert list(got) == expect
    assert list(O.top_n(np.array([0.0, 0.0, 0.0, 0.0]), 2)) == [0, 1]          # ties: lower index wins
    assert list(O.top_n(np.array([0.1, 0.5, 0.5, 0.2]), 1)) == [1]
    assert list(O.top_n(np.arange(10.0), 3)) == [7, 8, 9]                        # monotone -> the tail
    assert list(O.top_n(-np.arange(10.0), 3)) == [0, 1, 2]


def test_token_budget_rule():
    facts = json.load(open(os.path.join(GOLDEN, "paper_storage_facts.json")))
    assert facts["block_tokens"]["value"] == W.BLOCK == O.BLOCK
    # N = ceil(f |C|), robust to fp noise: 0.07*100 must give 7, not 8
    assert W.n_select_for(0.07, 100) == 7
    assert [W.n_select_for(f, n) for f, n in ((0.2, 64), (0.15, 512), (0.10, 1024), (0.10, 1000))] == [13, 77, 103, 100]
    assert W.n_select_for(0.0, 50) == 0 and W.n_select_for(1.0, 50) == 50
    # storage facts: bytes per token, all layers, K+V, 16-bit
    for name, f in facts["kv_mb_per_token"].items():
        mib = f["layers"] * f["kv_heads"] * f["head_dim"] * 2 * 2 / 2 ** 20
        assert abs(mib - f["value"]) / f["value"] < 0.3


# ----------------------------------------------------------------------------- fix + attend
def full_prefill_reference(w, theta):
    n = w.n_tok
    pos = np.arange(n)
    q = rope_complex(w.q.astype(np.float64), pos, theta)
    k = rope_complex(w.k_new.astype(np.float64), pos, theta)
    return dense_causal_gqa(q, k, w.v_new.astype(np.float64)), k


def test_full_recompute_equals_full_causal_prefill():
    w = small_workload(fracs=(1.0, 1.0, 1.0), lens=(20, 33, 16), question=5, offsets=(0, 7, 3))
    res = O.run_request(w, 0)
    ref, k_ref = full_prefill_reference(w, 1.0e4)
    assert np.array_equal(res.q_pos, np.arange(w.n_tok))
    np.testing.assert_allclose(res.out, ref, atol=1e-12)
    np.testing.assert_allclose(res.k_ctx, k_ref, atol=1e-12)
    np.testing.assert_allclose(res.v_ctx, w.v_new, atol=0)


def test_zero_recompute_at_cached_offsets_leaves_cache_unchanged():
    lens = (32, 16, 48)
    w = small_workload(fracs=(0.0, 0.0, 0.0), lens=lens, question=6, offsets=(0, 32, 48), order=(0, 1, 2))
    assert np.all(w.shift_descs[:, W.SHIFT_DELTA] == 0)
    res = O.run_request(w, 0)
    n_chunk = sum(lens)
    # cached rows come back bit-exact
    for c in range(3):
        blocks = w.store_tab[w.store_tab_off[c]: w.store_tab_off[c + 1]]
        s = int(w.segments[c][W.SEG_START])
        assert np.array_equal(res.k_ctx[s:s + lens[c]], O.read_k_pages(w.k_store, blocks, lens[c]))
        assert np.array_equal(res.v_ctx[s:s + lens[c]], O.read_v_pages(w.v_store, blocks, lens[c]))
    # only question tokens are queries; they equal plain attention of the question over cache + question
    assert np.array_equal(res.q_pos, n_chunk + np.arange(6))
    k_all = res.k_ctx.copy(); v_all = res.v_ctx.copy()
    q_full = np.zeros((w.n_tok, 4, 16))
    q_full[n_chunk:] = rope_complex(w.q[n_chunk:].astype(np.float64), res.q_pos, 1.0e4)
    ref = dense_causal_gqa(q_full, k_all, v_all)[n_chunk:]
    np.testing.assert_allclose(res.out, ref, atol=1e-12)


def test_dense_attention_form_on_row_subsets():
    """The matrix form of the attention (many rows at once): on every row of a prompt it is the library's
    causal attention; on a subset of rows in any order it gives those rows of it, and its log-sum-exp is
    that of the library softmax denominator; a row at position 0 returns the first value row."""
    rng = np.random.default_rng(21)
    n, hq, hkv, d = 53, 6, 2, 16
    q = rng.standard_normal((n, hq, d)); k = rng.standard_normal((n, hkv, d)); v = rng.standard_normal((n, hkv, d))
    full = dense_causal_gqa(q, k, v)
    out, lse = O.causal_attention_rows_dense(q, np.arange(n), k, v)
    np.testing.assert_allclose(out, full, atol=1e-12)
    rows = np.array([40, 0, 7, 52, 7])
    out_s, lse_s = O.causal_attention_rows_dense(q[rows], rows, k, v)
    np.testing.assert_allclose(out_s, full[rows], atol=1e-12)
    np.testing.assert_allclose(out_s[1], np.repeat(v[0], hq // hkv, axis=0), atol=1e-14)
    for j, p in enumerate(rows):
        for h in range(hq):
            logits = torch.from_numpy(k[: p + 1, h // (hq // hkv)] @ q[p, h] / math.sqrt(d))
            assert abs(float(torch.logsumexp(logits, 0)) - lse_s[j, h]) < 1e-12
    # no rows: empty results
    o0, l0 = O.causal_attention_rows_dense(q[:0], rows[:0], k, v)
    assert o0.shape == (0, hq, d) and l0.shape == (0, hq)


def test_attention_invariant_to_a_global_position_offset():
    base = small_workload(offsets=(0, 0, 0))
    k_sh, v_c, _ = O.shifted_context(base, 0)
    sel = [np.array([1, 5, 6]), np.array([0, 9, 30]), np.array([2, 3])]
    _, _, q_pos, q_row, out0, lse0 = O.fix_and_attend(base, 0, k_sh, v_c, sel)
    # same data, every position (cached keys, new keys, queries) moved by +1000
    off = 1000
    theta = base.spec.rope_theta
    k2 = O.rotate(k_sh, np.full(k_sh.shape[0], off), theta)
    k_ctx = k2.copy(); v_ctx = v_c.copy()
    k_ctx[q_pos] = O.rotate(base.k_new[q_row].astype(np.float64), q_pos + off, theta)
    v_ctx[q_pos] = base.v_new[q_row]
    q_rot = O.rotate(base.q[q_row].astype(np.float64), q_pos + off, theta)
    out1, lse1 = O.causal_attention_rows(q_rot, q_pos, k_ctx, v_ctx)
    np.testing.assert_allclose(out1, out0, atol=1e-10)
    np.testing.assert_allclose(lse1, lse0, atol=1e-10)


def test_zero_queries_average_the_values_and_lse_is_log_count():
    w = small_workload()
    w.q[:] = 0.0
    k_sh, v_c, _ = O.shifted_context(w, 0)
    sel = [np.array([0, 19]), np.array([4]), np.array([], dtype=np.int64)]
    k_ctx, v_ctx, q_pos, _, out, lse = O.fix_and_attend(w, 0, k_sh, v_c, sel)
    for j, p in enumerate(q_pos):
        for h in range(4):
            np.testing.assert_allclose(out[j, h], v_ctx[: p + 1, h // 2].mean(axis=0), atol=1e-13)
            assert abs(lse[j, h] - math.log(p + 1)) < 1e-13


def test_attention_bruteforce_scalar_loops_and_visibility_of_fixed_rows():
    w = W.config(1)                                                   # the tiny benchmark config
    res = O.run_request(w, 0)
    hq, hkv, d = 4, 2, 64
    assert res.out.shape == (55, hq, d)
    rng = np.random.default_rng(9)
    for j in rng.choice(55, size=6, replace=False):
        p = int(res.q_pos[j]); h = int(rng.integers(hq))
        qv = rope_complex(w.q[res.q_row[j]][None].astype(np.float64), [p], 1.0e4)[0, h]
        logits = []
        for l in range(p + 1):
            logits.append(sum(float(qv[e]) * float(res.k_ctx[l, h // 2, e]) for e in range(d)) / math.sqrt(d))
        mx = max(logits); z = sum(math.exp(v - mx) for v in logits)
        o = [sum(math.exp(logits[l] - mx) / z * float(res.v_ctx[l, h // 2, e]) for l in range(p + 1)) for e in range(d)]
        np.testing.assert_allclose(res.out[j, h], o, atol=1e-12)
        assert abs(res.lse[j, h] - (mx + math.log(z))) < 1e-12
    # fixed rows are the recomputed ones, stale rows are the shifted cache
    is_q = np.zeros(208, dtype=bool); is_q[res.q_pos] = True
    assert np.array_equal(res.k_ctx[~is_q], res.k_shifted[~is_q])
    np.testing.assert_allclose(res.k_ctx[is_q], rope_complex(w.k_new[res.q_row].astype(np.float64), res.q_pos, 1.0e4), atol=1e-12)
    assert np.array_equal(res.v_ctx[is_q], w.v_new[res.q_row].astype(np.float64))
    # 13 of 64 per chunk, first chunk takes its first 13 (all scores zero)
    assert [len(s) for s in res.selected] == [13, 13, 13]
    assert list(res.selected[0]) == list(range(13))


def test_query_row_order_does_not_matter():
    w = small_workload()
    k_sh, v_c, _ = O.shifted_context(w, 0)
    sel = [np.array([1, 5]), np.array([0, 9, 30]), np.array([2])]
    k_ctx, v_ctx, q_pos, q_row, out, lse = O.fix_and_attend(w, 0, k_sh, v_c, sel)
    perm = np.random.default_rng(4).permutation(len(q_pos))
    q_rot = O.rotate(w.q[q_row[perm]].astype(np.float64), q_pos[perm], 1.0e4)
    out_p, lse_p = O.causal_attention_rows(q_rot, q_pos[perm], k_ctx, v_ctx)
    np.testing.assert_allclose(out_p, out[perm], atol=1e-14)
    np.testing.assert_allclose(lse_p, lse[perm], atol=1e-14)


def test_padding_slots_are_never_keys():
    # chunk lengths that are not multiples of 16: poison the padding slots of the store
    w = small_workload(lens=(20, 33, 17), question=5)
    res0 = O.run_request(w, 0)
    for c, n in enumerate((20, 33, 17)):
        last = int(w.store_tab[w.store_tab_off[c + 1] - 1])
        w.k_store[last, :, n % 16:, :] = 1.0e6
        w.v_store[last, :, :, n % 16:] = -1.0e6
    res1 = O.run_request(w, 0)
    assert np.array_equal(res0.out, res1.out)
    assert all(np.array_equal(a, b) for a, b in zip(res0.scores, res1.scores))


def test_qkv_projection_splits_heads_in_q_k_v_order():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((3, 8)); wq = rng.standard_normal(((4 + 2 * 2) * 4, 8))
    q, k, v = O.qkv_project(x, wq, 4, 2, 4)
    y = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(wq))
    np.testing.assert_allclose(q[1, 2], y[1, 8:12].numpy(), atol=1e-13)
    np.testing.assert_allclose(k[2, 1], y[2, 16 + 4:16 + 8].numpy(), atol=1e-13)
    np.testing.assert_allclose(v[0, 0], y[0, 24:28].numpy(), atol=1e-13)


# ----------------------------------------------------------------------------- question-to-chunk mass
def _fixed_context(w, r=0):
    res = O.run_request(w, r)
    return res


def test_question_mass_uniform_softmax_closed_form():
    # all logits equal -> row at position p spreads 1/(p+1) on every visible key
    w = small_workload(lens=(20, 33, 16), question=5)
    w.q[:] = 0.0
    res = _fixed_context(w)
    got = O.question_chunk_mass(w, 0, res.k_ctx)
    starts, lens = (0, 20, 53, 69), (20, 33, 16, 5)
    want = np.zeros(4)
    for u in range(5):
        p = 69 + u
        for i in range(3):
            want[i] += lens[i] / (p + 1.0)
        want[3] += (u + 1) / (p + 1.0)
    np.testing.assert_allclose(got, want, rtol=1e-13)


def test_question_mass_is_the_block_sum_of_the_attention_matrix():
    # Eq. (2) with the question as the later chunk: sum of a_kl over question rows and chunk columns
    w = small_workload(lens=(12, 10, 14), question=6)
    res = _fixed_context(w)
    n_ctx = 42
    # every token's rotated query, in logical order (chunk rows are not needed but harmless)
    q_log = np.zeros((n_ctx, 4, 16))
    q_log[36:] = rope_complex(w.q[36:42].astype(np.float64), np.arange(36, 42), 1.0e4)
    a = attention_matrix(q_log, res.k_ctx)                            # [Hq, 42, 42], library softmax
    got = O.question_chunk_mass(w, 0, res.k_ctx)
    bounds = [(0, 12), (12, 22), (22, 36), (36, 42)]
    for i, (b0, b1) in enumerate(bounds):
        np.testing.assert_allclose(got[i], a[:, 36:42, b0:b1].sum(axis=(1, 2)).mean(), atol=1e-12)
    assert abs(got.sum() - 6.0) < 1e-12                               # every row's weights add up to one


def test_question_mass_bruteforce_scalar_loops():
    w = small_workload(lens=(5, 7), question=3, d=8, fracs=(0.4, 0.4), offsets=(0, 0), order=(1, 0))
    res = _fixed_context(w)
    segs = [tuple(int(v) for v in s) for s in w.segments]
    starts = [s[2] for s in segs] + [segs[-1][2] + segs[-1][3]]
    tok_q = segs[-1][6]
    want = [0.0] * len(segs)
    for u in range(3):
        p = starts[-2] + u
        for h in range(4):
            qv = rope_complex(w.q[tok_q + u][None].astype(np.float64), [p], 1.0e4)[0, h]
            logit = [sum(qv[e] * res.k_ctx[l, h // 2, e] for e in range(8)) / math.sqrt(8) for l in range(p + 1)]
            mx = max(logit)
            ex = [math.exp(v - mx) for v in logit]
            z = sum(ex)
            for i in range(len(segs)):
                want[i] += sum(ex[starts[i]:min(starts[i + 1], p + 1)]) / z / 4.0
    np.testing.assert_allclose(O.question_chunk_mass(w, 0, res.k_ctx), want, rtol=1e-12)


def test_question_mass_follows_a_dominant_key():
    w = small_workload(lens=(8, 8, 8), question=2)
    res = _fixed_context(w)
    k = res.k_ctx.copy()
    pos = 24 + np.arange(2)
    q_rot = O.rotate(w.q[24:26].astype(np.float64), pos, 1.0e4)
    k[11] = 0.0                                                       # one key of chunk 1 aligned with heads 0 and 2 of row 0
    k[11, 0, :] = 300.0 * np.sign(q_rot[0, 0, :])
    k[11, 1, :] = 300.0 * np.sign(q_rot[0, 2, :])
    m = O.segment_mass_rows(q_rot, pos, k, [0, 8, 16, 24, 26])
    assert m[0, 0, 1] > 1.0 - 1e-9 and m[0, 2, 1] > 1.0 - 1e-9
    np.testing.assert_allclose(m.sum(axis=2), 1.0, atol=1e-12)


# ----------------------------------------------------------------------------- focused chunks (Algorithm 1)
def test_focused_hand_worked_layer():
    # sorted scores 10, 9, 2, 1, 0.5 -> gaps 1, 7, 1, 0.5 (sum 9.5), p = .1053 .7368 .1053 .0526,
    # -p ln p = .2370 .2250 .2370 .1550; over i = 1..3 the jumps h_{i+1}-h_i are .2250 .2370 .1550:
    # i* = 2, the two top chunks (worked by hand from the algorithm's lines 4-9)
    inter = [2.0, 10.0, 0.5, 9.0, 1.0]
    f, l, f_all = O.predict_focused([inter], window=1)
    assert f == [1, 3] and l == 1 and f_all == [[1, 3]]
    p = np.array([1, 7, 1, 0.5]) / 9.5
    assert np.argmax((-p * np.log(p))[1:]) + 1 == 2


def test_focused_scores_accumulate_and_stop_rule_needs_w_equal_sets():
    a = [5.0, 1.0, 0.9, 0.8, 0.1]          # alone: sorted 5 1 .9 .8 .1 -> gaps 4 .1 .1 .7
    b = [0.0, 6.0, 0.0, 0.0, 0.0]          # cumulative after a+b: 5 7 .9 .8 .1 -> sorted 7 5 .9 .8 .1 -> gaps 2 4.1 .1 .7
    fa, la, _ = O.predict_focused([a], window=1)
    # gaps 4 .1 .1 .7 (sum 4.9): -p ln p = .166 .079 .079 .278 -> jumps over i=1..3: .079 .079 .278 -> i* = 3
    assert fa == [0, 1, 2] and la == 1
    f, l, f_all = O.predict_focused([a, b, [0.0] * 5, [0.0] * 5], window=2)
    # layer 2 cumulative gaps 2 4.1 .1 .7 (sum 6.9): -p ln p = .359 .309 .061 .232 -> jumps .309 .061 .232 -> i* = 1
    assert f_all[0] == [0, 1, 2] and f_all[1] == [1]
    assert f == [1] and l == 3 and len(f_all) == 3            # layers 2 and 3 agree -> stops at layer 3
    f, l, f_all = O.predict_focused([a, b], window=2)
    assert f is None and l is None and len(f_all) == 2         # never two equal sets in a row


def test_focused_degenerate_cases_keep_every_chunk():
    assert O.predict_focused([[1.0, 3.0]], window=1)[0] == [0, 1]                 # k < 3: no i in 1..k-2
    assert O.predict_focused([[2.0, 2.0, 2.0, 2.0]], window=1)[0] == [0, 1, 2, 3]  # no gap at all
    # k = 3: the only admissible i is 1
    assert O.predict_focused([[0.1, 0.2, 5.0]], window=1)[0] == [2]
    # invariants: result is a prefix of the descending order; scale of the scores does not matter
    rng = np.random.default_rng(3)
    for _ in range(50):
        x = rng.random(7)
        f1 = O.predict_focused([x], 1)[0]
        f2 = O.predict_focused([1000.0 * x], 1)[0]
        assert f1 == f2 and 1 <= len(f1) <= 5
        assert set(f1) == set(np.argsort(-x)[:len(f1)])


# ----------------------------------------------------------------------------- inter / intra, CCI, beta, gamma, CFO
def test_segment_matrix_is_the_block_sum_of_a_library_softmax():
    # full prefill (every token a query): M[t, s] = head-mean of the (t, s) block of the attention
    # matrix; the diagonal of that matrix is what intra leaves out (Eq. (2), Eq. (3))
    w = small_workload(lens=(12, 10, 14), question=6, fracs=(1.0, 1.0, 1.0))
    res = O.run_request(w, 0)
    assert len(res.q_pos) == 42 and np.array_equal(np.sort(res.q_pos), np.arange(42))
    order = np.argsort(res.q_pos)
    q_rot = rope_complex(w.q[res.q_row[order]].astype(np.float64), np.arange(42), 1.0e4)
    a = attention_matrix(q_rot, res.k_ctx)                            # [Hq, 42, 42]
    m, self_w = O.segment_attention_matrix(w, 0, res.k_ctx, res.q_pos, res.q_row)
    bounds = [(0, 12), (12, 22), (22, 36), (36, 42)]
    for t, (t0, t1) in enumerate(bounds):
        for s, (s0, s1) in enumerate(bounds):
            want = a[:, t0:t1, s0:s1].sum(axis=(1, 2)).mean() if s <= t else 0.0
            assert abs(m[t, s] - want) < 1e-12
        diag = np.mean([np.trace(a[h, t0:t1, t0:t1]) for h in range(4)])
        assert abs(self_w[t] - diag) < 1e-12
        strict = np.mean([np.tril(a[h, t0:t1, t0:t1], -1).sum() for h in range(4)])
        assert abs((m[t, t] - self_w[t]) - strict) < 1e-12            # intra: strictly earlier tokens
        assert abs(m[t].sum() - (t1 - t0)) < 1e-12                    # every row's weights add up to one


def test_segment_matrix_uniform_closed_form_and_row_subsets():
    w = small_workload(lens=(8, 5), question=3, fracs=(0.5, 0.4), offsets=(0, 0), order=(0, 1))
    w.q[:] = 0.0
    res = O.run_request(w, 0)
    m, self_w = O.segment_attention_matrix(w, 0, res.k_ctx, res.q_pos, res.q_row)
    bounds = [0, 8, 13, 16]
    want = np.zeros((3, 3)); want_self = np.zeros(3)
    for p in res.q_pos:
        t = max(i for i in range(3) if bounds[i] <= p)
        for s in range(3):
            want[t, s] += max(0, min(bounds[s + 1], p + 1) - bounds[s]) / (p + 1.0)
        want_self[t] += 1.0 / (p + 1.0)
    np.testing.assert_allclose(m, want, rtol=1e-13)
    np.testing.assert_allclose(self_w, want_self, rtol=1e-13)


def test_order_penalty_is_the_normalised_kendall_tau_distance():
    from scipy.stats import kendalltau
    rng = np.random.default_rng(8)
    for _ in range(40):
        n_old, n_new = int(rng.integers(2, 9)), int(rng.integers(2, 9))
        old = list(rng.choice(12, size=n_old, replace=False)); new = list(rng.choice(12, size=n_new, replace=False))
        common = [c for c in old if c in new]
        g = O.order_penalty(old, new)
        if len(common) < 2:
            assert g == 0.0
            continue
        tau = kendalltau(range(len(common)), [new.index(c) for c in common]).statistic   # (C - D) / T, no ties
        assert abs(g - (1.0 - tau) / 2.0) < 1e-12
    # the paper's own example: C1-C2-C3 against C2-C1-C3 for chunk C3 -> beta = 1 yet the order differs
    assert O.prefix_overlap([1, 2], [0.4, 0.6], [2, 1]) == 1.0
    assert O.order_penalty([1, 2], [2, 1]) == 1.0 and O.order_penalty([1, 2], [1, 2]) == 0.0


def test_prefix_overlap_cci_and_cfo_by_hand():
    # beta: 0.5 + 0.2 of a total 1.0 survive
    assert abs(O.prefix_overlap([7, 8, 9], [0.5, 0.3, 0.2], [9, 4, 7]) - 0.7) < 1e-15
    assert O.prefix_overlap([7, 8], [0.0, 0.0], [1]) == 1.0 and O.prefix_overlap([], [], [1, 2]) == 1.0
    assert O.prefix_overlap([7, 8], [0.5, 0.5], []) == 0.0
    # a, b: inter 1 and 2 from prefix chunks of 10 and 20 tokens, own length 10, intra 5
    a, b = O.chunk_ab([1.0, 2.0], [10, 20], 5.0, 10)
    assert abs(a - (1.0 / 100 + 2.0 / 200)) < 1e-15 and abs(b - 0.05) < 1e-15
    # CCI: sigmoid of the ratio of the layer means
    assert abs(O.cci([0.02, 0.04], [0.05, 0.07]) - 1.0 / (1.0 + math.exp(-0.5))) < 1e-15
    assert O.cci([0.0], [0.3]) == 0.5 and O.cci([0.0], [0.0]) == 0.5 and O.cci([0.1], [0.0]) == 1.0
    assert O.cci([0.3], [0.1]) > O.cci([0.2], [0.1]) > O.cci([0.1], [0.1])
    # CFO and N: beta' = 0.7 * (1 - 1/3), CFO = 1.0 * 0.6 * (1 - 0.4666..) = 0.32, N = ceil(0.32 * 100) = 32
    beta_adj, cfo, n = O.cache_fix_overhead(0.6, 0.7, 1.0 / 3.0, 1.0, 100)
    assert abs(beta_adj - 0.7 * 2.0 / 3.0) < 1e-15 and abs(cfo - 0.32) < 1e-12 and n == 32
    assert O.cache_fix_overhead(0.7, 1.0, 0.0, 1.0, 100)[1:] == (0.0, 0)            # same prefix, same order
    assert O.cache_fix_overhead(0.9, 0.0, 0.0, 2.0, 64)[1:] == (1.0, 64)            # clipped: recompute everything
    assert O.cache_fix_overhead(0.5, 0.86, 0.0, 1.0, 100)[2] == 7                   # 0.07 * 100: no spurious ceiling


# ----------------------------------------------------------------------------- layer-wise preloading (Algorithm 2)
def test_preload_depth_formula():
    # the paper's own example: 5 layers, prefill : load = 1 : 2 -> three layers ahead
    assert O.preload_depth(5, 1.0, 2.0) == 3
    assert O.preload_depth(5, 2.0, 2.0) == 1 and O.preload_depth(5, 3.0, 2.0) == 1 and O.preload_depth(7, 1.0, 0.0) == 1
    # what the formula is for: the other L - L_p layers must load within the compute time of L - 1 layers;
    # L_p is the smallest count that achieves it (brute force over all counts)
    rng = np.random.default_rng(4)
    for _ in range(200):
        L = int(rng.integers(1, 81)); tp = float(rng.uniform(0.1, 5.0)); tl = float(rng.uniform(0.1, 5.0))
        fits = [lp for lp in range(1, L + 1) if (L - lp) * (tl / L) <= (L - 1) * (tp / L) + 1e-12]
        assert O.preload_depth(L, tp, tl) == min(fits)


def test_preload_schedule_is_algorithm_2():
    # written out for 5 layers, depth 3 (0-based): before layer 0 -> 0..3, before 1 -> 4, then nothing new
    assert O.preload_schedule(5, 3) == [[0, 1, 2, 3], [4], [], [], []]
    assert O.preload_schedule(4, 1) == [[0, 1], [2], [3], []]
    for L in range(1, 12):
        for depth in range(1, L + 2):
            steps = O.preload_schedule(L, depth)
            flat = [j for s in steps for j in s]
            assert flat == list(range(L))                               # every layer once, in order
            for i, s in enumerate(steps):
                assert all(i <= j <= min(i + depth, L - 1) for j in s)   # never further than L_p ahead
                assert i in [j for t in steps[: i + 1] for j in t]       # a layer is asked for before it is computed


# ----------------------------------------------------------------------------- chunks without a cache next to reused ones
def test_miss_chunk_equals_a_cache_that_already_holds_its_fresh_keys():
    # A chunk with no chunk-cache (every token computed afresh) must give what a reused cache gives
    # when that cache happens to hold exactly the fresh K (rotated at its cached positions) and V.
    w = small_workload(lens=(20, 33, 16), question=5, fracs=(0.25, 1.0, 0.25), offsets=(0, 7, 0), dtype="f32")
    miss = 1                                                          # the middle chunk of the request
    ref = O.run_request(w, 0, miss_segments=[miss])
    seg = [int(v) for v in w.segments[miss]]
    start, n, tok = seg[2], seg[3], seg[6]
    chunk = w.spec.requests[0].chunks[miss]
    cached = rope_complex(w.k_new[tok:tok + n].astype(np.float64), 7 + np.arange(n), 1.0e4)
    blocks = w.store_tab[w.store_tab_off[chunk]: w.store_tab_off[chunk + 1]]
    for t in range(n):                                                # write the store pages (layouts of Sec. 4 paging)
        w.k_store[blocks[t // 16], :, t % 16, :] = cached[t]
        w.v_store[blocks[t // 16], :, :, t % 16] = w.v_new[tok + t]
    hit = O.run_request(w, 0)
    np.testing.assert_allclose(ref.k_shifted, hit.k_shifted, atol=2e-6)
    np.testing.assert_allclose(ref.out, hit.out, atol=2e-5)
    assert all(np.array_equal(a, b) for a, b in zip(ref.selected, hit.selected))
    assert np.array_equal(ref.selected[miss], np.arange(n))            # a miss recomputes every token


# ----------------------------------------------------------------------------- loop over layers
def test_layer_loop_without_a_stop_is_independent_single_layers():
    w = small_workload(lens=(20, 33, 16), question=5)
    scales = [1.0, 0.5, 2.0]
    recs = O.layer_loop(w, 0, 3, window=9, q_scales=scales)            # the window never fills: no stop
    k_sh, v_c, _ = O.shifted_context(w, 0)
    base = O.run_request(w, 0)
    for l, rec in enumerate(recs):
        assert rec["stop_layer"] is None and rec["focused"] is None
        assert all(np.array_equal(a, b) for a, b in zip(rec["selected"], base.selected))
        _, _, _, _, out, lse = O.fix_and_attend(w, 0, k_sh, v_c, base.selected, q=w.q.astype(np.float64) * scales[l])
        np.testing.assert_allclose(rec["out"], out, atol=1e-13)
        assert abs(rec["mass"].sum() - 5.0) < 1e-12
    np.testing.assert_allclose(recs[0]["out"], base.out, atol=1e-13)


def test_layer_loop_drops_unfocused_chunks_after_the_stop():
    w = small_workload(lens=(20, 33, 16), question=5, fracs=(0.5, 0.5, 0.5))
    recs = O.layer_loop(w, 0, 4, window=2, q_scales=[1.0, 1.0, 1.0, 1.0])
    # identical layers: the same set twice -> stop at layer 2, and with 3 chunks Algorithm 1 keeps one
    assert [r["stop_layer"] for r in recs] == [None, 2, 2, 2]
    f = recs[1]["focused"]
    assert len(f) == 1 and f == [int(np.argmax(recs[0]["mass"][:3]))]
    sizes = [[len(s) for s in r["selected"]] for r in recs]
    assert sizes[0] == sizes[1] == [10, 17, 8]
    assert sizes[2] == sizes[3] == [n if c in f else 0 for c, n in enumerate([10, 17, 8])]
    assert len(recs[2]["q_pos"]) == sum(sizes[2]) + 5                 # the question is always recomputed


# ---- the rest of the layer (Sec. 2.1, Sec. 3.4.3) ---------------------------------------------------
def test_rms_norm_against_the_library_routine_and_closed_forms():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 48)); g = 1.0 + 0.1 * rng.standard_normal(48)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(O.rms_norm(x, g, 1e-5), want, rtol=1e-12, atol=1e-14)
    # a constant row has root mean square |c|: it comes out as sign(c) * gain (eps aside)
    assert np.allclose(O.rms_norm(np.full((1, 48), -3.0), g, 0.0), -g)
    # scale invariance without eps; with eps the zero row stays zero instead of dividing by zero
    assert np.allclose(O.rms_norm(5.0 * x, g, 0.0), O.rms_norm(x, g, 0.0))
    assert np.array_equal(O.rms_norm(np.zeros((2, 48)), g, 1e-5), np.zeros((2, 48)))
    # eps sits inside the root: a row of ones gives gain / sqrt(1 + eps)
    assert np.allclose(O.rms_norm(np.ones((1, 48)), g, 3.0), g / 2.0)


def test_linear_is_x_times_w_transposed():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 12)); w = rng.standard_normal((9, 12))
    y = O.linear(x, w)
    assert y.shape == (5, 9)
    for i in range(5):
        for o in range(9):
            assert abs(y[i, o] - sum(x[i, c] * w[o, c] for c in range(12))) < 1e-12
    # a transposed operand would fail here: W picks input feature 3 into output feature 0
    w1 = np.zeros((2, 12)); w1[0, 3] = 1.0
    assert np.array_equal(O.linear(x, w1)[:, 0], x[:, 3]) and not O.linear(x, w1)[:, 1].any()


def test_silu_and_gated_ffn_input():
    t = np.array([-30.0, -1.0, 0.0, 1.0, 30.0])
    assert np.allclose(O.silu(t), torch.nn.functional.silu(torch.from_numpy(t)).numpy(), rtol=1e-13, atol=1e-15)
    assert O.silu(np.array([0.0]))[0] == 0.0 and abs(O.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    rng = np.random.default_rng(7)
    y = rng.standard_normal((4, 10)); wg = rng.standard_normal((6, 10)); wu = rng.standard_normal((6, 10))
    a = O.gated_ffn_in(y, wg, wu)
    for i in range(4):
        for f in range(6):
            gate, up = float(wg[f] @ y[i]), float(wu[f] @ y[i])
            assert abs(a[i, f] - gate / (1.0 + math.exp(-gate)) * up) < 1e-12
    # the activation is on the gate branch only: swapping the branches changes the result,
    # a zero gate matrix switches the unit off, a zero up matrix too
    assert not np.allclose(a, O.gated_ffn_in(y, wu, wg))
    assert not O.gated_ffn_in(y, np.zeros_like(wg), wu).any() and not O.gated_ffn_in(y, wg, np.zeros_like(wu)).any()


def test_layer_tail_residuals_and_a_library_layer():
    rng = np.random.default_rng(8)
    n, hq, d, hid, ffn = 6, 4, 8, 24, 40
    h = rng.standard_normal((n, hid)); o = rng.standard_normal((n, hq, d))
    w_o = rng.standard_normal((hid, hq * d)) * 0.2; g = 1.0 + 0.1 * rng.standard_normal(hid)
    wg = rng.standard_normal((ffn, hid)) * 0.2; wu = rng.standard_normal((ffn, hid)) * 0.2
    wd = rng.standard_normal((hid, ffn)) * 0.2
    h1, h2 = O.layer_tail(h, o, w_o, g, wg, wu, wd, 1e-5)
    # the same layer from the library's operators
    T = torch.from_numpy
    F = torch.nn.functional
    t1 = T(h) + F.linear(T(o).reshape(n, -1), T(w_o))
    y = F.rms_norm(t1, (hid,), T(g), eps=1e-5)
    t2 = t1 + F.linear(F.silu(F.linear(y, T(wg))) * F.linear(y, T(wu)), T(wd))
    assert np.allclose(h1, t1.numpy(), rtol=1e-12, atol=1e-13) and np.allclose(h2, t2.numpy(), rtol=1e-12, atol=1e-13)
    # both residual connections: with no output projection and no down projection the state passes through
    z1, z2 = O.layer_tail(h, o, np.zeros_like(w_o), g, wg, wu, np.zeros_like(wd), 1e-5)
    assert np.array_equal(z1, h) and np.array_equal(z2, h)
    # the second residual starts from h1, not from h
    _, z2 = O.layer_tail(h, o, w_o, g, wg, wu, np.zeros_like(wd), 1e-5)
    assert np.allclose(z2, h1)
    # heads are concatenated head-major into the output projection's input
    w_pick = np.zeros((hid, hq * d)); w_pick[0, 2 * d + 5] = 1.0
    p1, _ = O.layer_tail(np.zeros_like(h), o, w_pick, g, wg, wu, np.zeros_like(wd), 1e-5)
    assert np.allclose(p1[:, 0], o[:, 2, 5])


def _tiny_projected(dtype="f32", hidden=None):
    reqs = [W.RequestSpec([0, 1, 2], [0.3, 0.25, 0.4], 9), W.RequestSpec([2, 0], [0.5, 0.2], 5)]
    hq, hkv, d = 4, 2, 64
    return W.custom("tiny-layers", dtype, hq, hkv, d, 1.0e4, [40, 33, 50], [0, 7, 3], reqs, 0.5, seed=77,
                    hidden=hidden or (hq + 2 * hkv) * d)


def test_recompute_layers_attention_step_is_the_pinned_hot_path():
    """With an identity projection, unit gains and rows of unit mean square the layer's Q, K, V are
    slices of the hidden state, so its attention step must be run_request on those slices."""
    w = _tiny_projected()
    hq, hkv, d = w.spec.n_q_heads, w.spec.n_kv_heads, w.spec.head_dim
    hid = w.hidden.shape[1]
    w.hidden = (w.hidden / np.sqrt(np.mean(w.hidden.astype(np.float64) ** 2, axis=1, keepdims=True))).astype(np.float64)
    lw = W.layer_weights(w.spec, hid, 96)
    lw.w_qkv = np.eye(hid); lw.gain_attn = np.ones(hid); lw.eps = 0.0
    for r in range(w.n_requests):
        base = O.run_request(w, r)                               # selection from w.q, as the layer loop takes it
        got = O.recompute_layers(w, r, base.selected, [lw])[0]
        hd = w.hidden
        ref = O.run_request(w, r, selected_override=base.selected, q=hd[:, : hq * d].reshape(-1, hq, d),
                            k_new=hd[:, hq * d: (hq + hkv) * d].reshape(-1, hkv, d),
                            v_new=hd[:, (hq + hkv) * d:].reshape(-1, hkv, d))
        assert np.allclose(got["out"], ref.out, rtol=1e-10, atol=1e-12) and np.allclose(got["lse"], ref.lse, rtol=1e-10)


def test_recompute_layers_chain_and_pass_through():
    w = _tiny_projected(hidden=48)
    ws = [W.layer_weights(w.spec, 48, 96, layer=l) for l in range(3)]
    sel = O.run_request(w, 0).selected
    ls = O.recompute_layers(w, 0, sel, ws)
    q_pos, q_row = O.query_list(w, 0, sel)
    assert np.array_equal(ls[0]["h_in"], w.hidden[q_row].astype(np.float64))
    assert all(np.array_equal(ls[l + 1]["h_in"], ls[l]["h2"]) for l in range(2))          # the state is handed on
    assert not np.allclose(ls[0]["out"], ls[1]["out"])                                     # and the layers differ
    # each layer, fed its input alone, gives the same result (no hidden carry-over besides h)
    again = O.recompute_layers(w, 0, sel, [ws[2]], h_in=[ls[2]["h_in"]])[0]
    assert np.array_equal(again["h2"], ls[2]["h2"])
    # with no output and no down projection the hidden state passes every layer unchanged
    for lw in ws:
        lw.w_o = np.zeros_like(lw.w_o); lw.w_down = np.zeros_like(lw.w_down)
    ls = O.recompute_layers(w, 0, sel, ws)
    assert np.array_equal(ls[2]["h2"], w.hidden[q_row].astype(np.float64))


def test_recompute_layers_early_termination_matches_the_attention_only_loop():
    """With an identity projection and no output / down projection the hidden state never changes, so
    every layer is the same attention: the windowed recompute must then stop, drop rows and report
    masses exactly as layer_loop (pinned above) does on the hidden state's slices."""
    import copy
    w = _tiny_projected()
    hq, hkv, d = w.spec.n_q_heads, w.spec.n_kv_heads, w.spec.head_dim
    hid = w.hidden.shape[1]
    w.hidden = (w.hidden / np.sqrt(np.mean(w.hidden.astype(np.float64) ** 2, axis=1, keepdims=True))).astype(np.float64)
    lw = W.layer_weights(w.spec, hid, 96)
    lw.w_qkv = np.eye(hid); lw.gain_attn = np.ones(hid); lw.eps = 0.0
    lw.w_o = np.zeros_like(lw.w_o); lw.w_down = np.zeros_like(lw.w_down)
    w2 = copy.copy(w)
    w2.q = w.hidden[:, : hq * d].reshape(-1, hq, d)
    w2.k_new = w.hidden[:, hq * d: (hq + hkv) * d].reshape(-1, hkv, d)
    w2.v_new = w.hidden[:, (hq + hkv) * d:].reshape(-1, hkv, d)
    for r in range(w.n_requests):
        ref = O.layer_loop(w2, r, 4, 2, [1.0] * 4)
        got = O.recompute_layers(w, r, ref[0]["selected"], [lw] * 4, window=2)
        assert ref[1]["stop_layer"] == 2, "identical layers settle at the window"
        for a, b in zip(got, ref):
            assert a["stop_layer"] == b["stop_layer"] and a["focused"] == b["focused"]
            assert np.array_equal(a["q_pos"], b["q_pos"])
            assert np.allclose(a["mass"], b["mass"], rtol=1e-10, atol=1e-13)
            assert np.allclose(a["out"], b["out"], rtol=1e-10, atol=1e-12)
        # rows were really dropped where a chunk lost its focus, and the survivors kept their state
        n0, n3 = len(got[0]["q_pos"]), len(got[3]["q_pos"])
        n_chunks = len(ref[0]["selected"])
        if len(got[3]["focused"]) < n_chunks and any(len(s) for c, s in enumerate(ref[0]["selected"]) if c not in got[3]["focused"]):
            assert n3 < n0
        assert np.array_equal(got[3]["h_in"], w.hidden[O.query_list(w, r, got[3]["selected"])[1]])
