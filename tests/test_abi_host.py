"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/cc.h declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2502_15734_amd as P
    if not os.path.exists(P.library_path()):
        from paper_2502_15734_amd import build
        build.build(verbose=False)
    return P.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"cc_rope_shift", "cc_rope_place", "cc_scatter_kv", "cc_select", "cc_select_from_scores", "cc_sparse_prefill", "cc_gather_rows",
            "cc_qkv_project", "cc_create", "cc_destroy", "cc_question_mass", "cc_question_mass_workspace_bytes",
            "cc_focus_create", "cc_focus_update", "cc_focus_destroy", "cc_focus_layer", "cc_chunk_attention",
            "cc_chunk_attention_workspace_bytes", "cc_chunk_ab", "cc_chunk_cci", "cc_chunk_reuse", "cc_preload_depth",
            "cc_preloader_create", "cc_preloader_set_layer", "cc_preloader_acquire", "cc_preloader_release",
            "cc_preloader_issued", "cc_preloader_destroy", "cc_sparse_prefill_mass", "cc_sparse_prefill_pairs",
            "cc_sparse_prefill_pairs_workspace_bytes", "cc_rms_norm", "cc_linear", "cc_gated_linear",
            "cc_sparse_prefill_static", "cc_check_query_list", "cc_check_query_list_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in cc.h but not exported"


def test_status_strings(lib):
    assert lib.cc_status_string(0) == b"ok"
    for s in (-1, -2, -3, -4):
        assert len(lib.cc_status_string(s)) > 0


def test_create_validates_config():
    import paper_2502_15734_amd as P
    P.Context(32, 8, 128, 5.0e5, P.CC_BF16).close()
    P.Context(4, 2, 64, 1.0e4, P.CC_F32).close()
    for args, status in (((32, 8, 96, 5.0e5, P.CC_BF16), -2), ((32, 5, 128, 5.0e5, P.CC_BF16), -1),
                         ((32, 8, 128, -1.0, P.CC_BF16), -1), ((32, 8, 128, 5.0e5, 7), -2),
                         ((0, 8, 128, 5.0e5, P.CC_BF16), -1)):
        with pytest.raises(P.CacheCraftError) as e:
            P.Context(*args)
        assert e.value.status == status
    with pytest.raises(P.CacheCraftError):
        P.Context(32, 8, 128, 5.0e5, P.CC_BF16, block_size=32)


def test_calls_reject_bad_arguments_before_launch(lib):
    import paper_2502_15734_amd as P
    ctx = P.Context(8, 2, 128, 5.0e5, P.CC_BF16)
    h = ctx._h
    good = C.c_void_p(4096)          # a well-aligned non-null address; never dereferenced on these paths
    odd = C.c_void_p(4100)
    # cc_rope_shift: null pool, misaligned pool, V given on one side only, negative count
    assert lib.cc_rope_shift(h, None, None, 4, good, None, 4, good, good, good, 1, 16, None, None) == -1
    assert b"null" in lib.cc_last_error(h)
    assert lib.cc_rope_shift(h, odd, None, 4, good, None, 4, good, good, good, 1, 16, None, None) == -1
    assert lib.cc_rope_shift(h, good, good, 4, good, None, 4, good, good, good, 1, 16, None, None) == -1
    assert lib.cc_rope_shift(h, good, None, 4, good, None, 4, good, good, good, -1, 16, None, None) == -1
    assert lib.cc_rope_shift(h, good, None, 4, good, None, 4, good, good, good, 0, 16, None, None) == 0   # empty batch
    # a value map together with V pools (values are either copied or mapped, not both)
    assert lib.cc_rope_shift(h, good, good, 4, good, good, 4, good, good, good, 1, 16, good, None) == -1
    assert b"value map" in lib.cc_last_error(h)
    assert lib.cc_rope_place(h, None, None, 4, good, None, 4, good, good, good, 1, 16, None, None) == -1
    assert lib.cc_rope_place(h, good, None, 4, good, None, 4, good, good, good, 0, 16, None, None) == 0
    # cc_select: workspace too small / missing
    need = lib.cc_select_workspace_bytes(h, 100, 3)
    assert need >= 100 * 8 * 4
    assert lib.cc_select(h, good, 100, good, 8, good, good, 3, good, 1, 64, good, None, None, None, 10,
                         None, good, need - 1, None) == -3
    assert lib.cc_select(h, good, 100, good, 8, good, good, 3, good, 1, 64, good, None, None, None, 10,
                         None, None, need, None) == -1
    assert lib.cc_select(h, None, 100, good, 8, good, good, 3, good, 1, 64, good, None, None, None, 10,
                         None, good, need, None) == -1
    # cc_select_from_scores: null scores, workspace too small, empty segment list
    ws_sel = lib.cc_select_workspace_bytes(h, 100, 3)
    assert lib.cc_select_from_scores(h, None, 100, good, good, 3, good, None, None, None, 10, good, ws_sel, None) == -1
    assert lib.cc_select_from_scores(h, good, 100, good, good, 3, good, None, None, None, 10, good, 16, None) == -3
    assert lib.cc_select_from_scores(h, good, 100, good, good, 0, good, None, None, None, 10, good, ws_sel, None) == 0
    # cc_gather_rows: row size not a multiple of 16
    assert lib.cc_gather_rows(h, good, 10, good, 4, 24, good, None) == -1
    # cc_qkv_project: hidden not a multiple of 64
    assert lib.cc_qkv_project(h, good, good, 4, 100, good, good, good, None) == -1
    # cc_sparse_prefill: null output, max_q_per_req > n_q_tot, empty query list
    ws = lib.cc_sparse_prefill_workspace_bytes(h, 100, 3)
    args = [h, good, good, good, None, good, good, good, 10, 10, good, good, 8, good, good, 3, good, 1, 100, None]
    assert lib.cc_sparse_prefill(*args, None, None, good, ws, None) == -1
    args[9] = 11
    assert lib.cc_sparse_prefill(*args, good, None, good, ws, None) == -1
    args[8], args[9] = 0, 0
    assert lib.cc_sparse_prefill(*args, good, None, good, ws, None) == 0
    # shared values without a map, or with an empty pool
    from paper_2502_15734_amd.binding import SharedValues
    args[8], args[9] = 10, 10
    for bad in (SharedValues(4096, 8, None), SharedValues(None, 8, 4096), SharedValues(4096, 0, 4096), SharedValues(4100, 8, 4096)):
        args[19] = C.byref(bad)
        assert lib.cc_sparse_prefill(*args, good, None, good, ws, None) == -1 and b"shared values" in lib.cc_last_error(h)
    args[19] = None
    # rows of the compact list beyond n_ctx_tokens (the redo flags in the workspace are sized by it)
    few = [h, good, good, good, None, good, good, good, 10, 10, good, good, 8, good, good, 3, good, 1, 9, None]
    assert lib.cc_sparse_prefill(*few, good, None, good, ws, None) == -1 and b"n_ctx_tokens" in lib.cc_last_error(h)
    # cc_sparse_prefill_static: a plan larger than the built-in scratch is refused before anything else happens;
    # an empty query list is fine
    assert lib.cc_sparse_prefill_static(h, good, good, good, None, good, good, good, 10, 10, good, good, 8, good, good,
                                        3, good, 1, 4_000_000, None, good, None, None) == -3
    assert b"scratch" in lib.cc_last_error(h)
    assert lib.cc_sparse_prefill_static(h, good, good, good, None, good, good, good, 0, 0, good, good, 8, good, good,
                                        3, good, 1, 100, None, good, None, None) == 0
    # grid limits: more than 65535 requests (cc_sparse_prefill) or segments (cc_select) in one call are refused
    big = [h, good, good, good, None, good, good, good, 70000, 10, good, good, 8, good, good, 70000, good, 70000, 70000, None]
    wsb = lib.cc_sparse_prefill_workspace_bytes(h, 70000, 70000)
    assert lib.cc_sparse_prefill(*big, good, None, good, wsb, None) == -1 and b"65535" in lib.cc_last_error(h)
    need_big = lib.cc_select_workspace_bytes(h, 70000, 70000)
    assert lib.cc_select(h, good, 70000, good, 8, good, good, 70000, good, 1, 64, good, None, None, None, 10,
                         None, good, need_big, None) == -1 and b"65535" in lib.cc_last_error(h)
    # cc_check_query_list: missing result, tiny workspace
    wq = lib.cc_check_query_list_workspace_bytes(h, 100)
    assert wq >= 400
    assert lib.cc_check_query_list(h, good, 10, 100, None, good, wq, None) == -1
    assert lib.cc_check_query_list(h, good, 10, 100, good, good, wq - 1, None) == -3
    assert lib.cc_check_query_list(h, good, 10, 0, good, good, wq, None) == -1
    # cc_scatter_kv: null pool, misaligned rows, nothing to do
    assert lib.cc_scatter_kv(h, good, good, good, good, 4, None, good, 8, None) == -1
    assert lib.cc_scatter_kv(h, odd, good, good, good, 4, good, good, 8, None) == -1
    assert lib.cc_scatter_kv(h, good, good, good, good, 0, good, good, 8, None) == 0
    # cc_question_mass: missing lse, workspace too small, max_question_rows > n_q_tot, no segments
    wm = lib.cc_question_mass_workspace_bytes(h, 100, 3, 8)
    assert wm >= 3 * 8 * 8 * 4
    qm = [h, good, good, good, 10, 8, good, good, 8, good, good, 3, good, 1, 100]
    assert lib.cc_question_mass(*qm, None, good, good, wm, None) == -1
    assert lib.cc_question_mass(*qm, good, good, good, wm - 1, None) == -3
    assert lib.cc_question_mass(*qm, good, None, good, wm, None) == -1
    qm[5] = 11
    assert lib.cc_question_mass(*qm, good, good, good, wm, None) == -1
    qm[5], qm[11] = 8, 0
    assert lib.cc_question_mass(*qm, good, good, good, wm, None) == 0
    # cc_chunk_attention: n_pairs below the segment count, missing lse, self_mass without slot_map, tiny workspace
    wc = lib.cc_chunk_attention_workspace_bytes(h, 100, 3, 10, 10)
    ca = [h, good, good, good, good, 10, 10, good, good, 8, good, good, 3, good, 1, 100]
    assert lib.cc_chunk_attention(*ca, 2, good, good, good, good, wc, None) == -1
    assert lib.cc_chunk_attention(*ca, 6, None, good, good, good, wc, None) == -1
    ca[3] = None
    assert lib.cc_chunk_attention(*ca, 6, good, good, good, good, wc, None) == -1
    ca[3] = good
    assert lib.cc_chunk_attention(*ca, 6, good, good, good, good, wc - 1, None) == -3
    assert lib.cc_chunk_attention(*ca, 0, good, good, good, good, wc, None) == 0
    # cc_sparse_prefill_pairs: missing pair_mass, missing lse, too few pairs, tiny workspace, no segments
    wp = lib.cc_sparse_prefill_pairs_workspace_bytes(h, 100, 3, 10, 10, 3)
    assert wp >= 10 * 8 * 3 * 4
    pa = [h, good, good, good, None, good, good, good, 10, 10, good, good, 8, good, good, 3, good, 1, 3, 100]
    assert lib.cc_sparse_prefill_pairs(*pa, 6, None, good, good, good, None, good, good, wp, None) == -1
    assert lib.cc_sparse_prefill_pairs(*pa, 6, None, good, None, good, good, good, good, wp, None) == -1
    assert lib.cc_sparse_prefill_pairs(*pa, 2, None, good, good, good, good, good, good, wp, None) == -1
    assert lib.cc_sparse_prefill_pairs(*pa, 6, None, good, good, None, good, good, good, wp - 1, None) == -3
    pa[15] = 0
    assert lib.cc_sparse_prefill_pairs(*pa, 6, None, good, good, good, good, good, good, wp, None) == 0
    other = C.c_void_p(8192)
    # the dense operators of the layer: null tensors, x == y, hidden off the 16-byte grid, negative eps, no rows
    assert lib.cc_rms_norm(h, good, None, 1e-5, 4, 64, good, None) == -1
    assert lib.cc_rms_norm(h, good, good, 1e-5, 4, 63, good, None) == -1
    assert lib.cc_rms_norm(h, good, good, -1.0, 4, 64, good, None) == -1
    assert lib.cc_rms_norm(h, good, good, 1e-5, 0, 64, good, None) == 0
    assert lib.cc_linear(h, good, good, None, 4, 64, 64, good, None) == -1
    assert lib.cc_linear(h, good, None, None, 4, 64, 64, other, None) == -1
    assert lib.cc_linear(h, good, good, odd, 4, 64, 64, other, None) == -1
    assert lib.cc_linear(h, good, good, None, 0, 64, 64, other, None) == 0
    assert lib.cc_gated_linear(h, good, good, None, 4, 64, 64, other, None) == -1
    assert lib.cc_gated_linear(h, good, good, good, 4, 0, 64, other, None) == -1
    assert lib.cc_gated_linear(h, good, good, good, 0, 64, 64, other, None) == 0
    # null context
    assert lib.cc_rope_shift(None, good, None, 4, good, None, 4, good, good, good, 1, 16, None, None) == -1
    assert lib.cc_set_impl(h, 99) == -1
    for impl in (P.CC_IMPL_MFMA_NARROW, P.CC_IMPL_MFMA_WIDE, P.CC_IMPL_SCALAR, P.CC_IMPL_AUTO):
        assert lib.cc_set_impl(h, impl) == 0
    ctx.close()


def test_focus_tracker_follows_algorithm_1():
    """The library's host-side Algorithm 1 against the oracle's, layer by layer, on seeded score
    sequences that drift and then settle (so both the changing sets and the stop rule are hit)."""
    import numpy as np
    import paper_2502_15734_amd as P
    from oracle import cachecraft_oracle as O
    rng = np.random.default_rng(2025)
    stops = 0
    for case in range(60):
        k = int(rng.integers(1, 9))
        window = int(rng.integers(1, 4))
        n_layers = int(rng.integers(1, 12))
        base = rng.random(k) * (rng.random(k) < 0.6)
        layers = [np.float32(base * (1.0 if l >= 3 else 0.0) + rng.random(k) * (0.5 if l < 3 else 0.01))
                  for l in range(n_layers)]
        f_star, l_star, f_all = O.predict_focused([[float(v) for v in x] for x in layers], window)
        tr = P.FocusTracker(k, window)
        for l, x in enumerate(layers, start=1):
            stop, focused = tr.update(x)
            assert focused == f_all[l - 1], f"case {case} layer {l}"
            assert tr.layer == l
            if stop:
                assert (focused, l) == (f_star, l_star)
                stops += 1
                break
        else:
            assert f_star is None
        tr.close()
    assert stops >= 10
    # hand-worked layer (gaps 1, 7, 1, 0.5 -> the two top chunks) and argument checks
    tr = P.FocusTracker(5, 1)
    assert tr.update([2.0, 10.0, 0.5, 9.0, 1.0]) == (True, [1, 3])
    with pytest.raises(P.CacheCraftError):
        tr.update([float("nan")] * 5)
    with pytest.raises(P.CacheCraftError):
        P.FocusTracker(0, 1)
    with pytest.raises(P.CacheCraftError):
        P.FocusTracker(3, 0)


def test_reuse_scores_follow_the_oracle():
    """cc_chunk_ab / cc_chunk_cci / cc_chunk_reuse (host code of the library) against the oracle's
    formulas on seeded inputs, plus the argument checks."""
    import numpy as np
    import paper_2502_15734_amd as P
    from oracle import cachecraft_oracle as O
    rng = np.random.default_rng(77)
    for case in range(200):
        n_old, n_new = int(rng.integers(0, 8)), int(rng.integers(0, 8))
        old = [int(v) for v in rng.choice(10, size=n_old, replace=False)]
        new = [int(v) for v in rng.choice(10, size=n_new, replace=False)]
        inter = [float(v) for v in rng.random(n_old) * (rng.random(n_old) < 0.8)]
        lens = [int(v) for v in rng.integers(1, 2000, size=n_old)]
        clen = int(rng.integers(1, 1025))
        intra = float(rng.random() * clen)
        a, b = P.chunk_ab(inter, lens, intra, clen)
        ao, bo = O.chunk_ab(inter, lens, intra, clen)
        assert abs(a - ao) <= 1e-15 + 1e-12 * abs(ao) and abs(b - bo) <= 1e-15 + 1e-12 * abs(bo)
        layers_a = [a * float(v) for v in rng.random(3)]; layers_b = [b * float(v) for v in rng.random(3)]
        c = P.chunk_cci(layers_a, layers_b)
        assert abs(c - O.cci(layers_a, layers_b)) < 1e-12
        alpha = float(rng.choice([0.5, 1.0, 2.0]))
        got = P.chunk_reuse(old, inter, new, c, alpha, clen)
        beta, gamma = O.prefix_overlap(old, inter, new), O.order_penalty(old, new)
        beta_adj, cfo, n = O.cache_fix_overhead(c, beta, gamma, alpha, clen)
        assert abs(got["beta"] - beta) < 1e-12 and abs(got["gamma"] - gamma) < 1e-12
        assert abs(got["beta_adj"] - beta_adj) < 1e-12 and abs(got["cfo"] - cfo) < 1e-12
        assert got["n_recompute"] == n, f"case {case}"
    # the paper's example: same prefix chunks, swapped order -> beta 1, gamma 1
    r = P.chunk_reuse([1, 2], [0.4, 0.6], [2, 1], 0.7, 1.0, 100)
    assert r["beta"] == 1.0 and r["gamma"] == 1.0 and r["n_recompute"] == 70
    with pytest.raises(P.CacheCraftError):
        P.chunk_cci([float("nan")], [1.0])
    with pytest.raises(P.CacheCraftError):
        P.chunk_reuse([1], [-0.5], [1], 0.5, 1.0, 10)
    with pytest.raises(P.CacheCraftError):
        P.chunk_ab([1.0], [0], 1.0, 10)


def test_preload_depth_follows_the_oracle():
    import numpy as np
    import paper_2502_15734_amd as P
    from oracle import cachecraft_oracle as O
    assert P.preload_depth(5, 1.0, 2.0) == 3
    rng = np.random.default_rng(12)
    for _ in range(300):
        L = int(rng.integers(1, 129)); tp = float(rng.uniform(0.0, 4.0)); tl = float(rng.uniform(0.0, 4.0))
        assert P.preload_depth(L, tp, tl) == O.preload_depth(L, tp, tl)
    for bad in ((0, 1.0, 1.0), (4, -1.0, 1.0), (4, 1.0, float("nan"))):
        with pytest.raises(P.CacheCraftError):
            P.preload_depth(*bad)


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_15734_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr + res.stdout
