"""The loop over layers (preloaded store -> shift -> select from a score list -> recompute + attend ->
question-to-chunk mass -> Algorithm 1 -> budgets) against the oracle's loop, layer by layer."""
import math

import numpy as np
import pytest
import torch

import workload as W
from oracle import cachecraft_oracle as O
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("preload", [True, False])
def test_layer_loop_matches_the_oracle(preload):
    from paper_2502_15734_amd.layers import LayerLoop
    reqs = [W.RequestSpec([0, 1, 2, 3], [0.3, 0.2, 0.25, 0.4], 21), W.RequestSpec([3, 0, 4], [0.5, 0.15, 0.35], 40)]
    w = W.custom("layers", "bf16", 8, 2, 128, 5.0e5, [100, 77, 130, 64, 201], [0, 5, 0, 17, 3], reqs, 0.35, seed=41)
    n_layers, window = 5, 2
    scale = lambda l: 2.0 ** ((l % 3) - 1)
    # the score list both sides select from: the oracle's layer-0 scores, by token row
    scores = np.zeros(w.n_tok, dtype=np.float32)
    for r in range(w.n_requests):
        k_sh, _, _ = O.shifted_context(w, r)
        for sg, sc in zip(H.chunk_segments(w, r), O.score_request(w, r, k_sh)):
            scores[int(sg[W.SEG_TOK]): int(sg[W.SEG_TOK]) + int(sg[W.SEG_NTOK])] = sc
    ref = [O.layer_loop(w, r, n_layers, window, [scale(l) for l in range(n_layers)],
                        scores=[scores[int(sg[W.SEG_TOK]): int(sg[W.SEG_TOK]) + int(sg[W.SEG_NTOK])].astype(np.float64)
                                for sg in H.chunk_segments(w, r)]) for r in range(w.n_requests)]
    # every layer reuses the workload's one set of tensors; to make the layers differ, layer l's
    # queries are the workload's times a power of two (exact in bf16), installed per layer
    q0 = {}

    def layer_inputs(l, b):
        if "q" not in q0:
            q0["q"] = b.q.clone()
        torch.mul(q0["q"], scale(l), out=b.q)

    loop = LayerLoop(w, n_layers, window, layer_inputs=layer_inputs, preload=preload, depth=2)
    recs = loop.run(scores=scores, keep_outputs=True)
    assert any(rec["stop_layer"][0] is not None for rec in recs), "the test should reach a stop"
    for l, rec in enumerate(recs):
        cu = rec["cu_q"]
        for r in range(w.n_requests):
            o = ref[r][l]
            assert rec["stop_layer"][r] == o["stop_layer"] and rec["focused"][r] == o["focused"], f"layer {l + 1} request {r}"
            q0, q1 = int(cu[r]), int(cu[r + 1])
            assert q1 - q0 == len(o["q_pos"]), f"layer {l + 1} request {r}: rows"
            assert H.rel_l2(rec["out"][q0:q1], o["out"]) <= H.TOL["bf16"], f"layer {l + 1} request {r}: out"
            assert np.abs(rec["lse"][q0:q1] - o["lse"]).max() <= 4e-3
            s0, s1 = int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])
            np.testing.assert_allclose(rec["mass"][s0:s1], o["mass"], rtol=1e-2, atol=1e-3)
    assert recs[-1]["rows"] < recs[0]["rows"]                          # unfocused chunks are no longer recomputed
    loop.close()


def _decoder_workload(dtype):
    reqs = [W.RequestSpec([0, 1, 2, 3], [0.3, 0.2, 0.25, 0.4], 21), W.RequestSpec([3, 0, 4], [0.5, 0.15, 0.35], 40)]
    hq, hkv, d = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    return W.custom("decoder", dtype, hq, hkv, d, 5.0e5, [100, 77, 130, 64, 201], [0, 5, 0, 17, 3], reqs,
                    1.0 / math.sqrt(d), seed=43, hidden=256)


@pytest.mark.parametrize("dtype,impl", [("f32", "auto"), ("bf16", "auto"), ("bf16", "scalar")])
def test_decoder_loop_matches_the_oracle(dtype, impl):
    """Hidden states of the chosen rows through three whole layers.  fp32: the oracle runs freely
    beside the library.  bf16: every layer of the oracle starts from the library's own layer input
    (the bar is per layer; bf16 roundings of one layer's output are the next layer's input)."""
    import paper_2502_15734_amd as P
    from paper_2502_15734_amd.layers import DecoderLoop
    w = _decoder_workload(dtype)
    ffn = 640 if dtype == "bf16" else 160
    weights = [W.layer_weights(w.spec, 256, ffn, layer=l, qkv_scale=1.0 / 16) for l in range(3)]
    loop = DecoderLoop(w, weights, impl={"auto": P.CC_IMPL_AUTO, "scalar": P.CC_IMPL_SCALAR}[impl])
    recs = loop.run(keep=True)
    assert len(recs) == 3
    gsel = H.gpu_selection(w, loop.batch.sel_idx.cpu().numpy())
    tol = H.TOL[dtype] if dtype == "bf16" else 2e-5
    for r in range(w.n_requests):
        q0, q1 = int(w.cu_q[r]), int(w.cu_q[r + 1])
        forced = [rec["h_in"][q0:q1] for rec in recs] if dtype == "bf16" else None
        ref = O.recompute_layers(w, r, gsel[r], weights, h_in=forced)
        for l, (rec, o) in enumerate(zip(recs, ref)):
            what = f"request {r} layer {l + 1}"
            assert H.rel_l2(rec["h_in"][q0:q1], o["h_in"]) <= tol, what
            assert H.rel_l2(rec["out"][q0:q1], o["out"]) <= tol, f"{what}: attention {H.rel_l2(rec['out'][q0:q1], o['out']):.3e}"
            assert H.rel_l2(rec["h1"][q0:q1], o["h1"]) <= tol, what
            assert H.rel_l2(rec["h2"][q0:q1], o["h2"]) <= tol, f"{what}: h2 {H.rel_l2(rec['h2'][q0:q1], o['h2']):.3e}"
    # bf16, free-running: the oracle carries its own fp64 state from layer to layer while the library
    # carries bf16 roundings; every layer adds its own rounding (each of its operators is inside
    # the per-layer bar above) to what it inherited, so the gap may grow by about one bar per layer
    if dtype == "bf16":
        for r in range(w.n_requests):
            q0, q1 = int(w.cu_q[r]), int(w.cu_q[r + 1])
            free = O.recompute_layers(w, r, gsel[r], weights)
            for l, (rec, o) in enumerate(zip(recs, free)):
                drift = H.rel_l2(rec["h2"][q0:q1], o["h2"])
                assert drift <= tol * (l + 1), f"request {r} layer {l + 1}: free-running drift {drift:.3e}"
    # the layers do change the state
    assert H.rel_l2(recs[0]["h2"], recs[0]["h_in"]) > 0.1


@pytest.mark.parametrize("dtype,preload", [("f32", False), ("bf16", False), ("bf16", True)])
def test_decoder_loop_with_early_termination(dtype, preload):
    """Whole layers with Algorithm 1 deciding the focused chunks: from the layer after the stop the
    other chunks' rows leave the list and the survivors' hidden states are compacted."""
    from paper_2502_15734_amd.layers import DecoderLoop
    w = _decoder_workload(dtype)
    ffn = 640 if dtype == "bf16" else 160
    weights = [W.layer_weights(w.spec, 256, ffn, layer=l, qkv_scale=1.0 / 16) for l in range(4)]
    loop = DecoderLoop(w, weights, window=2, preload=preload, depth=2)
    recs = loop.run(keep=True)
    assert len(recs) == 4
    tol = H.TOL[dtype] if dtype == "bf16" else 2e-5
    # the rows layer 1 chose (the later lists are subsets of them)
    loop2 = DecoderLoop(w, weights[:1])
    loop2.run()
    gsel = H.gpu_selection(w, loop2.batch.sel_idx.cpu().numpy())
    for r in range(w.n_requests):
        forced = None
        if dtype == "bf16":
            forced = [rec["h_in"][int(rec["cu_q"][r]): int(rec["cu_q"][r + 1])] for rec in recs]
        ref = O.recompute_layers(w, r, gsel[r], weights, h_in=forced, window=2)
        for l, (rec, o) in enumerate(zip(recs, ref)):
            what = f"request {r} layer {l + 1}"
            q0, q1 = int(rec["cu_q"][r]), int(rec["cu_q"][r + 1])
            assert q1 - q0 == len(o["q_pos"]), f"{what}: rows {q1 - q0} vs {len(o['q_pos'])}"
            assert rec["stop_layer"][r] == o["stop_layer"] and rec["focused"][r] == o["focused"], what
            assert H.rel_l2(rec["h_in"][q0:q1], o["h_in"]) <= tol, what
            assert H.rel_l2(rec["out"][q0:q1], o["out"]) <= tol, what
            assert H.rel_l2(rec["h2"][q0:q1], o["h2"]) <= tol, f"{what}: h2 {H.rel_l2(rec['h2'][q0:q1], o['h2']):.3e}"
            s0, s1 = int(w.req_seg_off[r]), int(w.req_seg_off[r + 1])
            np.testing.assert_allclose(rec["mass"][s0:s1], o["mass"], rtol=1e-2 if dtype == "bf16" else 1e-4, atol=1e-3)
    assert recs[-1]["rows"] < recs[0]["rows"]
    loop.close()
