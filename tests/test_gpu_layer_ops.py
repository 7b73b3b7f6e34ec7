"""GPU parity of the dense operators around the attention (cc_rms_norm, cc_linear, cc_gated_linear)
against the oracle, through the C ABI: plain and MFMA kernels, ragged row counts, in-place
residuals, and the layer's tail composed from them."""
import math

import numpy as np
import pytest
import torch

import workload as W
from oracle import cachecraft_oracle as O
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _ctx(dtype, impl="auto"):
    import paper_2502_15734_amd as P
    ctx = P.Context(8, 2, 128, 5.0e5, P.CC_BF16 if dtype == "bf16" else P.CC_F32)
    ctx.set_impl({"auto": P.CC_IMPL_AUTO, "scalar": P.CC_IMPL_SCALAR, "narrow": P.CC_IMPL_MFMA_NARROW,
                  "wide": P.CC_IMPL_MFMA_WIDE}[impl])
    return ctx


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()


def _draw(rng, shape, scale, dtype):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return W.round_to_bf16(a) if dtype == "bf16" else a


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype,rows,hidden", [("bf16", 1, 256), ("bf16", 37, 4096), ("bf16", 301, 40),
                                               ("f32", 5, 36), ("f32", 130, 1024), ("bf16", 9, 8192),
                                               ("bf16", 3, 16384), ("f32", 6, 8192)])   # rows kept in registers / read twice
def test_rms_norm(dtype, rows, hidden):
    rng = np.random.default_rng(rows + hidden)
    x = _draw(rng, (rows, hidden), 1.5, dtype)
    x[0] *= 1e-3                                                      # a row whose mean square is close to eps
    g = _draw(rng, (hidden,), 0.1, dtype) + np.float32(1.0)
    g = W.round_to_bf16(g) if dtype == "bf16" else g
    ctx = _ctx(dtype)
    xd, gd = _dev(x, dtype), _dev(g, dtype)
    yd = torch.full_like(xd, float("nan"))
    ctx.rms_norm(xd, gd, 1e-5, yd); torch.cuda.synchronize()
    want = O.rms_norm(x, g, 1e-5)
    assert H.rel_l2(_host(yd), want) <= H.TOL[dtype]
    assert np.abs(_host(yd) - want).max() <= (2e-2 if dtype == "bf16" else 1e-5) * max(1.0, np.abs(want).max())
    ctx.rms_norm(xd, gd, 1e-5, xd); torch.cuda.synchronize()         # in place
    assert torch.equal(xd, yd)
    ctx.close()


LINEAR_CASES = [("f32", "auto", 37, 40, 50), ("f32", "auto", 130, 64, 256), ("bf16", "auto", 300, 256, 512),
                ("bf16", "auto", 256, 96, 256), ("bf16", "auto", 41, 72, 40), ("bf16", "scalar", 70, 256, 256),
                ("bf16", "narrow", 70, 256, 256), ("bf16", "wide", 513, 1024, 768),
                ("bf16", "auto", 1, 64, 256), ("bf16", "auto", 257, 128, 256),      # one and two 64-wide stages
                ("bf16", "auto", 2300, 192, 1280)]                                  # tile blocks with ragged edges


@pytest.mark.parametrize("dtype,impl,rows,n_in,n_out", LINEAR_CASES)
def test_linear_with_and_without_residual(dtype, impl, rows, n_in, n_out):
    rng = np.random.default_rng(rows * 7 + n_in)
    x = _draw(rng, (rows, n_in), 1.0, dtype)
    w = _draw(rng, (n_out, n_in), 1.0 / math.sqrt(n_in), dtype)
    res = _draw(rng, (rows, n_out), 1.0, dtype)
    ctx = _ctx(dtype, impl)
    xd, wd, rd = _dev(x, dtype), _dev(w, dtype), _dev(res, dtype)
    yd = torch.full((rows, n_out), float("nan"), dtype=xd.dtype, device="cuda")
    ctx.linear(xd, wd, yd); torch.cuda.synchronize()
    assert H.rel_l2(_host(yd), O.linear(x, w)) <= H.TOL[dtype]
    ctx.linear(xd, wd, yd, residual=rd); torch.cuda.synchronize()
    want = res.astype(np.float64) + O.linear(x, w)
    assert H.rel_l2(_host(yd), want) <= H.TOL[dtype]
    first = yd.clone()
    ctx.linear(xd, wd, rd, residual=rd); torch.cuda.synchronize()     # accumulate into the residual itself
    assert torch.equal(rd, first)
    ctx.close()


GATED_CASES = [("f32", "auto", 37, 40, 50), ("bf16", "auto", 300, 256, 384), ("bf16", "auto", 41, 72, 40),
               ("bf16", "scalar", 70, 256, 128), ("bf16", "wide", 513, 512, 640), ("bf16", "auto", 5, 64, 128)]


@pytest.mark.parametrize("dtype,impl,rows,n_in,n_ffn", GATED_CASES)
def test_gated_linear(dtype, impl, rows, n_in, n_ffn):
    rng = np.random.default_rng(rows * 11 + n_ffn)
    x = _draw(rng, (rows, n_in), 1.0, dtype)
    wg = _draw(rng, (n_ffn, n_in), 2.0 / math.sqrt(n_in), dtype)      # gates on both sides of the SiLU's bend
    wu = _draw(rng, (n_ffn, n_in), 1.0 / math.sqrt(n_in), dtype)
    ctx = _ctx(dtype, impl)
    yd = torch.full((rows, n_ffn), float("nan"), dtype=_dev(x, dtype).dtype, device="cuda")
    ctx.gated_linear(_dev(x, dtype), _dev(wg, dtype), _dev(wu, dtype), yd); torch.cuda.synchronize()
    want = O.gated_ffn_in(x, wg, wu)
    assert H.rel_l2(_host(yd), want) <= H.TOL[dtype]
    assert np.abs(_host(yd) - want).max() <= (3e-2 if dtype == "bf16" else 1e-5) * max(1.0, np.abs(want).max())
    ctx.close()


def _tail_on_gpu(ctx, lw, h, o, dtype):
    hd, od = _dev(h, dtype), _dev(o.reshape(o.shape[0], -1), dtype)
    h1 = torch.empty_like(hd); y = torch.empty_like(hd); h2 = torch.empty_like(hd)
    act = torch.empty((h.shape[0], lw.w_gate.shape[0]), dtype=hd.dtype, device="cuda")
    ctx.linear(od, _dev(lw.w_o, dtype), h1, residual=hd)
    ctx.rms_norm(h1, _dev(lw.gain_ffn, dtype), lw.eps, y)
    ctx.gated_linear(y, _dev(lw.w_gate, dtype), _dev(lw.w_up, dtype), act)
    ctx.linear(act, _dev(lw.w_down, dtype), h2, residual=h1)
    torch.cuda.synchronize()
    return _host(h1), _host(h2)


@pytest.mark.parametrize("dtype,rows,hidden,ffn", [("f32", 45, 64, 160), ("bf16", 333, 256, 640)])
def test_layer_tail_composed_from_the_calls(dtype, rows, hidden, ffn):
    spec = W.config_spec(2)
    spec.dtype = dtype
    lw = W.layer_weights(spec, hidden, ffn)
    rng = np.random.default_rng(rows)
    h = _draw(rng, (rows, hidden), 1.0, dtype)
    o = _draw(rng, (rows, spec.n_q_heads, spec.head_dim), 0.5, dtype)
    ctx = _ctx(dtype)
    h1, h2 = _tail_on_gpu(ctx, lw, h, o, dtype)
    w1, w2 = O.layer_tail(h, o, lw.w_o, lw.gain_ffn, lw.w_gate, lw.w_up, lw.w_down, lw.eps)
    assert H.rel_l2(h1, w1) <= H.TOL[dtype] and H.rel_l2(h2, w2) <= H.TOL[dtype]
    ctx.close()


def test_layer_tail_at_the_8b_model_shape_on_sampled_rows():
    """hidden 4096, feed-forward 14336, 32 heads of 128: the MFMA kernels on several full tiles and a
    ragged one; the oracle follows on sampled rows (a row depends on no other row)."""
    spec = W.config_spec(3)
    hidden, ffn, rows = 4096, 14336, 1000
    lw = W.layer_weights(spec, hidden, ffn)
    rng = np.random.default_rng(3)
    h = _draw(rng, (rows, hidden), 1.0, "bf16")
    o = _draw(rng, (rows, spec.n_q_heads, spec.head_dim), 0.5, "bf16")
    ctx = _ctx("bf16")
    h1, h2 = _tail_on_gpu(ctx, lw, h, o, "bf16")
    which = np.array([0, 127, 128, 255, 256, 511, 777, 999])
    w1, w2 = O.layer_tail(h[which], o[which], lw.w_o, lw.gain_ffn, lw.w_gate, lw.w_up, lw.w_down, lw.eps)
    assert H.rel_l2(h1[which], w1) <= 1e-2 and H.rel_l2(h2[which], w2) <= 1e-2
    assert np.isfinite(h2).all()
    ctx.close()
