"""ist_forward_full_static (the entry point for callers that cannot allocate: its intermediate values live
in a static device array inside the library) against ist_forward_full, through the C ABI: bit-identical
logits, on two calls in a row of which the second has the smaller input (the array keeps what the first
call left), with ragged widths (row padding that must read as zero), both storage types, dense and sparse
inputs, with and without the standardisation; and its size limit is an error, not a fault."""
import numpy as np
import pytest
import torch

import ist_harness as H
from test_gpu_parity import SHAPES, _mk

pytestmark = pytest.mark.gpu


def _both(name, normalize, B=None):
    cfg = SHAPES[name]
    B = cfg.B if B is None else B
    P = H.Problem(cfg, dev="cuda:0", normalize=normalize)
    bound = P.context()                                   # reference: workspace bound by the caller
    from paper_1910_02120_amd import ISTContext
    free = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, P.has_bias, max_B=cfg.B, bind=False,
                      normalize=normalize)                # nothing bound at all
    want = bound.forward_full(P.dW, P.db, B, X=P.dX, csr=P.dcsr)
    out = torch.full((B, cfg.dims[-1]), float("nan"), dtype=torch.float32, device="cuda:0")
    got = free.forward_full(P.dW, P.db, B, X=P.dX, csr=P.dcsr, logits=out, static=True)
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.equal(got, want), (name, normalize, B, float((got - want).abs().max()))
    assert torch.isfinite(got).all()
    bound.close()
    free.close()
    return P, got


@pytest.mark.parametrize("big,small", [("speech-small", "ragged-f32"), ("cfg4-small", "ragged-bf16"),
                                       ("cfg5-small", "csr-bf16-odd"), ("wide-out-f32", "width-one-blocks-f32")])
@pytest.mark.parametrize("normalize", [False, True], ids=["plain", "standardised"])
def test_static_forward_equals_the_bound_one_twice_in_a_row(big, small, normalize):
    _both(big, normalize)
    P, got = _both(small, normalize)          # smaller network, smaller batch, ragged rows
    _both(small, normalize, B=max(2, SHAPES[small].B // 2))   # and the same network on a shorter batch
    # the oracle agrees as well (the bound call's own parity test covers more shapes)
    from oracle import ist_oracle as orc
    cfg = P.cfg
    if cfg.input == "csr":
        rp, ci, va = orc.csr_slice(P.rp, P.ci, P.va, 0, cfg.B)
        want = orc.forward_full(P.Ws, P.bs, cfg.dtype, csr=(rp, ci, va.astype(np.float64)), normalize=normalize)
    else:
        want = orc.forward_full(P.Ws, P.bs, cfg.dtype, X=P.X.reshape(-1, cfg.dims[0])[:cfg.B], normalize=normalize)
    err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - want))) / float(np.max(np.abs(want)))
    assert err <= H.TOL[cfg.dtype], (small, err)


def test_static_forward_rejects_what_does_not_fit():
    from paper_1910_02120_amd import ISTContext, ISTError
    cfg = _mk("too-wide", "cfg2", dims=(16, 131072, 8), S=4, B=128, k=1)     # 128 x 131072 x 4 bytes = 64 MiB
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B, bind=False)
    W = [torch.zeros((cfg.dims[l], cfg.dims[l - 1]), device="cuda:0") for l in (1, 2)]
    b = [torch.zeros(cfg.dims[l], device="cuda:0") for l in (1, 2)]
    X = torch.zeros((cfg.B, cfg.dims[0]), device="cuda:0")
    out = torch.zeros((cfg.B, cfg.dims[-1]), device="cuda:0")
    with pytest.raises(ISTError) as e:
        ctx.forward_full(W, b, cfg.B, X=X, logits=out, static=True)
    assert e.value.status == -4 and "static scratch" in str(e.value)
    small = ctx.forward_full(W, b, 8, X=X, logits=out[:8], static=True)    # 8 rows of the same network do fit
    torch.cuda.synchronize()
    assert torch.equal(small, torch.zeros_like(small))
    with pytest.raises(ISTError) as e:                                      # the bound entry point still asks for ist_bind
        ctx.forward_full(W, b, 8, X=X, logits=out[:8])
    assert e.value.status == -6
    ctx.close()
