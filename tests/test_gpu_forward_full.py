"""ist_forward_full on the MI355X against the oracle's full-network forward pass: the logits of
the whole (unpartitioned) network on one batch, dense and CSR inputs, both storage types, with
and without the standardisation of Section 2.2; and that the call leaves the workspace fit for
ist_subnet_steps (rows of full width overlay the subnets' padded rows)."""
import numpy as np
import pytest
import torch

import ist_harness as H
from oracle import ist_oracle as orc
from test_gpu_parity import SHAPES

pytestmark = pytest.mark.gpu

CASES = ["cfg1", "ragged-f32", "ragged-bf16", "cfg3-small", "cfg4-small", "cfg5-small", "wide-out-f32",
         "one-hidden-B1-f32", "deep-bf16", "width-one-blocks-f32", "csr-bf16-odd", "csr-f32", "mid-out-bf16",
         "uneven-S5-bf16", "uneven-S7-csr-bf16"]


def _want(P, normalize):
    cfg = P.cfg
    bs = P.bs if P.has_bias else None
    if cfg.input == "csr":
        rp, ci, va = orc.csr_slice(P.rp, P.ci, P.va, 0, cfg.B)
        return orc.forward_full(P.Ws, bs, cfg.dtype, csr=(rp, ci, va.astype(np.float64)), normalize=normalize)
    return orc.forward_full(P.Ws, bs, cfg.dtype, X=P.X.reshape(-1, cfg.dims[0])[:cfg.B], normalize=normalize)


@pytest.mark.parametrize("normalize", [False, True], ids=["plain", "standardised"])
@pytest.mark.parametrize("name", CASES)
def test_full_network_logits_match_oracle(name, normalize):
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev="cuda:0", normalize=normalize)
    ctx = P.context()
    got = ctx.forward_full(P.dW, P.db, cfg.B, X=P.dX, csr=P.dcsr)
    torch.cuda.synchronize()
    want = _want(P, normalize)
    assert got.shape == want.shape
    err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - want))) / float(np.max(np.abs(want)))
    assert err <= H.TOL[cfg.dtype], (name, err)
    ctx.close()


@pytest.mark.parametrize("name", ["ragged-f32", "ragged-bf16", "csr-bf16-odd", "uneven-S5-bf16"])
def test_steps_after_a_full_forward_still_match_oracle(name):
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev="cuda:0")
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    ctx.forward_full(P.dW, P.db, cfg.B, X=P.dX, csr=P.dcsr)
    H.check_training(P, ctx)
    ctx.close()


def test_full_forward_argument_errors():
    from paper_1910_02120_amd import ISTError
    cfg = SHAPES["cfg1"]
    P = H.Problem(cfg, dev="cuda:0")
    ctx = P.context()
    with pytest.raises(ISTError) as e:
        ctx.forward_full(P.dW, P.db, cfg.B + 1, X=torch.zeros((cfg.B + 1) * cfg.dims[0], device="cuda:0"))
    assert e.value.status == -2
    ctx.close()


# ---------------------------------------------------------------- benchmark sizes
import ist_inputs as gen
from test_gpu_full_size import _device_weights

C = gen.CONFIGS


@pytest.mark.parametrize("name", ["cfg2", "cfg3"])
def test_full_size_logits_match_oracle(name):
    cfg = C[name]
    P = H.Problem(cfg, bias_scale=0.02)
    ctx = P.context()
    got = ctx.forward_full(P.dW, P.db, cfg.B, X=P.dX)
    torch.cuda.synchronize()
    want = _want(P, False)
    err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - want))) / float(np.max(np.abs(want)))
    assert err <= H.TOL[cfg.dtype], (name, err)
    ctx.close()


def test_extreme_classification_size_sampled_classes():
    """cfg5 at full size: the oracle evaluates the hidden layer whole and 48 sampled classes."""
    cfg = C["cfg5"]
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(gen.SEED_BASE + cfg.idx)
    rng = np.random.default_rng(55)
    dW, db = _device_weights(cfg, dev, g)
    one = gen.scaled(cfg, k=1, S=1)
    rp, ci, va, _ = gen.make_csr_batches(one)
    dcsr = (torch.from_numpy(rp).to(dev), torch.from_numpy(ci).to(dev), H.to_dev(va, cfg.dtype))
    from paper_1910_02120_amd import ISTContext
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B)
    got = ctx.forward_full(dW, db, cfg.B, csr=dcsr)
    torch.cuda.synchronize()
    pick = np.sort(rng.choice(cfg.dims[2], size=48, replace=False))
    tp = torch.from_numpy(pick.astype(np.int64)).to(dev)
    Ws = [H.to_f32(dW[0]).astype(np.float64), H.to_f32(dW[1].index_select(0, tp)).astype(np.float64)]
    bs = [H.to_f32(db[0]).astype(np.float64), H.to_f32(db[1].index_select(0, tp)).astype(np.float64)]
    r, c, v = orc.csr_slice(rp, ci, va, 0, cfg.B)
    want = orc.forward_full(Ws, bs, cfg.dtype, csr=(r, c, v.astype(np.float64)))
    sub = got.index_select(1, tp).cpu().numpy().astype(np.float64)
    err = float(np.max(np.abs(sub - want))) / float(np.max(np.abs(want)))
    assert err <= H.TOL[cfg.dtype], err
    ctx.close()


def test_wide_stress_size_against_library_matmul():
    """cfg4 at full size is out of the oracle's reach (three 65536-wide layers): a cross-check, not
    parity - the same layers with torch's matmul in float32 on the device, rounded where the path
    rounds."""
    cfg = C["cfg4"]
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(gen.SEED_BASE + cfg.idx)
    dW, db = _device_weights(cfg, dev, g)
    one = gen.scaled(cfg, k=1, S=1)
    X, _ = gen.make_dense_batches(one)
    dX = H.to_dev(X, cfg.dtype)
    from paper_1910_02120_amd import ISTContext
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B)
    got = ctx.forward_full(dW, db, cfg.B, X=dX)
    torch.cuda.synchronize()
    h = dX.reshape(-1, cfg.dims[0])[:cfg.B].float()
    for l in range(cfg.t):
        z = torch.empty((cfg.B, cfg.dims[l + 1]), dtype=torch.float32, device=dev)
        for r0 in range(0, cfg.dims[l + 1], 8192):
            r1 = min(cfg.dims[l + 1], r0 + 8192)
            z[:, r0:r1] = h @ dW[l][r0:r1].float().T + db[l][r0:r1].float()
        h = z if l == cfg.t - 1 else torch.relu(z).to(H.td(cfg.dtype)).float()
    err = float((got - h).abs().max()) / float(h.abs().max())
    assert err <= H.TOL[cfg.dtype], err
    ctx.close()


@pytest.mark.parametrize("name", ["cfg1", "ragged-bf16", "csr-f32"])
def test_round_then_full_forward_matches_oracle_end_to_end(name):
    """partition -> k local steps -> merge on the GPU, then the logits of the merged network, against the
    oracle's round followed by its full forward pass: every entry point of a round in one chain."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev="cuda:0")
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    P.gpu_steps(ctx, loss=False)
    ctx.merge(P.dW, P.db)
    got = ctx.forward_full(P.dW, P.db, cfg.B, X=P.dX, csr=P.dcsr)
    torch.cuda.synchronize()
    Ws = [w.copy() for w in P.Ws]
    bs = [b.copy() for b in P.bs]
    if cfg.input == "csr":
        orc.ist_round(Ws, bs, P.perms, cfg.S, cfg.lr, cfg.k, cfg.dtype, P.y,
                      csr=(P.rp, P.ci, P.va.astype(np.float64)))
        rp, ci, va = orc.csr_slice(P.rp, P.ci, P.va, 0, cfg.B)
        want = orc.forward_full(Ws, bs, cfg.dtype, csr=(rp, ci, va.astype(np.float64)))
    else:
        orc.ist_round(Ws, bs, P.perms, cfg.S, cfg.lr, cfg.k, cfg.dtype, P.y, X=P.X)
        want = orc.forward_full(Ws, bs, cfg.dtype, X=P.X.reshape(-1, cfg.dims[0])[:cfg.B])
    err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - want))) / float(np.max(np.abs(want)))
    assert err <= 2 * H.TOL[cfg.dtype], (name, err)
    ctx.close()
