"""Seeded random shapes: layer count, widths, S, batch, dtype, input kind, bias and standardisation drawn
per case.  Partition and merge bit for bit against the oracle, then k local steps: final parameters within
the stated tolerance and the loss of every step (the fixed shapes of test_gpu_parity.py carry the gates on
the change of the parameters; this file looks for shapes nobody thought of)."""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

import ist_harness as H

pytestmark = pytest.mark.gpu
C = gen.CONFIGS


def draw(case: int):
    rng = np.random.default_rng(77000 + case)
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    csr = rng.random() < 0.3
    t = int(rng.integers(2, 5))
    S = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
    big = rng.random() < 0.4
    hi = 2200 if big else 200
    hidden = [int(rng.integers(S, hi)) for _ in range(t - 1)]
    n_in = int(rng.integers(3, 1500 if csr else (600 if big else 150)))
    n_out = (int(rng.choice([1, 2, 10, 35, 100, 257, 300, 1000, 4097, 5000])) if rng.random() < 0.8
             else int(rng.integers(1, 400)))
    B = int(rng.integers(1, 520 if big else 70))
    k = int(rng.integers(1, 4))
    normalize = bool(rng.random() < 0.2 and B > 1)
    has_bias = bool(rng.random() < 0.85)
    base = "cfg5" if csr else ("cfg3" if dtype == "bf16" else "cfg2")
    kw = dict(dims=(n_in, *hidden, n_out), S=S, B=B, k=k, lr=0.05, dtype=dtype)
    if csr:
        kw["nnz_per_row"] = int(rng.integers(1, min(n_in, 30) + 1))
    return gen.scaled(C[base], name=f"random-{case}", **kw), has_bias, normalize


@pytest.mark.parametrize("case", range(24))
def test_random_shape_matches_oracle(case):
    cfg, has_bias, normalize = draw(case)
    print(f"{cfg.name}: {cfg.dtype} {cfg.input} dims={cfg.dims} S={cfg.S} B={cfg.B} k={cfg.k} "
          f"standardised={normalize} bias={has_bias}", flush=True)
    P = H.Problem(cfg, has_bias=has_bias, dev="cuda:0", normalize=normalize)
    ctx = P.context()
    ctx.set_checked(True)
    ctx.partition(P.dW, P.db, P.dperm)
    got = H.export_all(ctx, cfg)
    raw_W = [H.np_bits(w, cfg.dtype) for w in P.Ws]
    raw_b = [H.np_bits(b, cfg.dtype) for b in P.bs] if has_bias else [None] * cfg.t
    want = orc.partition(raw_W, raw_b, P.perms, cfg.S)
    for s in range(cfg.S):
        for l in range(cfg.t):
            assert np.array_equal(H.bits(got[s][0][l]), want[s][0][l]), (cfg.name, s, l)
            if has_bias:
                assert np.array_equal(H.bits(got[s][1][l]), want[s][1][l]), (cfg.name, s, l, "bias")
    # merge of the untrained subnets into poisoned matrices: owned entries return, the others keep the poison
    poison = [torch.full_like(w, 7.0) for w in P.dW]
    pb = [torch.full_like(b, 7.0) for b in P.db] if has_bias else None
    ctx.merge(poison, pb)
    torch.cuda.synchronize()
    full = [np.full(w.shape, H.np_bits(np.float32([7.0]), cfg.dtype)[0], dtype=raw_W[0].dtype) for w in raw_W]
    orc.merge(full, None, P.perms, cfg.S, want)
    for l in range(cfg.t):
        assert np.array_equal(H.bits(poison[l]), full[l]), (cfg.name, l, "merge")
    # k local steps
    subs = H.copy_subnets(P.oracle_subnets())
    loss_gpu = P.gpu_steps(ctx, k=cfg.k)
    loss_orc = P.oracle_steps(subs, k=cfg.k)
    worst = H.compare_subnets(H.export_all(ctx, cfg), subs, cfg, H.TOL[cfg.dtype])
    np.testing.assert_allclose(loss_gpu, loss_orc, rtol=H.LOSS_RTOL[cfg.dtype], atol=1e-6)
    print(f"{cfg.name}: worst parameter rel err {worst:.3e} (tol {H.TOL[cfg.dtype]})")
    ctx.close()
