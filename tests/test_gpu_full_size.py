"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

cfg2 and cfg3: a whole round against the oracle.  cfg4 and cfg5 are too large for
the oracle to run whole, so partition/merge are checked bit-exactly on sampled
rows, and training on one subnet for one local step (the oracle is fed the
subnet's parameters gathered from the full matrices with torch indexing, not
with anything the HIP path produced).
"""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

import ist_harness as H

pytestmark = pytest.mark.gpu
C = gen.CONFIGS


@pytest.mark.parametrize("name,normalize", [("cfg2", False), ("cfg3", False), ("cfg2", True), ("cfg3", True)])
def test_full_round_matches_oracle(name, normalize):
    cfg = C[name]
    P = H.Problem(cfg, bias_scale=0.02, normalize=normalize)
    ctx = P.context()
    ctx.set_checked(True)
    ctx.partition(P.dW, P.db, P.dperm)
    loss = P.gpu_steps(ctx)
    got = H.export_all(ctx, cfg)
    subs = P.oracle_subnets()
    want_loss = P.oracle_steps(subs)
    tol = H.TOL[cfg.dtype]
    worst = H.compare_subnets(got, subs, cfg, tol)
    np.testing.assert_allclose(loss, want_loss, rtol=5 * tol, atol=1e-4)
    # merged network: bit-exact placement of the trained blocks
    Wm = [w.clone() for w in P.dW]
    bm = [b.clone() for b in P.db]
    ctx.merge(Wm, bm)
    torch.cuda.synchronize()
    typed = [([H.np_bits(H.to_f32(w), cfg.dtype) for w in Wl], None) for Wl, _ in got]
    full = [H.np_bits(w, cfg.dtype).copy() for w in P.Ws]
    orc.merge(full, None, P.perms, cfg.S, typed)
    for l in range(cfg.t):
        assert np.array_equal(H.bits(Wm[l]), full[l])
    print(f"{name}: worst parameter rel err {worst:.3e} (tol {tol}); loss {loss[:, 0].mean():.4f} -> {loss[:, -1].mean():.4f}")
    ctx.close()


def _device_weights(cfg, dev, g):
    td = H.td(cfg.dtype)
    dW, db = [], []
    for l in range(1, cfg.t + 1):
        a = float(np.sqrt(6.0 / (cfg.dims[l] + cfg.dims[l - 1])))
        W = torch.empty((cfg.dims[l], cfg.dims[l - 1]), dtype=td, device=dev)
        rows = max(1, (1 << 26) // cfg.dims[l - 1])
        for r0 in range(0, cfg.dims[l], rows):
            r1 = min(cfg.dims[l], r0 + rows)
            W[r0:r1] = ((torch.rand((r1 - r0, cfg.dims[l - 1]), generator=g, device=dev) * 2 - 1) * a).to(td)
        dW.append(W)
        db.append((0.02 * torch.randn(cfg.dims[l], generator=g, device=dev)).to(td))
    return dW, db


def _host_subnet(cfg, dW, db, perms, s):
    """Subnet s gathered from the full parameters with torch indexing (float64 host arrays)."""
    Hs = orc.blocks(perms, cfg.S)
    Wl, bl = [], []
    for l in range(1, cfg.t + 1):
        W = dW[l - 1]
        if l < cfg.t:
            rows = torch.from_numpy(Hs[l - 1][s].astype(np.int64)).to(W.device)
            W = W.index_select(0, rows)
            b = db[l - 1].index_select(0, rows)
        else:
            b = db[l - 1]
        if l > 1:
            cols = torch.from_numpy(Hs[l - 2][s].astype(np.int64)).to(W.device)
            W = W.index_select(1, cols)
        Wl.append(np.ascontiguousarray(W.float().cpu().numpy(), dtype=np.float64))
        bl.append(np.ascontiguousarray(b.float().cpu().numpy(), dtype=np.float64))
    return Wl, bl


def _sampled_partition_check(cfg, ctx, dW, db, perms, rng, n_rows=6):
    """Bit-exact check of sampled rows of every subnet block against the oracle's gather
    applied to the same rows of the full matrices (copied to the host)."""
    Hs = orc.blocks(perms, cfg.S)
    for l in range(1, cfg.t + 1):
        R, Cc = ctx.subnet_shape(l)
        for s in rng.choice(cfg.S, size=min(2, cfg.S), replace=False):
            Wsub, bsub = ctx.subnet_export(int(s), l)
            torch.cuda.synchronize()
            ridx = Hs[l - 1][s] if l < cfg.t else np.arange(cfg.dims[l], dtype=np.int32)
            cidx = Hs[l - 2][s] if l > 1 else None
            pick = rng.choice(R, size=min(n_rows, R), replace=False)
            full_rows = dW[l - 1].index_select(0, torch.from_numpy(ridx[pick].astype(np.int64)).to(dW[l - 1].device))
            want = orc.gather(H.bits(full_rows), None, cidx)
            got = H.bits(Wsub.index_select(0, torch.from_numpy(pick.astype(np.int64)).to(Wsub.device)))
            assert np.array_equal(got, want), (l, s)
            wb = H.bits(db[l - 1].index_select(0, torch.from_numpy(ridx[pick].astype(np.int64)).to(db[l - 1].device)))
            assert np.array_equal(H.bits(bsub)[pick], wb), (l, s, "bias")


@pytest.mark.parametrize("name,normalize", [("cfg4", False), ("cfg5", False), ("cfg4", True), ("cfg5", True)])
def test_large_workload_sampled_parity(name, normalize):
    cfg = C[name]
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(gen.SEED_BASE + cfg.idx)
    rng = np.random.default_rng(cfg.idx)
    dW, db = _device_weights(cfg, dev, g)
    perms = gen.make_perms(cfg)
    dperm = [torch.from_numpy(p).to(dev) for p in perms]
    from paper_1910_02120_amd import ISTContext
    ctx = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B, normalize=normalize)
    ctx.partition(dW, db, dperm)
    _sampled_partition_check(cfg, ctx, dW, db, perms, rng)

    # ---- merge of the untrained partition into poisoned rows: owned entries return the
    # original bits (known from the inputs alone), unowned entries keep the poison ----
    Hs0 = orc.blocks(perms, cfg.S)
    saved = {}
    for l in range(1, cfg.t + 1):
        pick = torch.from_numpy(rng.choice(cfg.dims[l], size=4, replace=False).astype(np.int64)).to(dev)
        saved[l] = (pick, dW[l - 1].index_select(0, pick).clone())
        dW[l - 1].index_fill_(0, pick, 7.0)
    ctx.merge(dW, db)
    torch.cuda.synchronize()
    for l in range(1, cfg.t + 1):
        pick, orig = saved[l]
        new = H.bits(dW[l - 1].index_select(0, pick))
        ob = H.bits(orig)
        poison = H.bits(torch.full((1,), 7.0, dtype=orig.dtype, device=dev))[0]
        for i, r in enumerate(pick.cpu().numpy()):
            want = np.full(cfg.dims[l - 1], poison, dtype=ob.dtype)
            if l == 1:
                want[:] = ob[i]
            elif l < cfg.t:
                pos = int(np.flatnonzero(perms[l - 1] == r)[0])
                cidx = Hs0[l - 2][pos // (cfg.dims[l] // cfg.S)]
                want[cidx] = ob[i, cidx]
            else:
                want[:] = ob[i]                       # every column of the last layer has an owner
            assert np.array_equal(new[i], want), (name, l, int(r), "round trip")
        dW[l - 1].index_copy_(0, pick, orig)           # restore the inputs for what follows

    # ---- one local step on every subnet; subnet s0 is compared with the oracle ----
    s0 = int(rng.integers(cfg.S))
    one = gen.scaled(cfg, k=1)
    if cfg.input == "csr":
        rp, ci, va, y = gen.make_csr_batches(one)
        dcsr = (torch.from_numpy(rp).to(dev), torch.from_numpy(ci).to(dev), H.to_dev(va, cfg.dtype))
        dy = torch.from_numpy(y.reshape(-1)).to(dev)
        dX = None
    else:
        X, y = gen.make_dense_batches(one)
        dX, dy, dcsr = H.to_dev(X, cfg.dtype), torch.from_numpy(y.reshape(-1)).to(dev), None
    lr = 0.5 if cfg.input == "csr" else 0.05
    Wl, bl = _host_subnet(cfg, dW, db, perms, s0)
    lo = torch.zeros(cfg.S, dtype=torch.float32, device=dev)
    ctx.subnet_steps(dy, lr, 1, cfg.B, X=dX, csr=dcsr, loss_out=lo)
    torch.cuda.synchronize()
    if cfg.input == "csr":
        want_loss = orc.subnet_sgd(Wl, bl, y[s0], lr, 1, cfg.dtype, normalize=normalize,
                                   csr=orc.csr_slice(rp, ci, va.astype(np.float64), s0 * cfg.B, (s0 + 1) * cfg.B))
    else:
        want_loss = orc.subnet_sgd(Wl, bl, y[s0], lr, 1, cfg.dtype, X=X[s0].astype(np.float64), normalize=normalize)
    # the oracle worked in H^s order; export gives the same order
    tol = H.TOL[cfg.dtype]
    worst = 0.0
    for l in range(1, cfg.t + 1):
        Wg, bg = ctx.subnet_export(s0, l)
        torch.cuda.synchronize()
        e = H.rel_err(H.to_f32(Wg), Wl[l - 1])
        worst = max(worst, e)
        assert e <= tol, (name, l, e)
        scale = max(np.max(np.abs(bl[l - 1])), np.max(np.abs(Wl[l - 1])))
        eb = float(np.max(np.abs(H.to_f32(bg) - bl[l - 1]))) / scale
        assert eb <= tol, (name, l, "bias", eb)
        del Wg, bg
    assert abs(float(lo[s0]) - want_loss[0]) <= 5 * tol * abs(want_loss[0])
    print(f"{name}: subnet {s0} after one full-size step, worst rel err {worst:.3e}")

    # ---- merge after training: placement only (a consistency property: the trained values come
    # from ist_subnet_export, whose subnet s0 was compared with the oracle above) ----
    before = {}
    Hs = orc.blocks(perms, cfg.S)
    for l in range(1, cfg.t + 1):
        pick = torch.from_numpy(rng.choice(cfg.dims[l], size=4, replace=False).astype(np.int64)).to(dev)
        before[l] = (pick, dW[l - 1].index_select(0, pick).clone())
    ctx.merge(dW, db)
    torch.cuda.synchronize()
    for l in range(1, cfg.t + 1):
        pick, old = before[l]
        new = dW[l - 1].index_select(0, pick)
        for i, r in enumerate(pick.cpu().numpy()):
            if l < cfg.t:
                pos = int(np.flatnonzero(perms[l - 1] == r)[0])
                s, q = divmod(pos, cfg.dims[l] // cfg.S)
            else:
                s, q = None, int(r)
            want = H.bits(old[i:i + 1]).copy()
            for ss in ([s] if s is not None else range(cfg.S)):
                Wg, _ = ctx.subnet_export(ss, l)
                torch.cuda.synchronize()
                row = H.bits(Wg[q:q + 1])
                cidx = Hs[l - 2][ss] if l > 1 else np.arange(cfg.dims[0])
                want[0, cidx] = row[0]
                del Wg
            assert np.array_equal(H.bits(new[i:i + 1]), want), (name, l, int(r))
    ctx.close()


@pytest.mark.parametrize("name", ["cfg4", "cfg5"])
def test_resample_at_full_size_equals_merge_then_partition(name):
    """Bit-exact agreement of the one-pass re-sampling with the two calls it replaces, on the whole
    of every weight matrix and on sampled blocks of the new subnets, after one (small-batch) local
    step so that the subnets differ from the full network."""
    cfg = gen.scaled(C[name], B=8, k=1)
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(gen.SEED_BASE + 7 * cfg.idx)
    rng = np.random.default_rng(100 + cfg.idx)
    dW, db = _device_weights(cfg, dev, g)
    dperm = [torch.from_numpy(p).to(dev) for p in gen.make_perms(cfg, 0)]
    perm1 = [torch.from_numpy(p).to(dev) for p in gen.make_perms(cfg, 1)]
    if cfg.input == "csr":
        rp, ci, va, y = gen.make_csr_batches(cfg)
        data = dict(csr=(torch.from_numpy(rp).to(dev), torch.from_numpy(ci).to(dev), H.to_dev(va, cfg.dtype)), X=None)
    else:
        X, y = gen.make_dense_batches(cfg)
        data = dict(X=H.to_dev(X, cfg.dtype), csr=None)
    dy = torch.from_numpy(y.reshape(-1)).to(dev)
    from paper_1910_02120_amd import ISTContext
    ctxs = [ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B) for _ in range(2)]
    for c in ctxs:
        c.partition(dW, db, dperm)
        c.subnet_steps(dy, 0.5, 1, cfg.B, **data)
    a, b = ctxs
    Wb = [w.clone() for w in dW]
    bb = [x.clone() for x in db]
    a.resample(dW, db, perm1)
    b.merge(Wb, bb)
    b.partition(Wb, bb, perm1)
    torch.cuda.synchronize()
    for l in range(cfg.t):
        assert torch.equal(dW[l], Wb[l]), (name, l)
        assert torch.equal(db[l], bb[l]), (name, l, "bias")
    for l in range(1, cfg.t + 1):
        for s in rng.choice(cfg.S, size=2, replace=False):
            wa, xa = a.subnet_export(int(s), l)
            wb, xb = b.subnet_export(int(s), l)
            torch.cuda.synchronize()
            assert torch.equal(wa, wb) and torch.equal(xa, xb), (name, l, int(s))
            del wa, wb
    a.close()
    b.close()
