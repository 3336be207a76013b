"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The speech-like and image-like workloads (and the paper's 3 x 8192 speech model): whole
rounds against the oracle, the second round starting from the first round's merged
network.  The sparse extreme-classification workload: one whole round.  The wide stress
network is too large for the oracle to run whole (a round is 80 subnet-steps of several
seconds each), so partition/merge are checked bit-exactly on sampled rows, and training
on one subnet for all of its k = 10 local steps while the HIP path trains all eight
(the oracle is fed the subnet's parameters gathered from the full matrices with torch
indexing, not with anything the HIP path produced).  Large weights are drawn on the
device with torch's seeded generator in the recipe's distributions.
"""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

import ist_harness as H

pytestmark = pytest.mark.gpu
C = gen.CONFIGS


def _merge_check(ctx, P, got):
    """ist_merge of the trained subnets: bit-exact placement against the oracle's merge of the same
    (exported) subnets.  Returns the merged full network as float32 host arrays."""
    cfg = P.cfg
    Wm = [w.clone() for w in P.dW]
    bm = [b.clone() for b in P.db]
    ctx.merge(Wm, bm)
    torch.cuda.synchronize()
    typed = [([H.bits(w) for w in Wl], None) for Wl, _ in got]
    full = [H.np_bits(w, cfg.dtype).copy() for w in P.Ws]
    orc.merge(full, None, P.perms, cfg.S, typed)
    for l in range(cfg.t):
        assert np.array_equal(H.bits(Wm[l]), full[l]), (cfg.name, l, "merged weights")
    fb = [b.astype(np.float32).copy() for b in P.bs]
    dummy = [np.zeros(w.shape, dtype=np.float32) for w in P.Ws]
    f32subs = [([H.to_f32(w) for w in Wl], [H.to_f32(b) for b in bl]) for Wl, bl in got]
    orc.merge(dummy, fb, P.perms, cfg.S, f32subs, mode=cfg.dtype)
    for l in range(cfg.t):
        np.testing.assert_array_equal(H.to_f32(bm[l]), fb[l])
    return [H.to_f32(w) for w in Wm], [H.to_f32(b) for b in bm]


@pytest.mark.parametrize("name,normalize", [("cfg2", False), ("cfg3", False), ("cfg2", True), ("cfg3", True),
                                            ("speech8192", False)])
def test_full_rounds_match_oracle(name, normalize):
    """Two whole rounds at the benchmark's own S, B and k: partition, k local steps on every subnet, merge.
    The gate is per round from a common start: the second round (new permutations, new mini-batches)
    starts, on both sides, from the network the HIP path merged at the end of the first."""
    cfg = C[name]
    weights = None
    for rnd in (0, 1):
        P = H.Problem(cfg, rnd=rnd, bias_scale=0.02, normalize=normalize, weights=weights)
        ctx = P.context()
        ctx.set_checked(True)
        ctx.partition(P.dW, P.db, P.dperm)
        weak = tuple(f"b{l}" for l in range(1, cfg.t)) if normalize else ()   # no gradient: the mean is subtracted
        got, subs, loss, worst = H.check_training(P, ctx, weak=weak)
        weights = _merge_check(ctx, P, got)
        print(f"{name} round {rnd}: worst parameter rel err {worst:.3e} (tol {H.TOL[cfg.dtype]}); "
              f"loss {loss[:, 0].mean():.4f} -> {loss[:, -1].mean():.4f}")
        ctx.close()
        if name == "speech8192":
            break          # one round of the extra workload


def test_extreme_classification_whole_round():
    """The sparse-input, 670,091-class workload at its own S = 8, B = 256, k = 5: every subnet, every
    step, against the oracle (the recipe's host-generated weights; one hidden layer, so every weight
    has an owner and the merged network is compared whole)."""
    cfg = gen.scaled(C["cfg5"], lr=0.5)
    P = H.Problem(cfg, bias_scale=0.02)
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    got, subs, loss, worst = H.check_training(P, ctx)
    _merge_check(ctx, P, got)
    print(f"cfg5 whole round: worst parameter rel err {worst:.3e}; loss {loss[:, 0].mean():.4f} -> {loss[:, -1].mean():.4f}")
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


class _DeviceProblem(H.Problem):
    """The large workloads: weights live on the device only (an 18 GB host array is impractical); the
    oracle's subnets are gathered from them with torch indexing, the mini-batches come from the seeded
    host generators."""

    def __init__(self, cfg, dW, db, perms, dperm, normalize):
        self.cfg, self.dev, self.has_bias, self.normalize, self.scale = cfg, "cuda:0", True, normalize, None
        self.dW, self.db, self.perms, self.dperm = dW, db, perms, dperm
        if cfg.input == "csr":
            self.rp, self.ci, self.va, self.y = gen.make_csr_batches(cfg)
            self.X = None
            self.dcsr = (torch.from_numpy(self.rp).to(self.dev), torch.from_numpy(self.ci).to(self.dev),
                         H.to_dev(self.va, cfg.dtype))
            self.dX = None
        else:
            self.X, self.y = gen.make_dense_batches(cfg)
            self.dX, self.dcsr = H.to_dev(self.X, cfg.dtype), None
        self.dy = torch.from_numpy(self.y.reshape(-1).copy()).to(self.dev)

    def oracle_subnets(self, subnets=None):
        which = range(self.cfg.S) if subnets is None else subnets
        return [_host_subnet(self.cfg, self.dW, self.db, self.perms, s) for s in which]


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

    # ---- local steps on every subnet; subnet s0 is followed by the oracle: all k = 10 steps of the wide
    # stress network, two steps for the others (the sparse workload's whole round has a test of its own) ----
    s0 = int(rng.integers(cfg.S))
    k = cfg.k if (name == "cfg4" and not normalize) else 2
    lr = 0.5 if cfg.input == "csr" else 0.05
    P = _DeviceProblem(gen.scaled(cfg, k=k, lr=lr), dW, db, perms, dperm, normalize)
    weak = tuple(f"b{l}" for l in range(1, cfg.t)) if normalize else ()
    _, _, _, worst = H.check_training(P, ctx, weak=weak, subnets=[s0])
    print(f"{name}: subnet {s0} after {k} full-size steps, worst rel err {worst:.3e}")

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
