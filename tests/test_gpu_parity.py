"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Partition / merge indexing must be bit-exact.  Parameters after k local steps
must agree within max relative error 2e-3 (f32) or 3e-2 (bf16), measured per
parameter tensor as ||gpu - oracle||_inf / ||oracle||_inf.
"""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

import ist_harness as H

pytestmark = pytest.mark.gpu

C = gen.CONFIGS


def _mk(name, base, **kw):
    return gen.scaled(C[base], name=name, **kw)


# reduced shapes: several tiles plus ragged tails in every dimension
SHAPES = {
    "cfg1": C["cfg1"],
    "cfg1-nobias-S1": _mk("cfg1-S1", "cfg1", S=1),
    "ragged-f32": _mk("ragged-f32", "cfg2", dims=(100, 156, 204, 35), S=4, B=37, k=3, lr=0.05),
    "ragged-bf16": _mk("ragged-bf16", "cfg3", dims=(150, 264, 136, 10), S=8, B=45, k=4, lr=0.05),
    "cfg3-small": _mk("cfg3-small", "cfg3", dims=(384, 1024, 1024, 10), k=5, lr=0.05),
    "cfg4-small": _mk("cfg4-small", "cfg4", dims=(256, 1024, 512, 1024, 100), B=96, k=3, lr=0.05),
    "cfg5-small": _mk("cfg5-small", "cfg5", dims=(3001, 256, 5003), S=8, B=40, k=3, nnz_per_row=20,
                      lr=0.5),
    "wide-out-f32": _mk("wide-out-f32", "cfg2", dims=(96, 128, 4507), S=2, B=24, k=2, lr=0.5),
    # wide enough for the 256x256 block tiles (forward of layer 1, backward-data of layer 2)
    "big-tiles-bf16": _mk("big-tiles-bf16", "cfg3", dims=(520, 33280, 4352, 10), S=16, B=300, k=2,
                          lr=0.05),
    # the update product of a layer with at least 1024 blocks of 256 x 256 (persistent kernel that keeps the old
    # weights in its accumulators): 5808 = 22 x 256 + 176 rows and columns per subnet, 264 = 4 x 64 + 8 samples
    "wide-update-bf16": _mk("wide-update-bf16", "cfg3", dims=(264, 11616, 11616, 10), S=2, B=264, k=2, lr=0.05),
    # degenerate shapes: one hidden layer and a batch of one sample; a deeper net with S = N_l / 2
    "one-hidden-B1-f32": _mk("one-hidden-B1-f32", "cfg2", dims=(40, 64, 7), S=4, B=1, k=2, lr=0.05),
    "deep-bf16": _mk("deep-bf16", "cfg3", dims=(64, 128, 256, 128, 64, 12), S=4, B=20, k=3, lr=0.05),
    "width-one-blocks-f32": _mk("width-one-blocks-f32", "cfg2", dims=(24, 8, 8, 5), S=8, B=9, k=2, lr=0.05),
    # sparse first layer in bf16 (transposed storage): even row length with 128 rows per subnet, and
    # an odd row length with 8 rows per subnet
    "csr-bf16-even": _mk("csr-bf16-even", "cfg5", dims=(1000, 512, 77), S=4, B=21, k=2, nnz_per_row=12, lr=0.5),
    "csr-bf16-odd": _mk("csr-bf16-odd", "cfg5", dims=(777, 64, 50), S=8, B=10, k=2, nnz_per_row=7, lr=0.5),
    "speech-small": _mk("speech-small", "speech8192", dims=(256, 512, 512, 512, 35), k=3, lr=0.05),
    # more steps than row-loss slots of one reduction launch, and a class count that spans three
    # 64-wide lane groups of the narrow-output cross-entropy kernel; 300 classes take the wide kernel
    "many-steps-f32": _mk("many-steps-f32", "cfg2", dims=(48, 64, 130), S=2, B=10, k=19, lr=0.05),
    "mid-out-bf16": _mk("mid-out-bf16", "cfg3", dims=(64, 128, 300), S=4, B=12, k=2, lr=0.05),
    # wide output layer with a full 256-row batch: the row-statistics pass takes its 256x256 blocks
    "wide-out-bf16-B256": _mk("wide-out-bf16-B256", "cfg5", dims=(200, 512, 33001), S=8, B=256, k=2,
                              nnz_per_row=10, lr=0.5),
    # a wide bf16 output layer behind more than 128 hidden neurons per subnet: both cross-entropy passes recompute
    # the logits with 256 x 256 blocks (264 = 256 + 8 hidden neurons per subnet, 10500 = 41 x 256 + 4 classes: the
    # transposed dz pass walks a grid of 42 x 1 blocks per subnet, five bands of 8 block rows and one of 2)
    "wide-out-gemm-bf16": _mk("wide-out-gemm-bf16", "cfg3", dims=(100, 2112, 10500), S=8, B=256, k=2, lr=0.5),
    # hidden layers of at least 2048 neurons per subnet in f32: the bias kernel for wide layers (16-byte loads, eight
    # columns per lane) in its f32 form, with a batch that is not a multiple of its row groups
    "wide-hidden-f32": _mk("wide-hidden-f32", "cfg2", dims=(40, 4200, 4400, 7), S=2, B=70, k=2, lr=0.05),
    # more layers than one bias launch, one bias-copy launch or one shared update launch takes (16 / 16 / 4);
    # initial weights 1.5 x Xavier so that the gradient survives the 18 ReLU layers down to the first
    "very-deep-f32": _mk("very-deep-f32", "cfg2", dims=(16,) + (32,) * 18 + (5,), S=2, B=6, k=2, lr=0.05,
                         init_gain=1.5),
    "csr-f32": _mk("csr-f32", "cfg5", dims=(517, 96, 301), S=4, B=33, k=3, nnz_per_row=9,
                   dtype="f32", lr=0.5),
    # blocks of unequal width (S does not divide the hidden widths): 157 = 52 + 52 + 53 ..., a layer whose width
    # S does divide next to one it does not, and the sparse first layer (stored transposed)
    "uneven-S3-f32": _mk("uneven-S3-f32", "cfg2", dims=(100, 157, 203, 35), S=3, B=37, k=3, lr=0.05),
    "uneven-S5-bf16": _mk("uneven-S5-bf16", "cfg3", dims=(150, 263, 320, 137, 10), S=5, B=45, k=3, lr=0.05),
    "uneven-S7-csr-bf16": _mk("uneven-S7-csr-bf16", "cfg5", dims=(1000, 509, 77), S=7, B=21, k=2, nnz_per_row=12, lr=0.5),
    "uneven-S7-wide-out-f32": _mk("uneven-S7-wide-out-f32", "cfg2", dims=(96, 131, 4507), S=7, B=24, k=2, lr=0.5),
}


# Tensors on which no check of the change over the steps can have power, per shape: their gradient is
# (next to) zero by construction of the shape.
WEAK = {
    # one neuron per subnet and hidden layer: where that neuron's ReLU is off for the whole batch nothing below
    # the output bias moves
    "width-one-blocks-f32": ("W1", "b1", "W2", "b2", "W3"),
}


def _dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return "cuda:0"


@pytest.mark.parametrize("name", list(SHAPES))
def test_partition_and_merge_are_bit_exact(name):
    cfg = SHAPES[name]
    P = H.Problem(cfg, has_bias="nobias" not in name, dev=_dev())
    ctx = P.context()
    ctx.set_checked(True)
    ctx.partition(P.dW, P.db, P.dperm)
    got = H.export_all(ctx, cfg)
    raw_W = [H.np_bits(w, cfg.dtype) for w in P.Ws]
    raw_b = [H.np_bits(b, cfg.dtype) for b in P.bs] if P.has_bias else [None] * cfg.t
    want = orc.partition(raw_W, raw_b, P.perms, cfg.S)
    for s in range(cfg.S):
        for l in range(cfg.t):
            assert np.array_equal(H.bits(got[s][0][l]), want[s][0][l]), (name, s, l)
            if P.has_bias:
                assert np.array_equal(H.bits(got[s][1][l]), want[s][1][l]), (name, s, l, "bias")
    # merge(partition(W)) == W, into buffers that were poisoned first: what no subnet
    # owns must keep the poison, everything else must return bit for bit
    poison = [torch.full_like(w, 7.0) for w in P.dW]
    pb = [torch.full_like(b, 7.0) for b in P.db] if P.has_bias else None
    ctx.merge(poison, pb)
    torch.cuda.synchronize()
    full = [np.full(w.shape, H.np_bits(np.float32([7.0]), cfg.dtype)[0], dtype=raw_W[0].dtype)
            for w in raw_W]
    orc.merge(full, None, P.perms, cfg.S, want)
    for l in range(cfg.t):
        assert np.array_equal(H.bits(poison[l]), full[l]), (name, l)
    if P.has_bias:
        # hidden biases return bit for bit; the output bias is the oracle's mean of the S copies (the copies
        # themselves again when S is a power of two: every step of the pairwise sum and the scaling is exact)
        fb = [b.astype(np.float32).copy() for b in P.bs]
        f32subs = [([w for w in P.Ws], [H.to_f32(x) for x in bl]) for _, bl in got]
        for s in range(cfg.S):
            f32subs[s] = ([np.zeros(w.shape, dtype=np.float32) for w in want[s][0]], f32subs[s][1])
        orc.merge([np.zeros(w.shape, dtype=np.float32) for w in P.Ws], fb, P.perms, cfg.S, f32subs, mode=cfg.dtype)
        for l in range(cfg.t):
            assert np.array_equal(H.bits(pb[l]), H.np_bits(fb[l], cfg.dtype)), (name, l, "bias round trip")
            if l < cfg.t - 1 or cfg.S & (cfg.S - 1) == 0:
                assert np.array_equal(H.bits(pb[l]), raw_b[l]), (name, l, "bias round trip, exact")
    ctx.close()


@pytest.mark.parametrize("name", list(SHAPES))
def test_k_local_steps_match_oracle(name):
    cfg = SHAPES[name]
    P = H.Problem(cfg, has_bias="nobias" not in name, dev=_dev())
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    got, subs, loss, worst = H.check_training(P, ctx, weak=WEAK.get(name, ()))
    tol = H.TOL[cfg.dtype]
    # and the merged full network: owned entries from the subnets, the rest untouched
    Wm = [w.clone() for w in P.dW]
    bm = [b.clone() for b in P.db] if P.has_bias else None
    ctx.merge(Wm, bm)
    torch.cuda.synchronize()
    typed = [([H.np_bits(H.to_f32(w), cfg.dtype) for w in Wl],
              [None if b is None else H.to_f32(b) for b in bl]) for Wl, bl in got]
    full = [H.np_bits(w, cfg.dtype).copy() for w in P.Ws]
    orc.merge(full, None, P.perms, cfg.S, typed)
    for l in range(cfg.t):
        assert np.array_equal(H.bits(Wm[l]), full[l]), (name, l, "merge of trained subnets")
    if P.has_bias:
        fb = [b.astype(np.float32).copy() for b in P.bs]
        fl = [w.astype(np.float32).copy() for w in P.Ws]
        f32subs = [([H.to_f32(w) for w in Wl], [H.to_f32(b) for b in bl]) for Wl, bl in got]
        orc.merge(fl, fb, P.perms, cfg.S, f32subs, mode=cfg.dtype)
        for l in range(cfg.t):
            np.testing.assert_array_equal(H.to_f32(bm[l]), fb[l])
    print(f"{name}: worst parameter rel err {worst:.3e} (tol {tol})")
    ctx.close()


def test_steps_can_be_split_and_batches_reused():
    """Two calls of k/2 steps equal one call of k steps; stride 0 reuses a batch."""
    cfg = SHAPES["ragged-f32"]
    P = H.Problem(cfg, dev=_dev())
    a, b = P.context(), P.context()
    a.partition(P.dW, P.db, P.dperm)
    b.partition(P.dW, P.db, P.dperm)
    a.subnet_steps(P.dy, cfg.lr, 2, cfg.B, X=P.dX, stride_s=cfg.k * cfg.B, stride_k=cfg.B)
    b.subnet_steps(P.dy, cfg.lr, 1, cfg.B, X=P.dX, stride_s=cfg.k * cfg.B, stride_k=cfg.B)
    off = cfg.B
    b.subnet_steps(P.dy[off:], cfg.lr, 1, cfg.B, X=P.dX.reshape(-1, cfg.dims[0])[off:],
                   stride_s=cfg.k * cfg.B, stride_k=cfg.B)
    ga, gb = H.export_all(a, cfg), H.export_all(b, cfg)
    for s in range(cfg.S):
        for l in range(cfg.t):
            assert torch.equal(ga[s][0][l], gb[s][0][l])
    # same batch for every subnet and step: oracle fed with the repeated batch
    c = P.context()
    c.partition(P.dW, P.db, P.dperm)
    c.subnet_steps(P.dy, cfg.lr, 2, cfg.B, X=P.dX, stride_s=0, stride_k=0)
    subs = P.oracle_subnets()
    Xr = np.broadcast_to(P.X[0, 0], (cfg.S, 2) + P.X.shape[2:]).copy()
    yr = np.broadcast_to(P.y[0, 0], (cfg.S, 2, cfg.B)).copy()
    orc.subnet_steps(subs, cfg.lr, 2, "f32", yr, X=Xr)
    H.compare_subnets(H.export_all(c, cfg), subs, cfg, H.TOL["f32"])
    for x in (a, b, c):
        x.close()


def test_error_paths():
    from paper_1910_02120_amd import ISTContext, ISTError
    cfg = SHAPES["ragged-f32"]
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    with pytest.raises(ISTError) as e:
        ctx.subnet_steps(P.dy, cfg.lr, 1, cfg.B, X=P.dX)
    assert e.value.status == -6                       # steps before partition
    with pytest.raises(ISTError) as e:
        ctx.merge(P.dW, P.db)
    assert e.value.status == -6
    ctx.set_checked(True)
    bad = [p.clone() for p in P.dperm]
    bad[0][3] = bad[0][4]                             # duplicate -> not a permutation
    with pytest.raises(ISTError) as e:
        ctx.partition(P.dW, P.db, bad)
    assert e.value.status == -3
    bad[0][3] = 10 ** 6                               # out of range
    with pytest.raises(ISTError) as e:
        ctx.partition(P.dW, P.db, bad)
    assert e.value.status == -3
    # unchecked mode with the same bad permutation must stay in bounds (no fault)
    ctx.set_checked(False)
    ctx.partition(P.dW, P.db, bad)
    torch.cuda.synchronize()
    ctx.partition(P.dW, P.db, P.dperm)
    with pytest.raises(ISTError) as e:
        ctx.subnet_steps(P.dy, cfg.lr, 1, cfg.B + 1, X=P.dX)
    assert e.value.status == -2                       # B > max_B
    with pytest.raises(ISTError) as e:
        ISTContext((8, 3, 4), 4, bind=False)          # fewer hidden neurons than subnets
    assert e.value.status == -2
    ctx.close()


def test_k_zero_and_empty_step_list():
    cfg = SHAPES["cfg1"]
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    before = H.export_all(ctx, cfg)
    ctx.subnet_steps(P.dy, cfg.lr, 0, cfg.B, X=P.dX)
    after = H.export_all(ctx, cfg)
    for s in range(cfg.S):
        for l in range(cfg.t):
            assert torch.equal(before[s][0][l], after[s][0][l])
    ctx.close()


def test_profile_records_name_kernels_and_work():
    """Per-kernel profiling records: labels, launch counts and algorithmic flops of a known shape."""
    cfg = SHAPES["ragged-f32"]
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    ctx.profile_enable(True)
    ctx.profile_reset()
    ctx.partition(P.dW, P.db, P.dperm)
    P.gpu_steps(ctx)
    ctx.merge(P.dW, P.db)
    ks = ctx.profile_kernels()
    classes = ctx.profile_read()
    ctx.profile_enable(False)
    assert sum(k["launches"] for k in ks) == sum(n for _, n in classes.values())
    t = cfg.t
    widths = [cfg.width(l) for l in range(t + 1)]
    fwd = sum(2.0 * cfg.B * widths[l] * widths[l - 1] * cfg.S for l in range(1, t + 1)) * cfg.k
    got = sum(k["flops"] for k in ks if k["kernel_class"] == "gemm_forward")
    assert got == pytest.approx(fwd, rel=1e-12)
    assert all(k["ms"] > 0 for k in ks)
    assert any(k["label"].startswith("k_") and k["bytes"] > 0 for k in ks if k["kernel_class"] == "partition_copy")
    ctx.close()


@pytest.mark.parametrize("name", ["ragged-f32", "ragged-bf16", "csr-f32", "cfg5-small", "wide-out-f32"])
def test_batch_smaller_than_max_B(name):
    """A context sized for max_B runs smaller batches: same result as a context sized exactly."""
    from paper_1910_02120_amd import ISTContext
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev=_dev())
    big = ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, True, max_B=cfg.B + 19, device=_dev())
    big.partition(P.dW, P.db, P.dperm)
    H.check_training(P, big, weak=WEAK.get(name, ()))
    big.close()


@pytest.mark.parametrize("name", ["cfg5-small", "wide-out-f32", "ragged-bf16"])
def test_smaller_batch_after_a_larger_one(name):
    """The same context first trains on its largest batch, then, from a fresh partition, on a batch three
    samples shorter: what the first run left in the workspace (among it the columns of the transposed dz
    of a wide output layer beyond the new batch size) must not leak into the second."""
    cfg = SHAPES[name]
    small = gen.scaled(cfg, B=cfg.B - 3)
    Pb, Ps = H.Problem(cfg, dev=_dev()), H.Problem(small, dev=_dev())
    ctx = Pb.context()
    ctx.partition(Pb.dW, Pb.db, Pb.dperm)
    Pb.gpu_steps(ctx)
    ctx.partition(Ps.dW, Ps.db, Ps.dperm)
    H.check_training(Ps, ctx, weak=WEAK.get(name, ()))
    ctx.close()


def test_csr_with_empty_rows_and_unused_columns():
    """Samples without non-zeros see the bias only; weights of columns no sample touches stay put."""
    cfg = SHAPES["csr-f32"]
    P = H.Problem(cfg, dev=_dev())
    rows = len(P.rp) - 1
    keep = np.ones(len(P.ci), dtype=bool)
    for r in range(0, rows, 5):                      # every fifth sample loses all its features
        keep[P.rp[r]:P.rp[r + 1]] = False
    keep &= P.ci % 3 != 0                            # and a third of the columns never appears
    cnt = np.add.reduceat(keep.astype(np.int64), P.rp[:-1]) * (np.diff(P.rp) > 0)
    P.rp = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
    P.ci, P.va = P.ci[keep].copy(), P.va[keep].copy()
    assert (np.diff(P.rp) == 0).any()
    P.upload()
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    before = [s[0][0].copy() for s in P.oracle_subnets()]
    got, subs, loss, _ = H.check_training(P, ctx)
    unused = np.arange(cfg.dims[0]) % 3 == 0
    for s in range(cfg.S):                           # bit-exact: nothing may touch those columns
        w0 = H.np_bits(before[s].astype(np.float32), cfg.dtype)
        assert np.array_equal(H.bits(got[s][0][0])[:, unused], w0[:, unused])
    ctx.close()


@pytest.mark.parametrize("name", ["csr-f32", "csr-bf16-even", "cfg5-small"])
def test_csr_rows_that_repeat_a_column(name):
    """A sample's column list may name a column more than once: its values are summed, on both sides.  Every
    third row gets its second entry's column replaced by the first's (the lists stay ascending), so columns
    held by one sample, by several, and repeated inside a row all occur."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev=_dev())
    changed = 0
    for r in range(0, len(P.rp) - 1, 3):
        p0, p1 = int(P.rp[r]), int(P.rp[r + 1])
        if p1 - p0 >= 2:
            P.ci[p0 + 1] = P.ci[p0]
            changed += 1
    assert changed > 10
    P.upload()
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    _, _, _, worst = H.check_training(P, ctx)
    print(f"{name} with {changed} repeated columns: worst parameter rel err {worst:.3e} (tol {H.TOL[cfg.dtype]})")
    ctx.close()


@pytest.mark.parametrize("name", ["cfg3-small", "cfg5-small", "wide-update-bf16"])
def test_zero_learning_rate_changes_nothing(name):
    """lr = 0: every parameter keeps its bits (the update kernels that fold the old weights into their
    accumulators divide by lr and must step aside)."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    before = [[(H.bits(W).copy(), H.bits(b).copy()) for W, b in (ctx.subnet_export(s, l) for l in range(1, cfg.t + 1))]
              for s in range(cfg.S)]
    lo = torch.zeros(cfg.S * 2, dtype=torch.float32, device=P.dev)
    csr = None if P.dcsr is None else P.dcsr
    ctx.subnet_steps(P.dy, 0.0, 2, cfg.B, X=None if P.dX is None else P.dX.reshape(-1, cfg.dims[0]), csr=csr,
                     stride_s=cfg.k * cfg.B, stride_k=cfg.B, loss_out=lo)
    torch.cuda.synchronize()
    assert np.isfinite(lo.cpu().numpy()).all()
    for s in range(cfg.S):
        for l in range(1, cfg.t + 1):
            W, b = ctx.subnet_export(s, l)
            assert np.array_equal(H.bits(W), before[s][l - 1][0]), (s, l, "W")
            assert np.array_equal(H.bits(b), before[s][l - 1][1]), (s, l, "b")
    ctx.close()


@pytest.mark.parametrize("dims,S,B", [((12, 16, 1), 4, 6), ((20, 64, 64, 3), 64, 5)])
def test_single_class_and_as_many_subnets_as_neurons(dims, S, B):
    cfg = _mk(f"edge-{dims[-1]}-{S}", "cfg2", dims=dims, S=S, B=B, k=2, lr=0.05)
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    # one class: the loss is constant, nothing has a gradient; one neuron per subnet and layer: where its
    # ReLU is off for the whole batch nothing below the output bias moves
    H.check_training(P, ctx, weak=("W1", "b1", "W2", "b2") if dims[-1] == 1 else ("W1", "b1", "W2", "b2", "W3"))
    ctx.close()


# with the standardisation a hidden bias has no gradient at all (the mean is subtracted again)
WEAK_NORM = {n: tuple(f"b{l}" for l in range(1, len(SHAPES[n].dims) - 1)) for n in
             ["cfg1", "ragged-f32", "ragged-bf16", "cfg3-small", "cfg4-small", "big-tiles-bf16", "csr-f32", "cfg5-small",
              "deep-bf16", "uneven-S3-f32", "uneven-S5-bf16", "uneven-S7-csr-bf16"]}
# a batch of one sample standardises to zero everywhere: nothing below the output bias has a gradient
WEAK_NORM["one-hidden-B1-f32"] = ("W1", "b1", "W2")


@pytest.mark.parametrize("name", ["cfg1", "ragged-f32", "ragged-bf16", "cfg3-small", "cfg4-small", "big-tiles-bf16",
                                  "csr-f32", "cfg5-small", "one-hidden-B1-f32", "deep-bf16", "uneven-S3-f32",
                                  "uneven-S5-bf16", "uneven-S7-csr-bf16"])
def test_k_local_steps_with_standardisation_match_oracle(name):
    """Section 2.2: every hidden neuron's input standardised over the mini-batch before the ReLU."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev=_dev(), normalize=True)
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    _, _, _, worst = H.check_training(P, ctx, weak=WEAK_NORM.get(name, ()))
    print(f"{name} (standardised): worst parameter rel err {worst:.3e} (tol {H.TOL[cfg.dtype]})")
    ctx.close()


def _factors(cfg, paper):
    """Layer factors of Appendix A, equation (4).  paper: n^2 on the layers with both sides partitioned,
    1 elsewhere; otherwise moderate factors on every layer, so that the first (dense or sparse) and the
    output layer (stored logits, partial products, two-pass cross-entropy) take theirs too."""
    if paper:
        return [float(cfg.S ** 2) if 1 < l < cfg.t else 1.0 for l in range(1, cfg.t + 1)]
    return [1.5 if l == 1 else (0.5 if l == cfg.t else 2.0) for l in range(1, cfg.t + 1)]


@pytest.mark.parametrize("name,paper,normalize", [
    ("cfg1", True, False), ("cfg1", False, False), ("ragged-f32", False, False), ("ragged-bf16", False, False),
    ("cfg3-small", False, False), ("cfg4-small", False, False), ("cfg5-small", False, False),
    ("csr-f32", False, False), ("wide-out-f32", False, False), ("many-steps-f32", False, False),
    ("mid-out-bf16", False, False), ("deep-bf16", False, False), ("speech-small", False, False),
    ("cfg4-small", True, True), ("ragged-f32", False, True), ("cfg5-small", False, True),
    ("uneven-S5-bf16", True, False), ("uneven-S3-f32", False, False), ("wide-update-bf16", False, False)])
def test_k_local_steps_with_layer_factors_match_oracle(name, paper, normalize):
    """Appendix A, equation (4): the product of layer l multiplied by gamma_l in the forward pass, hence in
    both gradients.  With the standardisation the factor of a hidden layer only matters through epsilon."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev=_dev(), normalize=normalize, scale=_factors(cfg, paper))
    ctx = P.context()
    ctx.partition(P.dW, P.db, P.dperm)
    _, _, _, worst = H.check_training(P, ctx, weak=WEAK_NORM.get(name, ()) if normalize else WEAK.get(name, ()))
    print(f"{name} (factors {P.scale}): worst parameter rel err {worst:.3e} (tol {H.TOL[cfg.dtype]})")
    ctx.close()


@pytest.mark.parametrize("name", ["cfg1", "ragged-f32", "ragged-bf16", "cfg3-small", "cfg4-small", "cfg5-small",
                                  "csr-f32", "wide-out-f32", "deep-bf16", "width-one-blocks-f32", "cfg1-nobias-S1",
                                  "uneven-S3-f32", "uneven-S5-bf16", "uneven-S7-csr-bf16"])
def test_resample_equals_merge_then_partition(name):
    """ist_resample against the oracle: from the trained subnets as exported, the oracle's merge gives the
    full network and the oracle's partition by the next permutation gives the new subnets; both must come
    out of ist_resample bit for bit (Section 2.1: subnets are re-sampled after every J local iterations).
    Twice in a row (the two subnet buffers change roles).  A second context doing ist_merge followed by
    ist_partition must agree as well, and training continues identically afterwards."""
    cfg = SHAPES[name]
    has_bias = "nobias" not in name
    P = H.Problem(cfg, has_bias=has_bias, dev=_dev())
    a, b = P.context(), P.context()
    Wa, Wb = [w.clone() for w in P.dW], [w.clone() for w in P.dW]
    ba = [x.clone() for x in P.db] if has_bias else None
    bb = [x.clone() for x in P.db] if has_bias else None
    a.partition(Wa, ba, P.dperm)
    b.partition(Wb, bb, P.dperm)
    full_W = [H.np_bits(w, cfg.dtype).copy() for w in P.Ws]               # the oracle's full network, raw bits
    full_b = [x.astype(np.float32).copy() for x in P.bs] if has_bias else None
    old_perms = P.perms
    for rnd in (1, 2):
        P.gpu_steps(a, loss=False)
        P.gpu_steps(b, loss=False)
        trained = H.export_all(a, cfg)
        new_perms = gen.make_perms(cfg, rnd)
        perm = [torch.from_numpy(p).to(_dev()) for p in new_perms]
        a.profile_enable(True)
        a.profile_reset()
        a.resample(Wa, ba, perm)
        labels = {k["label"] for k in a.profile_kernels()}
        a.profile_enable(False)
        if name in ("cfg1", "cfg3-small", "cfg4-small"):   # aligned shapes take the one-pass kernels
            assert {"k_resample_rows", "k_resample_mid"} <= labels, labels
        # ---- the oracle's merge of the trained subnets, then its partition by the new permutation ----
        typed = [([H.bits(w) for w in Wl], None) for Wl, _ in trained]
        orc.merge(full_W, None, old_perms, cfg.S, typed)
        if has_bias:
            dummy = [np.zeros(w.shape, dtype=np.float32) for w in P.Ws]
            f32subs = [([H.to_f32(w) for w in Wl], [H.to_f32(x) for x in bl]) for Wl, bl in trained]
            orc.merge(dummy, full_b, old_perms, cfg.S, f32subs, mode=cfg.dtype)
        raw_b = [H.np_bits(x, cfg.dtype) for x in full_b] if has_bias else [None] * cfg.t
        want = orc.partition(full_W, raw_b, new_perms, cfg.S)
        torch.cuda.synchronize()
        for l in range(cfg.t):
            assert np.array_equal(H.bits(Wa[l]), full_W[l]), (name, rnd, l, "merged weights vs oracle")
            if has_bias:
                assert np.array_equal(H.bits(ba[l]), raw_b[l]), (name, rnd, l, "merged bias vs oracle")
        ga = H.export_all(a, cfg)
        for s in range(cfg.S):
            for l in range(cfg.t):
                assert np.array_equal(H.bits(ga[s][0][l]), want[s][0][l]), (name, rnd, s, l, "new subnet weights vs oracle")
                if has_bias:
                    assert np.array_equal(H.bits(ga[s][1][l]), want[s][1][l]), (name, rnd, s, l, "new subnet bias vs oracle")
        old_perms = new_perms
        # ---- and the two separate calls ----
        b.merge(Wb, bb)
        b.partition(Wb, bb, perm)
        torch.cuda.synchronize()
        for l in range(cfg.t):
            assert torch.equal(Wa[l], Wb[l]), (name, rnd, l, "merged weights")
            if has_bias:
                assert torch.equal(ba[l], bb[l]), (name, rnd, l, "merged bias")
        gb = H.export_all(b, cfg)
        for s in range(cfg.S):
            for l in range(cfg.t):
                assert torch.equal(ga[s][0][l], gb[s][0][l]), (name, rnd, s, l, "new subnet weights")
                if has_bias:
                    assert torch.equal(ga[s][1][l], gb[s][1][l]), (name, rnd, s, l, "new subnet bias")
    a.close()
    b.close()


def test_resample_rejects_a_bad_permutation_and_keeps_its_state():
    from paper_1910_02120_amd import ISTError
    cfg = SHAPES["ragged-f32"]
    P = H.Problem(cfg, dev=_dev())
    ctx = P.context()
    W, bsv = [w.clone() for w in P.dW], [x.clone() for x in P.db]
    ctx.set_checked(True)
    ctx.partition(W, bsv, P.dperm)
    P.gpu_steps(ctx, loss=False)
    before = H.export_all(ctx, cfg)
    W0 = [w.clone() for w in W]
    bad = [p.clone() for p in P.dperm]
    bad[0][1] = bad[0][2]
    with pytest.raises(ISTError) as e:
        ctx.resample(W, bsv, bad)
    assert e.value.status == -3
    after = H.export_all(ctx, cfg)
    for l in range(cfg.t):
        assert torch.equal(W[l], W0[l])
        for s in range(cfg.S):
            assert torch.equal(before[s][0][l], after[s][0][l])
    ctx.resample(W, bsv, P.dperm)          # and a good one still works
    ctx.close()
