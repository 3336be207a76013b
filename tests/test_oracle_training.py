"""Pins for the oracle's local SGD (Section 2.1 "Training Subnets", Appendix B).

The oracle is checked against things that are not the oracle: closed forms at
zero weights, central finite differences of an independently written loss,
PyTorch CPU autograd, a hand-written NumPy full-network SGD step (S = 1), the
masked-full-network definition of Appendix A, and invariants (independence of
subnets, representability of stored values).
"""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc


def _cfg(dims, S, B=6, k=3, dtype="f32", lr=0.1):
    return gen.ISTConfig("t", 1, tuple(dims), S=S, B=B, k=k, rounds=1, dtype=dtype, lr=lr)


def _np_forward_loss(Ws, bs, X, y, masks=None):
    """Independent formula: full network, optional 0/1 masks on hidden layers."""
    h = X.astype(np.float64)
    t = len(Ws)
    for l in range(1, t + 1):
        z = h @ Ws[l - 1].astype(np.float64).T
        if bs is not None and bs[l - 1] is not None:
            z = z + bs[l - 1].astype(np.float64)
        if l < t:
            h = np.maximum(z, 0.0)
            if masks is not None:
                h = h * masks[l - 1]
        else:
            z = z - z.max(axis=1, keepdims=True)
            lse = np.log(np.exp(z).sum(axis=1))
            return float(np.mean(lse - z[np.arange(len(y)), y])), z
    raise AssertionError


def test_zero_weights_closed_form():
    """W = 0: softmax is uniform, loss = ln C, and one step moves the last bias by
    -lr (1/C - onehot) averaged over the batch while all weights stay zero."""
    n0, n1, Cc, B = 5, 4, 7, 8
    rng = np.random.default_rng(1)
    X = rng.standard_normal((1, B, n0))
    y = rng.integers(0, Cc, (1, B)).astype(np.int32)
    W = [np.zeros((n1, n0)), np.zeros((Cc, n1))]
    b = [np.zeros(n1), np.zeros(Cc)]
    loss = orc.subnet_sgd(W, b, y, 0.5, 1, "exact", X=X)
    assert abs(loss[0] - np.log(Cc)) < 1e-14
    onehot = np.eye(Cc)[y[0]]
    np.testing.assert_allclose(b[1], -0.5 * (1.0 / Cc - onehot).mean(axis=0), atol=1e-15)
    assert not W[0].any() and not W[1].any() and not b[0].any()


def test_softmax_regression_closed_form():
    """t = 1 (no hidden layer): dW = (softmax - onehot)^T X / B written out."""
    n0, Cc, B = 6, 4, 9
    rng = np.random.default_rng(2)
    X = rng.standard_normal((1, B, n0))
    y = rng.integers(0, Cc, (1, B)).astype(np.int32)
    W0 = rng.standard_normal((Cc, n0)) * 0.3
    b0 = rng.standard_normal(Cc) * 0.1
    W, b = [W0.copy()], [b0.copy()]
    orc.subnet_sgd(W, b, y, 0.25, 1, "exact", X=X)
    z = X[0] @ W0.T + b0
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    g = (p - np.eye(Cc)[y[0]]) / B
    np.testing.assert_allclose(W[0], W0 - 0.25 * g.T @ X[0], atol=1e-14)
    np.testing.assert_allclose(b[0], b0 - 0.25 * g.sum(0), atol=1e-14)


@pytest.mark.parametrize("with_bias", [True, False])
def test_finite_difference_gradients(with_bias):
    cfg = _cfg((5, 8, 6, 4), S=2, B=7, k=1)
    Ws, bs = gen.make_weights(cfg, with_bias=with_bias, bias_scale=0.2)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    subs = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    rng = np.random.default_rng(3)
    for s in range(cfg.S):
        Wl, bl = subs[s]
        for w in Wl:                              # move away from the Xavier start
            w += 0.3 * rng.standard_normal(w.shape)
        ref = ([w.copy() for w in Wl], [None if v is None else v.copy() for v in bl])
        orc.subnet_sgd(Wl, bl if with_bias else None, y[s, :1], 1.0, 1, "exact", X=X[s, :1])
        params = [(ref[0][i], Wl[i]) for i in range(cfg.t)]
        if with_bias:
            params += [(ref[1][i], bl[i]) for i in range(cfg.t)]
        eps = 1e-6
        for p0, p1 in params:
            grad = p0 - p1                         # lr = 1
            flat = p0.reshape(-1)
            for idx in rng.choice(flat.size, size=min(12, flat.size), replace=False):
                keep = flat[idx]
                flat[idx] = keep + eps
                lp, _ = _np_forward_loss(ref[0], ref[1] if with_bias else None, X[s, 0], y[s, 0])
                flat[idx] = keep - eps
                lm, _ = _np_forward_loss(ref[0], ref[1] if with_bias else None, X[s, 0], y[s, 0])
                flat[idx] = keep
                fd = (lp - lm) / (2 * eps)
                assert abs(fd - grad.reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(fd)), (fd, grad.reshape(-1)[idx])


def test_k_steps_match_torch_autograd():
    cfg = _cfg((9, 12, 8, 5), S=2, B=6, k=4, lr=0.2)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    subs = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    for s in range(cfg.S):
        Wl, bl = subs[s]
        tw = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Wl]
        tb = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in bl]
        tl = []
        for j in range(cfg.k):
            h = torch.tensor(X[s, j], dtype=torch.float64)
            for l in range(cfg.t):
                h = h @ tw[l].T + tb[l]
                if l < cfg.t - 1:
                    h = torch.relu(h)
            loss = torch.nn.functional.cross_entropy(h, torch.tensor(y[s, j], dtype=torch.long))
            tl.append(float(loss.detach()))
            grads = torch.autograd.grad(loss, tw + tb)
            with torch.no_grad():
                for p, g in zip(tw + tb, grads):
                    p -= float(np.float32(cfg.lr)) * g
        loss = orc.subnet_sgd(Wl, bl, y[s], cfg.lr, cfg.k, "exact", X=X[s])
        np.testing.assert_allclose(loss, tl, rtol=1e-12)
        for a, b in zip(Wl + bl, tw + tb):
            np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-11, atol=1e-13)


def test_S1_round_is_a_full_network_sgd_step():
    cfg = _cfg((7, 10, 6, 3), S=1, B=5, k=1, lr=0.3)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    Ws = [w.astype(np.float64) for w in Ws]
    bs = [b.astype(np.float64) for b in bs]
    perms = [np.arange(cfg.dims[l], dtype=np.int32) for l in range(1, cfg.t)]
    X, y = gen.make_dense_batches(cfg)
    # hand-written full-network back-propagation
    x = X[0, 0].astype(np.float64)
    h1 = np.maximum(x @ Ws[0].T + bs[0], 0)
    h2 = np.maximum(h1 @ Ws[1].T + bs[1], 0)
    z = h2 @ Ws[2].T + bs[2]
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    g3 = (p - np.eye(cfg.dims[-1])[y[0, 0]]) / cfg.B
    g2 = (g3 @ Ws[2]) * (h2 > 0)
    g1 = (g2 @ Ws[1]) * (h1 > 0)
    lr = float(np.float32(cfg.lr))
    want_W = [Ws[0] - lr * g1.T @ x, Ws[1] - lr * g2.T @ h1, Ws[2] - lr * g3.T @ h2]
    want_b = [bs[0] - lr * g1.sum(0), bs[1] - lr * g2.sum(0), bs[2] - lr * g3.sum(0)]
    orc.ist_round(Ws, bs, perms, 1, cfg.lr, 1, "exact", y, X=X)
    for a, b in zip(Ws, want_W):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    for a, b in zip(bs[:-1], want_b[:-1]):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    # the output bias passes through the binary32 mean of the merge
    np.testing.assert_allclose(bs[-1], want_b[-1], rtol=0, atol=1e-7)
    # a random permutation with S = 1 gives the same step (neuron order is immaterial)
    Ws2, bs2 = gen.make_weights(cfg, bias_scale=0.1)
    Ws2 = [w.astype(np.float64) for w in Ws2]
    bs2 = [b.astype(np.float64) for b in bs2]
    orc.ist_round(Ws2, bs2, gen.make_perms(cfg), 1, cfg.lr, 1, "exact", y, X=X)
    for a, b in zip(Ws2, want_W):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


@pytest.mark.parametrize("dims,S", [((6, 12, 8, 5), 4), ((6, 13, 7, 5), 4), ((5, 11, 9, 3), 3)])
def test_subnet_equals_masked_full_network(dims, S):
    """Subnet loss = loss of the full network with every hidden neuron outside the
    subnet zeroed (Appendix A without the n^2 factor); also with blocks of unequal width."""
    cfg = _cfg(dims, S=S, B=9, k=1)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.3)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    subs = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    for s in range(cfg.S):
        masks = []
        for l in range(1, cfg.t):
            # membership from the split of the permutation a library routine makes
            m = np.zeros(cfg.dims[l])
            m[np.array_split(perms[l - 1], cfg.S)[s]] = 1.0
            masks.append(m)
        want, _ = _np_forward_loss(Ws, bs, X[s, 0], y[s, 0], masks)
        got = orc.subnet_sgd(*subs[s], y[s, :1], 0.0, 1, "exact", X=X[s, :1])[0]
        assert abs(got - want) < 1e-13


@pytest.mark.parametrize("normalize", [False, True])
@pytest.mark.parametrize("mode", ["exact", "f32", "bf16"])
def test_a_neuron_with_zero_parameters_is_inert(mode, normalize):
    """A hidden neuron whose incoming weights, bias and outgoing weights are all zero outputs ReLU(0) = 0,
    receives no gradient and passes none on: training a subnet with such neurons appended to its hidden
    layers leaves the real parameters exactly as training the subnet alone, and the added ones at zero.
    (What a device may rely on to keep blocks of unequal width in arrays of one common size.)"""
    cfg = _cfg((7, 5, 4, 6), S=1, B=8, k=4, dtype="bf16" if mode == "bf16" else "f32", lr=0.3)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.2)
    X, y = gen.make_dense_batches(cfg)
    Wa = [w.astype(np.float64) for w in Ws]
    ba = [b.astype(np.float64) for b in bs]
    pad = [0, 2, 1, 0]                                    # extra neurons per layer (hidden layers only)
    Wb = [np.zeros((w.shape[0] + pad[l + 1], w.shape[1] + pad[l])) for l, w in enumerate(Wa)]
    bb = [np.zeros(b.shape[0] + pad[l + 1]) for l, b in enumerate(ba)]
    for l in range(cfg.t):
        Wb[l][:Wa[l].shape[0], :Wa[l].shape[1]] = Wa[l]
        bb[l][:ba[l].shape[0]] = ba[l]
    la = orc.subnet_sgd(Wa, ba, y[0], cfg.lr, cfg.k, mode, X=X[0], normalize=normalize)
    lb = orc.subnet_sgd(Wb, bb, y[0], cfg.lr, cfg.k, mode, X=X[0], normalize=normalize)
    assert la.tobytes() == lb.tobytes()
    for l in range(cfg.t):
        r, c = Wa[l].shape
        assert Wb[l][:r, :c].tobytes() == Wa[l].tobytes() and bb[l][:r].tobytes() == ba[l].tobytes()
        assert not Wb[l][r:, :].any() and not Wb[l][:, c:].any() and not bb[l][r:].any()


def test_one_hidden_layer_subnet_logits_sum_to_full_network():
    """With one hidden layer and no output bias the subnets' logits add up to the
    full network's (the separability noted in Section 3.3)."""
    cfg = _cfg((6, 12, 5), S=3, B=4, k=1)
    Ws, _ = gen.make_weights(cfg, with_bias=False)
    perms = gen.make_perms(cfg)
    X, _y = gen.make_dense_batches(cfg)
    x = X[0, 0].astype(np.float64)
    full = np.maximum(x @ Ws[0].T, 0) @ Ws[1].T
    H = orc.blocks(perms, cfg.S)
    tot = 0
    for s in range(cfg.S):
        W1 = orc.gather(Ws[0], H[0][s], None).astype(np.float64)
        W2 = orc.gather(Ws[1], None, H[0][s]).astype(np.float64)
        tot = tot + np.maximum(x @ W1.T, 0) @ W2.T
    np.testing.assert_allclose(tot, full, atol=1e-12)


def test_subnets_are_independent():
    cfg = _cfg((6, 8, 8, 4), S=2, B=5, k=3)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    a = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    orc.subnet_steps(a, cfg.lr, cfg.k, "f32", y, X=X)
    X2 = X.copy()
    X2[1] += 1.0
    b = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    for w in b[1][0]:
        w *= 2.0
    orc.subnet_steps(b, cfg.lr, cfg.k, "f32", y, X=X2)
    for u, v in zip(a[0][0] + a[0][1], b[0][0] + b[0][1]):
        assert u.tobytes() == v.tobytes()
    assert any(u.tobytes() != v.tobytes() for u, v in zip(a[1][0], b[1][0]))


def test_csr_path_equals_dense_path():
    cfg = gen.ISTConfig("t", 5, (40, 8, 11), S=2, B=6, k=3, rounds=1, dtype="f32",
                        input="csr", nnz_per_row=5, label_dist="zipf", lr=0.2)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    perms = gen.make_perms(cfg)
    rp, ci, va, y = gen.make_csr_batches(cfg)
    Xd = gen.csr_to_dense(rp, ci, va, cfg.dims[0]).reshape(cfg.S, cfg.k, cfg.B, -1)
    a = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    la = orc.subnet_steps(a, cfg.lr, cfg.k, "exact", y, csr=(rp, ci, va.astype(np.float64)))
    b = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    lb = orc.subnet_steps(b, cfg.lr, cfg.k, "exact", y, X=Xd)
    np.testing.assert_allclose(la, lb, rtol=1e-13)
    for s in range(cfg.S):
        for u, v in zip(a[s][0] + a[s][1], b[s][0] + b[s][1]):
            np.testing.assert_allclose(u, v, rtol=0, atol=1e-14)
    # generator contract the CSR consumers rely on
    for r in range(len(rp) - 1):
        c = ci[rp[r]:rp[r + 1]]
        assert len(c) >= 1 and np.all(np.diff(c) > 0)
        assert abs(np.sum(va[rp[r]:rp[r + 1]].astype(np.float64) ** 2) - 1.0) < 1e-6


def test_rounding_matches_library_conversions():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-30, 30, 4000),
                        [1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 2.0 ** -127 * 1.5,
                         2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134, 0.0]])
    x32 = x.astype(np.float32).astype(np.float64)          # exactly representable in binary32
    want = torch.tensor(x32, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([orc.round_store(v, "bf16") for v in x32])
    assert np.array_equal(got, want)
    got32 = np.array([orc.round_store(v, "f32") for v in x])
    assert np.array_equal(got32, x.astype(np.float32).astype(np.float64))
    assert np.array_equal(gen.from_bf16_bits(gen.to_bf16_bits(x32.astype(np.float32))).astype(np.float64),
                          want)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_storage_emulation_keeps_values_representable_and_close(mode):
    cfg = _cfg((16, 24, 16, 6), S=2, B=8, k=4, dtype=mode, lr=0.1)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    e = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    orc.subnet_steps(e, cfg.lr, cfg.k, "exact", y, X=X)
    m = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    orc.subnet_steps(m, cfg.lr, cfg.k, mode, y, X=X)
    tol = 1e-5 if mode == "f32" else 3e-2
    for s in range(cfg.S):
        for u, v in zip(m[s][0] + m[s][1], e[s][0] + e[s][1]):
            assert np.array_equal(gen.quantize(u.astype(np.float32), mode).astype(np.float64), u)
            assert np.max(np.abs(u - v)) <= tol * np.max(np.abs(v))


def test_loss_decreases_on_a_learnable_problem():
    cfg = _cfg((16, 32, 32, 4), S=2, B=64, k=1, lr=0.5)
    Ws, bs = gen.make_weights(cfg)
    perms = gen.make_perms(cfg)
    X, y = gen.make_dense_batches(cfg)
    Xr = np.repeat(X, 30, axis=1)
    yr = np.repeat(y, 30, axis=1)
    subs = orc.to_f64(orc.partition(Ws, bs, perms, cfg.S))
    loss = orc.subnet_steps(subs, cfg.lr, 30, "exact", yr, X=Xr)
    assert np.all(loss[:, -1] < 0.7 * loss[:, 0])
