"""Pins for the per-neuron standardisation of Section 2.2 ("Correcting Distributional
Shift") in the oracle's local SGD: library batch normalisation with autograd, central
finite differences of an independently written loss, and properties that follow from the
definition (standardised activations, invariance to row scaling and bias shifts, zero bias
gradient of hidden layers)."""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

EPS = orc.NORM_EPS


def _cfg(dims, S, B=6, k=3, dtype="f32", lr=0.1):
    return gen.ISTConfig("t", 1, tuple(dims), S=S, B=B, k=k, rounds=1, dtype=dtype, lr=lr)


def _np_loss(Ws, bs, X, y, eps=EPS):
    """Independent formula with NumPy's mean / var (biased) per hidden neuron over the batch."""
    h = X.astype(np.float64)
    t = len(Ws)
    for l in range(1, t + 1):
        z = h @ Ws[l - 1].T + (bs[l - 1] if bs is not None else 0.0)
        if l < t:
            z = (z - z.mean(axis=0)) / np.sqrt(z.var(axis=0) + eps)
            h = np.maximum(z, 0.0)
        else:
            z = z - z.max(axis=1, keepdims=True)
            return float(np.mean(np.log(np.exp(z).sum(axis=1)) - z[np.arange(len(y)), y]))
    raise AssertionError


def _subnets(cfg, bias_scale=0.2, spread=0.3, seed=3):
    Ws, bs = gen.make_weights(cfg, bias_scale=bias_scale)
    subs = orc.to_f64(orc.partition(Ws, bs, gen.make_perms(cfg), cfg.S))
    rng = np.random.default_rng(seed)
    for Wl, _ in subs:
        for w in Wl:
            w += spread * rng.standard_normal(w.shape)
    return subs


def test_k_steps_match_torch_batch_norm_autograd():
    cfg = _cfg((9, 12, 8, 5), S=2, B=7, k=4, lr=0.2)
    X, y = gen.make_dense_batches(cfg)
    for s, (Wl, bl) in enumerate(_subnets(cfg)):
        tw = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Wl]
        tb = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in bl]
        tl = []
        for j in range(cfg.k):
            h = torch.tensor(X[s, j], dtype=torch.float64)
            for l in range(cfg.t):
                h = h @ tw[l].T + tb[l]
                if l < cfg.t - 1:
                    h = torch.nn.functional.batch_norm(h, None, None, training=True, eps=EPS)
                    h = torch.relu(h)
            loss = torch.nn.functional.cross_entropy(h, torch.tensor(y[s, j], dtype=torch.long))
            tl.append(float(loss.detach()))
            grads = torch.autograd.grad(loss, tw + tb)
            with torch.no_grad():
                for p, g in zip(tw + tb, grads):
                    p -= float(np.float32(cfg.lr)) * g
        loss = orc.subnet_sgd(Wl, bl, y[s], cfg.lr, cfg.k, "exact", X=X[s], normalize=True)
        np.testing.assert_allclose(loss, tl, rtol=1e-11)
        for a, b in zip(Wl + bl, tw + tb):
            np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-9, atol=1e-11)


def test_finite_difference_gradients_through_the_statistics():
    cfg = _cfg((5, 8, 6, 4), S=2, B=9, k=1)
    X, y = gen.make_dense_batches(cfg)
    rng = np.random.default_rng(5)
    for s, (Wl, bl) in enumerate(_subnets(cfg)):
        ref = ([w.copy() for w in Wl], [v.copy() for v in bl])
        orc.subnet_sgd(Wl, bl, y[s, :1], 1.0, 1, "exact", X=X[s, :1], normalize=True)
        h = 1e-6
        for p0, p1 in [(ref[0][i], Wl[i]) for i in range(cfg.t)] + [(ref[1][i], bl[i]) for i in range(cfg.t)]:
            grad = (p0 - p1).reshape(-1)              # lr = 1
            flat = p0.reshape(-1)
            for idx in rng.choice(flat.size, size=min(10, flat.size), replace=False):
                keep = flat[idx]
                flat[idx] = keep + h
                lp = _np_loss(ref[0], ref[1], X[s, 0], y[s, 0])
                flat[idx] = keep - h
                lm = _np_loss(ref[0], ref[1], X[s, 0], y[s, 0])
                flat[idx] = keep
                fd = (lp - lm) / (2 * h)
                assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(fd)), (fd, grad[idx])


def test_loss_equals_the_numpy_definition_and_differs_from_the_plain_net():
    cfg = _cfg((7, 10, 6, 3), S=2, B=8, k=1)
    X, y = gen.make_dense_batches(cfg)
    for s, (Wl, bl) in enumerate(_subnets(cfg)):
        W0, b0 = [w.copy() for w in Wl], [v.copy() for v in bl]
        ln = orc.subnet_sgd([w.copy() for w in W0], [v.copy() for v in b0], y[s, :1], 0.0, 1, "exact",
                            X=X[s, :1], normalize=True)[0]
        lp = orc.subnet_sgd([w.copy() for w in W0], [v.copy() for v in b0], y[s, :1], 0.0, 1, "exact",
                            X=X[s, :1])[0]
        assert abs(ln - _np_loss(W0, b0, X[s, 0], y[s, 0])) < 1e-13
        assert abs(ln - lp) > 1e-3


def test_invariance_to_row_scaling_and_bias_shift_and_zero_hidden_bias_gradient():
    """Standardisation removes a positive scale of a neuron's input row and any shift of its
    bias (up to eps): the loss does not move, and hidden biases receive no gradient."""
    cfg = _cfg((6, 8, 4), S=1, B=16, k=1)
    X, y = gen.make_dense_batches(cfg)
    (Wl, bl), = _subnets(cfg, spread=0.5)
    run = lambda W, b, lr=0.0: orc.subnet_sgd(W, b, y[0, :1], lr, 1, "exact", X=X[0, :1], normalize=True,
                                              eps=1e-14)[0]
    base = run([w.copy() for w in Wl], [v.copy() for v in bl])
    rng = np.random.default_rng(9)
    W2, b2 = [w.copy() for w in Wl], [v.copy() for v in bl]
    scale = rng.uniform(0.5, 3.0, W2[0].shape[0])
    W2[0] *= scale[:, None]
    b2[0] = b2[0] * scale + rng.standard_normal(b2[0].shape)
    assert abs(run(W2, b2) - base) < 1e-9
    W3, b3 = [w.copy() for w in Wl], [v.copy() for v in bl]
    run(W3, b3, lr=1.0)
    np.testing.assert_allclose(b3[0], bl[0], atol=1e-12)        # d loss / d b_1 = 0
    assert np.abs(b3[1] - bl[1]).max() > 1e-4                   # the output bias does move


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_storage_emulation_stays_close_to_exact(mode):
    cfg = _cfg((12, 16, 16, 5), S=2, B=10, k=3, dtype=mode, lr=0.05)
    X, y = gen.make_dense_batches(cfg)
    X = gen.quantize(X, mode)
    for s, (Wl, bl) in enumerate(_subnets(cfg, spread=0.1)):
        Wq = [gen.quantize(w, mode).astype(np.float64) for w in Wl]
        bq = [gen.quantize(v, mode).astype(np.float64) for v in bl]
        We, be = [w.copy() for w in Wq], [v.copy() for v in bq]
        orc.subnet_sgd(We, be, y[s], cfg.lr, cfg.k, "exact", X=X[s].astype(np.float64), normalize=True)
        orc.subnet_sgd(Wq, bq, y[s], cfg.lr, cfg.k, mode, X=X[s].astype(np.float64), normalize=True)
        tol = 1e-5 if mode == "f32" else 3e-2
        for a, b in zip(Wq, We):
            assert np.max(np.abs(a - b)) <= tol * np.max(np.abs(b))
            assert np.array_equal(gen.quantize(a, mode).astype(np.float64), a)   # representable
