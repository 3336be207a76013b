"""Pins for the scaled subnet forward pass of Appendix A (equation (4): the product of a layer
whose two sides are both partitioned is multiplied by n^2): the unbiasedness of each subnet's
scaled masked product, by exhaustive enumeration over every pair of layer partitions of tiny
layers in exact integer arithmetic (and what that implies for the sum over subnets); library autograd for the k-step recursion with per-layer factors; and the identity
that a uniform factor is plain SGD on rescaled weights."""
import itertools

import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc


def _cfg(dims, S, B=6, k=3, dtype="f32", lr=0.1):
    return gen.ISTConfig("t", 1, tuple(dims), S=S, B=B, k=k, rounds=1, dtype=dtype, lr=lr)


@pytest.mark.parametrize("N,S", [(4, 2), (3, 3)])
def test_scaled_masked_product_of_each_subnet_is_unbiased_by_enumeration(N, S):
    """Equation (4): f^(s)_l = n^2 m_l^s . (W_l (m_{l-1}^s . f)).  Over the independent uniform
    partitions of layers l-1 and l, P[m_{l,j}^s m_{l-1,i}^s = 1] = 1/n^2, so E f^(s)_l = W_l f for
    every single subnet s.  Their sum over the n subnets therefore has expectation n W_l f (an
    output neuron meets an input neuron in its own subnet with probability 1/n): the closing
    step of the appendix, which equates the sum with W_l f, holds with the factor n instead.
    Non-negative integers keep the ReLU of the read-out inactive and the arithmetic exact."""
    rng = np.random.default_rng(N * 10 + S)
    W = rng.integers(0, 6, size=(N, N)).astype(np.float64)
    f = rng.integers(0, 5, size=N).astype(np.float64)
    per_subnet = np.zeros((S, N))
    unscaled = np.zeros((S, N))
    count = 0
    for p_in in itertools.permutations(range(N)):
        for p_out in itertools.permutations(range(N)):
            p_in_a, p_out_a = np.array(p_in, dtype=np.int32), np.array(p_out, dtype=np.int32)
            for s in range(S):
                Hin, Hout = orc.block(p_in_a, S, s), orc.block(p_out_a, S, s)
                Ws = orc.gather(W, Hout, Hin)
                eye = np.eye(len(Hout))
                per_subnet[s, Hout] += orc.forward_full([Ws, eye], None, "exact", X=f[Hin][None, :],
                                                        scale=[float(S * S), 1.0])[0]
                unscaled[s, Hout] += orc.forward_full([Ws, eye], None, "exact", X=f[Hin][None, :])[0]
            count += 1
    for s in range(S):
        assert np.array_equal(per_subnet[s], count * (W @ f))
        # the factor is needed: without it a subnet's estimate is short by exactly n^2
        assert np.array_equal(unscaled[s] * S * S, count * (W @ f))
    # gathered over the subnets: n W f with the factor n^2, W f with the factor n
    assert np.array_equal(per_subnet.sum(axis=0), S * count * (W @ f))
    assert np.array_equal(unscaled.sum(axis=0) * S, count * (W @ f))


@pytest.mark.parametrize("normalize", [False, True])
def test_k_scaled_steps_match_torch_autograd(normalize):
    cfg = _cfg((9, 12, 8, 5), S=2, B=7, k=4, lr=0.05)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.2)
    X, y = gen.make_dense_batches(cfg)
    scale = [1.0, 4.0, 0.5]
    subs = orc.to_f64(orc.partition(Ws, bs, gen.make_perms(cfg), cfg.S))
    for s, (Wl, bl) in enumerate(subs):
        tw = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Wl]
        tb = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in bl]
        tl = []
        for j in range(cfg.k):
            h = torch.tensor(X[s, j], dtype=torch.float64)
            for l in range(cfg.t):
                h = scale[l] * (h @ tw[l].T) + tb[l]
                if l < cfg.t - 1:
                    if normalize:
                        h = torch.nn.functional.batch_norm(h, None, None, training=True, eps=orc.NORM_EPS)
                    h = torch.relu(h)
            loss = torch.nn.functional.cross_entropy(h, torch.tensor(y[s, j], dtype=torch.long))
            tl.append(float(loss.detach()))
            grads = torch.autograd.grad(loss, tw + tb)
            with torch.no_grad():
                for p, g in zip(tw + tb, grads):
                    p -= float(np.float32(cfg.lr)) * g
        loss = orc.subnet_sgd(Wl, bl, y[s], cfg.lr, cfg.k, "exact", X=X[s], normalize=normalize, scale=scale)
        np.testing.assert_allclose(loss, tl, rtol=1e-10)
        for l in range(cfg.t):
            np.testing.assert_allclose(Wl[l], tw[l].detach().numpy(), rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(bl[l], tb[l].detach().numpy(), rtol=1e-9, atol=1e-12)


def test_uniform_factor_is_plain_sgd_on_rescaled_weights():
    """Without biases, z_l = g W_l h is the plain network with weights g W_l; one step of the scaled
    net with rate lr moves g W_l by lr g^2 times the plain gradient."""
    cfg = _cfg((8, 10, 6, 4), S=1, B=5, k=1)
    Ws, _ = gen.make_weights(cfg, with_bias=False)
    X, y = gen.make_dense_batches(cfg)
    g = 3.0
    lr = float(np.float32(0.01))
    A = [np.ascontiguousarray(w, dtype=np.float64) for w in Ws]
    Bw = [g * np.ascontiguousarray(w, dtype=np.float64) for w in Ws]
    la = orc.subnet_sgd(A, None, y[0], lr, 1, "exact", X=X[0], scale=[g] * cfg.t)
    lb = orc.subnet_sgd(Bw, None, y[0], float(np.float32(lr * g * g)), 1, "exact", X=X[0])
    assert abs(la[0] - lb[0]) < 1e-12
    ratio = float(np.float32(lr * g * g)) / (lr * g * g)     # the rate is rounded to binary32 once
    for l in range(cfg.t):
        moved_a = g * A[l] - g * np.asarray(Ws[l], dtype=np.float64)
        moved_b = Bw[l] - g * np.asarray(Ws[l], dtype=np.float64)
        np.testing.assert_allclose(moved_a * ratio, moved_b, rtol=1e-9, atol=1e-15)


@pytest.mark.parametrize("mode", ["f32", "bf16"])
def test_factors_of_one_change_nothing(mode):
    cfg = _cfg((8, 12, 6, 4), S=2, B=5, k=3, dtype=mode)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    X, y = gen.make_dense_batches(cfg)
    a = orc.to_f64(orc.partition(Ws, bs, gen.make_perms(cfg), cfg.S))
    b = orc.to_f64(orc.partition(Ws, bs, gen.make_perms(cfg), cfg.S))
    la = orc.subnet_steps(a, cfg.lr, cfg.k, mode, y, X=X)
    lb = orc.subnet_steps(b, cfg.lr, cfg.k, mode, y, X=X, scale=[1.0] * cfg.t)
    assert np.array_equal(la, lb)
    for (Wa, ba), (Wb, bb) in zip(a, b):
        for l in range(cfg.t):
            assert np.array_equal(Wa[l], Wb[l]) and np.array_equal(ba[l], bb[l])
