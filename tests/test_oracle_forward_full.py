"""Pins for the oracle's full-network forward pass (Section 2.1: the network the subnets are cut
from; Section 2.2 for the standardised variant): library layers in float64, the pinned local-SGD
oracle with S = 1 (whose first loss is the cross-entropy of these logits, in every storage mode),
the masked-sum identity that ties the full first layer to the subnets' first layers, a
hand-computed 2-2-2 network, and the CSR input against its dense expansion."""
import numpy as np
import pytest
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc


def _cfg(dims, S=2, B=6, k=1, dtype="f32", **kw):
    return gen.ISTConfig("t", 1, tuple(dims), S=S, B=B, k=k, rounds=1, dtype=dtype, lr=0.1, **kw)


def _xent(logits, y):
    z = logits - logits.max(axis=1, keepdims=True)
    return float(np.mean(np.log(np.exp(z).sum(axis=1)) - z[np.arange(len(y)), y]))


def test_hand_computed_two_layer_network():
    # x = (1, -2); W1 = [[1, 0], [2, 1]], b1 = (0.5, -1): z1 = (1.5, -1) -> f1 = (1.5, 0)
    # W2 = [[2, -1], [0, 3]], b2 = (1, 1): logits = (4, 1)
    W = [np.array([[1.0, 0.0], [2.0, 1.0]]), np.array([[2.0, -1.0], [0.0, 3.0]])]
    b = [np.array([0.5, -1.0]), np.array([1.0, 1.0])]
    out = orc.forward_full(W, b, "exact", X=np.array([[1.0, -2.0]]))
    assert np.array_equal(out, np.array([[4.0, 1.0]]))


@pytest.mark.parametrize("normalize", [False, True])
def test_matches_torch_layers_in_float64(normalize):
    cfg = _cfg((11, 16, 12, 7), B=9)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.3)
    X, _ = gen.make_dense_batches(cfg)
    x = X[0, 0]
    h = torch.tensor(x, dtype=torch.float64)
    for l in range(cfg.t):
        h = torch.nn.functional.linear(h, torch.tensor(Ws[l], dtype=torch.float64),
                                       torch.tensor(bs[l], dtype=torch.float64))
        if l < cfg.t - 1:
            if normalize:
                h = torch.nn.functional.batch_norm(h, None, None, training=True, eps=orc.NORM_EPS)
            h = torch.relu(h)
    got = orc.forward_full(Ws, bs, "exact", X=x, normalize=normalize)
    np.testing.assert_allclose(got, h.numpy(), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("mode", ["exact", "f32", "bf16"])
@pytest.mark.parametrize("normalize", [False, True])
def test_first_loss_of_local_sgd_with_one_subnet(mode, normalize):
    """With S = 1 the subnet is the full network: the loss the SGD oracle reports for its first
    step (before any update) is the mean cross-entropy of forward_full's logits, with the
    activations rounded at the same places."""
    cfg = _cfg((10, 12, 8, 5), S=1, B=7, dtype="bf16" if mode == "bf16" else "f32")
    Ws, bs = gen.make_weights(cfg, bias_scale=0.2)
    X, y = gen.make_dense_batches(cfg)
    W64 = [np.ascontiguousarray(w, dtype=np.float64) for w in Ws]
    b64 = [np.ascontiguousarray(v, dtype=np.float64) for v in bs]
    logits = orc.forward_full(W64, b64, mode, X=X[0, 0], normalize=normalize)
    loss = orc.subnet_sgd([w.copy() for w in W64], [v.copy() for v in b64], y[0, :1], 0.1, 1, mode,
                          X=X[0, :1], normalize=normalize)
    assert abs(loss[0] - _xent(logits, y[0, 0])) < 1e-12


def test_full_first_layer_is_the_union_of_the_subnets_first_layers():
    """Every hidden neuron of layer 1 sits in exactly one subnet and every subnet sees the whole
    input (Section 2.1), so the full f_1 restricted to H_1^s equals subnet s's f_1."""
    cfg = _cfg((9, 12, 5), S=3, B=5)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.3)
    perms = gen.make_perms(cfg)
    X, _ = gen.make_dense_batches(cfg)
    x = X[0, 0]
    # logits of a one-hidden-layer net with an identity read-out of the hidden layer
    eye = [Ws[0], np.eye(cfg.dims[1])]
    full = orc.forward_full(eye, [bs[0], np.zeros(cfg.dims[1])], "f32", X=x)
    subs = orc.partition(Ws, bs, perms, cfg.S)
    for s in range(cfg.S):
        idx = orc.block(perms[0], cfg.S, s)
        Wl, bl = subs[s]
        sub = orc.forward_full([Wl[0], np.eye(len(idx))], [bl[0], np.zeros(len(idx))], "f32", X=x)
        assert np.array_equal(full[:, idx], sub)


def test_csr_input_equals_its_dense_expansion():
    cfg = _cfg((40, 8, 6), S=2, B=5, input="csr", nnz_per_row=4)
    Ws, bs = gen.make_weights(cfg, bias_scale=0.1)
    rp, ci, va, _ = gen.make_csr_batches(cfg)
    rp, ci, va = orc.csr_slice(rp, ci, va, 0, cfg.B)
    dense = np.zeros((cfg.B, cfg.dims[0]))
    for b in range(cfg.B):
        for p in range(rp[b], rp[b + 1]):
            dense[b, ci[p]] += va[p]
    a = orc.forward_full(Ws, bs, "f32", csr=(rp, ci, va.astype(np.float64)))
    b_ = orc.forward_full(Ws, bs, "f32", X=dense)
    assert np.array_equal(a, b_)
