"""Shared plumbing of the GPU parity tests: upload seeded inputs, run the HIP path
through the C ABI, run the oracle on the same inputs, compare."""
from __future__ import annotations

import numpy as np
import torch

import ist_inputs as gen
from oracle import ist_oracle as orc

TOL = {"f32": 2e-3, "bf16": 3e-2}   # max relative error on parameters after k local steps


def td(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_dev(a: np.ndarray, dtype: str, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(td(dtype)).contiguous()


def bits(x: torch.Tensor) -> np.ndarray:
    """Raw storage of a device tensor as unsigned integers (bit-exact comparisons)."""
    if x.dtype == torch.bfloat16:
        return x.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return x.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)


def np_bits(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return gen.to_bf16_bits(a).reshape(a.shape) if dtype == "bf16" else a.view(np.uint32)


def to_f32(x: torch.Tensor) -> np.ndarray:
    return x.float().cpu().numpy()


def rel_err(a: np.ndarray, b: np.ndarray) -> float:
    """||a - b||_inf / ||b||_inf over one parameter tensor."""
    den = float(np.max(np.abs(b)))
    num = float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))))
    return num / den if den > 0 else num


class Problem:
    """Seeded inputs of one configuration on the host and on the device."""

    def __init__(self, cfg: gen.ISTConfig, rnd: int = 0, bias_scale: float = 0.05, has_bias=True,
                 dev="cuda:0", normalize=False, scale=None):
        self.cfg, self.dev, self.has_bias, self.normalize = cfg, dev, has_bias, normalize
        self.scale = None if scale is None else [float(np.float32(v)) for v in scale]   # factors of Appendix A
        self.Ws, self.bs = gen.make_weights(cfg, with_bias=has_bias, bias_scale=bias_scale)
        self.perms = gen.make_perms(cfg, rnd)
        if cfg.input == "csr":
            self.rp, self.ci, self.va, self.y = gen.make_csr_batches(cfg, rnd)
            self.X = None
        else:
            self.X, self.y = gen.make_dense_batches(cfg, rnd)
        self.upload()

    def upload(self):
        cfg, dev = self.cfg, self.dev
        self.dW = [to_dev(w, cfg.dtype, dev) for w in self.Ws]
        self.db = [to_dev(b, cfg.dtype, dev) for b in self.bs] if self.has_bias else None
        self.dperm = [torch.from_numpy(p).to(dev) for p in self.perms]
        self.dy = torch.from_numpy(self.y.reshape(-1).copy()).to(dev)
        if cfg.input == "csr":
            self.dcsr = (torch.from_numpy(self.rp).to(dev), torch.from_numpy(self.ci).to(dev),
                         to_dev(self.va, cfg.dtype, dev))
            self.dX = None
        else:
            self.dX = to_dev(self.X, cfg.dtype, dev)
            self.dcsr = None

    def context(self):
        from paper_1910_02120_amd import ISTContext
        cfg = self.cfg
        return ISTContext(cfg.dims, cfg.S, cfg.dtype, cfg.input, self.has_bias, max_B=cfg.B,
                          device=self.dev, normalize=self.normalize, layer_scale=self.scale)

    def gpu_steps(self, ctx, k=None, loss=True):
        cfg = self.cfg
        k = cfg.k if k is None else k
        lo = torch.zeros(cfg.S * k, dtype=torch.float32, device=self.dev) if loss else None
        ctx.subnet_steps(self.dy, cfg.lr, k, cfg.B, X=self.dX, csr=self.dcsr,
                         stride_s=cfg.k * cfg.B, stride_k=cfg.B, loss_out=lo)
        return None if lo is None else lo.cpu().numpy().reshape(cfg.S, k)

    def oracle_subnets(self):
        """Subnets after partition, float64, permutation-block order."""
        return orc.to_f64(orc.partition(self.Ws, self.bs if self.has_bias else [None] * self.cfg.t,
                                        self.perms, self.cfg.S))

    def oracle_steps(self, subs, k=None, mode=None):
        cfg = self.cfg
        k = cfg.k if k is None else k
        mode = cfg.dtype if mode is None else mode
        if cfg.input == "csr":
            return orc.subnet_steps(subs, cfg.lr, k, mode, self.y, normalize=self.normalize, scale=self.scale,
                                    csr=(self.rp, self.ci, self.va.astype(np.float64)))
        return orc.subnet_steps(subs, cfg.lr, k, mode, self.y, X=self.X, normalize=self.normalize, scale=self.scale)


def export_all(ctx, cfg):
    """[(W list, b list)] per subnet as float32 host arrays, plus raw bits."""
    out = []
    for s in range(cfg.S):
        Wl, bl = [], []
        for l in range(1, cfg.t + 1):
            W, b = ctx.subnet_export(s, l)
            Wl.append(W)
            bl.append(b)
        out.append((Wl, bl))
    torch.cuda.synchronize()
    return out


def compare_subnets(gpu_subs, orc_subs, cfg, tol):
    """Max over parameter tensors of ||gpu - oracle||_inf / ||oracle||_inf."""
    worst = 0.0
    for s in range(cfg.S):
        for l in range(cfg.t):
            e = rel_err(to_f32(gpu_subs[s][0][l]), orc_subs[s][0][l])
            worst = max(worst, e)
            assert e <= tol, f"subnet {s} W_{l + 1}: rel err {e:.3e} > {tol}"
            if gpu_subs[s][1][l] is not None and orc_subs[s][1][l] is not None:
                ref = orc_subs[s][1][l]
                scale = max(float(np.max(np.abs(ref))), float(np.max(np.abs(orc_subs[s][0][l]))))
                e = float(np.max(np.abs(to_f32(gpu_subs[s][1][l]) - ref))) / scale
                worst = max(worst, e)
                assert e <= tol, f"subnet {s} b_{l + 1}: rel err {e:.3e} > {tol}"
    return worst
