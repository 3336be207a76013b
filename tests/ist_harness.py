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
                 dev="cuda:0", normalize=False, scale=None, weights=None):
        """weights: (Ws, bs) float32 host arrays to start from instead of the seeded initial ones (a later
        round that starts from an earlier round's merged network)."""
        self.cfg, self.dev, self.has_bias, self.normalize = cfg, dev, has_bias, normalize
        self.scale = None if scale is None else [float(np.float32(v)) for v in scale]   # factors of Appendix A
        if weights is None:
            self.Ws, self.bs = gen.make_weights(cfg, with_bias=has_bias, bias_scale=bias_scale)
        else:
            self.Ws, self.bs = weights
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

    def gpu_steps(self, ctx, k=None, loss=True, j0=0):
        """Steps j0 .. j0+k-1 of the cfg.k steps the data was drawn for."""
        cfg = self.cfg
        k = cfg.k if k is None else k
        assert j0 + k <= cfg.k or j0 == 0
        lo = torch.zeros(cfg.S * k, dtype=torch.float32, device=self.dev) if loss else None
        off = j0 * cfg.B
        X = None if self.dX is None else self.dX.reshape(-1, cfg.dims[0])[off:]
        csr = None if self.dcsr is None else (self.dcsr[0][off:], self.dcsr[1], self.dcsr[2])
        ctx.subnet_steps(self.dy[off:], cfg.lr, k, cfg.B, X=X, csr=csr,
                         stride_s=cfg.k * cfg.B, stride_k=cfg.B, loss_out=lo)
        return None if lo is None else lo.cpu().numpy().reshape(cfg.S, k)

    def oracle_subnets(self, subnets=None):
        """Subnets after partition, float64, permutation-block order (all, or those listed)."""
        subs = orc.to_f64(orc.partition(self.Ws, self.bs if self.has_bias else [None] * self.cfg.t,
                                        self.perms, self.cfg.S))
        return subs if subnets is None else [subs[s] for s in subnets]

    def oracle_run(self, k=None):
        """(start, result, loss): the oracle's subnets before and after the k local steps."""
        init = self.oracle_subnets()
        subs = copy_subnets(init)
        return init, subs, self.oracle_steps(subs, k)

    def oracle_steps(self, subs, k=None, mode=None, j0=0, subnets=None):
        """Steps j0 .. j0+k-1 on the oracle's subnets `subs` (those listed in `subnets`, default all),
        in place; returns loss [len(subs)][k]."""
        cfg = self.cfg
        k = cfg.k if k is None else k
        mode = cfg.dtype if mode is None else mode
        which = list(range(cfg.S)) if subnets is None else list(subnets)
        assert len(which) == len(subs)
        loss = np.zeros((len(subs), k))
        for n, s in enumerate(which):
            Wl, bl = subs[n]
            kw = dict(normalize=self.normalize, scale=self.scale)
            if cfg.input == "csr":
                r0 = (s * cfg.k + j0) * cfg.B
                kw["csr"] = orc.csr_slice(self.rp, self.ci, self.va.astype(np.float64), r0, r0 + k * cfg.B)
            else:
                kw["X"] = self.X[s, j0:j0 + k]
            loss[n] = orc.subnet_sgd(Wl, bl if self.has_bias else None, self.y[s, j0:j0 + k], cfg.lr, k, mode, **kw)
        return loss


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


def bf16_code(a: np.ndarray) -> np.ndarray:
    """Monotone integer code of the bfloat16 values nearest to `a`: neighbours differ by one (+0 and -0 coincide)."""
    b = gen.to_bf16_bits(np.ascontiguousarray(a, dtype=np.float32)).astype(np.int64).reshape(np.shape(a))
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 numbers at magnitude |x| (8 significant bits; at least the smallest normal's)."""
    _, e = np.frexp(np.maximum(np.abs(x), 2.0 ** -126))
    return np.ldexp(1.0, e - 8)


# ---------------------------------------------------------------------------------------------------
# The gate on the CHANGE of the parameters.  The tolerance on the final parameters (TOL) cannot see a
# wrong or missing update of a tensor that moves by less than the tolerance, so the change over the
# steps, dW = W_k - W_0, is compared as well.  Both sides start from the same bits, hence
# dW_gpu - dW_orc = W_gpu - W_orc.  Tensors are pooled per layer over the subnets that are compared
# (one grouped launch updates them all; a subnet that alone went wrong still shows, see SUBNET_*).
#
# STRICT, after the first local step (both sides have seen identical weights so far; what differs is
# the summation order, binary32 against the oracle's binary64 accumulation, and through it a few
# roundings of stored activations and, rarely, a ReLU that flips and changes a whole row of dW):
#   f32:  ||dW_gpu - dW_orc||_2 <= F32_RHO * ||dW_orc||_2, and
#         max |dW_gpu - dW_orc| <= DW_RTOL * max |dW_orc| + 2^-22 * max |W| (relative error of the gradient sums,
#         plus the storage rounding of the step); with the standardisation of Section 2.2 the activations are
#         centred on the ReLU's kink, flips are common (0.4 per step expected on the speech-like workload) and
#         the bound on the largest element is DW_RTOL_STANDARDISED instead;
#   bf16: most elements do not change at all in a step (the update is below half a unit in the last place
#         of the weight), so the stored bits are compared element by element: the two sides may disagree on at
#         most BF16_MISMATCH of the number of elements the oracle changed (updates at a rounding boundary,
#         where the summation order decides), and at most BF16_FAR of all elements may differ by more than
#         two units in the last place of the larger of their start and end value (the rows of flipped ReLUs).
#   Measured with the kernels as they stand: f32 0.0004 (largest element) and 2e-5 (norm); bf16 at most 3.1 % of
#   the changed elements (first layer of the wide stress network; 6 % with the standardisation) and 2e-5 far.
# A check has POWER when a kernel that never updated the tensor would fail it by a wide margin:
# POWER = what such a kernel would be off by / what is allowed; the tests assert POWER >= MIN_POWER on every
# tensor except those a shape declares weak (no gradient by construction; they are not gated either, what
# moves there is rounding noise).
#
# LOOSE, at the end of a run of k > 1 steps: differences compound from step to step (an element that
# rounded the other way perturbs every later activation; measured on the CPU with a copy of the oracle
# that only accumulates in binary32 instead of binary64: 12 % / 22 % of the changed first-layer weights /
# biases of the image-like workload disagree after its 20 steps, and the f32 weight change of the
# speech-like workload differs by 2.7 % after its 10 steps, through one flipped ReLU).  There the tolerance
# on the final parameters is the gate, and the change only has to be present and of the right size:
# ||dW_gpu - dW_orc||_2 <= LOOSE_RHO * ||dW_orc||_2 (a missing update gives 1).
# ---------------------------------------------------------------------------------------------------
DW_RTOL = 2e-3
DW_RTOL_STANDARDISED = 0.25
F32_RHO = 1e-2
BF16_MISMATCH = 0.08
BF16_FAR = 5e-3
SUBNET_MISMATCH = 0.5      # a single subnet of the pool: at most this share of its changed elements (+1)
MIN_POWER = 10.0
LOOSE_RHO = 0.5
LOSS_RTOL = {"f32": 2e-4, "bf16": 3e-3}   # the stated parameter tolerances divided by 10

COLLECT = None   # a list: checks append their statistics there instead of asserting (calibration runs)


def change_stats(gpu_subs, orc_subs, init_subs, cfg):
    """{tensor name ("W1", "b1", ...): statistics pooled over the given subnets}."""
    out = {}
    for l in range(cfg.t):
        for kind in (0, 1):
            if orc_subs[0][kind][l] is None or gpu_subs[0][kind][l] is None:
                continue
            st = dict(n=0, err=0.0, dmax=0.0, scale=0.0, sq_err=0.0, sq_d=0.0, n_changed=0, n_mism=0, n_far=0,
                      worst_subnet=0.0)
            for s in range(len(orc_subs)):
                g = np.asarray(to_f32(gpu_subs[s][kind][l]), dtype=np.float64)
                o = np.asarray(orc_subs[s][kind][l], dtype=np.float64)
                i = np.asarray(init_subs[s][kind][l], dtype=np.float64)
                st["n"] += o.size
                st["err"] = max(st["err"], float(np.max(np.abs(g - o))))
                st["dmax"] = max(st["dmax"], float(np.max(np.abs(o - i))))
                st["scale"] = max(st["scale"], float(np.max(np.abs(o))), float(np.max(np.abs(orc_subs[s][0][l]))))
                st["sq_err"] += float(np.sum((g - o) ** 2))
                st["sq_d"] += float(np.sum((o - i) ** 2))
                if cfg.dtype == "bf16":
                    cg, co, ci = bf16_code(g), bf16_code(o), bf16_code(i)
                    nc, nm = int((co != ci).sum()), int((cg != co).sum())
                    st["n_changed"] += nc
                    st["n_mism"] += nm
                    ulp = bf16_ulp(np.maximum(np.maximum(np.abs(i), np.abs(o)), np.abs(g)))
                    st["n_far"] += int((np.abs(g - o) > 2.0 * ulp).sum())
                    st["worst_subnet"] = max(st["worst_subnet"], nm / (nc + 1.0))
            st["rho"] = float(np.sqrt(st["sq_err"] / st["sq_d"])) if st["sq_d"] > 0 else (0.0 if st["sq_err"] == 0 else np.inf)
            st["move_over_tol"] = st["dmax"] / st["scale"] / TOL[cfg.dtype] if st["scale"] > 0 else 0.0
            out[("W" if kind == 0 else "b") + str(l + 1)] = st
    return out


def check_change(stats, cfg, strict, weak=(), tag="", standardised=False):
    """Asserts the gate described above on the pooled statistics of every tensor."""
    for name, st in stats.items():
        if strict and cfg.dtype == "f32":
            allowed = (DW_RTOL_STANDARDISED if standardised else DW_RTOL) * st["dmax"] + 2.0 ** -22 * st["scale"]
            # both bounds must hold, so a missing update fails by the larger of the two margins
            st["power"] = max(st["dmax"] / allowed if allowed > 0 else 0.0, 1.0 / F32_RHO if st["sq_d"] > 0 else 0.0)
            ok = st["err"] <= allowed and st["rho"] <= F32_RHO
        elif strict:
            allowed = max(1.0, BF16_MISMATCH * st["n_changed"])
            st["power"] = st["n_changed"] / allowed
            ok = (st["n_mism"] <= allowed and st["n_far"] <= max(1.0, BF16_FAR * st["n"])
                  and st["worst_subnet"] <= SUBNET_MISMATCH)
        else:
            st["power"] = 1.0 / LOOSE_RHO
            ok = st["rho"] <= LOOSE_RHO or st["sq_d"] == 0.0
        brief = {a: (float(f"{b:.3g}") if isinstance(b, float) else b) for a, b in st.items() if a not in ("sq_err", "sq_d")}
        print(f"  {cfg.name}{tag} {name} {'strict' if strict else 'loose'}{' (weak)' if name in weak else ''}: {brief}")
        if COLLECT is not None:
            COLLECT.append((cfg.name + tag, name, strict, dict(st), ok or name in weak))
            continue
        if name in weak:
            continue
        assert ok, f"{cfg.name}{tag} {name}: the change over the steps differs from the oracle's: {brief}"
        if strict:
            assert st["power"] >= MIN_POWER * (1 - 1e-9), f"{cfg.name}{tag} {name}: the check has no power here: {brief}"


def copy_subnets(subs):
    return [([w.copy() for w in Wl], [None if b is None else b.copy() for b in bl]) for Wl, bl in subs]


def compare_subnets(gpu_subs, orc_subs, cfg, tol):
    """Final parameters: max over tensors of ||gpu - oracle||_inf / ||oracle||_inf, asserted <= tol
    (bias vectors, which start near zero, are scaled by the larger of their own and their layer's weights' norm)."""
    worst = 0.0
    for s in range(len(orc_subs)):
        for l in range(cfg.t):
            e = rel_err(to_f32(gpu_subs[s][0][l]), orc_subs[s][0][l])
            worst = max(worst, e)
            assert COLLECT is not None or e <= tol, f"subnet {s} W_{l + 1}: rel err {e:.3e} > {tol}"
            if gpu_subs[s][1][l] is not None and orc_subs[s][1][l] is not None:
                ref = orc_subs[s][1][l]
                scale = max(float(np.max(np.abs(ref))), float(np.max(np.abs(orc_subs[s][0][l]))))
                e = float(np.max(np.abs(to_f32(gpu_subs[s][1][l]) - ref))) / scale
                worst = max(worst, e)
                assert COLLECT is not None or e <= tol, f"subnet {s} b_{l + 1}: rel err {e:.3e} > {tol}"
    return worst


def check_training(P, ctx, k=None, weak=(), subnets=None):
    """k local steps on the HIP path (ctx is partitioned) and on the oracle from the same start.  After
    the first step: the strict gate on the change of every tensor.  After all k: the tolerance on the final
    parameters, the loose gate on the change, and the losses of every step.
    subnets: indices of the subnets the oracle follows (default all).  Returns (gpu subnets as
    exported, oracle subnets after training, gpu loss [S][k], worst final relative error)."""
    cfg = P.cfg
    k = cfg.k if k is None else k
    tol = TOL[cfg.dtype]
    which = list(range(cfg.S)) if subnets is None else list(subnets)
    init = P.oracle_subnets(which)
    subs = copy_subnets(init)
    worst, done, losses_g, losses_o, got = 0.0, 0, [], [], None
    for kk, strict in ((1, True), (k - 1, False)):
        if kk <= 0:
            continue
        losses_g.append(P.gpu_steps(ctx, k=kk, j0=done))
        got = export_all(ctx, cfg)
        losses_o.append(P.oracle_steps(subs, k=kk, j0=done, subnets=which))
        done += kk
        sel = [got[s] for s in which]
        worst = max(worst, compare_subnets(sel, subs, cfg, tol))
        check_change(change_stats(sel, subs, init, cfg), cfg, strict, weak=weak, tag=f" after {done} step(s)",
                     standardised=bool(getattr(P, "normalize", False)))
    if not losses_g:
        return export_all(ctx, cfg), subs, np.zeros((cfg.S, 0)), 0.0
    loss_g, loss_o = np.concatenate(losses_g, axis=1), np.concatenate(losses_o, axis=1)
    if COLLECT is None:
        np.testing.assert_allclose(loss_g[which], loss_o, rtol=LOSS_RTOL[cfg.dtype], atol=1e-6)
    return got, subs, loss_g, worst
