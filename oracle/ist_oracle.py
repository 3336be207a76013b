"""ctypes front end of the CPU oracle (oracle/ist_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's
cpu_baseline leg; never by the product package.  The composition below follows
Section 2.1 of the IST paper: build the blocks, slice every weight matrix by
the blocks of its two endpoint layers, run k local SGD steps per subnet, copy
the blocks back.
"""
from __future__ import annotations

import ctypes as C
import hashlib
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ist_oracle.c")
_lib = None

MODE = {"exact": 0, "f32": 1, "bf16": 2}


def _cpu_tag() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    return hashlib.sha1(line.encode()).hexdigest()[:10]
    except OSError:
        pass
    return "generic"


def lib_path() -> str:
    return os.path.join(_HERE, "_build", f"libist_oracle_{_cpu_tag()}.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc for this host (the file name carries a hash of
    the CPU flags so a library built elsewhere with -march=native is not reused)."""
    out = lib_path()
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= os.path.getmtime(_SRC)):
        return out
    os.makedirs(os.path.dirname(out), exist_ok=True)
    tmp = out + f".tmp{os.getpid()}"
    cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
           "-std=c11", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = C.CDLL(build())
    p = C.c_void_p
    lib.ist_oracle_round.restype = C.c_double
    lib.ist_oracle_round.argtypes = [C.c_double, C.c_int32]
    lib.ist_oracle_round_array.restype = None
    lib.ist_oracle_round_array.argtypes = [p, C.c_int64, C.c_int32]
    lib.ist_oracle_block.restype = C.c_int64
    lib.ist_oracle_block.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p]
    for fn in (lib.ist_oracle_gather, lib.ist_oracle_scatter):
        fn.restype = None
        fn.argtypes = [p, C.c_int64, C.c_int64, p, C.c_int64, p, C.c_int64, p]
    lib.ist_oracle_merge_out_bias.restype = None
    lib.ist_oracle_merge_out_bias.argtypes = [p, C.c_int32, C.c_int64, C.c_int32, p]
    lib.ist_oracle_subnet_sgd_norm.restype = C.c_int32
    lib.ist_oracle_subnet_sgd_norm.argtypes = [C.c_int32, p, p, p, C.c_int32, p, p, p, p, p,
                                               C.c_int32, C.c_int32, C.c_double, C.c_int32, C.c_int32,
                                               C.c_double, p]
    lib.ist_oracle_subnet_sgd_scaled.restype = C.c_int32
    lib.ist_oracle_subnet_sgd_scaled.argtypes = [C.c_int32, p, p, p, C.c_int32, p, p, p, p, p,
                                                 C.c_int32, C.c_int32, C.c_double, C.c_int32, C.c_int32,
                                                 C.c_double, p, p]
    lib.ist_oracle_subnet_sgd.restype = C.c_int32
    lib.ist_oracle_subnet_sgd.argtypes = [C.c_int32, p, p, p, C.c_int32, p, p, p, p, p,
                                          C.c_int32, C.c_int32, C.c_double, C.c_int32, p]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def omp_threads() -> int:
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def round_store(x: float, mode: str) -> float:
    return float(_load().ist_oracle_round(float(x), MODE[mode]))


# ------------------------------------------------------------------ blocks
def block(perm: np.ndarray, S: int, s: int) -> np.ndarray:
    """H^s of one hidden layer: the s-th block of its permutation; when S does not divide the
    width the first N mod S subnets own one neuron more."""
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    N = perm.shape[0]
    if S <= 0 or not 0 <= s < S:
        raise ValueError("bad block request")
    out = np.empty(N // S + 1, dtype=np.int32)
    w = _load().ist_oracle_block(_ptr(perm), N, S, s, _ptr(out))
    if w < 0:
        raise ValueError("bad block request")
    return out[:w].copy()


def blocks(perms: Sequence[np.ndarray], S: int) -> List[List[np.ndarray]]:
    """H[l-1][s] for hidden layers l = 1..t-1."""
    return [[block(p, S, s) for s in range(S)] for p in perms]


def _endpoints(H, l: int, t: int, s: int):
    """Row and column index lists of W_l for subnet s (None = every neuron)."""
    ridx = None if l == t else H[l - 1][s]
    cidx = None if l == 1 else H[l - 2][s]
    return ridx, cidx


def gather(W: np.ndarray, ridx, cidx) -> np.ndarray:
    W = np.ascontiguousarray(W)
    nr = W.shape[0] if ridx is None else len(ridx)
    nc = W.shape[1] if cidx is None else len(cidx)
    out = np.empty((nr, nc), dtype=W.dtype)
    _load().ist_oracle_gather(_ptr(W), W.shape[1], W.dtype.itemsize, _ptr(ridx), nr,
                              _ptr(cidx), nc, _ptr(out))
    return out


def scatter(W: np.ndarray, ridx, cidx, sub: np.ndarray) -> None:
    assert W.flags.c_contiguous and W.dtype == sub.dtype
    sub = np.ascontiguousarray(sub)
    nr = W.shape[0] if ridx is None else len(ridx)
    nc = W.shape[1] if cidx is None else len(cidx)
    assert sub.shape == (nr, nc)
    _load().ist_oracle_scatter(_ptr(W), W.shape[1], W.dtype.itemsize, _ptr(ridx), nr,
                               _ptr(cidx), nc, _ptr(sub))


# --------------------------------------------------------- partition / merge
def partition(Ws, bs, perms, S: int):
    """subnets[s] = (W list, b list): W_l^s = W_l[H_l^s, H_{l-1}^s], hidden bias
    follows its neuron, the output bias is replicated.  Works on raw elements of
    any dtype (bit-exact)."""
    t = len(Ws)
    H = blocks(perms, S)
    subs = []
    for s in range(S):
        Wl, bl = [], []
        for l in range(1, t + 1):
            ridx, cidx = _endpoints(H, l, t, s)
            Wl.append(gather(Ws[l - 1], ridx, cidx))
            bfull = bs[l - 1] if bs is not None else None
            if bfull is None:
                bl.append(None)
            else:
                b2 = np.ascontiguousarray(bfull).reshape(-1, 1)
                bl.append(gather(b2, ridx, None).reshape(-1))
        subs.append((Wl, bl))
    return subs


def merge(Ws, bs, perms, S: int, subs, mode: str = "f32") -> None:
    """In place: copy every subnet block back; hidden biases follow their neuron;
    output bias = mean over subnets (float arrays only)."""
    t = len(Ws)
    H = blocks(perms, S)
    for s in range(S):
        for l in range(1, t + 1):
            ridx, cidx = _endpoints(H, l, t, s)
            scatter(Ws[l - 1], ridx, cidx, subs[s][0][l - 1])
            if bs is not None and bs[l - 1] is not None and l < t:
                b2 = bs[l - 1].reshape(-1, 1)
                scatter(b2, ridx, None, subs[s][1][l - 1].reshape(-1, 1))
    if bs is not None and bs[t - 1] is not None:
        stack = np.ascontiguousarray(
            np.stack([np.asarray(subs[s][1][t - 1], dtype=np.float64) for s in range(S)]))
        out = np.empty(stack.shape[1], dtype=np.float64)
        _load().ist_oracle_merge_out_bias(_ptr(stack), S, stack.shape[1], MODE[mode], _ptr(out))
        bs[t - 1][...] = out.astype(bs[t - 1].dtype)


# ------------------------------------------------------------------ training
NORM_EPS = 1e-5   # epsilon under the square root of the per-neuron standardisation


def subnet_sgd(Wl: List[np.ndarray], bl: Optional[List[Optional[np.ndarray]]], y: np.ndarray,
               lr: float, k: int, mode: str, X: Optional[np.ndarray] = None, csr=None,
               normalize: bool = False, eps: float = NORM_EPS, scale=None):
    """k local SGD steps on one subnet.  Wl/bl are float64 arrays updated in place.
    X: [k][B][n_0] float64, or csr = (rowptr[k*B+1], colidx, vals float64).
    normalize: standardise every hidden neuron's input over the mini-batch (Section 2.2).
    scale: factors gamma_l of the layer products (Appendix A, equation (4): n^2), None = 1.
    Returns loss[k]."""
    t = len(Wl)
    for w in Wl:
        assert w.dtype == np.float64 and w.flags.c_contiguous
    n = np.array([Wl[0].shape[1]] + [w.shape[0] for w in Wl], dtype=np.int64)
    y = np.ascontiguousarray(y, dtype=np.int32).reshape(k, -1)
    B = y.shape[1]
    assert y.min() >= 0 and y.max() < n[-1]
    Wp = (C.c_void_p * t)(*[w.ctypes.data for w in Wl])
    has_b = bl is not None and bl[0] is not None
    if has_b:
        for v in bl:
            assert v.dtype == np.float64 and v.flags.c_contiguous
        bp = (C.c_void_p * t)(*[v.ctypes.data for v in bl])
    else:
        bp = None
    loss = np.zeros(k, dtype=np.float64)
    if csr is None:
        X = np.ascontiguousarray(X, dtype=np.float64)
        assert X.shape == (k, B, n[0])
        args = (0, _ptr(X), None, None, None)
    else:
        rp, ci, va = csr
        rp = np.ascontiguousarray(rp, dtype=np.int32)
        ci = np.ascontiguousarray(ci, dtype=np.int32)
        va = np.ascontiguousarray(va, dtype=np.float64)
        assert rp.shape[0] == k * B + 1
        assert ci.size == 0 or (ci.min() >= 0 and ci.max() < n[0])
        args = (1, None, _ptr(rp), _ptr(ci), _ptr(va))
    sc = None if scale is None else np.ascontiguousarray(scale, dtype=np.float64)
    assert sc is None or sc.shape == (t,)
    rc = _load().ist_oracle_subnet_sgd_scaled(t, _ptr(n), Wp, bp, *args, _ptr(y), B, k,
                                              float(np.float32(lr)), MODE[mode], 1 if normalize else 0,
                                              float(eps), _ptr(sc), _ptr(loss))
    if rc:
        raise ValueError("ist_oracle_subnet_sgd rejected its arguments")
    return loss


def round_array(a: np.ndarray, mode: str) -> np.ndarray:
    """Storage rounding of every element (a float64 copy)."""
    out = np.array(a, dtype=np.float64, order="C", copy=True)
    _load().ist_oracle_round_array(_ptr(out), out.size, MODE[mode])
    return out


def forward_full(Ws, bs, mode: str, X: Optional[np.ndarray] = None, csr=None,
                 normalize: bool = False, eps: float = NORM_EPS, scale=None) -> np.ndarray:
    """Logits [B][N_t] of the full network of Section 2.1 on one batch, written out layer by
    layer: f_l = ReLU(W_l f_{l-1} + b_l), logits = W_t f_{t-1} + b_t; with `normalize` the input of
    every hidden neuron is standardised over the batch first (Section 2.2, biased variance).
    float64 arithmetic; hidden activations (and the standardised inputs) are rounded to the
    storage type where the device stores them, the logits are not.
    X [B][N_0], or csr = (rowptr [B+1], colidx, vals).  scale: factors gamma_l applied to the
    products W_l f_{l-1} (a subnet's forward pass in Appendix A, equation (4)); None for the full
    network, which has none."""
    t = len(Ws)
    if csr is None:
        f = np.asarray(X, dtype=np.float64)
    else:
        rp, ci, va = csr
        B = len(rp) - 1
        f = np.zeros((B, Ws[0].shape[1]))
        for bi in range(B):
            for p in range(int(rp[bi]), int(rp[bi + 1])):
                f[bi, int(ci[p])] += float(va[p])
    for l in range(1, t + 1):
        z = f @ np.asarray(Ws[l - 1], dtype=np.float64).T
        if scale is not None:
            z = float(scale[l - 1]) * z
        if bs is not None and bs[l - 1] is not None:
            z = z + np.asarray(bs[l - 1], dtype=np.float64)[None, :]
        if l == t:
            return z
        if normalize:
            mu = z.mean(axis=0, keepdims=True)
            var = ((z - mu) ** 2).mean(axis=0, keepdims=True)
            z = round_array((z - mu) / np.sqrt(var + eps), mode)
            f = np.maximum(z, 0.0)
        else:
            f = round_array(np.maximum(z, 0.0), mode)
    raise AssertionError("unreachable")


def csr_slice(rowptr, colidx, vals, r0: int, r1: int):
    """Rows r0..r1-1 of a CSR matrix, rowptr rebased to zero."""
    lo, hi = int(rowptr[r0]), int(rowptr[r1])
    return ((rowptr[r0:r1 + 1] - lo).astype(np.int32), colidx[lo:hi], vals[lo:hi])


def subnet_steps(subs_f64, lr: float, k: int, mode: str, y: np.ndarray,
                 X: Optional[np.ndarray] = None, csr=None, normalize: bool = False, scale=None):
    """Local SGD on every subnet independently (no communication between them).
    subs_f64[s] = (W list, b list) in float64, updated in place; X [S][k][B][N_0]
    or a CSR whose row (s*k + j)*B + b is sample b of step j of subnet s.
    Returns loss [S][k]."""
    S = len(subs_f64)
    B = y.shape[-1]
    losses = np.zeros((S, k))
    for s in range(S):
        Wl, bl = subs_f64[s]
        if csr is None:
            losses[s] = subnet_sgd(Wl, bl, y[s, :k], lr, k, mode, X=X[s, :k], normalize=normalize, scale=scale)
        else:
            losses[s] = subnet_sgd(Wl, bl, y[s, :k], lr, k, mode, normalize=normalize, scale=scale,
                                   csr=csr_slice(*csr, s * y.shape[1] * B, (s * y.shape[1] + k) * B))
    return losses


def to_f64(subs):
    return [([np.ascontiguousarray(w, dtype=np.float64) for w in Wl],
             [None if v is None else np.ascontiguousarray(v, dtype=np.float64) for v in bl])
            for Wl, bl in subs]


def ist_round(Ws, bs, perms, S: int, lr: float, k: int, mode: str, y, X=None, csr=None):
    """One IST round on float arrays: partition, k local steps per subnet, merge.
    Ws/bs (float32 or float64 arrays) are updated in place.  Returns
    (loss [S][k], subnets after training in float64)."""
    subs = to_f64(partition(Ws, bs, perms, S))
    loss = subnet_steps(subs, lr, k, mode, y, X=X, csr=csr)
    typed = [([w.astype(Ws[i].dtype) for i, w in enumerate(Wl)],
              [None if v is None else v.astype(Ws[0].dtype) for v in bl]) for Wl, bl in subs]
    merge(Ws, bs, perms, S, typed, mode="f32" if mode == "exact" else mode)
    return loss, subs
