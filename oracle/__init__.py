"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Loads ``liblccrf_oracle.so`` (built from ``lccrf_oracle.c`` by ``oracle/build.py``)
with ctypes and wraps it for numpy / CPU torch inputs.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import this package; the product
path never does, and this package imports nothing from the product: inputs are
handed in by the caller.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblccrf_oracle.so")
_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ip, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    i = ctypes.c_int
    lib.lccrf_oracle_forward_backward.argtypes = [vp, i, ip, i, i, i, dp, dp, dp]
    lib.lccrf_oracle_forward_backward.restype = i
    lib.lccrf_oracle_log_partition.argtypes = [vp, i, ip, i, i, i, dp]
    lib.lccrf_oracle_log_partition.restype = i
    lib.lccrf_oracle_marginals.argtypes = [vp, i, ip, i, i, i, dp, dp]
    lib.lccrf_oracle_marginals.restype = i
    lib.lccrf_oracle_viterbi.argtypes = [vp, i, ip, i, i, i, dp, vp, dp]
    lib.lccrf_oracle_viterbi.restype = i
    lib.lccrf_oracle_log_prob.argtypes = [vp, i, ip, ip, i, i, i, dp]
    lib.lccrf_oracle_log_prob.restype = i
    lib.lccrf_oracle_cross_entropy.argtypes = [vp, vp, i, ip, i, i, i, dp]
    lib.lccrf_oracle_cross_entropy.restype = i
    lib.lccrf_oracle_semi_markov_log_partition.argtypes = [vp, i, ip, i, i, i, i, dp]
    lib.lccrf_oracle_semi_markov_log_partition.restype = i
    lib.lccrf_oracle_sample.argtypes = [vp, i, ip, vp, i, i, i, vp, dp]
    lib.lccrf_oracle_sample.restype = i
    lib.lccrf_oracle_threads.argtypes = []
    lib.lccrf_oracle_threads.restype = i
    _lib = lib
    return lib


def _as_storage(phi):
    """Return (numpy array kept alive, dtype code, shape).  Accepts numpy float32/uint16
    (uint16 = raw bfloat16 bits) or CPU torch float32/bfloat16 tensors."""
    try:
        import torch
    except Exception:  # pragma: no cover
        torch = None
    if torch is not None and isinstance(phi, torch.Tensor):
        if phi.device.type != "cpu":
            raise ValueError("the oracle takes CPU tensors only")
        phi = phi.contiguous()
        if phi.dtype == torch.bfloat16:
            arr = phi.view(torch.int16).numpy().view(np.uint16)
            return arr, 1, tuple(phi.shape)
        if phi.dtype == torch.float32:
            return phi.numpy(), 0, tuple(phi.shape)
        raise ValueError(f"unsupported torch dtype {phi.dtype}")
    arr = np.ascontiguousarray(phi)
    if arr.dtype == np.float32:
        return arr, 0, arr.shape
    if arr.dtype == np.uint16:
        return arr, 1, arr.shape
    if arr.dtype == np.float64:
        a32 = arr.astype(np.float32)
        if not np.array_equal(a32.astype(np.float64), arr, equal_nan=True):
            raise ValueError("float64 potentials must be exactly representable in float32")
        return a32, 0, arr.shape
    raise ValueError(f"unsupported dtype {arr.dtype}")


def _lengths(lengths, B) -> Optional[np.ndarray]:
    if lengths is None:
        return None
    try:
        import torch
        if isinstance(lengths, torch.Tensor):
            lengths = lengths.cpu().numpy()
    except Exception:  # pragma: no cover
        pass
    l = np.ascontiguousarray(np.asarray(lengths, dtype=np.int32))
    assert l.shape == (B,)
    return l


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().lccrf_oracle_threads())


def forward_backward(phi, lengths=None):
    """alpha [B,N,T], beta [B,N,T] (rows past the length are NaN), logZ [B]; float64."""
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    alpha = np.full((B, N, T), np.nan)
    beta = np.full((B, N, T), np.nan)
    logZ = np.empty((B,))
    rc = lib.lccrf_oracle_forward_backward(_ptr(arr), dt, _ptr(l), B, N, T, _ptr(alpha), _ptr(beta), _ptr(logZ))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return alpha, beta, logZ


def log_partition(phi, lengths=None) -> np.ndarray:
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    logZ = np.empty((B,))
    rc = lib.lccrf_oracle_log_partition(_ptr(arr), dt, _ptr(l), B, N, T, _ptr(logZ))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return logZ


def marginals(phi, lengths=None):
    """(logZ [B], mu [B,N,T,T]) in float64."""
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    logZ = np.empty((B,))
    mu = np.empty((B, N, T, T))
    rc = lib.lccrf_oracle_marginals(_ptr(arr), dt, _ptr(l), B, N, T, _ptr(logZ), _ptr(mu))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return logZ, mu


def viterbi(phi, lengths=None, with_gap: bool = True):
    """(score [B] f64, tags [B,N] int32 with -1 past the length, gap [B] f64 or None)."""
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    score = np.empty((B,))
    tags = np.empty((B, N), dtype=np.int32)
    gap = np.empty((B,)) if with_gap else None
    rc = lib.lccrf_oracle_viterbi(_ptr(arr), dt, _ptr(l), B, N, T, _ptr(score), _ptr(tags), _ptr(gap))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return score, tags, gap


def log_prob(phi, tags, lengths=None) -> np.ndarray:
    """log p(tags) [B] float64: the path's score minus logZ (NaN where a tag is out of range)."""
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    y = np.ascontiguousarray(np.asarray(tags), dtype=np.int32)
    assert y.shape == (B, N)
    out = np.empty((B,))
    rc = lib.lccrf_oracle_log_prob(_ptr(arr), dt, _ptr(l), _ptr(y), B, N, T, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return out


def cross_entropy(phi_p, phi_q, lengths=None) -> np.ndarray:
    """H(p, q) [B] float64 = logZ_q - sum_e p(e) phi_q(e); entropy is cross_entropy(phi, phi)."""
    lib = _load()
    arr_p, dt, (B, N, T, T2) = _as_storage(phi_p)
    arr_q, dt_q, shape_q = _as_storage(phi_q)
    assert T == T2 and dt == dt_q and tuple(shape_q) == (B, N, T, T)
    l = _lengths(lengths, B)
    out = np.empty((B,))
    rc = lib.lccrf_oracle_cross_entropy(_ptr(arr_p), _ptr(arr_q), dt, _ptr(l), B, N, T, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return out


def entropy(phi, lengths=None) -> np.ndarray:
    return cross_entropy(phi, phi, lengths)


def kl_divergence(phi_p, phi_q, lengths=None) -> np.ndarray:
    """KL(p || q) [B] float64 = H(p, q) - H(p) (section "Entropy and KL Divergence")."""
    return cross_entropy(phi_p, phi_q, lengths) - cross_entropy(phi_p, phi_p, lengths)


def semi_markov_log_partition(phi, lengths=None) -> np.ndarray:
    """logZ [B] float64 of the semi-Markov CRF with potentials phi [B, N, K, T, T] (float32 numpy, or a
    torch float32 / bfloat16 tensor): phi[b, i, k, s, t] scores a segment tagged t that ends at i
    and covers k + 1 positions, after a segment tagged s."""
    lib = _load()
    arr, dt, shape = _as_storage(phi)
    B, N, K, T, T2 = shape
    assert T == T2
    l = _lengths(lengths, B)
    out = np.empty((B,))
    rc = lib.lccrf_oracle_semi_markov_log_partition(_ptr(arr), dt, _ptr(l), B, N, K, T, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return out


def sample(phi, uniforms, lengths=None):
    """Forward-filtering backward-sampling with the given uniforms [B, N] (float32 in [0, 1)):
    (tags [B, N] int32 with -1 past the length, margin [B] float64: how far, relative to the total
    weight, the closest draw of the chain was from picking a neighbouring tag)."""
    lib = _load()
    arr, dt, (B, N, T, T2) = _as_storage(phi)
    assert T == T2
    l = _lengths(lengths, B)
    u = np.ascontiguousarray(np.asarray(uniforms), dtype=np.float32)
    assert u.shape == (B, N)
    tags = np.empty((B, N), dtype=np.int32)
    margin = np.empty((B,))
    rc = lib.lccrf_oracle_sample(_ptr(arr), dt, _ptr(l), _ptr(u), B, N, T, _ptr(tags), _ptr(margin))
    if rc != 0:
        raise RuntimeError(f"oracle error {rc}")
    return tags, margin
