"""ctypes binding of ``liblccrf.so`` for torch device tensors.

Argument marshalling only: shapes, dtypes and devices are checked, pointers and the current
HIP stream are handed to the C ABI declared in ``include/lccrf.h``, and every step of the
computation runs in the library's kernels.  There is no fallback: if the shared library is
missing or an entry point reports an error, an exception is raised.

The three queries mirror the C entry points:
  ``lccrf_log_partition``  log-partition function      (paper, "Computing Probability of a
                           Structure and Partition Function"; forward algorithm of "Sequence Tagging")
  ``lccrf_marginals``      edge marginals = d logZ / d phi   (paper, "Computing Marginals", Eq. 3-4)
  ``lccrf_argmax``         most probable tag path, max-plus  (paper, "Computing Most Probable Structure")
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblccrf.so")

LCCRF_F32, LCCRF_BF16 = 0, 1
OP_LOGZ, OP_MARGINALS, OP_ARGMAX, OP_LOG_PROB, OP_ENTROPY, OP_SAMPLE, OP_CROSS_ENTROPY = 0, 1, 2, 3, 4, 5, 6
ALGO_AUTO, ALGO_SEQUENTIAL, ALGO_SCAN, ALGO_SEQUENTIAL_EXACT, ALGO_SEQUENTIAL_LANES = 0, 1, 2, 3, 4
MAX_T = 256

EXPORTS = (
    "lccrf_workspace_bytes", "lccrf_log_partition", "lccrf_marginals", "lccrf_argmax",
    "lccrf_log_partition_algo", "lccrf_marginals_algo", "lccrf_argmax_algo",
    "lccrf_marginals_timed", "lccrf_log_prob", "lccrf_entropy", "lccrf_cross_entropy", "lccrf_kl_divergence",
    "lccrf_sample", "lccrf_semi_markov_log_partition", "lccrf_log_partition_structured",
    "lccrf_marginals_structured", "lccrf_argmax_structured", "lccrf_set_scan_chunk", "lccrf_auto_algo",
    "lccrf_strerror", "lccrf_version", "lccrf_marginals_static", "lccrf_static_scratch_bytes",
    "lccrf_set_pair_poll_limit", "lccrf_set_lane_poll_limit", "lccrf_stream_probe", "lccrf_stream_probe_bytes", "lccrf_sample_seeded",
)

_lib = None


class LccrfError(RuntimeError):
    pass


def load_library() -> ctypes.CDLL:
    """Load ``liblccrf.so`` (built by ``build_ext.py``); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LccrfError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2308_03291_amd.build_ext` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.lccrf_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.lccrf_workspace_bytes.restype = sz
    base = [vp, i, vp, i, i, i]
    lib.lccrf_log_partition.argtypes = base + [vp, vp, sz, vp]
    lib.lccrf_marginals.argtypes = base + [vp, vp, vp, sz, vp]
    lib.lccrf_argmax.argtypes = base + [vp, vp, vp, sz, vp]
    lib.lccrf_log_partition_algo.argtypes = base + [vp, vp, sz, vp, i]
    lib.lccrf_marginals_algo.argtypes = base + [vp, vp, vp, sz, vp, i]
    lib.lccrf_argmax_algo.argtypes = base + [vp, vp, vp, sz, vp, i]
    lib.lccrf_marginals_timed.argtypes = base + [vp, vp, vp, sz, vp, i, vp, vp, vp]
    for n in ("lccrf_log_partition", "lccrf_marginals", "lccrf_argmax", "lccrf_marginals_timed",
              "lccrf_log_partition_algo", "lccrf_marginals_algo", "lccrf_argmax_algo", "lccrf_version"):
        getattr(lib, n).restype = i
    lib.lccrf_strerror.argtypes = [i]
    lib.lccrf_strerror.restype = ctypes.c_char_p
    lib.lccrf_version.argtypes = []
    lib.lccrf_log_prob.argtypes = [vp, i, vp, vp, i, i, i, vp, vp, sz, vp]
    lib.lccrf_log_prob.restype = i
    lib.lccrf_entropy.argtypes = base + [vp, vp, sz, vp]
    lib.lccrf_entropy.restype = i
    for n in ("lccrf_cross_entropy", "lccrf_kl_divergence"):
        getattr(lib, n).argtypes = [vp, vp, i, vp, i, i, i, vp, vp, sz, vp]
        getattr(lib, n).restype = i
    lib.lccrf_semi_markov_log_partition.argtypes = [vp, i, vp, i, i, i, i, vp, vp]
    lib.lccrf_semi_markov_log_partition.restype = i
    lib.lccrf_sample.argtypes = [vp, i, vp, vp, i, i, i, vp, vp, sz, vp]
    lib.lccrf_sample.restype = i
    lib.lccrf_sample_seeded.argtypes = [vp, i, vp, ctypes.c_uint64, i, i, i, vp, vp, sz, vp]
    lib.lccrf_sample_seeded.restype = i
    sbase = [vp, vp, vp, i, i, i]
    lib.lccrf_log_partition_structured.argtypes = sbase + [vp, vp, sz, vp]
    lib.lccrf_marginals_structured.argtypes = sbase + [vp, vp, vp, sz, vp]
    lib.lccrf_argmax_structured.argtypes = sbase + [vp, vp, vp, sz, vp]
    for n in ("lccrf_log_partition_structured", "lccrf_marginals_structured", "lccrf_argmax_structured"):
        getattr(lib, n).restype = i
    lib.lccrf_marginals_static.argtypes = base + [vp, vp, vp]
    lib.lccrf_marginals_static.restype = i
    lib.lccrf_static_scratch_bytes.argtypes = []
    lib.lccrf_static_scratch_bytes.restype = sz
    lib.lccrf_set_scan_chunk.argtypes = [i]
    lib.lccrf_set_scan_chunk.restype = i
    lib.lccrf_stream_probe.argtypes = [vp, vp, sz, i, vp, vp]
    lib.lccrf_stream_probe.restype = i
    lib.lccrf_stream_probe_bytes.argtypes = [sz, i]
    lib.lccrf_stream_probe_bytes.restype = sz
    lib.lccrf_set_pair_poll_limit.argtypes = [i]
    lib.lccrf_set_pair_poll_limit.restype = i
    lib.lccrf_set_lane_poll_limit.argtypes = [i]
    lib.lccrf_set_lane_poll_limit.restype = i
    lib.lccrf_auto_algo.argtypes = [i, i, i, i]
    lib.lccrf_auto_algo.restype = i
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().lccrf_strerror(int(code)).decode()


def set_scan_chunk(chunk: int) -> None:
    """Positions per chunk of ALGO_SCAN (0: default).  Size workspaces after calling this."""
    _check(load_library().lccrf_set_scan_chunk(int(chunk)), "lccrf_set_scan_chunk")


def set_lane_poll_limit(polls: int) -> None:
    """Looks the chain wave of ALGO_SEQUENTIAL_LANES spends on a late matrix (-1: default, 0: none)."""
    _check(load_library().lccrf_set_lane_poll_limit(int(polls)), "lccrf_set_lane_poll_limit")


def set_pair_poll_limit(polls: int) -> None:
    """Looks a paired workgroup takes for its partner's words before it gives its sequence up (-1: default,
    0: give up without looking)."""
    _check(load_library().lccrf_set_pair_poll_limit(int(polls)), "lccrf_set_pair_poll_limit")


def auto_algo(op: int, B: int, N: int, T: int) -> int:
    """The schedule ALGO_AUTO takes for `op` at this shape: ALGO_SEQUENTIAL, ALGO_SEQUENTIAL_LANES or ALGO_SCAN."""
    rc = load_library().lccrf_auto_algo(int(op), int(B), int(N), int(T))
    if rc < 0:
        _check(rc, "lccrf_auto_algo")
    return rc


def _check(rc: int, what: str):
    if rc != 0:
        raise LccrfError(f"{what} failed: {strerror(rc)} (status {rc})")


def _phi_args(phi: torch.Tensor) -> Tuple[int, int, int, int]:
    if phi.dim() != 4 or phi.shape[2] != phi.shape[3]:
        raise ValueError(f"phi must be [B, N, T, T], got {tuple(phi.shape)}")
    if not phi.is_cuda:
        raise ValueError("phi must live on the GPU")
    if not phi.is_contiguous():
        raise ValueError("phi must be contiguous")
    if phi.dtype == torch.float32:
        dt = LCCRF_F32
    elif phi.dtype == torch.bfloat16:
        dt = LCCRF_BF16
    else:
        raise ValueError(f"phi must be float32 or bfloat16, got {phi.dtype}")
    B, N, T, _ = phi.shape
    return dt, int(B), int(N), int(T)


def _len_ptr(lengths: Optional[torch.Tensor], B: int, device) -> Optional[int]:
    if lengths is None:
        return None
    if lengths.dtype != torch.int32 or lengths.shape != (B,) or lengths.device != device \
            or not lengths.is_contiguous():
        raise ValueError("lengths must be a contiguous int32 [B] tensor on phi's device")
    return lengths.data_ptr()


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def workspace_bytes(op: int, B: int, N: int, T: int, dtype: int) -> int:
    return int(load_library().lccrf_workspace_bytes(op, B, N, T, dtype))


def _workspace(op: int, B: int, N: int, T: int, dt: int, device, workspace: Optional[torch.Tensor]):
    need = workspace_bytes(op, B, N, T, dt)
    if need == 0:
        raise LccrfError(f"unsupported shape B={B} N={N} T={T} (1 <= T <= {MAX_T})")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    elif workspace.dtype != torch.uint8 or workspace.device != device or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 tensor on phi's device")
    return workspace, workspace.numel()


def lccrf_log_partition(phi: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        algo: int = ALGO_AUTO) -> torch.Tensor:
    """logZ [B] float32 on phi's device."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    ws, nws = _workspace(OP_LOGZ, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_log_partition_algo(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                                          out.data_ptr(), ws.data_ptr(), nws, _stream(phi.device), algo)
    _check(rc, "lccrf_log_partition")
    return out


def lccrf_marginals(phi: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                    out: Optional[torch.Tensor] = None, logZ: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, algo: int = ALGO_AUTO):
    """(logZ [B], marginals [B, N, T, T]) float32 on phi's device."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    ws, nws = _workspace(OP_MARGINALS, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, N, T, T, dtype=torch.float32, device=phi.device)
    if logZ is None:
        logZ = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_marginals_algo(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                                      logZ.data_ptr(), out.data_ptr(), ws.data_ptr(), nws,
                                      _stream(phi.device), algo)
    _check(rc, "lccrf_marginals")
    return logZ, out


def lccrf_marginals_static(phi: torch.Tensor, lengths: Optional[torch.Tensor], out: torch.Tensor,
                           logZ: torch.Tensor) -> None:
    """``lccrf_marginals`` into the caller's ``out`` [B, N, T, T] and ``logZ`` [B] (float32, on phi's device)
    with the library's built-in scratch buffer: nothing is allocated, here or in the library."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    for t, shape in ((out, (B, N, T, T)), (logZ, (B,))):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous() or t.device != phi.device:
            raise ValueError(f"outputs must be contiguous float32 tensors of shape {shape} on phi's device")
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_marginals_static(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                                        logZ.data_ptr(), out.data_ptr(), _stream(phi.device))
    _check(rc, "lccrf_marginals_static")


def lccrf_argmax(phi: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                 out: Optional[torch.Tensor] = None, score: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None, algo: int = ALGO_AUTO):
    """(best_score [B] float32, tags [B, N] int32 with -1 past the length)."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    ws, nws = _workspace(OP_ARGMAX, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, N, dtype=torch.int32, device=phi.device)
    if score is None:
        score = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_argmax_algo(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                                   score.data_ptr(), out.data_ptr(), ws.data_ptr(), nws,
                                   _stream(phi.device), algo)
    _check(rc, "lccrf_argmax")
    return score, out


def lccrf_log_prob(phi: torch.Tensor, tags: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """log p(tags) [B] float32: the path's score minus logZ (tags int32 [B, N] on phi's device)."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    if tags.dtype != torch.int32 or tuple(tags.shape) != (B, N) or not tags.is_contiguous() or tags.device != phi.device:
        raise LccrfError("tags must be a contiguous int32 [B, N] tensor on phi's device")
    ws, nws = _workspace(OP_LOG_PROB, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_log_prob(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), tags.data_ptr(), B, N, T,
                                out.data_ptr(), ws.data_ptr(), nws, _stream(phi.device))
    _check(rc, "lccrf_log_prob")
    return out


def lccrf_entropy(phi: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                  out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Entropy [B] float32 (nats) of every chain."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    ws, nws = _workspace(OP_ENTROPY, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_entropy(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                               out.data_ptr(), ws.data_ptr(), nws, _stream(phi.device))
    _check(rc, "lccrf_entropy")
    return out


def _two_chains(name, phi_p, phi_q, lengths, out, workspace):
    lib = load_library()
    dt, B, N, T = _phi_args(phi_p)
    if _phi_args(phi_q) != (dt, B, N, T) or phi_q.device != phi_p.device:
        raise LccrfError("phi_q must have phi_p's shape, dtype and device")
    ws, nws = _workspace(OP_CROSS_ENTROPY, B, N, T, dt, phi_p.device, workspace)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=phi_p.device)
    with torch.cuda.device(phi_p.device):
        rc = getattr(lib, name)(phi_p.data_ptr(), phi_q.data_ptr(), dt, _len_ptr(lengths, B, phi_p.device), B, N, T,
                                out.data_ptr(), ws.data_ptr(), nws, _stream(phi_p.device))
    _check(rc, name)
    return out


def lccrf_cross_entropy(phi_p: torch.Tensor, phi_q: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Cross-entropy H(p, q) [B] float32 (nats) of the chains of phi_p against those of phi_q."""
    return _two_chains("lccrf_cross_entropy", phi_p, phi_q, lengths, out, workspace)


def lccrf_kl_divergence(phi_p: torch.Tensor, phi_q: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Kullback-Leibler divergence KL(p || q) [B] float32 (nats)."""
    return _two_chains("lccrf_kl_divergence", phi_p, phi_q, lengths, out, workspace)


def lccrf_sample(phi: torch.Tensor, uniforms: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One sampled tag path per sequence [B, N] int32 (-1 past the length), drawn by forward-filtering
    backward-sampling from the given uniforms (float32 [B, N] in [0, 1) on phi's device)."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    if uniforms.dtype != torch.float32 or tuple(uniforms.shape) != (B, N) or not uniforms.is_contiguous() \
            or uniforms.device != phi.device:
        raise LccrfError("uniforms must be a contiguous float32 [B, N] tensor on phi's device")
    ws, nws = _workspace(OP_SAMPLE, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, N, dtype=torch.int32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_sample(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), uniforms.data_ptr(), B, N, T,
                              out.data_ptr(), ws.data_ptr(), nws, _stream(phi.device))
    _check(rc, "lccrf_sample")
    return out


def lccrf_sample_seeded(phi: torch.Tensor, seed: int, lengths: Optional[torch.Tensor] = None, *,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One sampled tag path per sequence [B, N] int32 (-1 past the length) with the uniforms drawn in the library by
    Philox4x32-10 under the 64-bit `seed` (counter b * N + i): reproducible from the seed alone."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    ws, nws = _workspace(OP_SAMPLE, B, N, T, dt, phi.device, workspace)
    if out is None:
        out = torch.empty(B, N, dtype=torch.int32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_sample_seeded(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), int(seed) & (2 ** 64 - 1), B, N, T,
                                     out.data_ptr(), ws.data_ptr(), nws, _stream(phi.device))
    _check(rc, "lccrf_sample_seeded")
    return out


def lccrf_semi_markov_log_partition(phi: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """logZ [B] float32 of the semi-Markov CRF with potentials phi [B, N, K, T, T] (float32 or bfloat16, on the
    GPU, contiguous): phi[b, i, k, s, t] scores a segment tagged t that ends at position i and covers k + 1
    positions, after a segment tagged s (row 0 for the first segment)."""
    lib = load_library()
    if phi.dim() != 5 or phi.shape[3] != phi.shape[4]:
        raise ValueError(f"phi must be [B, N, K, T, T], got {tuple(phi.shape)}")
    B, N, K, T, _ = (int(v) for v in phi.shape)
    dt, _, _, _ = _phi_args(phi.view(B, N * K, T, T))
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=phi.device)
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_semi_markov_log_partition(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, K, T,
                                                 out.data_ptr(), _stream(phi.device))
    _check(rc, "lccrf_semi_markov_log_partition")
    return out


def _structured_args(emit: torch.Tensor, trans: torch.Tensor):
    if emit.dtype != torch.float32 or trans.dtype != torch.float32 or emit.dim() != 3 or trans.dim() != 2:
        raise LccrfError("emit must be float32 [B, N, T] and trans float32 [T, T]")
    B, N, T = emit.shape
    if tuple(trans.shape) != (T, T) or not emit.is_contiguous() or not trans.is_contiguous() or not emit.is_cuda \
            or trans.device != emit.device:
        raise LccrfError("emit [B, N, T] and trans [T, T] must be contiguous tensors on one GPU")
    return B, N, T


def lccrf_log_partition_structured(emit: torch.Tensor, trans: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """logZ [B] of the chains with potentials trans[s, t] + emit[b, i, t] (never materialised)."""
    lib = load_library()
    B, N, T = _structured_args(emit, trans)
    ws, nws = _workspace(OP_LOGZ, B, N, T, LCCRF_F32, emit.device, workspace)
    if out is None:
        out = torch.empty(B, dtype=torch.float32, device=emit.device)
    with torch.cuda.device(emit.device):
        rc = lib.lccrf_log_partition_structured(emit.data_ptr(), trans.data_ptr(), _len_ptr(lengths, B, emit.device),
                                                B, N, T, out.data_ptr(), ws.data_ptr(), nws, _stream(emit.device))
    _check(rc, "lccrf_log_partition_structured")
    return out


def lccrf_marginals_structured(emit: torch.Tensor, trans: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                               out: Optional[torch.Tensor] = None, logZ: Optional[torch.Tensor] = None,
                               workspace: Optional[torch.Tensor] = None):
    """(logZ [B], marginals [B, N, T, T]) for potentials trans[s, t] + emit[b, i, t]."""
    lib = load_library()
    B, N, T = _structured_args(emit, trans)
    ws, nws = _workspace(OP_MARGINALS, B, N, T, LCCRF_F32, emit.device, workspace)
    if out is None:
        out = torch.empty(B, N, T, T, dtype=torch.float32, device=emit.device)
    if logZ is None:
        logZ = torch.empty(B, dtype=torch.float32, device=emit.device)
    with torch.cuda.device(emit.device):
        rc = lib.lccrf_marginals_structured(emit.data_ptr(), trans.data_ptr(), _len_ptr(lengths, B, emit.device),
                                            B, N, T, logZ.data_ptr(), out.data_ptr(), ws.data_ptr(), nws,
                                            _stream(emit.device))
    _check(rc, "lccrf_marginals_structured")
    return logZ, out


def lccrf_argmax_structured(emit: torch.Tensor, trans: torch.Tensor, lengths: Optional[torch.Tensor] = None, *,
                            out: Optional[torch.Tensor] = None, score: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None):
    """(best_score [B], tags [B, N]) for potentials trans[s, t] + emit[b, i, t]."""
    lib = load_library()
    B, N, T = _structured_args(emit, trans)
    ws, nws = _workspace(OP_ARGMAX, B, N, T, LCCRF_F32, emit.device, workspace)
    if out is None:
        out = torch.empty(B, N, dtype=torch.int32, device=emit.device)
    if score is None:
        score = torch.empty(B, dtype=torch.float32, device=emit.device)
    with torch.cuda.device(emit.device):
        rc = lib.lccrf_argmax_structured(emit.data_ptr(), trans.data_ptr(), _len_ptr(lengths, B, emit.device),
                                         B, N, T, score.data_ptr(), out.data_ptr(), ws.data_ptr(), nws,
                                         _stream(emit.device))
    _check(rc, "lccrf_argmax_structured")
    return score, out


def lccrf_marginals_timed(phi: torch.Tensor, lengths: Optional[torch.Tensor], out: torch.Tensor,
                          logZ: torch.Tensor, workspace: torch.Tensor, events, algo: int = ALGO_AUTO) -> None:
    """``lccrf_marginals`` with three ``torch.cuda.Event(enable_timing=True)`` objects recorded by
    the library before, between and after its two passes (benchmark instrumentation).  The
    events must have been recorded once before, so that their HIP handles exist."""
    lib = load_library()
    dt, B, N, T = _phi_args(phi)
    handles = [ctypes.c_void_p(e.cuda_event) for e in events]
    with torch.cuda.device(phi.device):
        rc = lib.lccrf_marginals_timed(phi.data_ptr(), dt, _len_ptr(lengths, B, phi.device), B, N, T,
                                       logZ.data_ptr(), out.data_ptr(), workspace.data_ptr(),
                                       workspace.numel(), _stream(phi.device), algo, *handles)
    _check(rc, "lccrf_marginals_timed")


def lccrf_stream_probe(src: torch.Tensor, dst: Optional[torch.Tensor], workgroups: int, sink: torch.Tensor) -> int:
    """Benchmark instrumentation: `workgroups` workgroups stream `src` (read only, or copied to `dst`); returns the
    bytes covered.  Enqueued on the current stream; the caller times it."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    if dst is not None and dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst is smaller than src")
    with torch.cuda.device(src.device):
        rc = lib.lccrf_stream_probe(src.data_ptr(), None if dst is None else dst.data_ptr(), nbytes, int(workgroups),
                                    sink.data_ptr(), _stream(src.device))
    _check(rc, "lccrf_stream_probe")
    return int(lib.lccrf_stream_probe_bytes(nbytes, int(workgroups)))
