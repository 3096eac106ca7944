"""Seeded synthetic inputs for the batched linear-chain CRF path.

This module only draws random tensors.  It holds none of the method's
arithmetic, so both the HIP path and the independent CPU oracle may be fed from
it without sharing any code of the dynamic program itself.

The paper benchmarks its linear-chain CRF on random potentials of a fixed shape
(appendix "Empirical comparisons", table of tested sizes), not on a dataset, so
random tensors of the stated shapes are the workload, not a stand-in for one.

Recipe (all draws on the CPU with `torch.Generator`, so every consumer sees the
same bits):

* workload k (1-based) has base seed ``SEED0 + k``;
* shared draws (lengths, then the tagging workload's transition matrix) use a
  generator seeded with ``base * 65536 + 65535``;
* sequence b's own draw uses a generator seeded with ``base * 65536 + b``, which
  makes any single sequence reproducible without drawing the others.

``phi[b, i, s, t]`` is the log-potential of tag s at position i-1 followed by tag
t at position i; one T x T matrix per position, as the paper's linear-chain CRF
takes them (section "Sequence Tagging").
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

SEED0 = 230803291


@dataclass(frozen=True)
class Workload:
    """Shape and value recipe of one synthetic workload."""

    key: str
    index: int  # 1-based; enters the seed
    B: int
    N: int
    T: int
    dtype: str  # "f32" or "bf16": storage type of phi
    len_lo: int  # lengths are uniform integers in [len_lo, len_hi]
    len_hi: int
    kind: str  # "iid" | "tagging"
    scale: float  # multiplies the unit normal draw
    note: str


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 4, 8, 5, "f32", 8, 8, "iid", 1.0,
                     "tiny; every one of the 5^8 tag paths can be enumerated"),
    "cfg2": Workload("cfg2", 2, 32, 64, 32, "f32", 32, 64, "iid", 1.0,
                     "ragged lengths uniform in [32, 64]"),
    "cfg3": Workload("cfg3", 3, 128, 128, 48, "f32", 16, 128, "tagging", 2.0,
                     "phi = emit[b,i,t] + trans[s,t]; emit std 2, trans std 1; lengths in [16, 128]"),
    "cfg4": Workload("cfg4", 4, 64, 512, 128, "f32", 512, 512, "iid", 1.0,
                     "large tag set; 2.1 GB of potentials streamed from HBM"),
    "cfg5": Workload("cfg5", 5, 4, 16384, 16, "bf16", 16384, 16384, "iid", 10.0,
                     "long, peaked (x10), bf16-stored potentials"),
    # The paper's own benchmark shapes for this model (table of tested sizes).
    "paper_lccrf": Workload("paper_lccrf", 6, 128, 256, 32, "f32", 256, 256, "iid", 1.0,
                            "the size the paper times its linear-chain CRF on"),
    "paper_hmm": Workload("paper_hmm", 7, 1, 128, 32, "f32", 128, 128, "iid", 1.0,
                          "the size the paper lists for its HMM"),
    # Beyond the five configurations: the largest tag set the library serves (profiles, timing sweeps).
    "t256": Workload("t256", 8, 64, 256, 256, "f32", 256, 256, "iid", 1.0,
                     "largest tag set: 4.3 GB of potentials, matrices streamed in row batches"),
    "long32": Workload("long32", 9, 8, 4096, 32, "f32", 4096, 4096, "iid", 1.0,
                       "long chains over 32 tags in a small batch: every query under the chunked scan"),
}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _base(w: Workload) -> int:
    return (SEED0 + w.index) * 65536


def lengths(w: Workload) -> torch.Tensor:
    """int32 [B] sequence lengths of workload ``w``."""
    g = _gen(_base(w) + 65535)
    if w.len_lo == w.len_hi:
        return torch.full((w.B,), w.len_lo, dtype=torch.int32)
    return torch.randint(w.len_lo, w.len_hi + 1, (w.B,), generator=g, dtype=torch.int64).to(torch.int32)


def shared_transitions(w: Workload) -> Optional[torch.Tensor]:
    """float32 [T, T] transition scores shared by all sequences (tagging workload only)."""
    if w.kind != "tagging":
        return None
    g = _gen(_base(w) + 65535)
    if w.len_lo != w.len_hi:  # keep the draw order: lengths first, then trans
        torch.randint(w.len_lo, w.len_hi + 1, (w.B,), generator=g, dtype=torch.int64)
    return torch.randn(w.T, w.T, generator=g, dtype=torch.float32)


def phi_sequence(w: Workload, b: int, trans: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Dense [N, T, T] log-potentials of sequence ``b`` in the workload's storage dtype."""
    g = _gen(_base(w) + b)
    if w.kind == "iid":
        x = torch.randn(w.N, w.T, w.T, generator=g, dtype=torch.float32)
        if w.scale != 1.0:
            x = x * w.scale
    elif w.kind == "tagging":
        if trans is None:
            trans = shared_transitions(w)
        emit = torch.randn(w.N, w.T, generator=g, dtype=torch.float32) * w.scale
        x = emit[:, None, :] + trans[None, :, :]
    else:  # pragma: no cover
        raise ValueError(w.kind)
    if w.dtype == "bf16":
        x = x.to(torch.bfloat16)
    return x.contiguous()


def phi_batch(w: Workload, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Dense [B, N, T, T] log-potentials.  ``out`` may be a preallocated tensor on any
    device (each sequence is drawn on the CPU and copied into its slot)."""
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    if out is None:
        out = torch.empty(w.B, w.N, w.T, w.T, dtype=dt)
    trans = shared_transitions(w)
    for b in range(w.B):
        out[b].copy_(phi_sequence(w, b, trans))
    return out


def random_case(seed: int, B: int, N: int, T: int, *, scale: float = 1.0, ragged: bool = False,
                min_len: int = 0, dtype: str = "f32"):
    """A free-form seeded case for sweeps over small or odd shapes.

    Returns ``(phi [B,N,T,T], lengths int32 [B])``.  With ``ragged`` the lengths
    are uniform in [min_len, N]; otherwise all equal N.
    """
    g = _gen(SEED0 * 7 + seed)
    phi = torch.randn(B, N, T, T, generator=g, dtype=torch.float32) * scale
    if ragged:
        lens = torch.randint(min_len, N + 1, (B,), generator=g, dtype=torch.int64).to(torch.int32)
    else:
        lens = torch.full((B,), N, dtype=torch.int32)
    if dtype == "bf16":
        phi = phi.to(torch.bfloat16)
    return phi.contiguous(), lens


def semi_markov_case(seed: int, B: int, N: int, K: int, T: int, *, scale: float = 1.0, ragged: bool = False,
                     min_len: int = 0, dtype: str = "f32"):
    """Seeded potentials of a semi-Markov CRF: ``(phi [B,N,K,T,T], lengths int32 [B])``, iid normal
    times ``scale`` (the paper's benchmark for this model is b=1, n=64, 32 tags, segments up to 8)."""
    g = _gen(SEED0 * 11 + seed)
    phi = torch.randn(B, N, K, T, T, generator=g, dtype=torch.float32) * scale
    if ragged:
        lens = torch.randint(min_len, N + 1, (B,), generator=g, dtype=torch.int64).to(torch.int32)
    else:
        lens = torch.full((B,), N, dtype=torch.int32)
    if dtype == "bf16":
        phi = phi.to(torch.bfloat16)
    return phi.contiguous(), lens
