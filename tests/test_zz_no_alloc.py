"""The entry point that allocates nothing, `lccrf_marginals_static`, against `lccrf_marginals`.

Both run the same kernels; the only difference is where the scratch lives (a buffer built into the
library instead of the caller's workspace).  Every case makes two calls in a row on the same GPU,
the second on a smaller input, so the second call finds the first call's contents in the buffer.
Results are held to the bar of the parity tests: logZ relative 1e-5, marginals absolute 1e-5
(1e-4 for bfloat16-stored potentials), exact zeros outside the chains.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads

pytestmark = pytest.mark.gpu

ETOOBIG = -7


@pytest.fixture(scope="module")
def crf():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03291_amd import binding
    binding.load_library()
    return binding


def _call_static(crf, phi, lens):
    """Through the C ABI: plain pointers, the current stream, outputs poisoned beforehand."""
    lib = crf.load_library()
    B, N, T, _ = phi.shape
    dt = crf.LCCRF_BF16 if phi.dtype == torch.bfloat16 else crf.LCCRF_F32
    mu = torch.full((B, N, T, T), float("nan"), device=phi.device)
    lz = torch.full((B,), float("nan"), device=phi.device)
    rc = lib.lccrf_marginals_static(ctypes.c_void_p(phi.data_ptr()), dt,
                                    ctypes.c_void_p(lens.data_ptr()) if lens is not None else None, B, N, T,
                                    ctypes.c_void_p(lz.data_ptr()), ctypes.c_void_p(mu.data_ptr()),
                                    ctypes.c_void_p(torch.cuda.current_stream(phi.device).cuda_stream))
    assert rc == 0, crf.strerror(rc)
    return lz, mu


def _compare(crf, phi_cpu, lens_cpu, what):
    dev = torch.device("cuda:0")
    phi = phi_cpu.to(dev)
    lens = None if lens_cpu is None else lens_cpu.to(dev)
    lz_s, mu_s = _call_static(crf, phi, lens)
    lz_w, mu_w = crf.lccrf_marginals(phi, lens)
    torch.cuda.synchronize()
    atol = 1e-4 if phi.dtype == torch.bfloat16 else 1e-5
    a, b = lz_s.cpu().numpy().astype(np.float64), lz_w.cpu().numpy().astype(np.float64)
    same_inf = np.isneginf(a) & np.isneginf(b)
    assert (same_inf | (np.abs(a - b) <= 1e-5 * np.maximum(1.0, np.abs(b)))).all(), f"{what}: logZ {a} vs {b}"
    ms, mw = mu_s.cpu().numpy(), mu_w.cpu().numpy()
    assert np.isfinite(ms).all(), f"{what}: non-finite marginals"
    err = float(np.abs(ms - mw).max())
    assert err <= atol, f"{what}: max |static - workspace| = {err:.3e}"
    assert np.array_equal(ms == 0, mw == 0), f"{what}: zeros outside the chains differ"


# (first call, then a smaller second call): one case per family of kernels the query dispatches to
PAIRS = [
    ("one wave per chain, then one launch for short chains", (6, 90, 24, "f32", True), (3, 40, 11, "f32", True)),
    ("four waves per chain", (5, 70, 48, "f32", True), (2, 33, 40, "f32", False)),
    ("two workgroups per chain (T = 128), then 16 waves per chain", (4, 40, 128, "f32", False), (3, 9, 100, "f32", True)),
    ("chunked scan over a long chain, bfloat16", (2, 2048, 16, "bf16", False), (1, 600, 13, "bf16", False)),
    ("largest tag sets", (2, 6, 256, "f32", True), (1, 4, 129, "f32", False)),
]


@pytest.mark.parametrize("what,first,second", PAIRS, ids=[p[0] for p in PAIRS])
def test_static_scratch_matches_workspace_call_twice_in_a_row(crf, what, first, second):
    for k, (B, N, T, dtype, ragged) in enumerate((first, second)):
        phi, lens = workloads.random_case(9100 + 10 * T + k, B, N, T, scale=1.5, ragged=ragged, min_len=0, dtype=dtype)
        _compare(crf, phi, lens if ragged else None, f"{what} [call {k + 1}: B={B} N={N} T={T} {dtype}]")


def test_static_scratch_refuses_what_does_not_fit(crf):
    lib = crf.load_library()
    limit = lib.lccrf_static_scratch_bytes()
    assert limit == 64 << 20
    B, N, T = 256, 1024, 128
    assert crf.workspace_bytes(crf.OP_MARGINALS, B, N, T, crf.LCCRF_F32) > limit
    fake = ctypes.c_void_p(4096)   # never dereferenced: the call is refused on the host
    assert lib.lccrf_marginals_static(fake, 0, None, B, N, T, fake, fake, None) == ETOOBIG
    assert "built-in" in crf.strerror(ETOOBIG)


def test_static_scratch_serves_the_headline_shape(crf):
    """The headline shape B=64, N=512, T=128 fits the built-in buffer (host arithmetic only)."""
    assert crf.workspace_bytes(crf.OP_MARGINALS, 64, 512, 128, crf.LCCRF_F32) <= crf.load_library().lccrf_static_scratch_bytes()
