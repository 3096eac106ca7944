"""GPU parity of the two-chain queries (lccrf_cross_entropy, lccrf_kl_divergence) against the CPU
oracle, which forms them from their definitions: H(p, q) = logZ_q - sum_e p(e) phi_q(e) from the
fp64 marginals of p, KL(p || q) = H(p, q) - H(p).  The library never forms marginals for them.

Tolerances: both results are differences of quantities of the size of logZ and of the expected
score, each carried in fp32 with fp64 offsets; the cross-entropy is held to 1e-5 of that size (the
bar of logZ itself), the KL divergence, whose expectation is formed from per-edge differences,
to 1e-5 of the sizes of logZ_p, logZ_q plus 1e-4 of itself."""
import math

import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import crf  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _pair(seed, B, N, T, scale_p=1.5, scale_q=1.0, dtype="f32", **kw):
    p, lens = workloads.random_case(seed, B, N, T, scale=scale_p, dtype=dtype, **kw)
    q, _ = workloads.random_case(seed + 7919, B, N, T, scale=scale_q, dtype=dtype)
    return p, q, lens


def _check(crf, oracle_mod, p, q, lens, what):
    lens_np = None if lens is None else lens.numpy()
    dl = None if lens is None else lens.cuda()
    dp, dq = p.cuda(), q.cuda()
    got_h = crf.lccrf_cross_entropy(dp, dq, dl).cpu().numpy().astype(np.float64)
    got_k = crf.lccrf_kl_divergence(dp, dq, dl).cpu().numpy().astype(np.float64)
    want_h = oracle_mod.cross_entropy(p, q, lens_np)
    want_k = oracle_mod.kl_divergence(p, q, lens_np)
    lzp = np.abs(oracle_mod.log_partition(p, lens_np))
    lzq = np.abs(oracle_mod.log_partition(q, lens_np))
    size = np.maximum(1.0, np.where(np.isfinite(lzp), lzp, 0) + np.where(np.isfinite(lzq), lzq, 0))
    for name, got, want, tol in (("cross-entropy", got_h, want_h, 1e-5 * (size + np.abs(np.nan_to_num(want_h, posinf=0)))),
                                 ("KL", got_k, want_k, 1e-5 * size + 1e-4 * np.abs(np.nan_to_num(want_k, posinf=0)))):
        same_special = (np.isnan(got) & np.isnan(want)) | (np.isinf(want) & (got == want))
        bad = ~same_special & ~(np.abs(got - want) <= tol)
        assert not bad.any(), f"{what}: {name} mismatch at {np.nonzero(bad)[0][:6]}: {got[bad][:4]} vs {want[bad][:4]}"


SHAPES = [(1, 5), (2, 1), (3, 7), (5, 8), (16, 40), (17, 9), (32, 65), (33, 6), (48, 33), (64, 12), (100, 9), (128, 10),
          (200, 4), (16, 300), (32, 200)]


@pytest.mark.parametrize("T,N", SHAPES)
def test_two_chains_sweep(crf, oracle_mod, T, N):
    p, q, lens = _pair(7000 + 13 * T + N, 5, N, T, ragged=True, min_len=0)
    _check(crf, oracle_mod, p, q, lens, f"T={T} N={N}")


@pytest.mark.parametrize("T", [4, 20, 128])
def test_equal_chains(crf, oracle_mod, T):
    """q = p: H(p, p) is the entropy (checked against lccrf_entropy too) and the divergence vanishes;
    a per-position constant added to q changes neither distribution."""
    p, lens = workloads.random_case(7100 + T, 4, 30, T, scale=2.0, ragged=True, min_len=1)
    dp, dl = p.cuda(), lens.cuda()
    H = crf.lccrf_entropy(dp, dl).cpu().numpy()
    Hpp = crf.lccrf_cross_entropy(dp, dp.clone(), dl).cpu().numpy()
    lz = np.abs(oracle_mod.log_partition(p, lens.numpy()))
    assert np.all(np.abs(Hpp - H) <= 2e-5 * np.maximum(1.0, lz))
    kl = crf.lccrf_kl_divergence(dp, dp.clone(), dl).cpu().numpy()
    assert np.all(np.abs(kl) <= 1e-5 * np.maximum(1.0, lz))
    shifted = (p + torch.linspace(-3, 3, 30).view(1, 30, 1, 1)).contiguous()
    kl = crf.lccrf_kl_divergence(dp, shifted.cuda(), dl).cpu().numpy()
    assert np.all(np.abs(kl) <= 2e-5 * np.maximum(1.0, lz) + 1e-3)   # the shifted copy is rounded to fp32


@pytest.mark.parametrize("T", [16, 48])
def test_two_chains_bf16_peaked_and_forbidden_edges(crf, oracle_mod, T):
    p, q, lens = _pair(7200 + T, 4, 60, T, scale_p=6.0, scale_q=3.0, dtype="bf16", ragged=True, min_len=20)
    _check(crf, oracle_mod, p, q, lens, f"peaked bf16 T={T}")
    p, q, _ = _pair(7300 + T, 5, 25, T)
    ninf = float("-inf")
    p[0, :, 3, :] = ninf             # p never leaves tag 3: q's values on those edges do not matter
    q[0, 5, 3, :] = ninf
    q[1, 10, :, 5] = ninf            # q forbids what p allows: +inf
    p[2, 12, :, :] = ninf            # p has no finite path: NaN
    mask = torch.rand(25, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
    p[3][mask] = ninf
    p[3, :, torch.arange(T), torch.arange(T)] = 0.0
    q[4, 12, :, :] = ninf            # q has no finite path, p has: +inf - (-inf) on the oracle's side is NaN
    _check(crf, oracle_mod, p, q, None, f"-inf T={T}")


@pytest.mark.parametrize("T,N,k", [(3, 70, 4), (16, 130, 8), (16, 1100, 16), (13, 300, 8), (24, 300, 8), (32, 530, 32)])
def test_two_chains_under_the_scan(crf, oracle_mod, T, N, k):
    """Long chains over few tags take the chunked scan: the expectation is then added up edge by edge
    in every chunk.  Small chunks so that short inputs cover many chunks, ragged and empty sequences,
    peaked bf16 potentials, forbidden edges, a chain without a finite path."""
    crf.set_scan_chunk(k)
    try:
        p, q, lens = _pair(7400 + 13 * T + N, 6, N, T, ragged=True, min_len=0)
        lens[0], lens[1] = N, 0
        _check(crf, oracle_mod, p, q, lens, f"scan T={T} N={N} chunk {k}")
        p, q, lens = _pair(7500 + 13 * T + N, 3, N, T, scale_p=6.0, scale_q=3.0, dtype="bf16", ragged=True, min_len=N // 2)
        _check(crf, oracle_mod, p, q, lens, f"scan peaked bf16 T={T} N={N} chunk {k}")
        if T >= 8:
            p, q, _ = _pair(7600 + 13 * T + N, 4, N, T)
            ninf = float("-inf")
            p[0, :, 3, :] = ninf
            q[0, 5, 3, :] = ninf
            q[1, 10, :, 5] = ninf
            p[2, 12, :, :] = ninf
            mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
            p[3][mask] = ninf
            p[3, :, torch.arange(T), torch.arange(T)] = 0.0
            _check(crf, oracle_mod, p, q, None, f"scan -inf T={T} N={N} chunk {k}")
    finally:
        crf.set_scan_chunk(0)


@pytest.mark.parametrize("key", ["cfg1", "cfg2", "cfg3", "cfg5"])
def test_two_chains_named_workloads(crf, oracle_mod, key):
    w = workloads.WORKLOADS[key]
    p = workloads.phi_batch(w)
    g = torch.Generator().manual_seed(99)
    q = (p.float() * 0.5 + 0.3 * torch.randn(p.shape, generator=g)).to(p.dtype).contiguous()
    _check(crf, oracle_mod, p, q, workloads.lengths(w), key)


def test_two_chains_at_config4_full_size(crf, oracle_mod):
    """Full-size config 4, the whole batch in one call: KL >= 0 on every sequence, and two full-length
    sequences of both queries against the oracle (q = 0.7 p, the same float32 products on both sides)."""
    w = workloads.WORKLOADS["cfg4"]
    p = torch.empty(w.B, w.N, w.T, w.T, dtype=torch.float32, device="cuda")
    workloads.phi_batch(w, out=p)
    q = (0.7 * p).contiguous()
    kl = crf.lccrf_kl_divergence(p, q).cpu().numpy().astype(np.float64)
    H = crf.lccrf_cross_entropy(p, q).cpu().numpy().astype(np.float64)
    assert (kl > 0).all() and np.isfinite(H).all()
    pick = [5, 62]
    pc = torch.stack([workloads.phi_sequence(w, b) for b in pick]).contiguous()
    qc = (0.7 * pc).contiguous()
    assert torch.equal(qc, q[pick].cpu())
    want_h = oracle_mod.cross_entropy(pc, qc, None)
    want_k = oracle_mod.kl_divergence(pc, qc, None)
    size = np.abs(oracle_mod.log_partition(pc, None)) + np.abs(oracle_mod.log_partition(qc, None))
    assert np.all(np.abs(H[pick] - want_h) <= 1e-5 * (size + np.abs(want_h))), f"{H[pick]} vs {want_h}"
    assert np.all(np.abs(kl[pick] - want_k) <= 1e-5 * size + 1e-4 * np.abs(want_k)), f"{kl[pick]} vs {want_k}"


def test_two_chains_argument_checks(crf):
    p = torch.zeros(2, 4, 3, 3, device="cuda")
    with pytest.raises(crf.LccrfError, match="shape"):
        crf.lccrf_cross_entropy(p, torch.zeros(2, 4, 4, 4, device="cuda"))
    with pytest.raises(crf.LccrfError, match="shape"):
        crf.lccrf_kl_divergence(p, p.to(torch.bfloat16))
    out = crf.lccrf_cross_entropy(p, p, torch.tensor([4, 0], dtype=torch.int32, device="cuda")).cpu().numpy()
    assert out[0] == pytest.approx(4 * math.log(3), rel=1e-6) and out[1] == 0.0


@pytest.mark.parametrize("T,N", [(129, 9), (130, 17), (192, 33), (200, 40), (255, 12), (256, 70)])
def test_two_chains_largest_tag_sets(crf, oracle_mod, T, N):
    """129 .. 256 tags: both tensors stream through the half chains in batches of 64 rows."""
    p, q, lens = _pair(7600 + 13 * T + N, 4, N, T, ragged=True, min_len=0)
    _check(crf, oracle_mod, p, q, lens, f"T={T} N={N}")


@pytest.mark.parametrize("T", [160, 256])
def test_two_chains_largest_tag_sets_replays_bf16_and_forbidden_edges(crf, oracle_mod, T):
    p, q, lens = _pair(7700 + T, 3, 24, T, scale_p=1.0, ragged=True, min_len=10)
    p[:, 5] *= 60.0
    p[:, 6] -= 300.0
    p[:, 11] += 500.0
    p[:, 17] *= 40.0
    _check(crf, oracle_mod, p, q, lens, f"jumps T={T}")
    p, q, lens = _pair(7800 + T, 3, 30, T, scale_p=5.0, scale_q=3.0, dtype="bf16", ragged=True, min_len=12)
    _check(crf, oracle_mod, p, q, lens, f"peaked bf16 T={T}")
    p, q, _ = _pair(7900 + T, 5, 14, T)
    ninf = float("-inf")
    p[0, :, 3, :] = ninf             # p never leaves tag 3: q's values on those edges do not matter
    q[0, 5, 3, :] = ninf
    q[1, 10, :, 5] = ninf            # q forbids what p allows: +inf
    p[2, 12, :, :] = ninf            # p has no finite path: NaN
    mask = torch.rand(14, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
    p[3][mask] = ninf
    p[3, :, torch.arange(T), torch.arange(T)] = 0.0
    q[4, 12, :, :] = ninf            # q has no finite path, p has
    _check(crf, oracle_mod, p, q, None, f"-inf T={T}")
