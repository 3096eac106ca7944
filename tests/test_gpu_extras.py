"""GPU parity of the queries derived from the partition function: log-probability of a given
path and entropy, against the CPU oracle (which computes them from their definitions: the
path's score minus logZ, and logZ - sum_e p(e) phi(e) over the oracle's own marginals).

Tolerances: log p(y) is the difference of two numbers of the size of logZ, so it inherits the
logZ bar as an absolute one: 1e-5 * max(1, |logZ|, |score|).  Entropy (float32 recursions over
up to N positions) is held to 1e-4 * max(1, H)."""
import math

import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import crf  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _check_log_prob(crf, oracle_mod, phi, lens, tags, what):
    got = crf.lccrf_log_prob(phi.cuda(), tags.cuda(), None if lens is None else lens.cuda()).cpu().numpy().astype(np.float64)
    lens_np = None if lens is None else lens.numpy()
    want = oracle_mod.log_prob(phi, tags.numpy(), lens_np)
    logZ = oracle_mod.log_partition(phi, lens_np)
    tol = 1e-5 * np.maximum(1.0, np.maximum(np.abs(logZ), np.abs(want + logZ)))
    both_nan = np.isnan(got) & np.isnan(want)
    bad = ~both_nan & ~(np.abs(got - want) <= tol)
    assert not bad.any(), f"{what}: log_prob mismatch {got[bad][:4]} vs {want[bad][:4]}"


def _check_entropy(crf, oracle_mod, phi, lens, what):
    got = crf.lccrf_entropy(phi.cuda(), None if lens is None else lens.cuda()).cpu().numpy().astype(np.float64)
    want = oracle_mod.entropy(phi, None if lens is None else lens.numpy())
    both_nan = np.isnan(got) & np.isnan(want)
    bad = ~both_nan & ~(np.abs(got - want) <= 1e-4 * np.maximum(1.0, np.abs(want)))
    assert not bad.any(), f"{what}: entropy mismatch at {np.nonzero(bad)[0][:6]}: {got[bad][:4]} vs {want[bad][:4]}"
    return np.abs(got - want)[~both_nan].max() if (~both_nan).any() else 0.0


SHAPES = [(1, 5), (2, 1), (3, 7), (5, 8), (16, 40), (17, 9), (32, 65), (33, 6), (48, 33), (64, 12), (100, 9), (128, 10),
          (200, 4)]


@pytest.mark.parametrize("T,N", SHAPES)
def test_log_prob_random_paths(crf, oracle_mod, T, N):
    phi, lens = workloads.random_case(6000 + 13 * T + N, 5, N, T, scale=1.5, ragged=True, min_len=0)
    g = torch.Generator().manual_seed(T * 100 + N)
    tags = torch.randint(0, T, (5, N), generator=g, dtype=torch.int32)
    _check_log_prob(crf, oracle_mod, phi, lens, tags, f"T={T} N={N}")


def test_log_prob_of_the_best_path_and_bad_tags(crf, oracle_mod):
    phi, lens = workloads.random_case(6100, 4, 30, 12, scale=2.0, ragged=True, min_len=5)
    _, best = crf.lccrf_argmax(phi.cuda(), lens.cuda())
    _check_log_prob(crf, oracle_mod, phi, lens, best.cpu(), "best path")   # -1 past the lengths is ignored
    tags = best.cpu().clone()
    tags[1, 2] = 12          # out of range inside the chain
    tags[2, 0] = -1
    got = crf.lccrf_log_prob(phi.cuda(), tags.cuda(), lens.cuda()).cpu().numpy()
    assert np.isnan(got[1]) and np.isnan(got[2]) and np.isfinite(got[0]) and np.isfinite(got[3])


def test_log_prob_bf16_and_long_chain(crf, oracle_mod):
    """Config 5 (the scan computes logZ): the score and logZ are ~1e5 each, their difference is not."""
    w = workloads.WORKLOADS["cfg5"]
    phi = workloads.phi_batch(w)
    lens = workloads.lengths(w)
    _, best = crf.lccrf_argmax(phi.cuda(), lens.cuda())
    _check_log_prob(crf, oracle_mod, phi, lens, best.cpu(), "cfg5 best path")
    g = torch.Generator().manual_seed(5)
    _check_log_prob(crf, oracle_mod, phi, lens, torch.randint(0, w.T, (w.B, w.N), generator=g, dtype=torch.int32), "cfg5 random path")


@pytest.mark.parametrize("T,N", SHAPES + [(16, 300), (32, 200), (48, 128)])
def test_entropy_sweep(crf, oracle_mod, T, N):
    phi, lens = workloads.random_case(6200 + 13 * T + N, 5, N, T, scale=1.5, ragged=True, min_len=0)
    _check_entropy(crf, oracle_mod, phi, lens, f"T={T} N={N}")


@pytest.mark.parametrize("T", [5, 32, 48, 128])
def test_entropy_closed_forms(crf, T):
    N = 20
    lens = torch.tensor([20, 7, 1, 0], dtype=torch.int32)
    H = crf.lccrf_entropy(torch.zeros(4, N, T, T, device="cuda"), lens.cuda()).cpu().numpy()
    assert np.allclose(H, lens.numpy() * math.log(T), rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("T", [16, 48])
def test_entropy_peaked_bf16_and_forbidden_edges(crf, oracle_mod, T):
    phi, lens = workloads.random_case(6300 + T, 4, 60, T, scale=6.0, ragged=True, min_len=20, dtype="bf16")
    _check_entropy(crf, oracle_mod, phi, lens, f"peaked bf16 T={T}")
    phi, _ = workloads.random_case(6400 + T, 4, 25, T)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 10, :, 5] = ninf
    phi[2, 12, :, :] = ninf          # no finite path: NaN on both sides
    mask = torch.rand(25, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
    phi[3][mask] = ninf
    phi[3, :, torch.arange(T), torch.arange(T)] = 0.0
    _check_entropy(crf, oracle_mod, phi, None, f"-inf T={T}")


@pytest.mark.parametrize("T,N", [(3, 256), (5, 700), (16, 300), (16, 1000), (20, 260), (24, 513), (32, 256), (32, 640)])
def test_entropy_under_the_scan(crf, oracle_mod, T, N):
    """Long chains in small batches take the chunked scan: the entropy is then added up edge by edge
    (H(y_0) + sum_i H(y_i | y_{i-1})) in the second pass, chunk by chunk."""
    phi, lens = workloads.random_case(6500 + 13 * T + N, 5, N, T, scale=1.5, ragged=True, min_len=0)
    lens[0] = N
    lens[1] = 1
    _check_entropy(crf, oracle_mod, phi, lens, f"scan T={T} N={N}")


def test_entropy_under_the_scan_peaked_bf16_and_forbidden_edges(crf, oracle_mod):
    w = workloads.WORKLOADS["cfg5"]
    _check_entropy(crf, oracle_mod, workloads.phi_batch(w), workloads.lengths(w), "cfg5")
    T, N = 16, 400
    phi, _ = workloads.random_case(6600, 4, N, T)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 210, :, 5] = ninf
    phi[2, 300, :, :] = ninf          # no finite path: NaN on both sides
    mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
    phi[3][mask] = ninf
    phi[3, :, torch.arange(T), torch.arange(T)] = 0.0
    _check_entropy(crf, oracle_mod, phi, None, "scan -inf")
    H = crf.lccrf_entropy(torch.zeros(3, 512, 32, 32, device="cuda"),
                          torch.tensor([512, 300, 0], dtype=torch.int32, device="cuda")).cpu().numpy()
    assert np.allclose(H, np.array([512, 300, 0]) * math.log(32), rtol=1e-5)


@pytest.mark.parametrize("key", ["cfg1", "cfg2", "cfg3"])
def test_entropy_named_workloads(crf, oracle_mod, key):
    w = workloads.WORKLOADS[key]
    _check_entropy(crf, oracle_mod, workloads.phi_batch(w), workloads.lengths(w), key)


def test_entropy_at_config4_full_size(crf, oracle_mod):
    """Full-size config 4, the whole batch in one call (the launch configuration the benchmark times):
    0 <= H <= L log T on all sequences, and three full-length sequences against the oracle, which forms
    H = logZ - sum_e p(e) phi(e) from its own float64 marginals."""
    w = workloads.WORKLOADS["cfg4"]
    phi = torch.empty(w.B, w.N, w.T, w.T, dtype=torch.float32, device="cuda")
    workloads.phi_batch(w, out=phi)
    H = crf.lccrf_entropy(phi).cpu().numpy().astype(np.float64)
    assert ((H >= 0) & (H <= w.N * math.log(w.T))).all()
    pick = [0, 29, 63]
    want = oracle_mod.entropy(torch.stack([workloads.phi_sequence(w, b) for b in pick]).contiguous(), None)
    assert np.all(np.abs(H[pick] - want) <= 1e-4 * np.maximum(1.0, np.abs(want))), f"{H[pick]} vs {want}"
    # the path's log-probability at full size: the best path of every sequence, three of them against the oracle
    _, best = crf.lccrf_argmax(phi)
    lp = crf.lccrf_log_prob(phi, best).cpu().numpy().astype(np.float64)
    phi_pick = torch.stack([workloads.phi_sequence(w, b) for b in pick]).contiguous()
    want_lp = oracle_mod.log_prob(phi_pick, best[pick].cpu().numpy(), None)
    want_lz = oracle_mod.log_partition(phi_pick, None)
    tol = 1e-5 * np.maximum(1.0, np.maximum(np.abs(want_lz), np.abs(want_lp + want_lz)))
    assert np.all(np.abs(lp[pick] - want_lp) <= tol), f"{lp[pick]} vs {want_lp}"


@pytest.mark.parametrize("T,N", [(129, 9), (130, 17), (192, 33), (200, 40), (255, 12), (256, 70)])
def test_entropy_largest_tag_sets(crf, oracle_mod, T, N):
    """129 .. 256 tags: the half chains stream every matrix in batches of 64 rows (three or four batches, ragged
    last batch, tag counts that are not multiples of 4)."""
    phi, lens = workloads.random_case(6500 + 13 * T + N, 4, N, T, scale=1.5, ragged=True, min_len=0)
    _check_entropy(crf, oracle_mod, phi, lens, f"T={T} N={N}")


@pytest.mark.parametrize("T", [160, 256])
def test_entropy_largest_tag_sets_replays_bf16_and_forbidden_edges(crf, oracle_mod, T):
    """Scale jumps between positions (the speculative step is rejected and the matrix streamed again), bfloat16
    potentials, -inf edges and a sequence without any finite path."""
    phi, lens = workloads.random_case(6600 + T, 3, 24, T, scale=1.0, ragged=True, min_len=10)
    phi[:, 5] *= 60.0
    phi[:, 6] -= 300.0
    phi[:, 11] += 500.0
    phi[:, 17] *= 40.0
    _check_entropy(crf, oracle_mod, phi, lens, f"jumps T={T}")
    phi, lens = workloads.random_case(6700 + T, 3, 30, T, scale=5.0, ragged=True, min_len=12, dtype="bf16")
    _check_entropy(crf, oracle_mod, phi, lens, f"peaked bf16 T={T}")
    phi, _ = workloads.random_case(6800 + T, 4, 14, T)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 10, :, 5] = ninf
    phi[2, 12, :, :] = ninf          # no finite path: NaN on both sides
    mask = torch.rand(14, T, T, generator=torch.Generator().manual_seed(7)) < 0.5
    phi[3][mask] = ninf
    phi[3, :, torch.arange(T), torch.arange(T)] = 0.0
    _check_entropy(crf, oracle_mod, phi, None, f"-inf T={T}")
