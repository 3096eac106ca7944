"""GPU parity of the chain-wave / producer-wave schedule (LCCRF_ALGO_SEQUENTIAL_LANES) against the CPU
oracle: log-partition and marginals, element by element, on seeded inputs, at the tolerances of
test_gpu_parity.py (logZ relative 1e-5, marginals absolute 1e-5 / 1e-4 for bfloat16).

The shapes span every block count of the kernels (8 .. 16, 17 .. 32, 33 .. 48, 52 .. 64 tags), tag counts
that are not a multiple of sixteen (zero padding inside the LDS tiles) or of four (matrices loaded element by
element, the last piece of a row cut short), chains shorter than the ring of tiles, the degenerate lengths 0, 1 and 2, and the inputs that must leave the linear domain: forbidden
edges (-inf), sequences with no finite path, scales that jump by hundreds of nats between positions and a
large common offset.
"""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import check_case, crf  # noqa: F401  (crf: the module-scoped binding fixture)

pytestmark = pytest.mark.gpu

TAGS = (8, 9, 10, 11, 12, 13, 16, 17, 20, 21, 30, 32, 33, 40, 45, 47, 48, 52, 64)


@pytest.mark.parametrize("T", TAGS)
@pytest.mark.parametrize("N", (1, 2, 3, 7, 33, 90))
def test_lanes_sweep_fp32(crf, oracle_mod, T, N):
    B = 6
    phi, _ = workloads.random_case(9000 + 13 * T + N, B, N, T, scale=1.5)
    lens = torch.tensor([N, 1, max(1, N // 2), 0, max(1, N - 1), min(N, 2)], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES, what=f"lanes T={T} N={N}",
               queries=("logz", "mu"))


@pytest.mark.parametrize("T,N", [(16, 70), (32, 41), (48, 33), (64, 25), (24, 9), (9, 50), (27, 40), (45, 33)])
def test_lanes_sweep_bf16(crf, oracle_mod, T, N):
    phi, _ = workloads.random_case(9100 + T + N, 3, N, T, scale=3.0, dtype="bf16")
    lens = torch.tensor([N, max(1, N // 3), N - 1 if N > 1 else 1], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES,
               what=f"lanes bf16 T={T} N={N}", queries=("logz", "mu"))


def test_lanes_no_lengths_argument(crf, oracle_mod):
    phi, _ = workloads.random_case(9200, 3, 50, 32)
    check_case(crf, oracle_mod, phi, None, algo=crf.ALGO_SEQUENTIAL_LANES, what="lanes, lengths = NULL",
               queries=("logz", "mu"))


@pytest.mark.parametrize("T", (13, 16, 29, 32, 45, 48, 64))
def test_lanes_forbidden_edges_take_the_log_domain_tail(crf, oracle_mod, T):
    N = 24
    phi, _ = workloads.random_case(9300 + T, 5, N, T)
    ninf = float("-inf")
    phi[0, 5, :, 7] = ninf                  # a forbidden tag in the forward half
    phi[0, 19, 3, :] = ninf                 # a tag without successors in the backward half
    phi[1, 8, :, :] = ninf                  # no finite path at all
    phi[2, 0, 0, 2] = ninf                  # a forbidden start tag
    phi[3, 12, :, 1:] = ninf                # only tag 0 allowed at the meeting position
    mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(5 + T)) < 0.3
    phi[4][mask] = ninf                     # sparse transitions everywhere
    phi[4, :, :, 0] = 0.0                   # (tag 0 always reachable: a finite path exists)
    lens = torch.tensor([N, N, N, N, N - 3], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES,
               what=f"lanes -inf T={T}", queries=("logz", "mu"))


@pytest.mark.parametrize("T,N", [(16, 64), (30, 40), (32, 40), (36, 44), (45, 30), (48, 21), (60, 25), (64, 30)])
def test_lanes_scale_jumps(crf, oracle_mod, T, N):
    """A common shift of a whole matrix is absorbed by the matrix's own power-of-two scale: the chain stays
    in the linear domain and the offsets carry the jumps."""
    phi, lens = workloads.random_case(9400 + T, 3, N, T, scale=1.0, ragged=True, min_len=N // 2)
    g = torch.Generator().manual_seed(199 + T)
    jump = (torch.randint(0, 3, (3, N, 1, 1), generator=g).to(torch.float32) - 1.0) * 300.0
    jump[:, ::5] = 0.0
    phi = (phi + jump).contiguous()
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES, what=f"lanes jumps T={T} N={N}",
               queries=("logz", "mu"))


@pytest.mark.parametrize("T", (16, 45, 48))
def test_lanes_wide_range_inside_a_matrix(crf, oracle_mod, T):
    """Entries of one matrix hundreds of nats apart: sums fall below the accepted range somewhere in the
    chain; those positions are taken in the log domain by the chain wave, and the fast path resumes once the
    vector fits scaled single precision again (both directions, both passes)."""
    N = 40
    phi, _ = workloads.random_case(9500 + T, 4, N, T, scale=1.0)
    phi[0, 7, : T // 2, :] -= 200.0
    phi[0, 30, :, T // 2:] -= 250.0
    phi[1, 11] *= 60.0
    phi[2, 25] *= 60.0
    phi[3, 3, 1:, :] -= 500.0
    phi[3, 36, :, 1:] -= 500.0
    check_case(crf, oracle_mod, phi, None, algo=crf.ALGO_SEQUENTIAL_LANES, what=f"lanes wide range T={T}",
               queries=("logz", "mu"))


def test_lanes_large_offset(crf, oracle_mod):
    phi, _ = workloads.random_case(9600, 2, 200, 16)
    phi = phi + 300.0
    check_case(crf, oracle_mod, phi, None, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES, what="lanes offset +300",
               queries=("logz", "mu"))


def test_lanes_peaked_long_chain_bf16(crf, oracle_mod):
    """The value distribution of the long-sequence configuration (bfloat16, ten times a standard normal)
    over a shorter chain: single positions drop into the log domain wherever the peaked matrices starve a tag."""
    phi, _ = workloads.random_case(9700, 2, 600, 16, scale=10.0, dtype="bf16")
    check_case(crf, oracle_mod, phi, None, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES, what="lanes peaked bf16",
               queries=("logz", "mu"))


@pytest.mark.parametrize("polls", (0, 1, 3, 40))
def test_lanes_chain_that_stops_waiting_finishes_in_the_log_domain(crf, oracle_mod, polls):
    """The bounded wait of the chain wave, made to expire from the host: with a limit of 0 looks nearly every
    chain leaves the fast path at its first position, with a few looks some leave it in the middle of a chain
    (wherever a producer happens to be late); every result still equals the oracle's, and every kernel ends."""
    crf.set_lane_poll_limit(polls)
    try:
        for T, N in ((11, 60), (16, 50), (32, 70), (45, 40), (48, 40), (64, 33)):
            phi, lens = workloads.random_case(9800 + T + polls, 5, N, T, scale=1.5, ragged=True, min_len=1)
            check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES,
                       what=f"lanes poll limit {polls} T={T}", queries=("logz", "mu"))
    finally:
        crf.set_lane_poll_limit(-1)


def test_lanes_more_sequences_than_compute_units(crf, oracle_mod):
    """Several workgroups a compute unit (and more than one round of them): 700 short sequences."""
    phi, lens = workloads.random_case(9900, 700, 12, 32, scale=1.0, ragged=True, min_len=0)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES, what="lanes B=700", queries=("logz", "mu"))


def test_lanes_refuses_what_it_does_not_serve(crf):
    dev = torch.device("cuda:0")
    for T in (5, 49, 50, 63, 68, 128):
        phi = torch.zeros(1, 4, T, T, device=dev)
        with pytest.raises(RuntimeError):
            crf.lccrf_log_partition(phi, algo=crf.ALGO_SEQUENTIAL_LANES)


def test_lanes_agree_with_the_one_wave_schedule(crf):
    """Both sequential schedules on the paper's benchmark shape (b=128, n=256, 32 tags; appendix "Empirical
    comparisons"): the same marginals within rounding."""
    w = workloads.WORKLOADS["paper_lccrf"]
    phi = workloads.phi_batch(w).cuda()
    lz_a, mu_a = crf.lccrf_marginals(phi, None, algo=crf.ALGO_SEQUENTIAL_LANES)
    lz_b, mu_b = crf.lccrf_marginals(phi, None, algo=crf.ALGO_SEQUENTIAL)
    assert torch.allclose(lz_a, lz_b, rtol=2e-6, atol=1e-5)
    assert float((mu_a - mu_b).abs().max()) < 4e-6
    s = mu_a.sum(dim=(2, 3))
    assert float((s - 1).abs().max()) < 2e-5


def test_auto_between_the_chain_wave_kernels_and_the_scan_on_long_chains(crf):
    """lccrf_auto_algo on a 256-unit device: the chain-wave kernels' time grows with the length of the chains, the
    scan's with the positions of the whole batch; long chains in small batches go to the scan, larger batches of the
    same length stay."""
    A = crf.auto_algo
    for op in (crf.OP_LOGZ, crf.OP_MARGINALS):
        assert A(op, 4, 16384, 32) == crf.ALGO_SCAN
        assert A(op, 16, 4096, 32) == crf.ALGO_SCAN
        assert A(op, 64, 2048, 32) == crf.ALGO_SCAN
        assert A(op, 128, 1024, 32) == crf.ALGO_SEQUENTIAL_LANES
        assert A(op, 128, 256, 32) == crf.ALGO_SEQUENTIAL_LANES      # the paper's shape
        assert A(op, 8, 4096, 48) == crf.ALGO_SCAN
        assert A(op, 16, 2048, 48) == crf.ALGO_SCAN
        assert A(op, 32, 1024, 48) == crf.ALGO_SEQUENTIAL_LANES
        assert A(op, 128, 128, 48) == crf.ALGO_SEQUENTIAL_LANES      # config 3
    assert A(crf.OP_LOGZ, 16, 1024, 64) == crf.ALGO_SEQUENTIAL_LANES
    assert A(crf.OP_MARGINALS, 16, 1024, 64) == crf.ALGO_SCAN
    assert A(crf.OP_MARGINALS, 32, 1024, 64) == crf.ALGO_SEQUENTIAL
