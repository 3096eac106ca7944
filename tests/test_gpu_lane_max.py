"""GPU parity of the max-plus chains run by a chain wave and helper waves (lccrf_argmax under
LCCRF_ALGO_SEQUENTIAL_LANES) against the CPU oracle, at the bars of test_gpu_parity.py (score relative 1e-5, tags
identical wherever the best path leads by more than 1e-3), and against the one-wave / four-wave kernels of the
plain sequential schedule, with which scores and tags must agree bit for bit, exact ties included: both add the
same operands in double precision and break ties towards the smaller tag.

The shapes span every instantiation (up to 16, 17 .. 32, 33 .. 48, 49 .. 64 tags; multiples of four, whose matrices
are loaded in 16-byte pieces, and other counts, loaded element by element), tag counts below the padded size, chains
shorter than the ring of matrices, the degenerate lengths 0, 1 and 2, forbidden edges and sequences with no finite
path.
"""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import check_case, crf  # noqa: F401  (crf: the module-scoped binding fixture)

pytestmark = pytest.mark.gpu

TAGS = (1, 2, 3, 4, 5, 8, 12, 13, 16, 17, 20, 24, 30, 32, 33, 36, 40, 45, 48, 49, 52, 57, 60, 63, 64)


def same_as_sequential(crf, phi, lens, what):
    dev = torch.device("cuda:0")
    d_phi = phi.to(dev)
    d_lens = None if lens is None else lens.to(dev)
    score_a, tags_a = crf.lccrf_argmax(d_phi, d_lens, algo=crf.ALGO_SEQUENTIAL_LANES)
    score_b, tags_b = crf.lccrf_argmax(d_phi, d_lens, algo=crf.ALGO_SEQUENTIAL)
    assert torch.equal(tags_a, tags_b), f"{what}: tags differ from the sequential schedule's"
    sa, sb = score_a.cpu().numpy(), score_b.cpu().numpy()
    assert np.array_equal(sa, sb, equal_nan=True), f"{what}: scores differ from the sequential schedule's"


@pytest.mark.parametrize("T", TAGS)
@pytest.mark.parametrize("N", (1, 2, 3, 7, 33, 90))
def test_lane_max_sweep_fp32(crf, oracle_mod, T, N):
    B = 6
    phi, _ = workloads.random_case(9000 + 13 * T + N, B, N, T, scale=1.5)
    lens = torch.tensor([N, 1, max(1, N // 2), 0, max(1, N - 1), min(N, 2)], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES, what=f"lane max T={T} N={N}", queries=("vit",))
    same_as_sequential(crf, phi, lens, f"lane max T={T} N={N}")


@pytest.mark.parametrize("T,N", [(16, 70), (32, 41), (48, 33), (64, 25), (24, 9), (8, 50), (36, 30), (7, 50), (37, 30), (45, 40)])
def test_lane_max_sweep_bf16(crf, oracle_mod, T, N):
    phi, _ = workloads.random_case(9100 + T + N, 3, N, T, scale=3.0, dtype="bf16")
    lens = torch.tensor([N, max(1, N // 3), N - 1 if N > 1 else 1], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES,
               what=f"lane max bf16 T={T} N={N}", queries=("vit",))
    same_as_sequential(crf, phi, lens, f"lane max bf16 T={T} N={N}")


def test_lane_max_no_lengths_argument(crf, oracle_mod):
    phi, _ = workloads.random_case(9200, 3, 50, 32)
    check_case(crf, oracle_mod, phi, None, algo=crf.ALGO_SEQUENTIAL_LANES, what="lane max, lengths = NULL", queries=("vit",))


@pytest.mark.parametrize("T", (6, 8, 16, 29, 32, 45, 48, 64))
def test_lane_max_forbidden_edges(crf, oracle_mod, T):
    N = 24
    phi, _ = workloads.random_case(9300 + T, 5, N, T)
    ninf = float("-inf")
    phi[0, 5, :, min(7, T - 1)] = ninf      # a forbidden tag in the forward half
    phi[0, 19, 3, :] = ninf                 # a tag without successors in the backward half
    phi[1, 8, :, :] = ninf                  # no finite path at all
    phi[2, 0, 0, 2] = ninf                  # a forbidden start tag
    phi[3, 12, :, 1:] = ninf                # only tag 0 allowed at the meeting position
    mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(5 + T)) < 0.3
    phi[4][mask] = ninf                     # sparse transitions everywhere
    phi[4, :, :, 0] = 0.0                   # (tag 0 always reachable: a finite path exists)
    lens = torch.tensor([N, N, N, N, N - 3], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES,
               what=f"lane max -inf T={T}", queries=("vit",))
    same_as_sequential(crf, phi, lens, f"lane max -inf T={T}")


@pytest.mark.parametrize("T,N", [(3, 60), (4, 60), (16, 64), (20, 33), (31, 40), (32, 40), (45, 30), (48, 30), (64, 21)])
def test_lane_max_exact_ties(crf, T, N):
    """Potentials from {0, 1, 2}: many paths share the best score exactly; the tie rule (the smallest tag at the
    meeting position, then the smallest predecessor and successor) must give the path of the other kernels."""
    g = torch.Generator().manual_seed(77 + T)
    phi = torch.randint(0, 3, (4, N, T, T), generator=g).to(torch.float32)
    lens = torch.tensor([N, N - 1, max(1, N // 2), 2], dtype=torch.int32)
    same_as_sequential(crf, phi, lens, f"lane max ties T={T} N={N}")
    same_as_sequential(crf, torch.zeros(2, N, T, T), None, f"lane max all-zero T={T} N={N}")


@pytest.mark.parametrize("polls", (0, 1, 3, 40))
def test_lane_max_chain_that_stops_waiting_goes_on_alone(crf, oracle_mod, polls):
    """The bounded wait of the chain wave, made to expire from the host: with a limit of 0 looks nearly every chain
    wave goes on alone from its first position, with a few looks some do so in the middle of a chain (wherever a
    helper happens to be late); every result still equals the oracle's, and every kernel ends."""
    crf.set_lane_poll_limit(polls)
    try:
        for T, N in ((11, 60), (16, 50), (32, 70), (45, 40), (48, 40), (64, 33)):
            phi, lens = workloads.random_case(9800 + T + polls, 5, N, T, scale=1.5, ragged=True, min_len=1)
            check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES,
                       what=f"lane max poll limit {polls} T={T}", queries=("vit",))
            same_as_sequential(crf, phi, lens, f"lane max poll limit {polls} T={T}")
    finally:
        crf.set_lane_poll_limit(-1)


@pytest.mark.parametrize("T,N,dtype", [(32, 1500, "f32"), (48, 700, "f32"), (16, 3000, "bf16"), (64, 300, "f32")])
def test_lane_max_long_chains(crf, oracle_mod, T, N, dtype):
    """Hundreds of trips round the rings of matrices and vectors, and a trace that takes several windows of
    pointers a direction."""
    phi, _ = workloads.random_case(9950 + T, 2, N, T, scale=2.0, dtype=dtype)
    lens = torch.tensor([N, N - 37], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL_LANES,
               what=f"lane max long chain T={T} N={N}", queries=("vit",))
    same_as_sequential(crf, phi, lens, f"lane max long chain T={T} N={N}")


def test_lane_max_more_sequences_than_compute_units(crf, oracle_mod):
    """Several workgroups a compute unit (and more than one round of them): 700 short sequences."""
    phi, lens = workloads.random_case(9900, 700, 12, 32, scale=1.0, ragged=True, min_len=0)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SEQUENTIAL_LANES, what="lane max B=700", queries=("vit",))


def test_lane_max_refuses_what_it_does_not_serve(crf):
    dev = torch.device("cuda:0")
    for T in (65, 68, 128):
        phi = torch.zeros(1, 4, T, T, device=dev)
        with pytest.raises(RuntimeError):
            crf.lccrf_argmax(phi, algo=crf.ALGO_SEQUENTIAL_LANES)


def test_lane_max_paper_shape(crf):
    """The paper's benchmark shape (b=128, n=256, 32 tags; appendix "Empirical comparisons"): the same tags and
    scores as the one-wave kernels."""
    w = workloads.WORKLOADS["paper_lccrf"]
    phi = workloads.phi_batch(w)
    same_as_sequential(crf, phi, None, "lane max paper shape")


def test_auto_takes_the_chain_wave_kernels_where_they_pay(crf):
    """lccrf_auto_algo for the argmax on a 256-unit device: batches whose workgroups are all resident at once, up to
    48 tags; the max-plus scan only where it is quicker still."""
    A = lambda B, N, T: crf.auto_algo(crf.OP_ARGMAX, B, N, T)
    assert A(128, 256, 32) == crf.ALGO_SEQUENTIAL_LANES     # the paper's shape
    assert A(32, 64, 32) == crf.ALGO_SEQUENTIAL_LANES       # config 2
    assert A(128, 128, 48) == crf.ALGO_SEQUENTIAL_LANES     # config 3
    assert A(256, 256, 16) == crf.ALGO_SEQUENTIAL_LANES
    assert A(64, 512, 16) == crf.ALGO_SEQUENTIAL_LANES      # quicker than the scan there
    assert A(64, 1024, 16) == crf.ALGO_SCAN
    assert A(4, 16384, 16) == crf.ALGO_SCAN                 # config 5
    assert A(1024, 64, 32) == crf.ALGO_SEQUENTIAL           # too many sequences at once
    assert A(32, 256, 64) == crf.ALGO_SEQUENTIAL            # more than 48 tags
    assert A(32, 64, 30) == crf.ALGO_SEQUENTIAL_LANES       # any tag count up to 48
    assert A(128, 128, 45) == crf.ALGO_SEQUENTIAL_LANES
    assert A(4, 8, 5) == crf.ALGO_SEQUENTIAL                # config 1: too short to pay
