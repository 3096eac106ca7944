"""GPU parity of the chunked scan schedule (ALGO_SCAN) against the CPU oracle, and against the
sequential schedule: the scan regroups the same semiring products (associativity), so every
result must agree to the tolerances of test_gpu_parity.py whatever the chunk size is."""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import _path_score, check_case, crf  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

SUMS = ("logz", "mu")   # the scan of the max-plus semiring stops at 32 tags
ALL = ("logz", "mu", "vit")


@pytest.fixture
def chunk(crf):
    """Sets the scan's chunk size for one test and restores the default afterwards."""
    yield crf.set_scan_chunk
    crf.set_scan_chunk(0)


def _lens_around_chunks(N, k):
    """Lengths that hit empty, one-position, chunk-aligned and ragged-tail cases."""
    cand = [0, 1, 2, k - 1, k, k + 1, 2 * k, 2 * k + 1, N - 1, N]
    return torch.tensor([min(max(c, 0), N) for c in cand], dtype=torch.int32)


@pytest.mark.parametrize("k", [4, 7, 64])
@pytest.mark.parametrize("T,N", [(1, 9), (2, 5), (5, 8), (5, 130), (13, 65), (16, 1), (16, 3), (16, 64), (16, 300)])
def test_scan_fp32(crf, oracle_mod, chunk, T, N, k):
    chunk(k)
    lens = _lens_around_chunks(N, k)
    phi, _ = workloads.random_case(5000 + 31 * T + N, len(lens), N, T, scale=1.5)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan T={T} N={N} k={k}")


@pytest.mark.parametrize("k", [4, 64])
def test_scan_one_chunk_and_many_chunks(crf, oracle_mod, chunk, k):
    """Degenerate chunk counts: the whole chain in one chunk (C = 1) and the smallest chunks."""
    N = 64
    chunk(k)
    phi, lens = workloads.random_case(5100 + k, 6, N, 16, scale=2.0, ragged=True, min_len=1)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan C={N // k}")


@pytest.mark.parametrize("T", [16, 27])
def test_scan_chunks_longer_than_the_fused_kernel_takes(crf, oracle_mod, chunk, T):
    """Chunks of more than 64 positions run the two passes inside the chunks as two launches with the
    vectors in the workspace (shorter ones: one launch, vectors in LDS)."""
    chunk(100)
    phi, lens = workloads.random_case(5150 + T, 4, 1700, T, scale=2.0, ragged=True, min_len=90)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan chunk 100 T={T}", queries=SUMS)
    H = crf.lccrf_entropy(phi.cuda(), lens.cuda()).cpu().numpy()
    want = oracle_mod.entropy(phi, lens.numpy())
    assert np.all(np.abs(H - want) <= 2e-4 * np.maximum(1.0, np.abs(want)))


def test_scan_bf16(crf, oracle_mod, chunk):
    chunk(16)
    phi, lens = workloads.random_case(5200, 5, 200, 16, scale=3.0, ragged=True, min_len=3, dtype="bf16")
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what="scan bf16")


def test_scan_forbidden_edges_and_dead_chains(crf, oracle_mod, chunk):
    """-inf potentials are structural zeros of the chunk products; a chain with no finite path
    gives logZ = -inf and zero marginals."""
    chunk(8)
    T, N = 16, 50
    phi, _ = workloads.random_case(5300, 5, N, T)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf                       # tag 3 can never be left
    phi[1, 20, :, 7] = ninf                      # a forbidden tag at one position
    phi[2, 30, :, :] = ninf                      # no finite path at all
    mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(5)) < 0.6
    phi[3][mask] = ninf                          # sparse transition structure
    phi[3, :, torch.arange(T), torch.arange(T)] = 0.0
    lens = torch.tensor([50, 50, 50, 50, 33], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what="scan -inf")


def test_scan_scale_jumps_take_the_exact_product(crf, oracle_mod, chunk):
    """Matrices whose entries span hundreds of nats, and scales that jump between positions: the
    linear-domain chunk product must be rejected and the exact log-domain product used."""
    chunk(8)
    T, N = 16, 70
    phi, lens = workloads.random_case(5400, 4, N, T, scale=1.0, ragged=True, min_len=N // 2)
    g = torch.Generator().manual_seed(17)
    jump = (torch.randint(0, 3, (4, N, 1, 1), generator=g).to(torch.float32) - 1.0) * 300.0
    phi = phi + jump
    wide = torch.randint(0, 2, (4, N, T, T), generator=g).to(torch.float32) * -150.0
    wide[:, ::3] = 0.0
    phi = (phi + wide).contiguous()
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what="scan jumps", queries=("logz", "mu"))


def test_scan_large_offsets(crf, oracle_mod, chunk):
    chunk(16)
    phi, lens = workloads.random_case(5500, 3, 120, 16, scale=1.0, ragged=True, min_len=60)
    phi = (phi + 40.0).contiguous()
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what="scan offsets")


def test_scan_agrees_with_sequential(crf):
    phi, lens = workloads.random_case(5600, 4, 1000, 16, scale=2.0, ragged=True, min_len=500)
    dphi, dl = phi.cuda(), lens.cuda()
    lz_a, mu_a = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SCAN)
    lz_b, mu_b = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SEQUENTIAL)
    lz_c = crf.lccrf_log_partition(dphi, dl, algo=crf.ALGO_SCAN)
    assert torch.allclose(lz_a, lz_b, rtol=2e-6, atol=0)
    assert torch.allclose(lz_c, lz_b, rtol=2e-6, atol=0)
    assert float((mu_a - mu_b).abs().max()) < 5e-6


def test_scan_viterbi_matches_sequential_path(crf):
    """Generic potentials have a unique best path: both schedules must return it."""
    phi, lens = workloads.random_case(5650, 5, 3000, 16, scale=2.0, ragged=True, min_len=1)
    dphi, dl = phi.cuda(), lens.cuda()
    s_a, y_a = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SCAN)
    s_b, y_b = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SEQUENTIAL)
    assert torch.equal(y_a, y_b)
    assert torch.allclose(s_a, s_b, rtol=1e-6, atol=0)


@pytest.mark.parametrize("T,N,k", [(17, 900, 0), (24, 2100, 8), (32, 3000, 0), (32, 1500, 4), (29, 700, 32)])
def test_scan_viterbi_17_to_32_tags_matches_sequential_path(crf, chunk, T, N, k):
    """The max-plus scan at 17 .. 32 tags (chunk products of 32 x 32 matrices in double precision, a 4 x 4 block a
    lane; with 64 chunks or more a sequence the boundary phase runs over groups of chunks): the path and the score of
    the sequential schedule (float32), a path of the best score (bfloat16, where exact ties occur)."""
    chunk(k)
    for dtype in ("f32", "bf16"):
        phi, lens = workloads.random_case(5670 + T, 4, N, T, scale=2.0, ragged=True, min_len=1, dtype=dtype)
        dphi, dl = phi.cuda(), lens.cuda()
        s_a, y_a = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SCAN)
        s_b, y_b = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SEQUENTIAL)
        assert torch.equal(s_a, s_b), dtype
        if dtype == "f32":      # generic potentials: a unique best path
            assert torch.equal(y_a, y_b)
        else:                   # bfloat16 potentials tie exactly now and then: any path with the best score
            phi64 = phi.to(torch.float32).numpy().astype(np.float64)
            for b_ in range(phi.shape[0]):
                L = int(lens[b_])
                y = y_a[b_, :L].cpu().numpy()
                assert (y_a[b_, L:] == -1).all() and ((y >= 0) & (y < T)).all()
                got = _path_score(phi64[b_], y, L)
                assert abs(got - float(s_a[b_])) <= 1e-5 * max(1.0, abs(got))


def test_auto_takes_the_max_plus_scan_on_long_chains_of_17_to_32_tags(crf):
    A = lambda B, N, T: crf.auto_algo(crf.OP_ARGMAX, B, N, T)
    assert A(8, 4096, 32) == crf.ALGO_SCAN
    assert A(1, 8192, 24) == crf.ALGO_SCAN
    assert A(4, 16384, 17) == crf.ALGO_SCAN
    assert A(32, 1024, 32) == crf.ALGO_SEQUENTIAL_LANES
    assert A(16, 512, 32) == crf.ALGO_SEQUENTIAL_LANES
    assert A(128, 256, 32) == crf.ALGO_SEQUENTIAL_LANES       # the paper's shape
    assert A(8, 4096, 33) == crf.ALGO_SEQUENTIAL_LANES        # no max-plus scan above 32 tags


def test_scan_viterbi_many_chunks_cross_the_trace_window(crf, chunk):
    """More chunks than one window of the chunk-level back-trace holds."""
    chunk(4)
    phi, lens = workloads.random_case(5660, 2, 5000, 3, scale=2.0, ragged=True, min_len=4500)
    dphi, dl = phi.cuda(), lens.cuda()
    s_a, y_a = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SCAN)
    s_b, y_b = crf.lccrf_argmax(dphi, dl, algo=crf.ALGO_SEQUENTIAL)
    assert torch.equal(y_a, y_b)
    assert torch.allclose(s_a, s_b, rtol=1e-6, atol=0)


def test_scan_repeat_runs_are_bit_identical(crf):
    phi, lens = workloads.random_case(5700, 3, 400, 16, scale=2.0, ragged=True, min_len=100)
    dphi, dl = phi.cuda(), lens.cuda()
    lz_a, mu_a = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SCAN)
    lz_b, mu_b = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SCAN)
    assert torch.equal(lz_a, lz_b) and torch.equal(mu_a, mu_b)


@pytest.mark.parametrize("k", [4, 7, 32])
@pytest.mark.parametrize("T,N", [(17, 9), (20, 65), (24, 1), (31, 130), (32, 3), (32, 64), (32, 300)])
def test_scan_up_to_32_tags(crf, oracle_mod, chunk, T, N, k):
    """Tag sets of 17 .. 32: chunk products in four 16 x 16 blocks."""
    chunk(k)
    lens = _lens_around_chunks(N, k)
    phi, _ = workloads.random_case(5900 + 31 * T + N, len(lens), N, T, scale=1.5)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan T={T} N={N} k={k}", queries=ALL)


def test_scan_32_tags_bf16_forbidden_edges_jumps_and_offsets(crf, oracle_mod, chunk):
    chunk(16)
    T, N = 32, 200
    phi, lens = workloads.random_case(5910, 5, N, T, scale=3.0, ragged=True, min_len=3, dtype="bf16")
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what="scan T=32 bf16", queries=ALL)
    chunk(8)
    T, N = 29, 50
    phi, _ = workloads.random_case(5920, 5, N, T)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 20, :, 27] = ninf
    phi[2, 30, :, :] = ninf
    mask = torch.rand(N, T, T, generator=torch.Generator().manual_seed(5)) < 0.6
    phi[3][mask] = ninf
    phi[3, :, torch.arange(T), torch.arange(T)] = 0.0
    lens = torch.tensor([50, 50, 50, 50, 33], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what="scan T=29 -inf", queries=ALL)
    T, N = 32, 70
    phi, lens = workloads.random_case(5930, 4, N, T, scale=1.0, ragged=True, min_len=N // 2)
    g = torch.Generator().manual_seed(17)
    jump = (torch.randint(0, 3, (4, N, 1, 1), generator=g).to(torch.float32) - 1.0) * 300.0
    wide = torch.randint(0, 2, (4, N, T, T), generator=g).to(torch.float32) * -150.0
    wide[:, ::3] = 0.0
    check_case(crf, oracle_mod, (phi + jump + wide).contiguous(), lens, algo=crf.ALGO_SCAN, what="scan T=32 jumps",
               queries=ALL)
    chunk(16)
    phi, lens = workloads.random_case(5940, 3, 120, 24, scale=1.0, ragged=True, min_len=60)
    check_case(crf, oracle_mod, (phi + 40.0).contiguous(), lens, algo=crf.ALGO_SCAN, what="scan T=24 offsets", queries=ALL)


@pytest.mark.parametrize("scale", [5.0, 8.0, 10.0, 12.0])
@pytest.mark.parametrize("T", [19, 32])
def test_scan_32_tags_precision_ladder(crf, oracle_mod, chunk, T, scale):
    """Chunk products of 17 .. 32 tags start in single precision and pass to double precision where
    their exponent range runs out: scales on both sides of that boundary (it lies near 8), long
    chunks, so that some chunks give up late and others never, and group products above them."""
    chunk(32)
    phi, lens = workloads.random_case(5950 + T, 3, 2100, T, scale=scale, ragged=True, min_len=1500)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan T={T} scale {scale}", queries=ALL)


def test_scan_32_tags_agrees_with_sequential_on_the_paper_shape(crf):
    w = workloads.WORKLOADS["paper_lccrf"]
    dphi = workloads.phi_batch(w).cuda()
    lz_a, mu_a = crf.lccrf_marginals(dphi, None, algo=crf.ALGO_SCAN)
    lz_b, mu_b = crf.lccrf_marginals(dphi, None, algo=crf.ALGO_SEQUENTIAL)
    lz_c = crf.lccrf_log_partition(dphi, None, algo=crf.ALGO_SCAN)
    assert torch.allclose(lz_a, lz_b, rtol=2e-6, atol=0)
    assert torch.allclose(lz_c, lz_b, rtol=2e-6, atol=0)
    assert float((mu_a - mu_b).abs().max()) < 5e-6


@pytest.mark.parametrize("k", [4, 7, 32])
@pytest.mark.parametrize("T,N", [(33, 9), (40, 65), (48, 1), (48, 130), (49, 40), (64, 3), (64, 64), (64, 150), (57, 90)])
def test_scan_up_to_64_tags(crf, oracle_mod, chunk, T, N, k):
    """Tag sets of 33 .. 64: chunk products in 3 x 3 or 4 x 4 blocks of 16 x 16, one wave per block column of
    the running product; the chunks themselves by the four-wave chain kernels."""
    chunk(k)
    lens = _lens_around_chunks(N, k)
    phi, _ = workloads.random_case(6900 + 31 * T + N, len(lens), N, T, scale=1.5)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan T={T} N={N} k={k}", queries=SUMS)


@pytest.mark.parametrize("T", [48, 64])
def test_scan_64_tags_bf16_forbidden_edges_jumps_and_offsets(crf, oracle_mod, chunk, T):
    chunk(16)
    N = 200
    phi, lens = workloads.random_case(6910 + T, 5, N, T, scale=3.0, ragged=True, min_len=3, dtype="bf16")
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what=f"scan T={T} bf16", queries=SUMS)
    chunk(8)
    N = 50
    phi, _ = workloads.random_case(6920 + T, 5, N, T - 3)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 20, :, 27] = ninf
    phi[2, 30, :, :] = ninf
    mask = torch.rand(N, T - 3, T - 3, generator=torch.Generator().manual_seed(5)) < 0.6
    phi[3][mask] = ninf
    phi[3, :, torch.arange(T - 3), torch.arange(T - 3)] = 0.0
    lens = torch.tensor([50, 50, 50, 50, 33], dtype=torch.int32)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SCAN, what=f"scan T={T - 3} -inf", queries=SUMS)
    N = 70
    phi, lens = workloads.random_case(6930 + T, 4, N, T, scale=1.0, ragged=True, min_len=N // 2)
    g = torch.Generator().manual_seed(17)
    jump = (torch.randint(0, 3, (4, N, 1, 1), generator=g).to(torch.float32) - 1.0) * 300.0
    wide = torch.randint(0, 2, (4, N, T, T), generator=g).to(torch.float32) * -150.0
    wide[:, ::3] = 0.0
    check_case(crf, oracle_mod, (phi + jump + wide).contiguous(), lens, algo=crf.ALGO_SCAN, what=f"scan T={T} jumps",
               queries=SUMS)
    chunk(16)
    phi, lens = workloads.random_case(6940 + T, 3, 120, T - 7, scale=1.0, ragged=True, min_len=60)
    check_case(crf, oracle_mod, (phi + 40.0).contiguous(), lens, algo=crf.ALGO_SCAN, what=f"scan T={T - 7} offsets",
               queries=SUMS)


@pytest.mark.parametrize("scale", [5.0, 8.0, 10.0])
@pytest.mark.parametrize("T", [41, 64])
def test_scan_64_tags_precision_ladder(crf, oracle_mod, chunk, T, scale):
    """Single precision first, double precision where its exponent range runs out, with group products
    above the chunk products (many chunks).  Scales up to 10, the peaked case of the long-chain workload
    (float32 potentials of scale 12 over 64 tags bring every schedule, the exact sequential one included,
    to 7e-6 .. 1e-5 of the oracle: the rounding of arguments of magnitude 60 in float32)."""
    chunk(16)
    phi, lens = workloads.random_case(6950 + T, 2, 1100, T, scale=scale, ragged=True, min_len=900)
    check_case(crf, oracle_mod, phi, lens, algo=crf.ALGO_SCAN, what=f"scan T={T} scale {scale}", queries=SUMS)


def test_scan_config3_agrees_with_sequential(crf):
    w = workloads.WORKLOADS["cfg3"]
    dphi, dl = workloads.phi_batch(w).cuda(), workloads.lengths(w).cuda()
    lz_a, mu_a = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SCAN)
    lz_b, mu_b = crf.lccrf_marginals(dphi, dl, algo=crf.ALGO_SEQUENTIAL)
    lz_c = crf.lccrf_log_partition(dphi, dl, algo=crf.ALGO_SCAN)
    assert torch.allclose(lz_a, lz_b, rtol=2e-6, atol=0)
    assert torch.allclose(lz_c, lz_b, rtol=2e-6, atol=0)
    assert float((mu_a - mu_b).abs().max()) < 5e-6


def test_scan_needs_a_small_tag_set(crf):
    phi, _ = workloads.random_case(5800, 2, 8, 65)
    with pytest.raises(crf.LccrfError, match="not available"):
        crf.lccrf_marginals(phi.cuda(), None, algo=crf.ALGO_SCAN)
    phi, _ = workloads.random_case(5801, 2, 8, 33)
    with pytest.raises(crf.LccrfError, match="not available"):
        crf.lccrf_argmax(phi.cuda(), None, algo=crf.ALGO_SCAN)
    with pytest.raises(crf.LccrfError, match="invalid argument"):
        crf.set_scan_chunk(3)


def test_config5_sequential_schedule(crf, oracle_mod):
    """Config 5 under the sequential schedule (the default now takes the scan for it)."""
    w = workloads.WORKLOADS["cfg5"]
    phi = workloads.phi_batch(w)
    lens = workloads.lengths(w)
    check_case(crf, oracle_mod, phi, lens, poison=False, algo=crf.ALGO_SEQUENTIAL, what="cfg5 sequential")
