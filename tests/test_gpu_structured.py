"""GPU parity of the structured calls (emit [B,N,T] + trans [T,T]) against the CPU oracle run on the
materialised dense potentials phi[b,i,s,t] = trans[s,t] + emit[b,i,t]: the definition of what
the structured form stands for.  Tolerances as in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import check_case, crf, _close_logz, _path_score, LOGZ_RTOL, GAP_MIN  # noqa: F401

pytestmark = pytest.mark.gpu


def _make(seed, B, N, T, scale_e=2.0, scale_t=1.0):
    g = torch.Generator().manual_seed(seed)
    emit = torch.randn(B, N, T, generator=g) * scale_e
    trans = torch.randn(T, T, generator=g) * scale_t
    return emit.contiguous(), trans.contiguous()


def _check(crf, oracle_mod, emit, trans, lens, what):
    B, N, T = emit.shape
    phi = (emit[:, :, None, :] + trans[None, None]).contiguous()   # the same float32 additions the kernels make
    lens_np = None if lens is None else lens.numpy()
    eff = np.full((B,), N) if lens is None else np.clip(lens_np, 0, N)
    de, dtr = emit.cuda(), trans.cuda()
    dl = None if lens is None else lens.cuda()

    lz = crf.lccrf_log_partition_structured(de, dtr, dl).cpu().numpy()
    want_lz, want_mu = oracle_mod.marginals(phi, lens_np)
    _close_logz(lz, want_lz, what + " logZ")

    lz2, mu = crf.lccrf_marginals_structured(de, dtr, dl)
    _close_logz(lz2.cpu().numpy(), want_lz, what + " marginals.logZ")
    got_mu = mu.cpu().numpy().astype(np.float64)
    assert np.isfinite(got_mu).all()
    assert np.abs(got_mu - want_mu).max() <= 1e-5, f"{what}: max |mu - oracle| = {np.abs(got_mu - want_mu).max():.3e}"
    for b in range(B):
        assert not got_mu[b, eff[b]:].any() and (eff[b] == 0 or not got_mu[b, 0, 1:].any())

    score, tags = crf.lccrf_argmax_structured(de, dtr, dl)
    want_score, want_tags, gap = oracle_mod.viterbi(phi, lens_np)
    _close_logz(score.cpu().numpy(), want_score, what + " score")
    tags = tags.cpu().numpy()
    phi64 = phi.numpy().astype(np.float64)
    for b in range(B):
        L = int(eff[b])
        assert (tags[b, L:] == -1).all()
        y = tags[b, :L]
        assert ((y >= 0) & (y < T)).all()
        if gap[b] > GAP_MIN:
            assert np.array_equal(y, want_tags[b, :L]), f"{what}: path differs in sequence {b}"
        elif np.isfinite(want_score[b]):
            assert abs(_path_score(phi64[b], y, L) - want_score[b]) <= LOGZ_RTOL * max(1.0, abs(want_score[b]))


@pytest.mark.parametrize("T,N", [(1, 4), (2, 9), (5, 8), (9, 33), (16, 40), (17, 12), (32, 65), (33, 7), (45, 50), (48, 33),
                                 (64, 20), (63, 5), (65, 9), (100, 21), (127, 6), (128, 40)])
def test_structured_sweep(crf, oracle_mod, T, N):
    emit, trans = _make(7000 + 17 * T + N, 5, N, T)
    lens = torch.tensor([N, max(N - 1, 0), min(2, N), 1, 0], dtype=torch.int32)
    _check(crf, oracle_mod, emit, trans, lens, f"structured T={T} N={N}")


@pytest.mark.parametrize("T", (9, 13, 21, 30, 45, 63))
def test_structured_big_batches_off_the_16_byte_grid(crf, oracle_mod, T):
    """More sequences than the chain-wave kernels take: the one-wave and four-wave kernels with a tag count that is
    no multiple of four (a row of emission scores loaded as one piece a lane where another row follows it, element
    by element for the last row of the tensor: full lengths, so that row is worked on)."""
    B, N = 300, 12
    for op in (crf.OP_MARGINALS, crf.OP_ARGMAX):
        assert crf.auto_algo(op, B, N, T) == crf.ALGO_SEQUENTIAL
    emit, trans = _make(7100 + T, B, N, T)
    _check(crf, oracle_mod, emit, trans, None, f"structured B={B} T={T}")


def test_structured_config3(crf, oracle_mod):
    """Config 3 is exactly this structure (emissions of scale 2 plus one transition matrix)."""
    w = workloads.WORKLOADS["cfg3"]
    g = torch.Generator().manual_seed(33)
    emit = (torch.randn(w.B, w.N, w.T, generator=g) * 2.0).contiguous()
    trans = torch.randn(w.T, w.T, generator=g).contiguous()
    _check(crf, oracle_mod, emit, trans, workloads.lengths(w), "structured cfg3 shape")


def test_structured_with_forbidden_transitions(crf, oracle_mod):
    """BIO-style constraints: -inf entries in the transition matrix."""
    T, N = 9, 30
    emit, trans = _make(7100, 4, N, T)
    trans[0, 2] = trans[0, 4] = trans[1, 4] = trans[3, 2] = float("-inf")
    trans[:, 8] = float("-inf")
    trans[8, 8] = 0.0
    _check(crf, oracle_mod, emit, trans, None, "structured with -inf")


def test_structured_agrees_with_dense_call(crf):
    emit, trans = _make(7200, 8, 100, 32)
    phi = (emit[:, :, None, :] + trans[None, None]).contiguous().cuda()
    lz_a, mu_a = crf.lccrf_marginals_structured(emit.cuda(), trans.cuda())
    lz_b, mu_b = crf.lccrf_marginals(phi)
    assert torch.allclose(lz_a, lz_b, rtol=1e-6, atol=0)
    assert float((mu_a - mu_b).abs().max()) < 2e-6
    s_a, y_a = crf.lccrf_argmax_structured(emit.cuda(), trans.cuda())
    s_b, y_b = crf.lccrf_argmax(phi)
    assert torch.equal(y_a, y_b) and torch.equal(s_a, s_b)


@pytest.mark.parametrize("T", (17, 20, 21, 24, 30, 32, 40, 45, 48))
@pytest.mark.parametrize("N", (2, 7, 45))
def test_structured_on_the_chain_wave_kernels(crf, oracle_mod, T, N):
    """8 .. 48 tags, batches that leave the chip latency-bound: the sum queries take the chain-wave / producer-wave
    kernels, whose producers form trans + emit in registers (tag counts that are no multiple of four element by
    element)."""
    assert crf.auto_algo(crf.OP_MARGINALS, 6, N, T) == crf.ALGO_SEQUENTIAL_LANES
    emit, trans = _make(7250 + 3 * T + N, 6, N, T)
    lens = torch.tensor([N, 1, max(1, N // 2), 0, max(1, N - 1), min(N, 2)], dtype=torch.int32)
    _check(crf, oracle_mod, emit, trans, lens, f"structured lanes T={T} N={N}")


@pytest.mark.parametrize("T", (8, 9, 13, 16))
def test_structured_on_the_chain_wave_kernels_up_to_16_tags(crf, oracle_mod, T):
    """8 .. 16 tags take the chain-wave kernels for chains of 16 positions or more in batches of at most one sequence
    a compute unit (shorter chains do not pay their start)."""
    B, N = 6, 45
    assert crf.auto_algo(crf.OP_MARGINALS, B, N, T) == crf.ALGO_SEQUENTIAL_LANES
    assert crf.auto_algo(crf.OP_MARGINALS, B, 12, T) == crf.ALGO_SEQUENTIAL
    emit, trans = _make(7255 + T, B, N, T)
    lens = torch.tensor([N, 1, N // 2, 0, N - 1, 2], dtype=torch.int32)
    _check(crf, oracle_mod, emit, trans, lens, f"structured lanes T={T} N={N}")


@pytest.mark.parametrize("T", (32, 45, 48))
def test_structured_chain_wave_kernels_leave_the_linear_domain(crf, oracle_mod, T):
    """Forbidden transitions and peaked emissions: positions the scaled single-precision step rejects are taken in
    the log domain by the chain wave, from trans + emit as well; and with the wait for a matrix made to expire from
    the host the whole chain is."""
    N = 60
    emit, trans = _make(7260 + T, 4, N, T, scale_e=6.0)
    trans[0, 2] = trans[0, 4] = trans[1, 4] = trans[3, 2] = float("-inf")
    trans[:, T - 1] = float("-inf")
    trans[T - 1, T - 1] = 0.0
    emit[1, 17, :] = -400.0
    emit[1, 17, 5] = 0.0
    lens = torch.tensor([N, N, N - 9, 3], dtype=torch.int32)
    _check(crf, oracle_mod, emit, trans, lens, f"structured lanes -inf and peaks T={T}")
    crf.set_lane_poll_limit(0)
    try:
        _check(crf, oracle_mod, emit, trans, lens, f"structured lanes, poll limit 0, T={T}")
    finally:
        crf.set_lane_poll_limit(-1)


@pytest.mark.parametrize("T", (8, 13, 16, 32, 45, 48))
def test_structured_argmax_on_the_chain_wave_kernels(crf, oracle_mod, T):
    """Up to 48 tags the structured argmax takes the max-plus chain-wave kernels where the dense
    one does (their helpers form trans + emit in registers): tags and scores of the dense call bit for bit, exact
    ties (integer scores) and forbidden transitions included; and with the wait for a matrix made to expire."""
    B, N = 6, 70
    assert crf.auto_algo(crf.OP_ARGMAX, B, N, T) == crf.ALGO_SEQUENTIAL_LANES
    g = torch.Generator().manual_seed(7280 + T)
    emit = torch.randint(0, 3, (B, N, T), generator=g).to(torch.float32)
    trans = torch.randint(0, 3, (T, T), generator=g).to(torch.float32)
    trans[0, 2] = trans[3, 1] = float("-inf")
    lens = torch.tensor([N, N - 1, 1, 0, 2, N // 2], dtype=torch.int32)
    phi = (emit[:, :, None, :] + trans[None, None]).contiguous().cuda()
    for polls in (-1, 0, 2):
        crf.set_lane_poll_limit(polls)
        try:
            s_a, y_a = crf.lccrf_argmax_structured(emit.cuda(), trans.cuda(), lens.cuda())
        finally:
            crf.set_lane_poll_limit(-1)
        s_b, y_b = crf.lccrf_argmax(phi, lens.cuda(), algo=crf.ALGO_SEQUENTIAL)
        assert torch.equal(y_a, y_b) and torch.equal(s_a, s_b), f"poll limit {polls}"
    emit, trans = _make(7290 + T, B, N, T)
    _check(crf, oracle_mod, emit, trans, lens, f"structured argmax lanes T={T}")


def test_structured_needs_a_supported_tag_set(crf):
    emit, trans = _make(7300, 2, 6, 129)
    with pytest.raises(crf.LccrfError, match="not available"):
        crf.lccrf_log_partition_structured(emit.cuda(), trans.cuda())


@pytest.fixture
def chunk(crf):
    """Sets the scan's chunk size for one test and restores the default afterwards."""
    yield crf.set_scan_chunk
    crf.set_scan_chunk(0)


def _scan_lens(N, k):
    cand = [0, 1, 2, k - 1, k, k + 1, 2 * k + 1, N - 1, N]
    return torch.tensor([min(max(c, 0), N) for c in cand], dtype=torch.int32)


@pytest.mark.parametrize("k", [0, 4, 7])
@pytest.mark.parametrize("T,N", [(1, 70), (5, 130), (13, 257), (16, 300), (17, 120), (32, 140), (33, 300), (45, 320),
                                 (48, 288), (64, 130), (63, 71)])
def test_structured_under_the_scan(crf, oracle_mod, chunk, T, N, k):
    """Long chains in small batches: the structured calls take the chunked scan (sum queries up to 64 tags, the argmax
    up to 16; the dense argmax may prefer its chain-wave kernels there, which structured potentials do not have)
    whenever the dense call of the same shape would, with the chunk's potentials formed from the transition
    entries in registers and the streamed emissions."""
    chunk(k)
    lens = _scan_lens(N, k or 8)
    B = len(lens)
    assert crf.auto_algo(crf.OP_MARGINALS, B, N, T) == crf.ALGO_SCAN
    emit, trans = _make(7400 + 13 * T + N + k, B, N, T)
    _check(crf, oracle_mod, emit, trans, lens, f"structured scan T={T} N={N} k={k}")


@pytest.mark.parametrize("T,N,k", [(8, 1100, 16), (16, 2100, 8), (30, 700, 8)])
def test_structured_scan_many_chunks(crf, oracle_mod, chunk, T, N, k):
    """64 chunks or more a sequence: the boundary phase itself runs over groups of chunks."""
    chunk(k)
    lens = torch.tensor([N, N - 3, N // 2 + 1, 1], dtype=torch.int32)
    assert crf.auto_algo(crf.OP_MARGINALS, 4, N, T) == crf.ALGO_SCAN
    emit, trans = _make(7500 + T, 4, N, T, scale_e=1.0, scale_t=0.7)
    _check(crf, oracle_mod, emit, trans, lens, f"structured scan, many chunks, T={T} N={N} k={k}")


@pytest.mark.parametrize("T,N", [(17, 1500), (32, 2000), (27, 1100)])
def test_structured_argmax_under_the_max_plus_scan_at_17_to_32_tags(crf, oracle_mod, T, N):
    """Long chains: the structured argmax takes the max-plus scan where the dense one does (chunk products from the
    transition entries in registers and the streamed emissions): the dense call's tags and scores bit for bit."""
    B = 2
    assert crf.auto_algo(crf.OP_ARGMAX, B, N, T) == crf.ALGO_SCAN
    emit, trans = _make(7650 + T, B, N, T)
    trans[0, 2] = trans[3, 1] = float("-inf")
    lens = torch.tensor([N, N - 41], dtype=torch.int32)
    phi = (emit[:, :, None, :] + trans[None, None]).contiguous().cuda()
    s_a, y_a = crf.lccrf_argmax_structured(emit.cuda(), trans.cuda(), lens.cuda())
    s_b, y_b = crf.lccrf_argmax(phi, lens.cuda(), algo=crf.ALGO_SEQUENTIAL)
    assert torch.equal(y_a, y_b) and torch.equal(s_a, s_b)
    _check(crf, oracle_mod, emit, trans, lens, f"structured max-plus scan T={T} N={N}")


@pytest.mark.parametrize("T,N", [(9, 200), (16, 160), (24, 120), (40, 256)])
def test_structured_scan_with_forbidden_transitions_and_peaked_emissions(crf, oracle_mod, T, N):
    """-inf transitions (the zero pattern of the chunk products) and emissions of scale 12 (the single-precision
    product gives up, the double-precision one or the exact one takes over)."""
    assert crf.auto_algo(crf.OP_MARGINALS, 3, N, T) == crf.ALGO_SCAN
    emit, trans = _make(7600 + T, 3, N, T, scale_e=12.0, scale_t=3.0)
    trans[0, 2] = trans[1, 0] = trans[3, 2] = float("-inf")
    trans[:, T - 1] = float("-inf")
    trans[T - 1, T - 1] = 0.0
    lens = torch.tensor([N, N - 1, 37], dtype=torch.int32)
    _check(crf, oracle_mod, emit, trans, lens, f"structured scan with -inf, T={T}")


def test_structured_scan_agrees_with_dense_scan(crf):
    emit, trans = _make(7700, 4, 512, 16)
    assert crf.auto_algo(crf.OP_ARGMAX, 4, 512, 16) == crf.ALGO_SCAN
    phi = (emit[:, :, None, :] + trans[None, None]).contiguous().cuda()
    lz_a, mu_a = crf.lccrf_marginals_structured(emit.cuda(), trans.cuda())
    lz_b, mu_b = crf.lccrf_marginals(phi)
    assert torch.allclose(lz_a, lz_b, rtol=2e-6, atol=0)
    assert float((mu_a - mu_b).abs().max()) < 5e-6
    s_a, y_a = crf.lccrf_argmax_structured(emit.cuda(), trans.cuda())
    s_b, y_b = crf.lccrf_argmax(phi)
    assert torch.equal(y_a, y_b) and torch.equal(s_a, s_b)
