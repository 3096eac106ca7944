"""GPU parity of lccrf_sample (forward-filtering backward-sampling from caller-supplied uniforms)
against the CPU oracle on the same uniforms.

A sampled tag is an integer decided by floating point (is the cumulative weight above u * total?).
The oracle decides in float64, the GPU in float32, so the two may differ when a draw falls within
rounding distance of a boundary between two tags, and from then on the chains condition on
different tags.  The oracle reports, per sequence, how close its closest draw came to a boundary
(relative to the total weight): sequences whose margin exceeds MARGIN must match tag for tag; the
others must still be valid paths of positive probability.  Frequencies are checked separately."""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import crf  # noqa: F401  (fixture)
import philox_host

pytestmark = pytest.mark.gpu

MARGIN = 2e-4


def _check(crf, oracle_mod, phi, lens, seed, what, min_exact=0.5):
    B, N, T, _ = phi.shape
    u = torch.rand(B, N, generator=torch.Generator().manual_seed(seed))
    got = crf.lccrf_sample(phi.cuda(), u.cuda(), None if lens is None else lens.cuda()).cpu().numpy()
    lens_np = None if lens is None else lens.numpy()
    want, margin = oracle_mod.sample(phi, u.numpy(), lens_np)
    eff = np.full((B,), N) if lens_np is None else np.clip(lens_np, 0, N)
    clear = margin > MARGIN
    for b in range(B):
        L = int(eff[b])
        assert (got[b, L:] == -1).all(), f"{what}: tags past the length of sequence {b}"
        assert ((got[b, :L] >= 0) & (got[b, :L] < T)).all()
        if clear[b]:
            assert np.array_equal(got[b], want[b]), f"{what}: sample differs in sequence {b} (margin {margin[b]:.2e})"
    lp = oracle_mod.log_prob(phi, got, lens_np)
    feasible = np.isfinite(oracle_mod.log_partition(phi, lens_np))
    assert np.isfinite(lp[feasible]).all(), f"{what}: a sampled path has probability 0"
    assert clear.mean() >= min_exact, f"{what}: too few sequences with a clear margin to test anything"


@pytest.mark.parametrize("T,N", [(1, 5), (2, 9), (5, 8), (16, 40), (17, 12), (32, 65), (33, 7), (48, 33), (64, 12),
                                 (100, 9), (128, 30), (129, 5), (200, 6)])
def test_sample_sweep(crf, oracle_mod, T, N):
    phi, lens = workloads.random_case(8000 + 13 * T + N, 6, N, T, scale=1.5, ragged=True, min_len=0)
    _check(crf, oracle_mod, phi, lens, 100 + T, f"sample T={T} N={N}")


def test_sample_bf16_and_forbidden_edges(crf, oracle_mod):
    phi, lens = workloads.random_case(8100, 4, 50, 16, scale=3.0, ragged=True, min_len=10, dtype="bf16")
    _check(crf, oracle_mod, phi, lens, 7, "sample bf16")
    phi, _ = workloads.random_case(8200, 4, 20, 12)
    ninf = float("-inf")
    phi[0, :, 3, :] = ninf
    phi[1, 10, :, 5] = ninf
    phi[2, 12, :, :] = ninf          # no finite path: tags all 0 on both sides
    _check(crf, oracle_mod, phi, None, 8, "sample -inf")
    got = crf.lccrf_sample(phi.cuda(), torch.rand(4, 20).cuda()).cpu().numpy()
    assert (got[2] == 0).all() and (got[1, 10] != 5)


def _draws_miss(oracle_mod, phi_b, L, y, u_b, what):
    """How far (relative to the total weight) the worst draw of the path y [L] of ONE sequence lies outside the
    interval of its tag, given the path's own tag above it, with the oracle's fp64 alpha.  phi_b: [N, T, T] CPU
    tensor, u_b: [N] float64."""
    N, T, _ = phi_b.shape
    if L == 0:
        return 0.0
    alpha, _, _ = oracle_mod.forward_backward(phi_b.unsqueeze(0).contiguous(), np.array([L], dtype=np.int32))
    phi32 = phi_b.to(torch.float32).numpy()
    y = y[:L].astype(np.int64)
    assert ((y >= 0) & (y < T)).all()
    logw = alpha[0, :L].copy()                                       # [L, T] over the candidate tag s
    logw[:L - 1] += phi32[np.arange(1, L), :, y[1:]].astype(np.float64)   # + phi_{i+1}(s, y_{i+1})
    w = np.exp(logw - logw.max(axis=1, keepdims=True))
    cum = np.cumsum(w, axis=1)
    tot = cum[:, -1]
    target = u_b[:L] * tot
    upper = cum[np.arange(L), y]
    lower = upper - w[np.arange(L), y]
    assert (w[np.arange(L), y] > 0).all(), f"{what}: a tag of weight 0 was drawn"
    below = np.maximum(lower - target, 0.0) / tot                    # the draw lies below the tag's interval
    # above the interval is allowed only for the last tag of positive weight (the rounding rule)
    is_last = np.array([y[i] == np.nonzero(w[i] > 0)[0][-1] for i in range(L)])
    above = np.where(is_last, 0.0, np.maximum(target - upper, 0.0) / tot)
    return max(float(below.max()), float(above.max()))


def _check_every_draw(crf, oracle_mod, phi, lens, seed, what, tol=1e-4):
    """Long chains: the oracle's closest draw is almost surely within rounding of a boundary somewhere
    along thousands of positions, after which the two chains condition on different tags.  So every
    draw of the GPU's path is checked on its own, given the GPU's own tag above it: with the oracle's
    fp64 alpha, u_i * total must lie in the interval of the chosen tag, up to tol of the total."""
    B, N, T, _ = phi.shape
    u = torch.rand(B, N, generator=torch.Generator().manual_seed(seed))
    got = crf.lccrf_sample(phi.cuda(), u.cuda(), None if lens is None else lens.cuda()).cpu().numpy()
    lens_np = np.full((B,), N) if lens is None else np.clip(lens.numpy(), 0, N)
    un = u.numpy().astype(np.float64)
    worst = 0.0
    for b in range(B):
        L = int(lens_np[b])
        assert (got[b, L:] == -1).all(), f"{what}: tags past the length of sequence {b}"
        worst = max(worst, _draws_miss(oracle_mod, phi[b], L, got[b], un[b], f"{what} sequence {b}"))
    assert worst <= tol, f"{what}: a draw misses its tag's interval by {worst:.2e} of the total weight"


def test_sample_config4_full_size(crf, oracle_mod):
    """Full-size config 4, the whole batch in one call: every tag in range on all sequences, and every draw of
    three full-length sequences against the oracle's fp64 interval of its tag."""
    w = workloads.WORKLOADS["cfg4"]
    phi = torch.empty(w.B, w.N, w.T, w.T, dtype=torch.float32, device="cuda")
    workloads.phi_batch(w, out=phi)
    u = torch.rand(w.B, w.N, generator=torch.Generator().manual_seed(44))
    got = crf.lccrf_sample(phi, u.cuda()).cpu().numpy()
    assert ((got >= 0) & (got < w.T)).all()
    un = u.numpy().astype(np.float64)
    for b in (1, 30, 63):
        miss = _draws_miss(oracle_mod, workloads.phi_sequence(w, b), w.N, got[b], un[b], f"cfg4 sequence {b}")
        assert miss <= 1e-4, f"cfg4 sequence {b}: a draw misses its tag's interval by {miss:.2e} of the total weight"


@pytest.mark.parametrize("T,N", [(3, 6000), (5, 700), (16, 3000), (20, 300), (32, 600), (48, 400), (128, 200)])
def test_sample_long_chains(crf, oracle_mod, T, N):
    """Several windows of the table of maps, the segmented walk for small tag sets, and (T <= 32) the forward
    pass under the chunked scan."""
    phi, lens = workloads.random_case(8400 + 13 * T + N, 4, N, T, scale=1.5, ragged=True, min_len=N // 2)
    lens[0] = N
    _check_every_draw(crf, oracle_mod, phi, lens, 200 + T, f"long T={T} N={N}")


@pytest.mark.parametrize("T,N", [(4, 13000), (16, 2500), (130, 400), (200, 300)])
def test_sample_many_windows_edge_lengths(crf, oracle_mod, T, N):
    """Sequences of several windows walked all at once: with empty and one-position sequences, lengths
    that end inside the first window or exactly on a window boundary, and a chain without a finite path."""
    wp = 16384 // T
    phi, lens = workloads.random_case(8500 + T, 7, N, T, scale=1.5, ragged=True, min_len=N // 3)
    lens[0], lens[1], lens[2], lens[3], lens[4] = 0, 1, 2, min(N, wp + 1), min(N, 2 * wp + 1)
    _check_every_draw(crf, oracle_mod, phi, lens, 300 + T, f"windows T={T} N={N}")
    phi[5, N // 2, :, :] = float("-inf")
    got = crf.lccrf_sample(phi.cuda(), torch.rand(7, N).cuda(), lens.cuda()).cpu().numpy()
    L5 = int(lens[5])
    if L5 > N // 2:
        assert (got[5, :L5] == 0).all() and (got[5, L5:] == -1).all()


def test_sample_config5(crf, oracle_mod):
    w = workloads.WORKLOADS["cfg5"]
    _check_every_draw(crf, oracle_mod, workloads.phi_batch(w), workloads.lengths(w), 12, "cfg5")


def test_sample_frequencies(crf):
    """Many independent draws from one small chain: path frequencies match the probabilities that
    lccrf_log_prob assigns (5 sigma)."""
    T, N, M = 3, 4, 200000
    phi1, _ = workloads.random_case(8300, 1, N, T, scale=1.2)
    phi = phi1.expand(M, N, T, T).contiguous().cuda()
    u = torch.rand(M, N, generator=torch.Generator().manual_seed(3)).cuda()
    tags = crf.lccrf_sample(phi, u)
    codes = (tags.long() * (T ** torch.arange(N - 1, -1, -1, device="cuda"))).sum(1)
    freq = torch.bincount(codes, minlength=T ** N).double() / M
    all_paths = torch.cartesian_prod(*[torch.arange(T)] * N).to(torch.int32).cuda()
    lp = crf.lccrf_log_prob(phi1.expand(T ** N, N, T, T).contiguous().cuda(), all_paths.contiguous())
    p = lp.double().exp()
    assert abs(float(p.sum()) - 1.0) < 1e-4
    assert float((freq - p).abs().max()) < 5 * float((p.max() / M) ** 0.5)


@pytest.mark.parametrize("key", ["cfg2", "cfg3"])
def test_sample_named_workloads(crf, oracle_mod, key):
    w = workloads.WORKLOADS[key]
    _check(crf, oracle_mod, workloads.phi_batch(w), workloads.lengths(w), 11, key, min_exact=0.3)


@pytest.mark.parametrize("T,N,seed", [(5, 8, 1), (16, 300, 2 ** 40 + 7), (48, 33, 12345), (128, 40, 2 ** 63 + 5), (32, 700, 99)])
def test_sample_seeded_matches_the_host_generator(crf, oracle_mod, T, N, seed):
    """The seeded variant draws its uniforms in the library; regenerated on the host they must give, fed to
    lccrf_sample, the same tags bit for bit, and fed to the oracle the same tags wherever its margin is clear."""
    phi, lens = workloads.random_case(8600 + T, 5, N, T, scale=1.5, ragged=True, min_len=1)
    lens[0] = N
    dphi, dl = phi.cuda(), lens.cuda()
    got = crf.lccrf_sample_seeded(dphi, seed, dl)
    again = crf.lccrf_sample_seeded(dphi, seed, dl)
    other = crf.lccrf_sample_seeded(dphi, seed + 1, dl)
    u = philox_host.uniforms(seed, 5, N)
    fed = crf.lccrf_sample(dphi, torch.from_numpy(u).cuda(), dl)
    assert torch.equal(got, again) and torch.equal(got, fed)
    assert not torch.equal(got, other)
    want, margin = oracle_mod.sample(phi, u, lens.numpy())
    g = got.cpu().numpy()
    for b in range(5):
        if margin[b] > MARGIN:
            assert np.array_equal(g[b], want[b]), f"sequence {b} (margin {margin[b]:.2e})"
    lp = oracle_mod.log_prob(phi, g, lens.numpy())
    assert np.isfinite(lp).all()
