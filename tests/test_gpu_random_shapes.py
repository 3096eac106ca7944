"""A seeded sweep over many random shapes, length mixes, scales and both input types: every query
against the CPU oracle, with the scan's chunk size varied too.  The systematic tests cover the
known boundaries one by one; this one looks for interactions between them."""
import numpy as np
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import check_case, crf  # noqa: F401  (fixture)
from test_gpu_two_chains import _check as check_two_chains

pytestmark = pytest.mark.gpu


def _cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(count):
        T = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 15, 16, 17, 24, 31, 32, 33, 40, 48, 63, 64, 65, 96, 127, 128, 129, 160]))
        if T <= 32 and rng.random() < 0.4:
            N = int(rng.integers(256, 900))          # long enough for the scan under AUTO
            B = int(rng.integers(1, 4))
        else:
            N = int(rng.integers(1, max(2, min(200, 6000 // T))))
            B = int(rng.integers(1, 7))
        scale = float(rng.choice([0.3, 1.0, 3.0, 8.0]))
        dtype = "bf16" if rng.random() < 0.3 else "f32"
        ragged = rng.random() < 0.7
        chunk = int(rng.choice([0, 0, 4, 9, 16, 64]))
        out.append((k, B, N, T, scale, dtype, ragged, chunk))
    return out


@pytest.mark.parametrize("k,B,N,T,scale,dtype,ragged,chunk", _cases(20230803, 120))
def test_random_shape(crf, oracle_mod, k, B, N, T, scale, dtype, ragged, chunk):
    phi, lens = workloads.random_case(70000 + k, B, N, T, scale=scale, ragged=ragged, min_len=0, dtype=dtype)
    crf.set_scan_chunk(chunk)
    try:
        what = f"case {k}: B={B} N={N} T={T} scale={scale} {dtype} chunk={chunk}"
        check_case(crf, oracle_mod, phi, lens if ragged else None, poison=(dtype == "f32"), what=what)
        lens_np = lens.numpy() if ragged else None
        dl = lens.cuda() if ragged else None
        H = crf.lccrf_entropy(phi.cuda(), dl).cpu().numpy().astype(np.float64)
        want = oracle_mod.entropy(phi, lens_np)
        assert np.all(np.abs(H - want) <= 2e-4 * np.maximum(1.0, np.abs(want))), f"{what}: entropy {H} vs {want}"
        if k % 3 == 0:   # a second chain over the same sequences: cross-entropy and KL divergence
            q, _ = workloads.random_case(80000 + k, B, N, T, scale=0.5 * scale, dtype=dtype)
            check_two_chains(crf, oracle_mod, phi, q, lens if ragged else None, what)
    finally:
        crf.set_scan_chunk(0)


def _off_grid_cases(seed, count):
    rng = np.random.default_rng(seed)
    tags = [6, 9, 10, 11, 13, 14, 18, 21, 22, 23, 27, 30, 35, 37, 41, 45, 46, 50, 55, 61, 70, 99, 131, 190, 201, 255]
    out = []
    for k in range(count):
        T = int(tags[k % len(tags)])
        N = int(rng.integers(1, max(2, min(120, 5000 // T))))
        B = int(rng.integers(1, 6))
        scale = float(rng.choice([0.3, 1.0, 3.0, 8.0]))
        dtype = "bf16" if rng.random() < 0.35 else "f32"
        ragged = rng.random() < 0.5          # (unragged: the last matrix of the tensor is worked on)
        out.append((k, B, N, T, scale, dtype, ragged))
    return out


@pytest.mark.parametrize("k,B,N,T,scale,dtype,ragged", _off_grid_cases(20230804, 78))
def test_random_shape_off_the_16_byte_grid(crf, oracle_mod, k, B, N, T, scale, dtype, ragged):
    """Tag counts that are no multiple of four, every schedule that serves the shape: the rows of a matrix start at
    any multiple of the element size, and the kernels load pieces of four columns from wherever they start."""
    phi, lens = workloads.random_case(90000 + k, B, N, T, scale=scale, ragged=ragged, min_len=0, dtype=dtype)
    what = f"off-grid case {k}: B={B} N={N} T={T} scale={scale} {dtype}"
    algos = [crf.ALGO_AUTO, crf.ALGO_SEQUENTIAL]
    if T <= 64:
        algos.append(crf.ALGO_SCAN)
    for algo in algos:
        q = ("logz", "mu", "vit") if algo != crf.ALGO_SCAN or T <= 32 else ("logz", "mu")
        check_case(crf, oracle_mod, phi, lens if ragged else None, poison=(dtype == "f32"), algo=algo, what=f"{what} algo={algo}", queries=q)
    if T <= 64:
        q = ("logz", "mu", "vit") if 8 <= T <= 48 else ("vit",)
        check_case(crf, oracle_mod, phi, lens if ragged else None, poison=(dtype == "f32"), algo=crf.ALGO_SEQUENTIAL_LANES,
                   what=f"{what} lanes", queries=q)
