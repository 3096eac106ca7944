"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, sizes workspaces sensibly and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2308_03291_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2308_03291_amd import build_ext
        build_ext.build()
    return binding.load_library()


def _declared_functions():
    """Every function declared in any header under include/."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(lccrf_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert "lccrf_log_partition" in names and "lccrf_marginals" in names and "lccrf_argmax" in names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared under include/ but not exported"
    assert set(names) == set(binding.EXPORTS)


def test_version_and_strerror(lib):
    assert lib.lccrf_version() >= 100
    assert binding.strerror(0) == "ok"
    for code in range(-7, 0):
        assert "unknown" not in binding.strerror(code)
    assert "unknown" in binding.strerror(-99)


def test_workspace_sizes(lib):
    for op in (binding.OP_LOGZ, binding.OP_MARGINALS, binding.OP_ARGMAX):
        n = binding.workspace_bytes(op, 64, 512, 128, binding.LCCRF_F32)
        assert n > 0 and n % 256 == 0
        # scratch is O(B N T), a 1/T fraction of the potentials
        assert n <= 64 * 512 * 128 * 16 + 4096 * 8
    assert binding.workspace_bytes(binding.OP_MARGINALS, 0, 8, 8, 0) == 0
    assert binding.workspace_bytes(binding.OP_MARGINALS, 1, 8, 257, 0) == 0
    assert binding.workspace_bytes(binding.OP_MARGINALS, 1, 8, 8, 7) == 0
    assert binding.workspace_bytes(9, 1, 8, 8, 0) == 0


def test_auto_schedule_is_reported_without_a_gpu(lib):
    """lccrf_auto_algo is host arithmetic: long chains over few tags in small batches take the scan.  (Without a
    device there are no compute units to count and the chain-wave kernels are never chosen; their share of AUTO
    is asserted on the GPU.)"""
    assert binding.auto_algo(binding.OP_MARGINALS, 4, 16384, 16) == binding.ALGO_SCAN       # config 5
    assert binding.auto_algo(binding.OP_ARGMAX, 4, 16384, 16) == binding.ALGO_SCAN
    assert binding.auto_algo(binding.OP_MARGINALS, 64, 512, 128) == binding.ALGO_SEQUENTIAL  # config 4
    assert binding.auto_algo(binding.OP_MARGINALS, 128, 256, 32) == binding.ALGO_SCAN        # the paper's size
    assert binding.auto_algo(binding.OP_ARGMAX, 128, 256, 32) == binding.ALGO_SEQUENTIAL     # max-plus scan: 16 tags
    assert binding.auto_algo(binding.OP_ENTROPY, 128, 256, 32) == binding.ALGO_SEQUENTIAL
    assert binding.auto_algo(binding.OP_MARGINALS, 32, 64, 32) == binding.ALGO_SCAN          # config 2: chunks of 8
    assert binding.auto_algo(binding.OP_MARGINALS, 32, 63, 32) == binding.ALGO_SEQUENTIAL    # fewer than eight chunks
    assert binding.auto_algo(binding.OP_ARGMAX, 256, 256, 16) == binding.ALGO_SEQUENTIAL
    assert binding.auto_algo(binding.OP_MARGINALS, 256, 256, 16) == binding.ALGO_SCAN
    assert binding.auto_algo(binding.OP_MARGINALS, 4, 8, 5) == binding.ALGO_SEQUENTIAL       # config 1
    assert binding.auto_algo(binding.OP_MARGINALS, 128, 128, 48) == binding.ALGO_SEQUENTIAL  # config 3: too many positions
    assert binding.auto_algo(binding.OP_MARGINALS, 32, 256, 48) == binding.ALGO_SCAN         # 33 .. 64 tags, small batch
    assert binding.auto_algo(binding.OP_ENTROPY, 32, 256, 48) == binding.ALGO_SEQUENTIAL     # entropy by edges: 32 tags at most
    assert binding.auto_algo(binding.OP_SAMPLE, 32, 256, 48) == binding.ALGO_SEQUENTIAL
    # long chains pay whatever the batch holds, while the batch is small
    assert binding.auto_algo(binding.OP_MARGINALS, 4, 16384, 32) == binding.ALGO_SCAN
    assert binding.auto_algo(binding.OP_LOGZ, 128, 1024, 32) == binding.ALGO_SCAN
    assert binding.auto_algo(binding.OP_LOGZ, 256, 4096, 32) == binding.ALGO_SEQUENTIAL
    assert binding.auto_algo(binding.OP_MARGINALS, 8, 4096, 48) == binding.ALGO_SCAN
    assert binding.auto_algo(binding.OP_MARGINALS, 64, 4096, 48) == binding.ALGO_SEQUENTIAL
    assert binding.auto_algo(binding.OP_MARGINALS, 16, 1024, 64) == binding.ALGO_SCAN
    with pytest.raises(binding.LccrfError):
        binding.auto_algo(binding.OP_MARGINALS, 1, 8, 0)
    with pytest.raises(binding.LccrfError):
        binding.auto_algo(99, 1, 8, 4)


def test_bad_arguments_are_rejected_without_a_gpu(lib):
    fake = 4096  # a non-null, aligned "pointer" that is never dereferenced on these paths
    ws = 1 << 20
    EINVAL, ENULL, EWS, EALIGN = -1, -2, -3, -4
    assert lib.lccrf_log_partition(fake, 0, None, 0, 4, 4, fake, fake, ws, None) == EINVAL
    assert lib.lccrf_log_partition(fake, 0, None, 1, 4, 300, fake, fake, ws, None) == EINVAL
    assert lib.lccrf_log_partition(fake, 5, None, 1, 4, 4, fake, fake, ws, None) == EINVAL
    assert lib.lccrf_log_partition(None, 0, None, 1, 4, 4, fake, fake, ws, None) == ENULL
    assert lib.lccrf_log_partition(fake, 0, None, 1, 4, 4, None, fake, ws, None) == ENULL
    assert lib.lccrf_log_partition(fake, 0, None, 1, 4, 4, fake, None, ws, None) == EWS
    assert lib.lccrf_log_partition(fake, 0, None, 1, 4, 4, fake, fake, 8, None) == EWS
    assert lib.lccrf_log_partition(fake + 4, 0, None, 1, 4, 4, fake, fake, ws, None) == EALIGN
    assert lib.lccrf_log_partition(fake, 0, None, 1, 4, 4, fake, fake + 16, ws, None) == EALIGN
    assert lib.lccrf_marginals(fake, 0, None, 1, 4, 4, None, None, fake, ws, None) == ENULL
    assert lib.lccrf_marginals(fake, 0, None, 1, 4, 4, None, fake + 4, fake, ws, None) == EALIGN
    assert lib.lccrf_argmax(fake, 0, None, 1, 4, 4, None, None, fake, ws, None) == ENULL
    assert lib.lccrf_argmax_algo(fake, 0, None, 1, 4, 4, None, fake, fake, ws, None, 17) == EINVAL


def test_tuning_knobs_check_their_range(lib):
    assert lib.lccrf_set_scan_chunk(3) == -1 and lib.lccrf_set_scan_chunk(5000) == -1
    assert lib.lccrf_set_scan_chunk(0) == 0
    assert lib.lccrf_set_pair_poll_limit(-2) == -1 and lib.lccrf_set_pair_poll_limit((1 << 24) + 1) == -1
    assert lib.lccrf_set_pair_poll_limit(0) == 0 and lib.lccrf_set_pair_poll_limit(-1) == 0
    assert lib.lccrf_set_lane_poll_limit(-2) == -1 and lib.lccrf_set_lane_poll_limit((1 << 24) + 1) == -1
    assert lib.lccrf_set_lane_poll_limit(0) == 0 and lib.lccrf_set_lane_poll_limit(-1) == 0
    # the chunk enters the workspace size: a call sized under one setting is refused under a larger need
    small = binding.workspace_bytes(binding.OP_MARGINALS, 2, 4096, 16, 0)
    assert lib.lccrf_set_scan_chunk(4) == 0
    try:
        assert binding.workspace_bytes(binding.OP_MARGINALS, 2, 4096, 16, 0) > small
        fake = 4096
        assert lib.lccrf_marginals(fake, 0, None, 2, 4096, 16, fake, fake, fake, small, None) == -3
    finally:
        assert lib.lccrf_set_scan_chunk(0) == 0


def test_host_philox_known_answers():
    """The host copy of Philox4x32-10 (tests/philox_host.py), which the seeded sampling test regenerates the
    library's uniforms with, against the known-answer vectors published with the generator."""
    import numpy as np
    import philox_host
    def one(counter, key):
        return [int(x) for x in philox_host.philox4x32_10([np.uint64(c) for c in counter], key)]
    assert one([0, 0, 0, 0], [0, 0]) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert one([0xffffffff] * 4, [0xffffffff] * 2) == [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]
    u = philox_host.uniforms(12345, 3, 7)
    assert u.shape == (3, 7) and u.dtype == np.float32 and (u >= 0).all() and (u < 1).all()


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(ValueError):
        binding.lccrf_log_partition(torch.zeros(1, 2, 3, 3))
    with pytest.raises(ValueError):
        binding.lccrf_marginals(torch.zeros(1, 2, 3, 4))


def test_product_does_not_import_the_oracle():
    """The product path must never route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2308_03291_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "lccrf_oracle" not in text, f
