"""The library enqueues kernels only (no allocation, no memset, no synchronisation), so a call can be
captured in a HIP graph and replayed: every replay must give what the eager call gives on the same
inputs, also after the inputs in the captured buffers have changed."""
import pytest
import torch

from paper_2308_03291_amd import workloads
from test_gpu_parity import crf  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _capture_and_replay(crf, shapes_seed, B, N, T, scan):
    dev = torch.device("cuda:0")
    algo = crf.ALGO_SCAN if scan else crf.ALGO_SEQUENTIAL
    phi0, lens0 = workloads.random_case(shapes_seed, B, N, T, scale=1.5, ragged=True, min_len=1)
    phi = phi0.to(dev)
    lens = lens0.to(dev)
    mu = torch.empty(B, N, T, T, device=dev)
    lz = torch.empty(B, device=dev)
    tags = torch.empty(B, N, dtype=torch.int32, device=dev)
    score = torch.empty(B, device=dev)
    ws = torch.empty(max(crf.workspace_bytes(op, B, N, T, 0) for op in (1, 2)), dtype=torch.uint8, device=dev)

    def call():
        crf.lccrf_marginals(phi, lens, out=mu, logZ=lz, workspace=ws, algo=algo)
        crf.lccrf_argmax(phi, lens, out=tags, score=score, workspace=ws, algo=algo if T <= 16 else crf.ALGO_SEQUENTIAL)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()                      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(3):
        new_phi, new_lens = workloads.random_case(shapes_seed + 1 + rep, B, N, T, scale=1.0 + rep, ragged=True, min_len=1)
        phi.copy_(new_phi)
        lens.copy_(new_lens)
        for out in (mu, lz, score):
            out.fill_(float("nan"))
        tags.fill_(-9)
        graph.replay()
        torch.cuda.synchronize()
        got = (mu.clone(), lz.clone(), tags.clone(), score.clone())
        call()                      # the same inputs, eagerly
        torch.cuda.synchronize()
        assert torch.equal(got[0], mu) and torch.equal(got[1], lz), f"replay {rep}: marginals differ from the eager call"
        assert torch.equal(got[2], tags) and torch.equal(got[3], score), f"replay {rep}: argmax differs from the eager call"


@pytest.mark.parametrize("B,N,T", [(6, 40, 12), (5, 33, 48), (3, 20, 128)])
def test_graph_replay_sequential(crf, B, N, T):
    _capture_and_replay(crf, 9000 + T, B, N, T, scan=False)


def test_graph_replay_scan(crf):
    _capture_and_replay(crf, 9100, 3, 700, 16, scan=True)
    _capture_and_replay(crf, 9200, 2, 300, 32, scan=True)
