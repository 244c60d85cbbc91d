"""The whole hot path recorded into one HIP graph and replayed: every library call is a
sequence of kernel launches on the caller's stream (no host synchronisation, no memset node,
the work-list counters are cleared by kernels), so a caller may capture a layer and replay it
per denoising step. Each replay is checked bit for bit against the eager result, with eager
runs of the same path between the replays."""
import pytest
import torch

import paper_2603_08982_amd as sv
from workloads import budget_pairs, get_workload, make_qkv
from helpers import dev, init_centroids

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["default", "candidate_lists"])
def kmeans_mode(request):
    """The library's default, and the later k-means iterations forced onto candidate lists (more
    kernels, queues filled through atomics) whatever the number of centroids."""
    from paper_2603_08982_amd.binding import kmeans_list_threshold
    before = kmeans_list_threshold(1) if request.param == "candidate_lists" else kmeans_list_threshold(0)
    yield request.param
    kmeans_list_threshold(before)


@pytest.mark.parametrize("overlap", [False, True])
@pytest.mark.parametrize("name", ["mini_video", "mini_video_tail"])
def test_captured_layer_replays_bit_exactly(name, overlap, kmeans_mode):
    wl = get_workload(name)
    Q, K, V = make_qkv(wl, dev())
    cq0 = init_centroids(Q, wl.Cq, wl.seed, 0, wl.n_tail)
    ck0 = init_centroids(K, wl.Ck, wl.seed, 1, wl.n_tail)
    budget = budget_pairs(wl.rho, wl.N, wl.N)

    def eager():
        cq, ck = cq0.clone(), ck0.clone()
        O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail)
        torch.cuda.synchronize()
        return O, r["mask_bits"], cq, ck

    O_ref, mask_ref, cq_ref, ck_ref = eager()

    cq, ck = cq0.clone(), ck0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # one uncaptured pass on the capture stream first
        sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail, overlap=overlap)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cq.copy_(cq0)
        ck.copy_(ck0)
        O, r = sv.attention_layer(Q, K, V, cq, ck, wl.iters, budget, wl.n_tail, overlap=overlap)
    for _ in range(3):
        O.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, O_ref)
        assert torch.equal(r["mask_bits"], mask_ref)
        assert torch.equal(cq, cq_ref) and torch.equal(ck, ck_ref)
        eager()
