"""svgear_permute_static (scratch inside the library, no allocation) against svgear_permute:
two calls in a row on the same GPU, the second with a smaller input, every output bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2603_08982_amd as sv

pytestmark = pytest.mark.gpu


def _case(seed, B, H, N, C, n_tail, d, dtype):
    g = torch.Generator().manual_seed(seed)
    labels = torch.randint(0, C, (B, H, N - n_tail), generator=g, dtype=torch.int32)
    labels[..., ::7] = C - 1       # a large cluster
    labels[labels == 1] = 0        # an empty one
    K = torch.randn(B, H, N, d, generator=g).to(dtype)
    V = torch.randn(B, H, N, d, generator=g).to(dtype)
    return labels.cuda(), K.cuda(), V.cuda()


def _same(a, b):
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8)) if a.dtype.is_floating_point else torch.equal(a, b)


def test_static_scratch_permute_matches_workspace_permute_on_consecutive_calls():
    lib = sv.load_library()
    assert lib.svgear_permute_static_capacity() == 8 << 20
    # the second call is smaller in every dimension: it must not see what the first one left
    cases = [(0, 1, 6, 9000, 300, 37, 128, torch.bfloat16), (1, 1, 3, 2500, 17, 0, 64, torch.float32)]
    for seed, B, H, N, C, n_tail, d, dtype in cases:
        labels, K, V = _case(seed, B, H, N, C, n_tail, d, dtype)
        print(f"case seed={seed} B={B} H={H} N={N} C={C} tail={n_tail} d={d} {dtype}", flush=True)
        # outputs preallocated by the caller: the static call itself touches no allocator
        out = (torch.full((B, H, N), -1, dtype=torch.int32, device="cuda"),
               torch.full((B, H, C + 2), -1, dtype=torch.int32, device="cuda"),
               [torch.zeros_like(K), torch.zeros_like(V)])
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        perm_s, off_s, (Kp_s, Vp_s) = sv.permute(labels, C, [K, V], n_tail, static_scratch=True, out=out)
        after = torch.cuda.memory_stats()["allocation.all.allocated"]
        assert after == before, "the static-scratch call went through torch's allocator"
        perm, off, (Kp, Vp) = sv.permute(labels, C, [K, V], n_tail)
        torch.cuda.synchronize()
        assert torch.equal(perm_s, perm) and torch.equal(off_s, off)
        assert _same(Kp_s, Kp) and _same(Vp_s, Vp)
        # and it is a stable sort by label with the tail last (independent of the other entry point)
        lab = labels[0, 0].cpu().numpy()
        ref = np.concatenate([np.argsort(lab, kind="stable"), np.arange(N - n_tail, N)]).astype(np.int32)
        assert np.array_equal(perm_s[0, 0].cpu().numpy(), ref)


def test_static_scratch_rejects_sizes_beyond_its_capacity():
    lib = sv.load_library()
    B, H, N, C = 1, 40, 75600, 1500
    assert lib.svgear_permute_workspace(B, H, N, C) > lib.svgear_permute_static_capacity()
    labels = torch.zeros(B, H, N, dtype=torch.int32, device="cuda")
    with pytest.raises(sv.SvgearError, match="workspace"):
        sv.permute(labels, C, [], 0, static_scratch=True)
