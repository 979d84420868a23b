"""The entry point that allocates nothing: sqap_attn_scores_noalloc runs the retention-score kernel on the
library's built-in scratch array.  It must give the bits sqap_attn_scores_batch gives with a caller's
workspace, on consecutive calls of different sizes (the array keeps the previous call's contents), also when
replayed from a HIP graph, and must refuse what the array cannot hold."""
import ctypes

import numpy as np
import pytest

from paper_2509_09090_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from tests import gpu_util
    return gpu_util


def _case(G, nb, S, H, d, seed):
    qs, ks = [], []
    for b in range(nb):
        q, k = wl.query_and_keys(S, H, d, wl.rng_for(98, S, wl.T_Q, seed * 100 + b))
        qs.append(q)
        ks.append(k)
    return qs, ks, G.to_dev(np.stack(qs)), G.to_dev(np.stack(ks))


def test_noalloc_matches_the_workspace_entry_point_on_two_calls_in_a_row(G, oracle):
    import torch
    from paper_2509_09090_amd import binding as B
    # the second call is smaller than the first; the third takes the single-workgroup kernel (no scratch)
    for i, (nb, S, H, d, v0, nv) in enumerate([(16, 276, 32, 128, 0, 256), (3, 61, 8, 32, 7, 40), (2, 100, 3, 24, 5, 60)]):
        qs, ks, qd, kd = _case(G, nb, S, H, d, i)
        ref = torch.zeros(nb, nv, dtype=torch.float32, device="cuda")
        B.sqap_attn_scores_batch(qd, kd, v0, nv, ref, G.score_workspace(nb, S, H, d, nv))
        out = torch.full((nb, nv), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        B.sqap_attn_scores_noalloc(qd, kd, v0, nv, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32)), (nb, S, H, d)
        for b in (0, nb - 1):
            assert np.allclose(out[b].cpu().numpy(), oracle.attn_scores(qs[b], ks[b], v0, nv), rtol=2e-4, atol=1e-7)


def test_noalloc_replayed_from_a_graph(G, oracle):
    """Capture forbids allocation; every replay, with eager calls of another size in between, gives the eager bits."""
    import torch
    from paper_2509_09090_amd import binding as B
    nb, S, H, d, v0, nv = 16, 276, 32, 128, 0, 256
    qs, ks, qd, kd = _case(G, nb, S, H, d, 7)
    qs2, ks2, qd2, kd2 = _case(G, 2, 61, 8, 32, 8)
    ref = torch.zeros(nb, nv, dtype=torch.float32, device="cuda")
    B.sqap_attn_scores_batch(qd, kd, v0, nv, ref, G.score_workspace(nb, S, H, d, nv))
    out = torch.zeros(nb, nv, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.sqap_attn_scores_noalloc(qd, kd, v0, nv, out)          # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.sqap_attn_scores_noalloc(qd, kd, v0, nv, out)
    small = torch.zeros(2, 40, dtype=torch.float32, device="cuda")
    for rep in range(3):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32)), rep
        B.sqap_attn_scores_noalloc(qd2, kd2, 7, 40, small)       # eager work on the same array between replays
        torch.cuda.synchronize()
        assert np.allclose(small[1].cpu().numpy(), oracle.attn_scores(qs2[1], ks2[1], 7, 40), rtol=2e-4, atol=1e-7)


def test_noalloc_refuses_what_the_array_cannot_hold(G):
    from paper_2509_09090_amd import binding as B
    L = B.lib()
    p = ctypes.c_void_p(4096)
    assert L.sqap_attn_scores_noalloc(p, p, 65, 276, 32, 128, 0, 256, p, None) == B.EUNSUPPORTED
    assert b"64" in L.sqap_last_error()
    assert L.sqap_attn_scores_noalloc(p, p, 64, 4096, 32, 128, 0, 4096, p, None) == B.EUNSUPPORTED
    assert b"524288" in L.sqap_last_error()
    assert L.sqap_attn_scores_noalloc(p, p, -1, 276, 32, 128, 0, 256, p, None) == B.EINVAL
    assert L.sqap_attn_scores_noalloc(None, None, 0, 276, 32, 128, 0, 256, None, None) == B.OK
