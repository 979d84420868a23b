"""GPU parity: the HIP library against the CPU oracle, element by element, on
the same seeded inputs, through the C ABI.  Integer outputs (indices, int4
codes, int32 accumulators, scales' bit patterns) must be identical; fp16
outputs must be within 1e-2 + 1e-3|ref| (and are expected to be bit-equal,
since the epilogue arithmetic is pinned)."""
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


# ------------------------------------------------------------------ top-k / rows / gather
@pytest.mark.parametrize("batch,n,k", [(1, 64, 32), (1, 256, 128), (1, 256, 64), (16, 256, 128),
                                       (3, 1, 1), (2, 7, 3), (2, 255, 254), (2, 300, 1),
                                       (2, 1000, 17), (2, 2048, 1000), (2, 2049, 5), (3, 5000, 2500),
                                       (1, 65536, 4097), (2, 4096, 4096), (4, 256, 256)])
def test_topk_random(G, oracle, batch, n, k):
    s = wl.scores(batch, n, wl.rng_for(90, n, wl.T_SCORES, k))
    assert np.array_equal(G.gpu_prune_topk(s, k), oracle.prune_topk(s, k))


@pytest.mark.parametrize("n", [64, 256, 4096])
def test_topk_adversarial(G, oracle, n):
    rng = np.random.default_rng(n)
    cases = {
        "all_equal": np.full(n, 0.5, np.float32),
        "two_valued": np.tile(np.array([1.0, 0.0], np.float32), n // 2),
        "descending": np.linspace(1, 0, n).astype(np.float32),
        "ascending": np.linspace(0, 1, n).astype(np.float32),
        "dups": (np.round(rng.random(n) * 10) / 10).astype(np.float32),
        "signed_zero": np.array([0.0, -0.0] * (n // 2), np.float32),
        "with_nan": np.where(np.arange(n) % 5 == 0, np.nan, np.arange(n) % 7).astype(np.float32),
        "all_nan": np.full(n, np.nan, np.float32),
        "infs": np.array([np.inf, -np.inf, 1.0, np.inf] * (n // 4), np.float32),
        "negatives": -np.arange(n, dtype=np.float32),
        "denormals": (np.arange(n) % 9).astype(np.float32) * np.float32(1e-45),
    }
    for name, s in cases.items():
        for k in (1, 2, n // 2 - 1, n // 2, n // 2 + 1, n - 1, n):
            got = G.gpu_prune_topk(s[None, :], k)
            assert np.array_equal(got, oracle.prune_topk(s[None, :], k)), (name, k)


def test_topk_zero_sizes(G):
    import torch
    from paper_2509_09090_amd import binding as B
    s = torch.zeros((2, 8), dtype=torch.float32, device="cuda")
    out = torch.zeros((2, 0), dtype=torch.int32, device="cuda")
    B.sqap_prune_topk(s, 0, out)          # keep_k = 0: legal no-op
    with pytest.raises(B.SqapError):
        B.sqap_prune_topk(s, 9, torch.zeros((2, 9), dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("batch,S,v0,nv,k", [(1, 276, 0, 256, 128), (16, 276, 0, 256, 128),
                                             (3, 30, 4, 16, 5), (2, 700, 100, 500, 123),
                                             (2, 20, 0, 20, 0), (2, 20, 3, 0, 0), (1, 64, 0, 64, 32)])
def test_kept_rows_and_gather(G, oracle, batch, S, v0, nv, k):
    s = wl.scores(batch, max(nv, 1), wl.rng_for(91, S, wl.T_SCORES, k))[:, :nv]
    idx = oracle.prune_topk(s, k) if nv else np.zeros((batch, 0), np.int32)
    rows = oracle.kept_rows(idx, S, v0, nv)
    assert np.array_equal(G.gpu_kept_rows(idx, S, v0, nv), rows)
    X, _ = wl.activations(batch * S, 64, 2, 20.0, wl.rng_for(91, S, wl.T_X, k))
    assert np.array_equal(G.gpu_gather(X, rows).view(np.uint16), X[rows].view(np.uint16))


@pytest.mark.parametrize("batch,S,v0,nv,k", [(16, 276, 0, 256, 128), (1, 276, 0, 256, 64), (3, 30, 4, 16, 5),
                                             (2, 700, 100, 500, 123), (2, 20, 0, 20, 0), (2, 2500, 7, 2048, 1000),
                                             (2, 5000, 100, 4096, 77), (2, 40, 5, 30, 30),
                                             (2, 1500, 3, 1000, 400), (2, 2100, 0, 900, 10), (3, 600, 88, 512, 511)])
def test_prune_rows_fused(G, oracle, batch, S, v0, nv, k):
    import torch
    from paper_2509_09090_amd import binding as B
    s = wl.scores(batch, nv, wl.rng_for(96, S, wl.T_SCORES, k))
    idx = torch.full((batch, k), -1, dtype=torch.int32, device="cuda")
    rows = torch.full((batch * (S - nv + k),), -1, dtype=torch.int32, device="cuda")
    B.sqap_prune_rows(G.to_dev(s), k, S, v0, idx, rows)
    torch.cuda.synchronize()
    idx_o = oracle.prune_topk(s, k)
    assert np.array_equal(idx.cpu().numpy(), idx_o)
    assert np.array_equal(rows.cpu().numpy(), oracle.kept_rows(idx_o, S, v0, nv))


# ------------------------------------------------------------------ quantizer
@pytest.mark.parametrize("M,K", [(64, 512), (148, 4096), (37, 11008), (5, 8), (3, 16), (9, 2056),
                                 (2, 16384), (1, 4096), (8, 11008),
                                 (1025, 520), (1024, 4096), (1031, 11008)])       # two rows per block from 1024 rows on
def test_quantize_act(G, oracle, M, K):
    X, _ = wl.activations(M, K, max(1, wl.n_outliers_for(K)), 30.0, wl.rng_for(92, M, wl.T_X, K))
    q, s = G.gpu_quantize(X)
    qo, so, _ = oracle.quantize_rows(X)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16))
    assert np.array_equal(q, qo)


def test_quantize_act_fused_gather(G, oracle):
    X, _ = wl.activations(276, 4096, 41, 30.0, wl.rng_for(92, 1, wl.T_X, 1))
    rows = np.sort(np.random.default_rng(5).choice(276, 148, replace=False)).astype(np.int32)
    q, s = G.gpu_quantize(X, rows=rows)
    qo, so, _ = oracle.quantize_rows(X, rows=rows)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16)) and np.array_equal(q, qo)


@pytest.mark.parametrize("M,K", [(7, 16), (5, 64), (33, 512), (148, 4096), (3, 16384), (37, 11008), (9, 1536), (4, 48),
                                 (6, 10240)])
def test_quantize_act_rotated(G, oracle, M, K):
    X, _ = wl.activations(M, K, max(1, wl.n_outliers_for(K)), 30.0, wl.rng_for(93, M, wl.T_X, K))
    q, s = G.gpu_quantize(X, rotate=True)
    qo, so, _ = oracle.quantize_rows(X, rotate=True)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16))
    assert np.array_equal(q, qo)


def test_quantize_special_rows(G, oracle):
    K = 64
    X = np.zeros((7, K), np.float16)
    X[6, :4] = np.array([-10, 10, -7, 3], np.float16) * np.float16(2.0 ** -24)   # the only way to code -8: the clamp
    X[1, 3] = np.float16(6e-8)            # smallest subnormal: scale floor path
    X[2] = np.float16(65504.0)
    X[3, ::2] = np.float16(-1.5)
    X[4] = np.linspace(-7, 7, K).astype(np.float16)   # exact .5 ties with scale 1
    X[5, 0], X[5, 1] = np.float16(7.0), np.float16(2.5)
    q, s = G.gpu_quantize(X)
    qo, so, _ = oracle.quantize_rows(X)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16)) and np.array_equal(q, qo)


def test_quantizer_quotient_is_the_ieee_quotient(G):
    """Every (half, half) pair: the fast quotient of the quantizer equals the division operator."""
    import torch
    from paper_2509_09090_amd import binding as B
    c = torch.zeros((1,), dtype=torch.int64, device="cuda")
    B.sqap_selftest_quotient(c)
    torch.cuda.synchronize()
    assert int(c.item()) == 0


def test_quantize_weight(G, oracle):
    W = wl.weights(512, 512, wl.rng_for(94, 0, wl.T_W))
    q, s = G.gpu_quantize(W, weight=True)
    qo, so, _ = oracle.quantize_rows(W)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16)) and np.array_equal(q, qo)
    q, s = G.gpu_quantize(W, weight=True, rotate=True)
    qo, so, _ = oracle.quantize_rows(W, rotate=True)
    assert np.array_equal(s.view(np.uint16), so.view(np.uint16)) and np.array_equal(q, qo)


# ------------------------------------------------------------------ full selection rule (Eq. 1-5)
def _gpu_select(G, s, gw, gh, k_attn, total, cam, radius, cap=None):
    import torch
    from paper_2509_09090_amd import binding as B
    s2 = np.atleast_2d(s).astype(np.float32)
    cap = gw * gh if cap is None else cap
    idx = torch.full((s2.shape[0], cap), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((s2.shape[0],), -7, dtype=torch.int32, device="cuda")
    B.sqap_prune_select(G.to_dev(s2), gw, gh, k_attn, total, None if cam is None else G.to_dev(cam), radius, idx, cnt)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cnt.cpu().numpy()


def _oracle_select(oracle, s, gw, gh, k_attn, total, cam, radius):
    out = []
    for b, row in enumerate(np.atleast_2d(s)):
        centre = None
        if cam is not None:
            centre = oracle.project_token(cam[b, 0:9], cam[b, 9:21], cam[b, 21:24], cam[b, 24], cam[b, 25])
        out.append(oracle.prune_select(row, gw, gh, k_attn, total, centre, radius))
    return out


@pytest.mark.parametrize("gw,gh,batch,k_attn,total,radius,with_cam", [
    (16, 16, 16, 64, 128, 2, True),       # the workload's grid: 256 visual tokens, half kept
    (16, 16, 3, 100, 128, 0, False),      # no ring
    (16, 16, 4, 0, 60, 1, True),          # no attention set
    (16, 16, 4, 128, 128, 3, True),       # the union exceeds the total: it is not cut
    (16, 16, 2, 10, 256, 1, True),        # keep everything
    (32, 32, 3, 300, 700, 4, True),       # the largest grid, 16 tokens per lane
    (5, 3, 6, 2, 9, 1, True),             # ragged small grid
    (1, 9, 2, 1, 5, 0, False),            # one column
    (16, 16, 2, 20, 40, 1000, True),      # a ring that covers the grid
    (7, 11, 5, 0, 0, 0, False),           # nothing kept
])
def test_prune_select(G, oracle, gw, gh, batch, k_attn, total, radius, with_cam):
    rng = wl.rng_for(96, gw * 100 + gh, wl.T_SCORES, extra=k_attn)
    s = wl.scores(batch, gw * gh, rng)
    s[0, : (gw * gh) // 2] = 0.5                       # a run of equal scores: ties by index
    cam = wl.cameras(batch, gw, gh, 14.0, wl.rng_for(96, gw * 100 + gh, wl.T_CAMERA)) if with_cam else None
    idx, cnt = _gpu_select(G, s, gw, gh, k_attn, total, cam, radius)
    want = _oracle_select(oracle, s, gw, gh, k_attn, total, cam, radius)
    for b in range(batch):
        assert cnt[b] == len(want[b]), b
        assert np.array_equal(idx[b, : cnt[b]], want[b]), b
        assert np.all(idx[b, cnt[b]:] == -1)


def test_prune_select_projection_edge_cases(G, oracle):
    """Points on patch borders, outside the image, behind the camera: the token is decided in binary64
    on both sides, so the sets agree exactly."""
    gw = gh = 16
    s = wl.scores(8, 256, wl.rng_for(97, 0, wl.T_SCORES))
    cam = np.zeros((8, 26))
    cam[:, 0:9] = np.array([[100.0, 0, 112], [0, 100, 112], [0, 0, 1]]).reshape(-1)
    cam[:, 9:21] = np.hstack([np.eye(3), np.zeros((3, 1))]).reshape(-1)
    cam[:, 24:26] = 14.0
    pts = [(0, 0, 1), (0.14, 0.28, 1), (-1.12, -1.12, 1), (-1.1201, 0, 1), (5, 5, 1), (0, 0, -1), (0, 0, 0),
           (1.0 / 3, 2.0 / 3, 7.0 / 9)]
    cam[:, 21:24] = np.array(pts)
    idx, cnt = _gpu_select(G, s, gw, gh, 32, 96, cam, 2)
    want = _oracle_select(oracle, s, gw, gh, 32, 96, cam, 2)
    for b in range(8):
        assert cnt[b] == len(want[b]) and np.array_equal(idx[b, : cnt[b]], want[b]), b


def test_prune_select_feeds_the_row_list(G, oracle):
    """The selected tokens shorten the sequence exactly as the top-k tokens do."""
    s = wl.scores(4, 256, wl.rng_for(98, 0, wl.T_SCORES))
    cam = wl.cameras(4, 16, 16, 14.0, wl.rng_for(98, 0, wl.T_CAMERA))
    idx, cnt = _gpu_select(G, s, 16, 16, 64, 128, cam, 1, cap=128)
    assert np.all(cnt == 128)
    rows = G.gpu_kept_rows(idx, 276, 0, 256)
    assert np.array_equal(rows, oracle.kept_rows(np.stack(_oracle_select(oracle, s, 16, 16, 64, 128, cam, 1)), 276, 0, 256))


# ------------------------------------------------------------------ channel-wise activations (Section 3.3)
def _gpu_channelwise(G, X, W, rows=None, rotate=False, batches=1):
    import torch
    from paper_2509_09090_amd import binding as B
    flags = B.ROTATE_HADAMARD if rotate else 0
    x, w = G.to_dev(X), G.to_dev(W)
    r = None if rows is None else G.to_dev(rows.astype(np.int32))
    K, N = X.shape[1], W.shape[0]
    M = X.shape[0] if rows is None else rows.size
    amax = torch.full((K,), 123.0, dtype=torch.float32, device="cuda")         # cleared by the call
    c = torch.zeros((K,), dtype=torch.float16, device="cuda")
    if batches == 1:
        B.sqap_channel_scales(x, r, amax, c, flags)
    else:                                                                       # same rows in several calls
        order = np.arange(M) if rows is None else rows
        parts = np.array_split(order, batches)
        for i, part in enumerate(parts):
            B.sqap_channel_scales(x, G.to_dev(part.astype(np.int32)), amax, c, flags, accumulate=i > 0)
    xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((M,), dtype=torch.float16, device="cuda")
    B.sqap_quantize_act_channelwise(x, r, c, xq, sx, flags)
    wq = torch.zeros((N, K // 2), dtype=torch.uint8, device="cuda")
    sw = torch.zeros((N,), dtype=torch.float16, device="cuda")
    B.sqap_quantize_weight_folded(w, c, wq, sw, flags)
    torch.cuda.synchronize()
    return c.cpu().numpy(), xq.cpu().numpy(), sx.cpu().numpy(), wq.cpu().numpy(), sw.cpu().numpy()


@pytest.mark.parametrize("M,K,N,rotate,gather,batches", [
    (148, 4096, 96, False, False, 1),      # the workload's hidden size
    (300, 11008, 40, False, True, 3),      # the FFN width, gathered rows, calibration in three calls
    (64, 512, 64, True, False, 1),         # rotated first
    (37, 2048, 33, True, True, 2),
    (5, 64, 3, False, False, 1),           # a single group of eight per thread, most threads idle
    (700, 16384, 8, True, False, 1),       # the widest rows, more rows than calibration blocks
])
def test_channelwise_quantization(G, oracle, M, K, N, rotate, gather, batches):
    rng = wl.rng_for(99, M, wl.T_X, extra=K)
    S = M + 9 if gather else M
    X, _ = wl.activations(S, K, max(1, wl.n_outliers_for(K)), 30.0, rng)
    X[:, 3] = 0                                                  # a dead channel: smallest scale, codes 0
    W = wl.weights(N, K, rng)
    rows = rng.permutation(S)[:M].astype(np.int32) if gather else None
    c, xq, sx, wq, sw = _gpu_channelwise(G, X, W, rows, rotate, batches)
    co = oracle.channel_scales(X, rows=rows, rotate=rotate)
    assert np.array_equal(c.view(np.uint16), co.view(np.uint16))
    xqo, sxo = oracle.quantize_rows_channelwise(X, co, rows=rows, rotate=rotate)
    assert np.array_equal(xq, xqo) and np.array_equal(sx.view(np.uint16), sxo.view(np.uint16))
    wqo, swo = oracle.quantize_rows_folded(W, co, rotate=rotate)
    assert np.array_equal(wq, wqo) and np.array_equal(sw.view(np.uint16), swo.view(np.uint16))


def test_channelwise_linear_end_to_end(G, oracle):
    """Calibrate, quantize both sides, run the W4A4 linear: exact accumulators, outputs at the parity bar."""
    rng = wl.rng_for(99, 1, wl.T_W)
    X, _ = wl.activations(148, 4096, 41, 30.0, rng)
    W = wl.weights(256, 4096, rng)
    c, xq, sx, wq, sw = _gpu_channelwise(G, X, W)
    Y, acc = G.gpu_linear(xq, sx, wq, sw)
    Yo, acco = oracle.w4a4_linear(xq, sx, wq, sw)
    assert np.array_equal(acc, acco) and G.assert_fp16_close(Y, Yo) == 0
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.linalg.norm(Y.astype(np.float64) - ref) / np.linalg.norm(ref) < 0.35


# ------------------------------------------------------------------ linear
def _random_packed(rng, R, K):
    return rng.integers(0, 256, size=(R, K // 2), dtype=np.uint8)


@pytest.mark.parametrize("M,N,K", [(32, 512, 512), (1, 32, 32), (8, 4096, 4096), (148, 512, 1024),
                                   (300, 700, 352), (70, 33, 96), (257, 300, 128), (5, 1000, 11008),
                                   (148, 1024, 11008), (513, 544, 640),
                                   # ragged last tile row of the 256-row tiles: 2, 3, 5 and 7 of its 8 row groups hold tokens
                                   (576, 1280, 4096), (608, 512, 2048), (672, 768, 1024), (736, 512, 512),
                                   (2368, 512, 4096)])
def test_linear_random_codes(G, oracle, M, N, K):
    """Uniform random codes (including -8) exercise every tile edge and the exact int32 sum."""
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    Xq, Wq = _random_packed(rng, M, K), _random_packed(rng, N, K)
    sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    Y, acc = G.gpu_linear(Xq, sx, Wq, sw)
    Yo, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
    assert np.array_equal(acc, acco)
    assert G.assert_fp16_close(Y, Yo) == 0


def test_dispatch_order_selftest(G):
    """Workgroup b of a launch runs on XCD b % 8: what the persistent GEMM kernels rely on."""
    from paper_2509_09090_amd import binding as B
    table = B.sqap_selftest_dispatch()
    assert len(table) == 256 and all(table[b] == table[b % 8] for b in range(256)), table


@pytest.mark.parametrize("M,N,K", [(600, 768, 1024), (148, 1024, 2048), (84, 512, 1024)])
def test_linear_fallback_kernels(G, oracle, M, N, K):
    """With the persistent kernels switched off the one-tile-per-workgroup kernels give the same bits."""
    rng = np.random.default_rng(M + N + K)
    Xq, Wq = _random_packed(rng, M, K), _random_packed(rng, N, K)
    sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    Y1, acc1 = G.gpu_linear(Xq, sx, Wq, sw)
    from paper_2509_09090_amd import binding as B
    B.sqap_set_persistent_kernels(False)
    try:
        Y2, acc2 = G.gpu_linear(Xq, sx, Wq, sw)
    finally:
        B.sqap_set_persistent_kernels(True)
    _, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
    assert np.array_equal(acc1, acco) and np.array_equal(acc2, acco)
    assert np.array_equal(Y1.view(np.uint16), Y2.view(np.uint16))


def test_linear_extreme_codes(G, oracle):
    """All codes -8 on both sides: the largest accumulator the format allows (64 K)."""
    M, N, K = 40, 64, 11008
    Xq = np.full((M, K // 2), 0x88, np.uint8)
    Wq = np.full((N, K // 2), 0x88, np.uint8)
    sx = np.full(M, 1.0, np.float16)
    sw = np.full(N, 2.0 ** -10, np.float16)
    Y, acc = G.gpu_linear(Xq, sx, Wq, sw)
    assert np.all(acc == 64 * K)
    Yo, _ = oracle.w4a4_linear(Xq, sx, Wq, sw)
    assert G.assert_fp16_close(Y, Yo) == 0


def test_config0_end_to_end(G, oracle):
    """Configuration 0: prune 64 -> 32 tokens, quantize, one 512x512 W4A4 linear."""
    c = wl.toy_config()
    idx = G.gpu_prune_topk(c["scores"], c["keep_k"])
    idx_o = oracle.prune_topk(c["scores"], c["keep_k"])
    assert np.array_equal(idx, idx_o)
    rows = G.gpu_kept_rows(idx, 64, 0, 64)
    assert np.array_equal(rows, oracle.kept_rows(idx_o, 64, 0, 64))
    Xq, sx = G.gpu_quantize(c["X"], rows=rows)
    Xq_o, sx_o, _ = oracle.quantize_rows(c["X"], rows=rows)
    assert np.array_equal(Xq, Xq_o) and np.array_equal(sx.view(np.uint16), sx_o.view(np.uint16))
    Wq, sw = G.gpu_quantize(c["W"], weight=True)
    Wq_o, sw_o, _ = oracle.quantize_rows(c["W"])
    assert np.array_equal(Wq, Wq_o) and np.array_equal(sw.view(np.uint16), sw_o.view(np.uint16))
    Y, acc = G.gpu_linear(Xq, sx, Wq, sw)
    Yo, acco = oracle.w4a4_linear(Xq_o, sx_o, Wq_o, sw_o)
    assert Y.shape == (32, 512)
    assert np.array_equal(acc, acco)
    assert G.assert_fp16_close(Y, Yo) == 0


def test_attn_scores(G, oracle):
    import torch
    from paper_2509_09090_amd import binding as B
    # (100, 3, 24) and (5000, 2, 32) take the general kernel: head size not a power of two, a long sequence
    for (S, H, d, v0, nv) in [(276, 32, 128, 0, 256), (37, 4, 16, 3, 20), (1000, 5, 64, 10, 990), (300, 128, 8, 1, 299),
                              (4096, 2, 256, 0, 4096), (100, 3, 24, 5, 60), (5000, 2, 32, 100, 4000), (50, 130, 16, 0, 50)]:
        q, k = wl.query_and_keys(S, H, d, wl.rng_for(95, S, wl.T_Q))
        qd, kd = G.to_dev(q), G.to_dev(k)
        out = torch.zeros(nv, dtype=torch.float32, device="cuda")
        ws = G.score_workspace(1, S, H, d, nv)
        B.sqap_attn_scores(qd, kd, v0, nv, out, ws)
        torch.cuda.synchronize()
        ref = oracle.attn_scores(q, k, v0, nv)
        assert np.allclose(out.cpu().numpy(), ref, rtol=2e-4, atol=1e-7), (S, H, d)
        again = torch.zeros(nv, dtype=torch.float32, device="cuda")      # same bits on every call, same workspace
        B.sqap_attn_scores(qd, kd, v0, nv, again, ws)
        torch.cuda.synchronize()
        assert torch.equal(out, again), (S, H, d)
        if ws is not None:
            assert int(ws[:256].view(torch.int32).abs().sum()) == 0     # the counter is back at zero


def test_attn_scores_on_two_streams(G, oracle):
    """Calls that overlap on two streams do not disturb each other when each has its own workspace."""
    import torch
    from paper_2509_09090_amd import binding as B
    S, H, d, v0, nv = 276, 32, 128, 0, 256
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    data = []
    for i in range(2):
        q, k = wl.query_and_keys(S, H, d, wl.rng_for(97, S, wl.T_Q, i))
        data.append((q, k, G.to_dev(q), G.to_dev(k), torch.zeros(nv, dtype=torch.float32, device="cuda"),
                     G.score_workspace(1, S, H, d, nv)))
    torch.cuda.synchronize()
    for rep in range(20):
        for i in range(2):
            q, k, qd, kd, out, ws = data[i]
            B.sqap_attn_scores(qd, kd, v0, nv, out, ws, stream=streams[i].cuda_stream)
    torch.cuda.synchronize()
    for q, k, qd, kd, out, ws in data:
        assert np.allclose(out.cpu().numpy(), oracle.attn_scores(q, k, v0, nv), rtol=2e-4, atol=1e-7)


@pytest.mark.gpu
def test_attn_scores_batch(G, oracle):
    """One launch for a batch of observations gives each what the single call gives, and the oracle's values."""
    import torch
    from paper_2509_09090_amd import binding as B
    # (batch, S, H, d, vis_begin, n_vis)
    for (nb, S, H, d, v0, nv) in [(16, 276, 32, 128, 0, 256), (3, 61, 5, 32, 7, 40), (5, 4096, 32, 16, 0, 4096)]:
        qs, ks = [], []
        for b in range(nb):
            q, k = wl.query_and_keys(S, H, d, wl.rng_for(96, S, wl.T_Q, b))
            qs.append(q)
            ks.append(k)
        qd, kd = G.to_dev(np.stack(qs)), G.to_dev(np.stack(ks))
        out = torch.zeros(nb, nv, dtype=torch.float32, device="cuda")
        ws = G.score_workspace(nb, S, H, d, nv)
        B.sqap_attn_scores_batch(qd, kd, v0, nv, out, ws)
        torch.cuda.synchronize()
        one = torch.zeros(nv, dtype=torch.float32, device="cuda")
        for b in ([0, nb - 1] if S > 1000 else range(nb)):
            ref = oracle.attn_scores(qs[b], ks[b], v0, nv)
            assert np.allclose(out[b].cpu().numpy(), ref, rtol=2e-4, atol=1e-7), (nb, S, H, d, b)
            B.sqap_attn_scores(qd[b], kd[b], v0, nv, one, ws)
            torch.cuda.synchronize()
            assert np.allclose(out[b].cpu().numpy(), one.cpu().numpy(), rtol=1e-6, atol=1e-9), (nb, S, H, d, b)


@pytest.mark.parametrize("M,N,K", [(600, 768, 1024),     # 3 x 3 tiles of 256 x 256 over 256 workgroups: every tile is shared
                                   (148, 1024, 2048),    # narrow tiles, finished together by their contributors
                                   (84, 512, 11008)])
def test_linear_replayed_from_a_graph(G, oracle, M, N, K):
    """A captured launch of the split (persistent) kernels carries the launch epoch it was captured with:
    every replay, with new operands and eager launches on the same workspace in between, must still
    give the exact result."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(4242 + M)
    Wq = _random_packed(rng, N, K)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    W = B.sqap_weight_pack(G.to_dev(Wq), G.to_dev(sw))
    xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    sxd = torch.zeros((M,), dtype=torch.float16, device="cuda")
    Y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
    ws = torch.empty((B.sqap_workspace_bytes(M, N, K),), dtype=torch.uint8, device="cuda")
    ws.random_(0, 256)                  # the workspace needs no initialisation
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.sqap_w4a4_linear(xq, sxd, W, Y, acc, ws)          # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.sqap_w4a4_linear(xq, sxd, W, Y, acc, ws)
    for rep in range(4):
        Xq = _random_packed(rng, M, K)
        sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
        xq.copy_(G.to_dev(Xq))
        sxd.copy_(G.to_dev(sx))
        Y.fill_(float("nan"))
        acc.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        Yo, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
        assert np.array_equal(acc.cpu().numpy(), acco), rep
        assert G.assert_fp16_close(Y.cpu().numpy(), Yo) == 0
        # eager launch on the same workspace between replays
        Y2 = torch.zeros_like(Y)
        B.sqap_w4a4_linear(xq, sxd, W, Y2, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y)
    W.free()


# ------------------------------------------------------------------ small-M (decode) path
@pytest.mark.parametrize("M,N,K", [(1, 4096, 4096), (2, 544, 640), (3, 33, 64), (4, 11008, 4096),
                                   (7, 4096, 11008), (8, 1000, 11008), (8, 32000, 4096), (1, 32, 128),
                                   (8, 64, 64), (5, 96, 1088),
                                   # few row groups with long rows: every wavefront walks its ring two or three times
                                   (1, 8192, 8192), (3, 2048, 16384), (2, 96, 8320), (8, 4096, 11008)])
def test_small_m_linear(G, oracle, M, N, K):
    rng = np.random.default_rng(M * 11 + N * 5 + K)
    Xq, Wq = _random_packed(rng, M, K), _random_packed(rng, N, K)
    sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    Y, acc = G.gpu_linear(Xq, sx, Wq, sw)
    Yo, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
    assert np.array_equal(acc, acco)
    assert G.assert_fp16_close(Y, Yo) == 0


def test_group_with_many_row_groups_per_wavefront(G, oracle):
    """A launch long enough for the form of the kernel that parks outputs in LDS (every wavefront gets
    more row groups than it has slots, so the slots are also emptied mid-run), with problems of different
    token counts, one whose N does not allow 16-byte stores (stored at once, inside the same launch), one
    with the integer accumulators asked for, and an output pitch above N."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(78)
    shapes = [(5, 262144, 64), (8, 262144, 64), (1, 262144, 64), (8, 262144, 64), (3, 131076, 64), (8, 262144, 64),
              (2, 262144, 64), (8, 196608, 128), (7, 262144, 64), (4, 262144, 64)]
    assert sum(-(-N // 32) for _, N, _ in shapes) > 17 * 4096        # more than 16 row groups per wavefront
    problems, refs = [], []
    for i, (M, N, K) in enumerate(shapes):
        Xq = _random_packed(rng, M, K)
        sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
        Wq = _random_packed(rng, N, K)
        sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
        W = B.sqap_weight_pack(G.to_dev(Wq), G.to_dev(sw))
        pitch = N + 16 if i % 2 else N
        Y = torch.full((M, pitch), float("nan"), dtype=torch.float16, device="cuda")[:, :N]
        acc = torch.full((M, N), -1, dtype=torch.int32, device="cuda") if i in (2, 4) else None
        problems.append((G.to_dev(Xq), G.to_dev(sx), W, Y, acc))
        refs.append(oracle.w4a4_linear(Xq, sx, Wq, sw))
    g = B.sqap_group_create(problems)
    for _ in range(2):
        g.run()
    torch.cuda.synchronize()
    for (xq_d, sx_d, W, Y, acc), (Yo, acco) in zip(problems, refs):
        if acc is not None:
            assert np.array_equal(acc.cpu().numpy(), acco)
        assert G.assert_fp16_close(Y.cpu().numpy(), Yo) == 0
    g.free()
    for pr in problems:
        pr[2].free()


def test_group_of_small_m_linears(G, oracle):
    """One launch over several independent problems of different shapes, two of them sharing an input."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(77)
    shapes = [(8, 4096, 4096), (8, 4096, 4096), (1, 11008, 4096), (3, 4096, 11008), (8, 96, 64), (5, 1000, 640)]
    keep, problems, refs = [], [], []
    shared_x = None
    for i, (M, N, K) in enumerate(shapes):
        if i == 1:
            Xq, sx = shared_x
        else:
            Xq = _random_packed(rng, M, K)
            sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
        if i == 0:
            shared_x = (Xq, sx)
        Wq = _random_packed(rng, N, K)
        sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
        xq_d, sx_d = G.to_dev(Xq), G.to_dev(sx)
        W = B.sqap_weight_pack(G.to_dev(Wq), G.to_dev(sw))
        Y = torch.full((M, N + 8), float("nan"), dtype=torch.float16, device="cuda")[:, :N]   # pitch > N
        acc = torch.full((M, N), -1, dtype=torch.int32, device="cuda")
        problems.append((xq_d, sx_d, W, Y, acc))
        refs.append(oracle.w4a4_linear(Xq, sx, Wq, sw))
    g = B.sqap_group_create(problems)
    for _ in range(2):                       # a group is reusable
        g.run()
    torch.cuda.synchronize()
    for (xq_d, sx_d, W, Y, acc), (Yo, acco) in zip(problems, refs):
        assert np.array_equal(acc.cpu().numpy(), acco)
        assert G.assert_fp16_close(Y.cpu().numpy(), Yo) == 0
    g.free()
    for pr in problems:
        pr[2].free()
