"""GPU parity at the full sizes of the workload configurations, in the launch
configuration bench.py times.  Where the oracle can form the whole product in
seconds it is compared element by element; otherwise on sampled outputs that
the oracle computes one by one from the same inputs.  Every oracle input is
made by the seeded generator and quantized by the oracle itself: nothing the
HIP path produced is fed to it."""
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


def _gpu_pipeline(G, scores, keep, S, nv, X, W, want_acc=False):
    """prune -> rows -> quantize (gather fused) -> weight quantize/pack -> linear; returns numpy."""
    import torch
    from paper_2509_09090_amd import binding as B
    dev = "cuda"
    batch = scores.shape[0]
    M = batch * (S - nv + keep)
    N, K = W.shape
    sc, Xd, Wd = G.to_dev(scores), G.to_dev(X), G.to_dev(W)
    idx = torch.empty((batch, keep), dtype=torch.int32, device=dev)
    rows = torch.empty((M,), dtype=torch.int32, device=dev)
    Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
    sx = torch.empty((M,), dtype=torch.float16, device=dev)
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    sw = torch.empty((N,), dtype=torch.float16, device=dev)
    Y = torch.full((M, N), float("nan"), dtype=torch.float16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    ws = torch.zeros((max(B.sqap_workspace_bytes(M, N, K), 256),), dtype=torch.uint8, device=dev)
    B.sqap_prune_topk(sc, keep, idx)
    B.sqap_kept_rows(idx, S, 0, nv, rows)
    B.sqap_quantize_act(Xd, rows, Xq, sx)
    B.sqap_quantize_weight(Wd, Wq, sw)
    Wh = B.sqap_weight_pack(Wq, sw)
    B.sqap_w4a4_linear(Xq, sx, Wh, Y, acc, ws)
    torch.cuda.synchronize()
    err_word = int(ws[4000:4008].view(torch.int64)[0]) if ws.numel() > 4096 else 0
    out = dict(idx=idx.cpu().numpy(), rows=rows.cpu().numpy(), Xq=Xq.cpu().numpy(), sx=sx.cpu().numpy(),
               Wq=Wq.cpu().numpy(), sw=sw.cpu().numpy(), Y=Y.cpu().numpy(),
               acc=None if acc is None else acc.cpu().numpy(), err_word=err_word)
    Wh.free()
    return out


def _oracle_front(oracle, scores, keep, S, nv, X, W):
    idx = oracle.prune_topk(scores, keep)
    rows = oracle.kept_rows(idx, S, 0, nv)
    Xq, sx, _ = oracle.quantize_rows(X, rows=rows)
    Wq, sw, _ = oracle.quantize_rows(W)
    return idx, rows, Xq, sx, Wq, sw


def _check_front(g, o):
    idx, rows, Xq, sx, Wq, sw = o
    assert np.array_equal(g["idx"], idx)
    assert np.array_equal(g["rows"], rows)
    assert np.array_equal(g["Xq"], Xq)
    assert np.array_equal(g["sx"].view(np.uint16), sx.view(np.uint16))
    assert np.array_equal(g["Wq"], Wq)
    assert np.array_equal(g["sw"].view(np.uint16), sw.view(np.uint16))


def _check_samples(G, oracle, g, o, n_samples, seed):
    _, _, Xq, sx, Wq, sw = o
    M, N = g["Y"].shape
    rng = np.random.default_rng(seed)
    ms = rng.integers(0, M, n_samples).astype(np.int32)
    ns = rng.integers(0, N, n_samples).astype(np.int32)
    # always include the corners and the last row/column of every 256-tile edge
    edge_m = np.array([0, M - 1, min(255, M - 1), min(256, M - 1)], np.int32)
    edge_n = np.array([0, N - 1, min(255, N - 1), min(256, N - 1)], np.int32)
    mm, nn = np.meshgrid(edge_m, edge_n, indexing="ij")
    ms, ns = np.concatenate([ms, mm.ravel()]), np.concatenate([ns, nn.ravel()])
    acc_o, y_o = oracle.linear_samples(Xq, sx, Wq, sw, ms, ns)
    if g["acc"] is not None:
        assert np.array_equal(g["acc"][ms, ns], acc_o)
    assert G.assert_fp16_close(g["Y"][ms, ns], y_o) == 0
    assert not np.isnan(g["Y"].astype(np.float32)).any()      # every output was written


def test_config1_one_layer_all_linears(G, oracle):
    """Configuration 1: 276 tokens, 256 visual pruned to 128 (M = 148), the 7 linears of one layer.
    q is compared in full (with accumulators); the others on 3000 sampled outputs each."""
    c = wl.CONFIGS[1]
    scores = wl.scores(1, wl.N_VISUAL, wl.rng_for(1, 0, wl.T_SCORES))
    for li, (name, N, K) in enumerate(wl.LAYER_LINEARS):
        X = wl.layer_input(1, 0, li, wl.SEQ_LEN)
        W = wl.layer_weight(1, 0, li)
        g = _gpu_pipeline(G, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W, want_acc=(name in ("q", "down")))
        o = _oracle_front(oracle, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W)
        assert g["Y"].shape == (148, N) and g["err_word"] == 0
        _check_front(g, o)
        if name == "q":
            Yo, acco = oracle.w4a4_linear(o[2], o[3], o[4], o[5])
            assert np.array_equal(g["acc"], acco)
            assert G.assert_fp16_close(g["Y"], Yo) == 0
        else:
            _check_samples(G, oracle, g, o, 3000, seed=li)


@pytest.mark.parametrize("li", [4, 6])          # gate/up (4096 -> 11008) and down (11008 -> 4096)
def test_config3_batched_prefill(G, oracle, li):
    """Configuration 3 as bench.py runs it: 16 observations, M = 2368, persistent stream-K launch."""
    c = wl.CONFIGS[3]
    name, N, K = wl.LAYER_LINEARS[li]
    scores = wl.scores(c["batch"], wl.N_VISUAL, wl.rng_for(3, 0, wl.T_SCORES))
    X = wl.layer_input(3, 0, li, c["batch"] * wl.SEQ_LEN)
    W = wl.layer_weight(3, 0, li)
    g = _gpu_pipeline(G, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W, want_acc=True)
    o = _oracle_front(oracle, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W)
    assert g["Y"].shape == (2368, N) and g["err_word"] == 0
    _check_front(g, o)
    # every one of the 2368 x N accumulators and outputs against the full oracle product
    Yo, acco = oracle.w4a4_linear(o[2], o[3], o[4], o[5])
    assert np.array_equal(g["acc"], acco)
    assert G.assert_fp16_close(g["Y"], Yo) == 0


def test_config3_without_acc_output_matches(G, oracle):
    """The timed launch passes no accumulator buffer: same Y either way."""
    c = wl.CONFIGS[3]
    scores = wl.scores(c["batch"], wl.N_VISUAL, wl.rng_for(3, 0, wl.T_SCORES))
    X = wl.layer_input(3, 0, 6, c["batch"] * wl.SEQ_LEN)
    W = wl.layer_weight(3, 0, 6)
    a = _gpu_pipeline(G, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W, want_acc=True)
    b = _gpu_pipeline(G, scores, c["keep_k"], wl.SEQ_LEN, wl.N_VISUAL, X, W, want_acc=False)
    assert np.array_equal(a["Y"].view(np.uint16), b["Y"].view(np.uint16))


@pytest.mark.parametrize("M,keep", [(276, 256), (84, 64)])
def test_config2_stack_shapes(G, oracle, M, keep):
    """Configuration 2: layers 0-1 run on all 276 tokens, the rest on 64 + 20 = 84; two linears each."""
    scores = wl.scores(1, wl.N_VISUAL, wl.rng_for(2, 0, wl.T_SCORES))
    for li in (1, 6):
        X = wl.layer_input(2, 3, li, wl.SEQ_LEN)
        W = wl.layer_weight(2, 3, li)
        g = _gpu_pipeline(G, scores, keep, wl.SEQ_LEN, wl.N_VISUAL, X, W, want_acc=True)
        o = _oracle_front(oracle, scores, keep, wl.SEQ_LEN, wl.N_VISUAL, X, W)
        assert g["Y"].shape[0] == M and g["err_word"] == 0
        _check_front(g, o)
        _check_samples(G, oracle, g, o, 3000, seed=200 + li)


@pytest.mark.parametrize("M", [1, 8])
def test_config4_decode_group(G, oracle, M):
    """Configuration 4: one group launch over the 7 linears of two layers plus the lm_head at M tokens."""
    import torch
    from paper_2509_09090_amd import binding as B
    probs, refs = [], []
    specs = [(l, li) for l in (0, 1) for li in range(7)] + [(0, 7)]
    for (l, li) in specs:
        name, N, K = wl.LM_HEAD if li == 7 else wl.LAYER_LINEARS[li]
        X = wl.layer_input(4, l, li, M)
        W = wl.layer_weight(4, l, li)
        Xq_o, sx_o, _ = oracle.quantize_rows(X)
        Wq_o, sw_o, _ = oracle.quantize_rows(W)
        Xq, sx = G.gpu_quantize(X)
        Wq, sw = G.gpu_quantize(W, weight=True)
        assert np.array_equal(Xq, Xq_o) and np.array_equal(sx.view(np.uint16), sx_o.view(np.uint16))
        assert np.array_equal(Wq, Wq_o) and np.array_equal(sw.view(np.uint16), sw_o.view(np.uint16))
        Wh = B.sqap_weight_pack(G.to_dev(Wq), G.to_dev(sw))
        Y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        probs.append((G.to_dev(Xq), G.to_dev(sx), Wh, Y, acc))
        refs.append((Xq_o, sx_o, Wq_o, sw_o))
    grp = B.sqap_group_create(probs)
    grp.run()
    torch.cuda.synchronize()
    for (xq, sx, Wh, Y, acc), (Xq_o, sx_o, Wq_o, sw_o) in zip(probs, refs):
        Yo, acco = oracle.w4a4_linear(Xq_o, sx_o, Wq_o, sw_o)        # M <= 8: the full product is cheap
        assert np.array_equal(acc.cpu().numpy(), acco)
        assert G.assert_fp16_close(Y.cpu().numpy(), Yo) == 0
    grp.free()
    for pr in probs:
        pr[2].free()


def _random_packed(rng, R, K):
    return rng.integers(0, 256, (R, K // 2), dtype=np.uint8)


def _linear_with_error_word(G, Xq, sx, Wq, sw, pitch_extra=0):
    """pack + linear on canonical operands; returns (Y, acc, workspace error word)."""
    import torch
    from paper_2509_09090_amd import binding as B
    M, N, K = Xq.shape[0], Wq.shape[0], 2 * Wq.shape[1]
    W = B.sqap_weight_pack(G.to_dev(Wq), G.to_dev(sw))
    Y = torch.full((M, N + pitch_extra), float("nan"), dtype=torch.float16, device="cuda")[:, :N]
    acc = torch.full((M, N), -123456789, dtype=torch.int32, device="cuda")
    ws = torch.empty((max(B.sqap_workspace_bytes(M, N, K), 4096),), dtype=torch.uint8, device="cuda")
    ws.random_(0, 256)                                  # garbage, error word included: the launch must clear it
    B.sqap_w4a4_linear(G.to_dev(Xq), G.to_dev(sx), W, Y, acc, ws)
    torch.cuda.synchronize()
    err = B.workspace_error(ws) if B.sqap_workspace_bytes(M, N, K) else 0
    out = Y.cpu().numpy(), acc.cpu().numpy(), err
    W.free()
    return out


# The pruning-ratio sweep (ratios 0.3 .. 0.6 of 256 visual tokens + 20 text tokens: M = 199, 174, 148, 122) through
# the shapes of a layer's linears, separate and with q|k|v / gate|up packed as one weight, and the vocabulary
# head at the two token counts of the 32-layer stack.  M = 199 and 174 take two 96-row tiles: the joint
# split-K finish at N = 4096 and the single-finisher stream-K launch at N = 11008 and above.
@pytest.mark.parametrize("M,N,K", [(M, N, K) for M in (199, 174, 148, 122)
                                   for (N, K) in ((4096, 4096), (11008, 4096), (4096, 11008))] +
                         [(199, 12288, 4096), (122, 22016, 4096), (148, 12288, 4096), (148, 22016, 4096),
                          (84, 12288, 4096), (84, 22016, 4096), (276, 12288, 4096), (276, 22016, 4096),
                          (84, 32000, 4096), (276, 32000, 4096)])
def test_ratio_sweep_and_head_shapes(G, oracle, M, N, K):
    """Both kernels that serve this range: whole outputs per workgroup (the default) and K split between workgroups."""
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    Xq, Wq = _random_packed(rng, M, K), _random_packed(rng, N, K)
    sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    Yo, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
    for which in (1, 0):
        B.sqap_set_mid_m_kernel(which)
        try:
            Y, acc, err = _linear_with_error_word(G, Xq, sx, Wq, sw, pitch_extra=8 if N == 4096 else 0)
        finally:
            B.sqap_set_mid_m_kernel(1)
        if which == 0:                   # the kernel with whole outputs per workgroup never touches the workspace
            assert err == 0
        assert np.array_equal(acc, acco), which
        assert G.assert_fp16_close(Y, Yo) == 0, which


# The kernel with whole outputs per workgroup at the edges of its range: token counts around the 16-row groups
# and the 160-row blocks (one, two and four blocks), channel counts that are no multiple of 16 (guarded stores,
# odd pitches), the shortest K it takes and a K with unequal shares for the four wavefronts.
@pytest.mark.parametrize("M,N,K", [(9, 4096, 4096), (16, 512, 1024), (17, 1000, 2048), (33, 33, 1024), (160, 4096, 4096),
                                   (161, 4096, 4096), (320, 2064, 2048), (321, 4096, 1024), (511, 1536, 2304),
                                   (48, 16, 11008), (100, 12288, 1280), (148, 50, 4096), (640, 256, 1024)])
def test_whole_output_kernel_edge_shapes(G, oracle, M, N, K):
    rng = np.random.default_rng(M * 13 + N * 5 + K)
    Xq, Wq = _random_packed(rng, M, K), _random_packed(rng, N, K)
    sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-4).astype(np.float16)
    Y, acc, err = _linear_with_error_word(G, Xq, sx, Wq, sw, pitch_extra=0 if N % 8 else 24)
    Yo, acco = oracle.w4a4_linear(Xq, sx, Wq, sw)
    if M >= 512:                         # the stream-K kernel: it owns the workspace's error word
        assert err == 0
    assert np.array_equal(acc, acco)
    assert G.assert_fp16_close(Y, Yo) == 0


@pytest.mark.parametrize("M", [1, 8])
def test_config4_decode_headline_launch(G, oracle, M):
    """The launch bench.py times for configuration 4: ONE group launch over the seven 7B-shaped linears of 16
    layers plus the vocabulary head, long enough (17 248 row groups) for the 16-wavefront form of the
    small-M kernel: row groups handed out on demand, outputs parked in LDS slots, K = 4096 (8 ring rounds)
    and K = 11008 (21.5 rounds: a padded last round and a refill across the row-group boundary).  The eight
    packed weights are shared by the layers (memory), every problem has its own input and output; every
    output and accumulator is compared with the oracle's full product.  One problem per layer has an output
    pitch above N."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(4400 + M)
    layers = 16
    shapes = [(N, K) for (_, N, K) in wl.LAYER_LINEARS] + [(wl.LM_HEAD[1], wl.LM_HEAD[2])]
    Wq = [_random_packed(rng, N, K) for (N, K) in shapes]
    sw = [(rng.random(N) * 0.01 + 1e-4).astype(np.float16) for (N, _) in shapes]
    Wh = [B.sqap_weight_pack(G.to_dev(a), G.to_dev(b)) for a, b in zip(Wq, sw)]
    problems, hosts = [], []
    for l in range(layers):
        for i in range(7 if l + 1 < layers else 8):
            N, K = shapes[i]
            Xq = _random_packed(rng, M, K)
            sx = (rng.random(M) * 2 + 0.01).astype(np.float16)
            pitch = N + 8 if i == 3 else N
            Y = torch.full((M, pitch), float("nan"), dtype=torch.float16, device="cuda")[:, :N]
            acc = torch.full((M, N), -1, dtype=torch.int32, device="cuda")
            problems.append((G.to_dev(Xq), G.to_dev(sx), Wh[i], Y, acc))
            hosts.append((Xq, sx, i))
    g = B.sqap_group_create(problems)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_prob, row_groups, per_rg, per_wg, slots = g.info()
    assert n_prob == len(problems) and row_groups == sum(-(-shapes[i][0] // 32) for _, _, i in hosts)
    if cus == 256:
        # the form the benchmark's 225-problem launch takes: skinny_kernel<1, 16> with LDS output slots
        assert (per_rg, per_wg) == (1, 16) and 4 <= slots < 16 and row_groups >= 4 * cus * 16
        assert g.info(256) == g.info()
    g.run()
    torch.cuda.synchronize()
    for (xq_d, sx_d, W, Y, acc), (Xq, sx, i) in zip(problems, hosts):
        Yo, acco = oracle.w4a4_linear(Xq, sx, Wq[i], sw[i])
        assert np.array_equal(acc.cpu().numpy(), acco)
        assert G.assert_fp16_close(Y.cpu().numpy(), Yo) == 0
    g.free()
    for w in Wh:
        w.free()


def test_streamk_is_deterministic(G):
    """Integer partial sums commute: repeated launches give bit-identical outputs."""
    import torch
    from paper_2509_09090_amd import binding as B
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    M, N, K = 2368, 4096, 4096
    Xq = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    Wq = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=g)
    sx = (torch.rand((M,), device="cuda", generator=g) + 0.1).half()
    sw = (torch.rand((N,), device="cuda", generator=g) * 0.01 + 0.001).half()
    W = B.sqap_weight_pack(Wq, sw)
    ws = torch.zeros((B.sqap_workspace_bytes(M, N, K),), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(4):
        Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        B.sqap_w4a4_linear(Xq, sx, W, Y, None, ws)
        torch.cuda.synchronize()
        outs.append(Y)
    for Y in outs[1:]:
        assert torch.equal(Y.view(torch.int16), outs[0].view(torch.int16))
    W.free()
