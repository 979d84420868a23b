"""GPU parity of the decoder glue (RMSNorm / SwiGLU fused into the quantizer, rotary embedding,
attention, residual add) against the CPU oracle, through the C-ABI."""
import numpy as np
import pytest

from paper_2509_09090_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    from tests import gpu_util
    return gpu_util


def _acts(rng, M, K, outliers=True):
    X = rng.standard_normal((M, K)).astype(np.float32)
    if outliers and K >= 100:
        ch = rng.choice(K, size=max(1, K // 100), replace=False)
        X[:, ch] *= 30.0
    return X.astype(np.float16)


@pytest.mark.parametrize("M,K,rotate,gather,with_delta,channelwise", [
    (5, 64, False, False, False, False), (148, 4096, False, True, True, False), (37, 11008, False, False, True, False),
    (33, 512, True, False, False, False), (148, 4096, True, True, True, False), (20, 2056, False, False, True, True),
    (64, 4096, True, False, False, True), (3, 16384, False, False, True, False)])
def test_rmsnorm_quantize(G, oracle, M, K, rotate, gather, with_delta, channelwise):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(M * 13 + K)
    src_rows = M + 9 if gather else M
    X = _acts(rng, src_rows, K)
    rows = np.sort(rng.choice(src_rows, size=M, replace=False)).astype(np.int32) if gather else None
    delta = _acts(rng, M, K, outliers=False) if with_delta else None
    gamma = (1 + 0.2 * rng.standard_normal(K)).astype(np.float16)
    eps = 1e-5
    xs_o, y_o = oracle.rmsnorm_rows(X, gamma, eps, rows=rows, delta=delta)
    cs = None
    if channelwise:
        cs = oracle.channel_scales(y_o, rotate=rotate)
        q_o, s_o = oracle.quantize_rows_channelwise(y_o, cs, rotate=rotate)
    else:
        q_o, s_o, _ = oracle.quantize_rows(y_o, rotate=rotate)
    dev = lambda a: None if a is None else G.to_dev(a)
    Xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((M,), dtype=torch.float16, device="cuda")
    xs = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    y = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    B.sqap_rmsnorm_quantize_act(dev(X), dev(rows), dev(gamma), eps, Xq, sx, delta=dev(delta),
                                flags=B.ROTATE_HADAMARD if rotate else 0, col_scales=dev(cs), xsum_out=xs, y_out=y)
    torch.cuda.synchronize()
    assert np.array_equal(xs.cpu().numpy().view(np.uint16), xs_o.view(np.uint16))
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y_o.view(np.uint16))
    assert np.array_equal(sx.cpu().numpy().view(np.uint16), np.asarray(s_o).view(np.uint16))
    assert np.array_equal(Xq.cpu().numpy(), q_o)
    # the half-precision result alone (no quantizer), and the quantizer without the optional outputs
    y2 = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    B.sqap_rmsnorm_quantize_act(dev(X), dev(rows), dev(gamma), eps, None, None, delta=dev(delta), y_out=y2)
    Xq2 = torch.zeros_like(Xq)
    B.sqap_rmsnorm_quantize_act(dev(X), dev(rows), dev(gamma), eps, Xq2, sx, delta=dev(delta),
                                flags=B.ROTATE_HADAMARD if rotate else 0, col_scales=dev(cs))
    torch.cuda.synchronize()
    assert torch.equal(y2, y) and torch.equal(Xq2, Xq)


def test_rmsnorm_sum_of_squares_is_exact_on_the_device(G, oracle):
    """Rows whose squares span 80 binary orders and rows of extreme values: the exact sum decides r."""
    import torch
    from paper_2509_09090_amd import binding as B
    K = 4096
    rng = np.random.default_rng(77)
    rows = []
    r = np.full(K, 2.0 ** -24, dtype=np.float16)
    r[7] = np.float16(65504.0)
    rows.append(r)
    rows.append(np.full(K, 2.0 ** -24, dtype=np.float16))
    rows.append(np.full(K, 65504.0, dtype=np.float16))
    rows.append(np.zeros(K, dtype=np.float16))
    for _ in range(12):
        r = (rng.standard_normal(K) * np.exp(rng.uniform(-15, 8, K))).astype(np.float64)
        rows.append(np.clip(r, -60000, 60000).astype(np.float16))
    X = np.stack(rows)
    gamma = np.ones(K, np.float16)
    for eps in (0.0, 1e-6):
        if eps == 0.0:
            Xe = np.delete(X, 3, axis=0)          # a zero row with eps = 0 has no finite norm
        else:
            Xe = X
        _, y_o = oracle.rmsnorm_rows(Xe, gamma, eps)
        y = torch.zeros(Xe.shape, dtype=torch.float16, device="cuda")
        B.sqap_rmsnorm_quantize_act(G.to_dev(Xe), None, G.to_dev(gamma), eps, None, None, y_out=y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().view(np.uint16), y_o.view(np.uint16)), eps


def test_silu_of_every_half_value(G, oracle):
    """silu is a function of one half value: all 63488 finite ones, against the oracle, bit for bit."""
    import torch
    from paper_2509_09090_amd import binding as B
    bits = np.arange(65536, dtype=np.uint16)
    g = bits.view(np.float16)
    g = g[np.isfinite(g)]
    assert len(g) == 63488
    g = g.reshape(62, 1024)
    Gm = np.concatenate([g, g, g])
    Um = np.concatenate([np.ones_like(g), np.full_like(g, 0.333), np.full_like(g, -7.5)])
    h_o = oracle.swiglu(Gm, Um)
    h = torch.zeros(Gm.shape, dtype=torch.float16, device="cuda")
    B.sqap_swiglu_quantize_act(G.to_dev(Gm), G.to_dev(Um), None, None, h_out=h)
    torch.cuda.synchronize()
    got = h.cpu().numpy()
    assert np.array_equal(got.view(np.uint16), h_o.view(np.uint16)), int(np.count_nonzero(got.view(np.uint16) != h_o.view(np.uint16)))


@pytest.mark.parametrize("M,F,channelwise,sliced", [(148, 11008, False, True), (7, 64, False, False), (33, 2056, True, False),
                                                     (8, 11008, False, True)])
def test_swiglu_quantize(G, oracle, M, F, channelwise, sliced):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(M + F)
    GU = (rng.standard_normal((M, 2 * F)) * 2.5).astype(np.float16)     # gate | up as a fused linear writes them
    Gn, Un = GU[:, :F], GU[:, F:]
    h_o = oracle.swiglu(Gn, Un)
    cs = None
    if channelwise:
        cs = oracle.channel_scales(h_o)
        q_o, s_o = oracle.quantize_rows_channelwise(h_o, cs)
    else:
        q_o, s_o, _ = oracle.quantize_rows(h_o)
    gu = G.to_dev(GU)
    if sliced:
        Gd, Ud = gu[:, :F], gu[:, F:]
    else:
        Gd, Ud = G.to_dev(np.ascontiguousarray(Gn)), G.to_dev(np.ascontiguousarray(Un))
    Xq = torch.zeros((M, F // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((M,), dtype=torch.float16, device="cuda")
    h = torch.zeros((M, F), dtype=torch.float16, device="cuda")
    B.sqap_swiglu_quantize_act(Gd, Ud, Xq, sx, col_scales=None if cs is None else G.to_dev(cs), h_out=h)
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy().view(np.uint16), h_o.view(np.uint16))
    assert np.array_equal(sx.cpu().numpy().view(np.uint16), np.asarray(s_o).view(np.uint16))
    assert np.array_equal(Xq.cpu().numpy(), q_o)


@pytest.mark.parametrize("S,H,d", [(276, 32, 128), (5, 3, 16), (148, 4, 64), (700, 6, 64)])
def test_rope(G, oracle, S, H, d):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(S + H + d)
    width = 3 * H * d                                           # rotated where it lies inside a fused q|k|v row
    Y = rng.standard_normal((S, width)).astype(np.float16)
    pos = np.sort(rng.choice(max(400, 2 * S), size=S, replace=False)).astype(np.int32)
    want = Y.copy()
    want[:, :H * d] = oracle.rope(Y[:, :H * d].reshape(S, H, d), pos).reshape(S, H * d)
    want[:, H * d:2 * H * d] = oracle.rope(Y[:, H * d:2 * H * d].reshape(S, H, d), pos).reshape(S, H * d)
    y = G.to_dev(Y)
    p = G.to_dev(pos)
    B.sqap_rope(y[:, :H * d], p, H, d)
    B.sqap_rope(y[:, H * d:2 * H * d], p, H, d)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert np.array_equal(got[:, 2 * H * d:].view(np.uint16), Y[:, 2 * H * d:].view(np.uint16))      # v untouched
    g, w = got.astype(np.float64), want.astype(np.float64)
    assert np.all(np.abs(g - w) <= 1e-2 + 1e-3 * np.abs(w))
    assert np.count_nonzero(got.view(np.uint16) != want.view(np.uint16)) <= got.size // 200          # both are binary64 -> half


def test_rope_append_equals_rotation_plus_row_copy(G, oracle):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(41)
    S, H, d, past = 9, 4, 64, 5
    width = H * d
    QKV = rng.standard_normal((S, 3 * width)).astype(np.float16)
    pos = (np.arange(S) * 3 + 2).astype(np.int32)
    a = G.to_dev(QKV)
    b = G.to_dev(QKV)
    p = G.to_dev(pos)
    cache = torch.full((past + S + 2, 2 * width + 16), 7.0, dtype=torch.float16, device="cuda")    # wider pitch, guard rows
    B.sqap_rope_append(a, p, H, d, cache[past:past + S, :2 * width])
    B.sqap_rope(b[:, :2 * width], p, 2 * H, d)
    torch.cuda.synchronize()
    an, bn, cn = a.cpu().numpy(), b.cpu().numpy(), cache.cpu().numpy()
    assert np.array_equal(an[:, :width].view(np.uint16), bn[:, :width].view(np.uint16))                  # q rotated in place
    assert np.array_equal(an[:, width:].view(np.uint16), QKV[:, width:].view(np.uint16))                 # k, v columns untouched
    assert np.array_equal(cn[past:past + S, :width].view(np.uint16), bn[:, width:2 * width].view(np.uint16))
    assert np.array_equal(cn[past:past + S, width:2 * width].view(np.uint16), QKV[:, 2 * width:].view(np.uint16))
    assert np.all(cn[:past] == 7.0) and np.all(cn[past + S:] == 7.0) and np.all(cn[:, 2 * width:] == 7.0)
    want_q = oracle.rope(QKV[:, :width].reshape(S, H, d), pos).reshape(S, width)
    assert G.assert_fp16_close(an[:, :width], want_q) >= 0


@pytest.mark.parametrize("Sq,Sk,H,d", [(276, 276, 32, 128), (148, 148, 8, 128), (1, 149, 32, 128), (8, 156, 4, 64),
                                       (70, 70, 3, 16), (33, 97, 2, 32), (1, 1, 1, 16)])
def test_attention(G, oracle, Sq, Sk, H, d):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(Sq * 3 + Sk + H + d)
    width = H * d
    QKV = rng.standard_normal((Sk, 3 * width)).astype(np.float16)
    QKV[:, :width] *= 2.0                                      # sharper softmax rows
    Qn = QKV[Sk - Sq:, :width].reshape(Sq, H, d)
    Kn = QKV[:, width:2 * width].reshape(Sk, H, d)
    Vn = QKV[:, 2 * width:].reshape(Sk, H, d)
    want = oracle.attention(Qn, Kn, Vn).reshape(Sq, width)
    qkv = G.to_dev(QKV)
    O = torch.full((Sq, width), float("nan"), dtype=torch.float16, device="cuda")
    B.sqap_attention(qkv[Sk - Sq:, :width], qkv[:, width:2 * width], qkv[:, 2 * width:], H, d, O)
    torch.cuda.synchronize()
    assert G.assert_fp16_close(O.cpu().numpy(), want) >= 0


def test_attention_batch(G, oracle):
    """Sequences stacked as row blocks: each gets what a single call gives."""
    import torch
    from paper_2509_09090_amd import binding as B
    nb, S, H, d = 5, 41, 3, 64
    rng = np.random.default_rng(12)
    width = H * d
    QKV = rng.standard_normal((nb * S, 3 * width)).astype(np.float16)
    qkv = G.to_dev(QKV)
    O = torch.full((nb * S, width), float("nan"), dtype=torch.float16, device="cuda")
    B.sqap_attention(qkv[:, :width], qkv[:, width:2 * width], qkv[:, 2 * width:], H, d, O, batch=nb)
    torch.cuda.synchronize()
    got = O.cpu().numpy()
    for b in range(nb):
        blk = QKV[b * S:(b + 1) * S]
        want = oracle.attention(blk[:, :width].reshape(S, H, d), blk[:, width:2 * width].reshape(S, H, d),
                                blk[:, 2 * width:].reshape(S, H, d)).reshape(S, width)
        assert G.assert_fp16_close(got[b * S:(b + 1) * S], want) >= 0


@pytest.mark.parametrize("H,d,past,quantize", [(32, 128, 148, True), (4, 64, 0, True), (3, 16, 5, True),
                                                (8, 128, 1100, True), (2, 96, 70, False), (32, 128, 63, False)])
def test_decode_attention_in_one_launch(G, oracle, H, d, past, quantize):
    """Rotation + cache append + attention (+ activation quantizer) of one new token in one launch:
    the cache row against the oracle's rotation, the output against the oracle's attention over the
    oracle's own rotated rows, the codes against the oracle's quantizer of the oracle's output within
    one quantization step (the outputs differ within the fp16 tolerance, so codes may flip at
    rounding boundaries) and, bit for bit, against the library's own quantizer on the same output."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(H * 1000 + d + past)
    width = H * d
    QKV = rng.standard_normal((1, 3 * width)).astype(np.float16)
    QKV[:, :width] *= 2.0
    prefix = rng.standard_normal((past, 2 * width)).astype(np.float16)          # rotated keys | values already cached
    pos = np.array([past + 3], dtype=np.int32)
    q_rot = oracle.rope(QKV[:, :width].reshape(1, H, d), pos)
    k_rot = oracle.rope(QKV[:, width:2 * width].reshape(1, H, d), pos)
    Kn = np.concatenate([prefix[:, :width].reshape(past, H, d), k_rot], axis=0)
    Vn = np.concatenate([prefix[:, width:].reshape(past, H, d), QKV[:, 2 * width:].reshape(1, H, d)], axis=0)
    want = oracle.attention(q_rot, Kn, Vn).reshape(1, width)

    pitch = 2 * width + 16
    cache = torch.full((past + 3, pitch), 7.0, dtype=torch.float16, device="cuda")
    cache[:past, :2 * width] = G.to_dev(prefix)
    qkv, p = G.to_dev(QKV), G.to_dev(pos)
    O = torch.full((1, width), float("nan"), dtype=torch.float16, device="cuda")
    Xq = torch.full((1, width // 2), 0x5a, dtype=torch.uint8, device="cuda") if quantize else None
    sx = torch.full((1,), float("nan"), dtype=torch.float16, device="cuda") if quantize else None
    counter = torch.zeros((1,), dtype=torch.int32, device="cuda") if quantize else None
    for _ in range(2):                                                         # the second call finds the counter at zero again
        B.sqap_decode_attention(qkv, p, H, d, cache[:, :2 * width], past, O, Xq, sx, counter)
    torch.cuda.synchronize()
    cn, got = cache.cpu().numpy(), O.cpu().numpy()
    assert np.array_equal(qkv.cpu().numpy().view(np.uint16), QKV.view(np.uint16))                      # only read
    assert np.array_equal(cn[:past, :2 * width].view(np.uint16), prefix.view(np.uint16))               # earlier rows untouched
    assert np.all(cn[past + 1:] == 7.0) and np.all(cn[:, 2 * width:] == 7.0)
    assert G.assert_fp16_close(cn[past:past + 1, :width], k_rot.reshape(1, width)) <= width // 100
    assert np.array_equal(cn[past:past + 1, width:2 * width].view(np.uint16), QKV[:, 2 * width:].view(np.uint16))
    assert G.assert_fp16_close(got, want) >= 0
    # the separate calls give the same cache row (bits) and an output within the tolerance
    qkv2 = G.to_dev(QKV)
    cache2 = cache.clone()
    cache2[past] = 7.0
    O2 = torch.empty_like(O)
    B.sqap_rope_append(qkv2, p, H, d, cache2[past:past + 1, :2 * width])
    if d in (16, 32, 64, 128):
        B.sqap_attention(qkv2[:, :width], cache2[:past + 1, :width], cache2[:past + 1, width:2 * width], H, d, O2)
        torch.cuda.synchronize()
        assert G.assert_fp16_close(got, O2.cpu().numpy()) >= 0
    torch.cuda.synchronize()
    assert np.array_equal(cache2.cpu().numpy().view(np.uint16), cn.view(np.uint16))
    if quantize:
        assert int(counter.item()) == 0
        q_o, s_o, _ = oracle.quantize_rows(want)
        step = float(np.asarray(s_o, dtype=np.float64)[0])
        s_g = float(sx.cpu().numpy().astype(np.float64)[0])
        assert abs(s_g - step) <= 2e-3 * step + 1e-6                          # scale = half(max / 7) of outputs 1e-3 apart
        deq_g = oracle.unpack_int4(Xq.cpu().numpy()).astype(np.float64) * s_g
        deq_o = oracle.unpack_int4(q_o).astype(np.float64) * step
        assert np.all(np.abs(deq_g - deq_o) <= 1.02 * step + 1e-6)
        q2 = torch.empty_like(Xq)
        s2 = torch.empty_like(sx)
        B.sqap_quantize_act(O, None, q2, s2)
        torch.cuda.synchronize()
        assert torch.equal(q2, Xq) and torch.equal(s2.view(torch.int16), sx.view(torch.int16))


def test_decode_attention_replayed_from_a_graph(G, oracle):
    """The folded quantizer's arrival counter is put back to zero by the last workgroup, so a captured
    launch replays: new inputs per replay, an eager call on the same counter in between, each result
    against the oracle and the counter at zero afterwards."""
    import torch
    from paper_2509_09090_amd import binding as B
    H, d, past = 8, 64, 37
    width = H * d
    rng = np.random.default_rng(977)
    prefix = rng.standard_normal((past, 2 * width)).astype(np.float16)
    cache = torch.zeros((past + 1, 2 * width), dtype=torch.float16, device="cuda")
    cache[:past] = G.to_dev(prefix)
    qkv = torch.zeros((1, 3 * width), dtype=torch.float16, device="cuda")
    pos = G.to_dev(np.array([past], dtype=np.int32))
    O = torch.zeros((1, width), dtype=torch.float16, device="cuda")
    Xq = torch.zeros((1, width // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((1,), dtype=torch.float16, device="cuda")
    counter = torch.zeros((1,), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.sqap_decode_attention(qkv, pos, H, d, cache, past, O, Xq, sx, counter)       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.sqap_decode_attention(qkv, pos, H, d, cache, past, O, Xq, sx, counter)
    for rep in range(4):
        QKV = rng.standard_normal((1, 3 * width)).astype(np.float16)
        qkv.copy_(G.to_dev(QKV))
        O.fill_(float("nan"))
        Xq.fill_(0x5a)
        graph.replay()
        torch.cuda.synchronize()
        p = np.array([past], dtype=np.int32)
        q_rot = oracle.rope(QKV[:, :width].reshape(1, H, d), p)
        k_rot = oracle.rope(QKV[:, width:2 * width].reshape(1, H, d), p)
        Kn = np.concatenate([prefix[:, :width].reshape(past, H, d), k_rot], axis=0)
        Vn = np.concatenate([prefix[:, width:].reshape(past, H, d), QKV[:, 2 * width:].reshape(1, H, d)], axis=0)
        assert G.assert_fp16_close(O.cpu().numpy(), oracle.attention(q_rot, Kn, Vn).reshape(1, width)) >= 0, rep
        assert int(counter.item()) == 0, rep
        q2, s2 = torch.empty_like(Xq), torch.empty_like(sx)
        B.sqap_quantize_act(O, None, q2, s2)
        torch.cuda.synchronize()
        assert torch.equal(q2, Xq) and torch.equal(s2.view(torch.int16), sx.view(torch.int16)), rep
        O3, q3, s3 = torch.empty_like(O), torch.empty_like(Xq), torch.empty_like(sx)
        B.sqap_decode_attention(qkv, pos, H, d, cache, past, O3, q3, s3, counter)      # eager, same counter
        torch.cuda.synchronize()
        assert torch.equal(O3.view(torch.int16), O.view(torch.int16)) and torch.equal(q3, Xq), rep


def test_residual_add(G, oracle):
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(4)
    X = _acts(rng, 37, 4096)
    D = _acts(rng, 37, 4096, outliers=False)
    x = G.to_dev(X)
    B.sqap_residual_add(x, G.to_dev(D))
    torch.cuda.synchronize()
    assert np.array_equal(x.cpu().numpy().view(np.uint16), oracle.residual_add(X, D).view(np.uint16))


def _layer_case(oracle, G, seed, hidden, H, d, F, batch, S, rotate):
    import torch
    from paper_2509_09090_amd import binding as B
    from paper_2509_09090_amd import decoder
    rng = np.random.default_rng(seed)
    M = batch * S
    x = _acts(rng, M, hidden)
    pend = (0.5 * rng.standard_normal((M, hidden))).astype(np.float16)
    pos = np.tile(np.arange(S) * 2 + 1, batch).astype(np.int32)        # pruned sequences keep their old positions
    ws, packed = {}, {}
    for name, (N, K) in dict(qkv=(3 * hidden, hidden), o=(hidden, hidden), gate_up=(2 * F, hidden), down=(hidden, F)).items():
        W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float16)
        q, s, _ = oracle.quantize_rows(W, rotate=rotate and name == "qkv")
        ws[name] = (q, s)
        packed[name] = B.sqap_weight_pack(G.to_dev(q), G.to_dev(s))
    g1 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
    g2 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
    w = decoder.LayerWeights(packed["qkv"], packed["o"], packed["gate_up"], packed["down"], G.to_dev(g1), G.to_dev(g2))
    return x, pend, pos, ws, w, g1, g2, M


@pytest.mark.parametrize("hidden,H,d,F,batch,S,rotate", [(256, 4, 64, 512, 2, 19, False), (512, 4, 128, 1024, 1, 70, True)])
def test_decoder_layer(G, oracle, hidden, H, d, F, batch, S, rotate):
    """One layer through decoder.layer_forward against the oracle's chain.  Everything up to the
    rotary embedding is exact; attention is compared within the fp16 tolerance; the rest of the
    layer is then continued on both sides from the DEVICE's attention output and is exact again."""
    import torch
    from paper_2509_09090_amd import binding as B
    from paper_2509_09090_amd import decoder
    x, pend, pos, ws, w, g1, g2, M = _layer_case(oracle, G, 21 + hidden, hidden, H, d, F, batch, S, rotate)
    buf = decoder.LayerBuffers(M, hidden, F)
    x_out = torch.zeros((M, hidden), dtype=torch.float16, device="cuda")
    d_out = torch.zeros((M, hidden), dtype=torch.float16, device="cuda")
    decoder.layer_forward(w, buf, G.to_dev(x), G.to_dev(pend), G.to_dev(pos), batch, H, d, x_out, d_out, rotate=rotate)
    torch.cuda.synchronize()
    attn_dev = buf.attn[:M].cpu().numpy()
    qkv_dev = buf.qkv[:M].cpu().numpy()
    st = oracle.decoder_layer(x, pend, pos, batch, ws, g1, g2, H, d, rotate=rotate, attn_override=attn_dev)
    # value part of the fused q|k|v output is untouched by the rotation: exact
    assert np.array_equal(qkv_dev[:, 2 * hidden:].view(np.uint16), st["qkv"][:, 2 * hidden:].view(np.uint16))
    assert G.assert_fp16_close(qkv_dev[:, :hidden], st["q_rot"]) >= 0
    assert G.assert_fp16_close(qkv_dev[:, hidden:2 * hidden], st["k_rot"]) >= 0
    # the device's attention is within tolerance of the oracle's on the oracle's own q, k, v ...
    assert G.assert_fp16_close(attn_dev, st["attn"]) >= 0
    # ... and from the device's attention output on, both sides agree bit for bit
    assert np.array_equal(x_out.cpu().numpy().view(np.uint16), st["x2"].view(np.uint16))
    assert np.array_equal(buf.hq[:M].cpu().numpy(), st["hq"])
    assert np.array_equal(buf.sh[:M].cpu().numpy().view(np.uint16), np.asarray(st["sh"]).view(np.uint16))
    assert G.assert_fp16_close(d_out.cpu().numpy(), st["d"]) == 0
    w.free()


def test_glue_at_full_size_on_sampled_rows(G, oracle):
    """Configuration 3's sizes (16 observations x 148 tokens = 2368 rows): the fused quantizers on sampled
    rows bit for bit, attention on sampled (observation, head) pairs within the fp16 tolerance."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(2368)
    M, K, F, nb, S, H, d = 2368, wl.HIDDEN, wl.FFN, 16, 148, wl.N_HEADS, wl.HEAD_DIM
    sample = np.sort(rng.choice(M, size=24, replace=False))
    # RMSNorm + residual + quantize, K = 4096
    X = _acts(rng, M, K)
    D = _acts(rng, M, K, outliers=False)
    gamma = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    Xq = torch.zeros((M, K // 2), dtype=torch.uint8, device="cuda")
    sx = torch.zeros((M,), dtype=torch.float16, device="cuda")
    xs = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    B.sqap_rmsnorm_quantize_act(G.to_dev(X), None, G.to_dev(gamma), 1e-5, Xq, sx, delta=G.to_dev(D), xsum_out=xs)
    torch.cuda.synchronize()
    xs_o, y_o = oracle.rmsnorm_rows(X[sample], gamma, 1e-5, delta=D[sample])
    q_o, s_o, _ = oracle.quantize_rows(y_o)
    assert np.array_equal(xs.cpu().numpy()[sample].view(np.uint16), xs_o.view(np.uint16))
    assert np.array_equal(Xq.cpu().numpy()[sample], q_o)
    assert np.array_equal(sx.cpu().numpy()[sample].view(np.uint16), np.asarray(s_o).view(np.uint16))
    # SwiGLU + quantize, F = 11008, gate | up as one fused output
    GU = (rng.standard_normal((M, 2 * F)) * 2).astype(np.float16)
    gu = G.to_dev(GU)
    Hq = torch.zeros((M, F // 2), dtype=torch.uint8, device="cuda")
    sh = torch.zeros((M,), dtype=torch.float16, device="cuda")
    B.sqap_swiglu_quantize_act(gu[:, :F], gu[:, F:], Hq, sh)
    torch.cuda.synchronize()
    h_o = oracle.swiglu(GU[sample, :F], GU[sample, F:])
    q_o, s_o, _ = oracle.quantize_rows(h_o)
    assert np.array_equal(Hq.cpu().numpy()[sample], q_o)
    assert np.array_equal(sh.cpu().numpy()[sample].view(np.uint16), np.asarray(s_o).view(np.uint16))
    # attention over 16 sequences of 148 tokens, 32 heads of 128
    QKV = rng.standard_normal((nb * S, 3 * H * d)).astype(np.float16)
    qkv = G.to_dev(QKV)
    O = torch.full((nb * S, H * d), float("nan"), dtype=torch.float16, device="cuda")
    B.sqap_attention(qkv[:, :H * d], qkv[:, H * d:2 * H * d], qkv[:, 2 * H * d:], H, d, O, batch=nb)
    torch.cuda.synchronize()
    got = O.cpu().numpy()
    assert not np.isnan(got).any()
    for (b, h) in ((0, 0), (7, 13), (15, 31)):
        blk = QKV[b * S:(b + 1) * S]
        cut = lambda part: np.ascontiguousarray(blk[:, part * H * d + h * d: part * H * d + (h + 1) * d]).reshape(S, 1, d)
        want = oracle.attention(cut(0), cut(1), cut(2)).reshape(S, d)
        assert G.assert_fp16_close(got[b * S:(b + 1) * S, h * d:(h + 1) * d], want) >= 0


def test_decoder_layer_with_a_key_value_cache(G, oracle):
    """Prefill 21 tokens into the cache, then three single-token steps: the cache rows are what the prefill and
    the steps wrote, attention runs over all of them, and everything downstream of it is exact."""
    import torch
    from paper_2509_09090_amd import decoder
    hidden, H, d, F, S, steps = 256, 4, 64, 512, 21, 3
    x, pend, pos, ws, w, g1, g2, M = _layer_case(oracle, G, 77, hidden, H, d, F, 1, S, False)
    rng = np.random.default_rng(78)
    buf = decoder.LayerBuffers(S, hidden, F)
    kv = torch.zeros((S + steps, 2 * hidden), dtype=torch.float16, device="cuda")
    x_out = torch.zeros((S, hidden), dtype=torch.float16, device="cuda")
    d_out = torch.zeros((S, hidden), dtype=torch.float16, device="cuda")
    decoder.layer_forward(w, buf, G.to_dev(x), G.to_dev(pend), G.to_dev(pos), 1, H, d, x_out, d_out, kv=kv, past=0)
    torch.cuda.synchronize()
    st = oracle.decoder_layer(x, pend, pos, 1, ws, g1, g2, H, d, attn_override=buf.attn[:S].cpu().numpy())
    cache = kv.cpu().numpy()
    assert G.assert_fp16_close(cache[:S, :hidden], st["k_rot"]) >= 0
    assert np.array_equal(cache[:S, hidden:].view(np.uint16), st["qkv"][:, 2 * hidden:].view(np.uint16))
    assert G.assert_fp16_close(buf.attn[:S].cpu().numpy(), st["attn"]) >= 0
    assert G.assert_fp16_close(d_out.cpu().numpy(), st["d"]) == 0
    past = S
    for step in range(steps):
        xt = _acts(rng, 1, hidden)
        pt = np.array([int(pos[-1]) + 1 + step], np.int32)
        x1 = torch.zeros((1, hidden), dtype=torch.float16, device="cuda")
        d1 = torch.zeros((1, hidden), dtype=torch.float16, device="cuda")
        before = kv.cpu().numpy()[:past]
        decoder.layer_forward(w, buf, G.to_dev(xt), None, G.to_dev(pt), 1, H, d, x1, d1, kv=kv, past=past,
                              fold_quantizer=step % 2 == 1)        # the quantizer as its own launch, then folded in
        torch.cuda.synchronize()
        after = kv.cpu().numpy()
        assert np.array_equal(after[:past].view(np.uint16), before.view(np.uint16))          # earlier rows untouched
        st = oracle.decoder_layer(xt, None, pt, 1, ws, g1, g2, H, d, attn_override=buf.attn[:1].cpu().numpy(),
                                  past_k=before[:, :hidden], past_v=before[:, hidden:])
        assert G.assert_fp16_close(after[past:past + 1, :hidden], st["k_rot"]) >= 0
        assert np.array_equal(after[past:past + 1, hidden:].view(np.uint16), st["qkv"][:, 2 * hidden:].view(np.uint16))
        assert G.assert_fp16_close(buf.attn[:1].cpu().numpy(), st["attn"]) >= 0               # over the device's own cache
        assert np.array_equal(x1.cpu().numpy().view(np.uint16), st["x2"].view(np.uint16))
        assert G.assert_fp16_close(d1.cpu().numpy(), st["d"]) == 0
        past += 1
    w.free()
