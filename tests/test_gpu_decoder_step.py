"""A decode step as one launch (sqap_decoder_step) against the oracle's layer chain and against the chain of
separate launches.  The caches are prefilled by the chain of launches (itself checked against the oracle in
test_gpu_glue.py); each step's per-layer attention output (attn_trace) is fed to the oracle, so everything
downstream of the attention (o, both norms, gate|up, SwiGLU, down, the head) is compared bit for bit, and
the attention output itself and the appended cache rows within the fp16 tolerance."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from tests import gpu_util
    return gpu_util


def _acts(rng, M, K, outliers=True):
    x = rng.standard_normal((M, K)).astype(np.float32)
    if outliers:
        ch = rng.choice(K, size=max(1, K // 100), replace=False)
        x[:, ch] *= 30.0
    return x.astype(np.float16)


def _model(oracle, G, rng, hidden, H, d, F, L, vocab, capacity):
    """Random layers: oracle-quantized weights (host copies for the oracle, packed handles for the device)."""
    import torch
    from paper_2509_09090_amd import binding as B, decoder
    host, dev = [], []
    for l in range(L):
        ws, packed = {}, {}
        for name, (N, K) in dict(qkv=(3 * hidden, hidden), o=(hidden, hidden), gate_up=(2 * F, hidden), down=(hidden, F)).items():
            W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float16)
            q, s, _ = oracle.quantize_rows(W)
            ws[name] = (q, s)
            packed[name] = B.sqap_weight_pack(G.to_dev(q), G.to_dev(s))
        g1 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
        g2 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
        kv = torch.zeros((capacity, 2 * hidden), dtype=torch.float16, device="cuda")
        host.append((ws, g1, g2))
        dev.append((decoder.LayerWeights(packed["qkv"], packed["o"], packed["gate_up"], packed["down"], G.to_dev(g1),
                                         G.to_dev(g2)), kv))
    Wh = (rng.standard_normal((vocab, hidden)) / np.sqrt(hidden)).astype(np.float16)
    hq, hs, _ = oracle.quantize_rows(Wh)
    gf = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
    head = B.sqap_weight_pack(G.to_dev(hq), G.to_dev(hs))
    return host, dev, (hq, hs), gf, head


def _oracle_step(oracle, host, head_host, gf, x_tok, pos, caches_before, attn_trace, H, d):
    """The oracle's chain for one token, continuing from the device's attention outputs; returns per-layer
    states and the logits."""
    hidden = x_tok.shape[1]
    x, pend, states = x_tok, None, []
    for l, (ws, g1, g2) in enumerate(host):
        before = caches_before[l]
        st = oracle.decoder_layer(x, pend, pos, 1, ws, g1, g2, H, d, attn_override=attn_trace[l:l + 1],
                                  past_k=before[:, :hidden], past_v=before[:, hidden:])
        states.append(st)
        x, pend = st["x2"], st["d"]
    _, y = oracle.rmsnorm_rows(x, gf, 1e-5, delta=pend)
    q, s, _ = oracle.quantize_rows(y)
    logits, _ = oracle.w4a4_linear(q, s, *head_host)
    return states, logits


def _wide_token(rng, K):
    """A token whose elements span thirty binary orders: neighbours differ by more than 2^14 in most groups of
    eight, which is where the norm's sum of squares leaves its binary64 path."""
    x = rng.standard_normal((1, K)) * np.exp2(rng.uniform(-20, 10, (1, K)))
    return np.clip(x, -6e4, 6e4).astype(np.float16)


@pytest.mark.parametrize("hidden,H,d,F,L,vocab,S,wide", [(256, 4, 64, 512, 3, 1000, 21, False),       # most workgroups idle in every phase
                                                         (256, 4, 64, 512, 2, 1000, 9, True),         # tokens of wide dynamic range
                                                         (1024, 8, 128, 2816, 2, 5008, 40, False),   # several groups per workgroup, ragged shares
                                                         (512, 4, 128, 1408, 2, 3008, 300, False),   # a cache longer than one attention chunk
                                                         (4096, 32, 128, 11008, 1, 32000, 148, False)])   # the 7B layer shape and head
def test_decoder_step_matches_the_oracle_and_the_launch_chain(G, oracle, hidden, H, d, F, L, vocab, S, wide):
    import torch
    from paper_2509_09090_amd import binding as B, decoder
    rng = np.random.default_rng(hidden + L)
    steps = 3
    host, dev, head_host, gf, head = _model(oracle, G, rng, hidden, H, d, F, L, vocab, S + steps)
    gf_d = G.to_dev(gf)
    # prefill S tokens into the caches with the chain of launches
    buf = decoder.LayerBuffers(S, hidden, F)
    pos = (np.arange(S) * 2 + 1).astype(np.int32)
    xa = torch.zeros((S, hidden), dtype=torch.float16, device="cuda")
    da = torch.zeros((S, hidden), dtype=torch.float16, device="cuda")
    xb, db = torch.zeros_like(xa), torch.zeros_like(xa)
    src, pend = G.to_dev(_acts(rng, S, hidden)), None
    for l, (w, kv) in enumerate(dev):
        xo, do = (xa, da) if l % 2 == 0 else (xb, db)
        decoder.layer_forward(w, buf, src, pend, G.to_dev(pos), 1, H, d, xo, do, kv=kv, past=0)
        src, pend = xo, do
    torch.cuda.synchronize()

    dec = B.sqap_decoder_create([(w.qkv, w.o, w.gate_up, w.down, w.gamma_attn, w.gamma_mlp, kv) for (w, kv) in dev],
                                H, d, gf_d, head)
    logits = torch.zeros((vocab,), dtype=torch.float16, device="cuda")
    trace = torch.zeros((L, hidden), dtype=torch.float16, device="cuda")
    chain_logits = torch.zeros((1, vocab), dtype=torch.float16, device="cuda")
    past = S
    for step in range(steps):
        x_tok = _wide_token(rng, hidden) if wide else _acts(rng, 1, hidden)
        pt = np.array([int(pos[-1]) + 1 + 2 * step], np.int32)
        x_d, p_d = G.to_dev(x_tok), G.to_dev(pt)
        before = [kv.cpu().numpy()[:past].copy() for (_, kv) in dev]
        # the chain of launches on copies of the caches (same kernels for the attention, so the same bits)
        kv_copy = [kv.clone() for (_, kv) in dev]
        x1a, x1b, d1a, d1b = (torch.zeros((1, hidden), dtype=torch.float16, device="cuda") for _ in range(4))
        src, pend = x_d, None
        for l, (w, _) in enumerate(dev):
            xo, do = (x1a, d1a) if l % 2 == 0 else (x1b, d1b)
            decoder.layer_forward(w, buf, src, pend, p_d, 1, H, d, xo, do, kv=kv_copy[l], past=past)
            src, pend = xo, do
        B.sqap_rmsnorm_quantize_act(src, None, gf_d, 1e-5, buf.xq[:1], buf.sx[:1], delta=pend)
        B.sqap_w4a4_linear(buf.xq[:1], buf.sx[:1], head, chain_logits, None, buf.ws)
        # the step as one launch
        logits.fill_(float("nan"))
        dec.step(x_d[0], p_d, past, logits, trace)
        torch.cuda.synchronize()
        assert dec.status() == 0
        got = logits.cpu().numpy()
        assert np.array_equal(got.view(np.uint16), chain_logits[0].cpu().numpy().view(np.uint16)), step
        for l, (_, kv) in enumerate(dev):
            assert torch.equal(kv[:past + 1].view(torch.int16), kv_copy[l][:past + 1].view(torch.int16)), (step, l)
        # the oracle, continuing from the device's attention outputs
        tr = trace.cpu().numpy()
        states, logits_o = _oracle_step(oracle, host, head_host, gf, x_tok, pt, before, tr, H, d)
        for l, st in enumerate(states):
            after = dev[l][1].cpu().numpy()
            assert np.array_equal(after[:past].view(np.uint16), before[l].view(np.uint16))          # earlier rows untouched
            assert G.assert_fp16_close(after[past:past + 1, :hidden], st["k_rot"]) >= 0
            assert np.array_equal(after[past:past + 1, hidden:].view(np.uint16), st["qkv"][:, 2 * hidden:].view(np.uint16))
            assert G.assert_fp16_close(tr[l:l + 1], st["attn"]) >= 0          # attention over the device's own cache
        assert G.assert_fp16_close(got[None, :], logits_o) == 0
        past += 1
    dec.free()
    head.free()
    for (w, _) in dev:
        w.free()


def test_decoder_step_replayed_from_a_graph(G, oracle):
    """The barrier generation moves on in device memory: replays of a captured step, with eager steps in
    between, all give the eager result (the step is a pure function of the caches' first `past` rows)."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(5)
    hidden, H, d, F, L, vocab, S = 512, 4, 128, 1408, 2, 3008, 30
    host, dev, head_host, gf, head = _model(oracle, G, rng, hidden, H, d, F, L, vocab, S + 1)
    for (_, kv) in dev:
        kv[:S] = G.to_dev((0.5 * rng.standard_normal((S, 2 * hidden))).astype(np.float16))
    gf_d = G.to_dev(gf)
    dec = B.sqap_decoder_create([(w.qkv, w.o, w.gate_up, w.down, w.gamma_attn, w.gamma_mlp, kv) for (w, kv) in dev],
                                H, d, gf_d, head)
    x_d, p_d = G.to_dev(_acts(rng, 1, hidden))[0], G.to_dev(np.array([77], np.int32))
    ref = torch.zeros((vocab,), dtype=torch.float16, device="cuda")
    out = torch.zeros_like(ref)
    dec.step(x_d, p_d, S, ref)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dec.step(x_d, p_d, S, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dec.step(x_d, p_d, S, out)
    for rep in range(4):
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert dec.status() == 0
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), rep
        eager = torch.zeros_like(ref)
        dec.step(x_d, p_d, S, eager)          # an eager step between replays
        torch.cuda.synchronize()
        assert torch.equal(eager.view(torch.int16), ref.view(torch.int16)), rep
    dec.free()
    head.free()
    for (w, _) in dev:
        w.free()


def test_decoder_step_gives_up_instead_of_waiting(G, oracle):
    """With a wait limit of zero a step never waits for another workgroup: it ends, says so in the status word,
    and the decoder is as good as new afterwards (the next step with the default limit gives the reference)."""
    import torch
    from paper_2509_09090_amd import binding as B
    rng = np.random.default_rng(11)
    hidden, H, d, F, L, vocab, S = 512, 4, 128, 1408, 3, 3008, 25
    host, dev, head_host, gf, head = _model(oracle, G, rng, hidden, H, d, F, L, vocab, S + 1)
    for (_, kv) in dev:
        kv[:S] = G.to_dev((0.5 * rng.standard_normal((S, 2 * hidden))).astype(np.float16))
    gf_d = G.to_dev(gf)
    dec = B.sqap_decoder_create([(w.qkv, w.o, w.gate_up, w.down, w.gamma_attn, w.gamma_mlp, kv) for (w, kv) in dev],
                                H, d, gf_d, head)
    x_d, p_d = G.to_dev(_acts(rng, 1, hidden))[0], G.to_dev(np.array([40], np.int32))
    ref = torch.zeros((vocab,), dtype=torch.float16, device="cuda")
    out = torch.zeros_like(ref)
    dec.step(x_d, p_d, S, ref)
    torch.cuda.synchronize()
    assert dec.status() == 0
    dec.set_wait_limit(0)
    dec.step(x_d, p_d, S, out)
    torch.cuda.synchronize()                 # the launch ends although nobody waited for anybody
    assert dec.status() != 0
    dec.set_wait_limit(-1)
    for _ in range(2):
        out.fill_(float("nan"))
        dec.step(x_d, p_d, S, out)
        torch.cuda.synchronize()
        assert dec.status() == 0
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    dec.free()
    head.free()
    for (w, _) in dev:
        w.free()
