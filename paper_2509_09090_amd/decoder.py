"""One Llama-shaped decoder layer as a sequence of library calls (argument marshalling only: every
step runs in the HIP kernels).  The paper runs its W4A4 linears inside such a decoder
(Implementation Details; Section 3.3) without restating it; the order of operations here is the
published pre-normalisation layer:

    y1 = RMSNorm(x + pending) -> int4        sqap_rmsnorm_quantize_act   (also writes x + pending)
    q|k|v = W_qkv y1                         sqap_w4a4_linear            (one GEMM, N = 3 * hidden)
    q, k <- rotary(q, k)                     sqap_rope                   (one launch: 2 * heads columns;
                                             sqap_rope_append with a key/value cache: append folded in)
    a = causal attention(q, k, v)            sqap_attention
    o = W_o quant(a)                         sqap_quantize_act + sqap_w4a4_linear
                                             (one token with a cache: rotation, append and attention are one
                                             launch, sqap_decode_attention, which can take this quantizer along)
    y2 = RMSNorm(x + o) -> int4              sqap_rmsnorm_quantize_act   (residual add fused)
    g|u = W_gu y2                            sqap_w4a4_linear            (N = 2 * ffn)
    h = silu(g) * u -> int4                  sqap_swiglu_quantize_act
    d = W_down h                             sqap_w4a4_linear
The last residual add (x + d) is left pending and fused into the next layer's first call.
"""
import torch

from . import binding as B


class LayerWeights:
    """Packed weights and norm gains of one layer (device resident)."""

    def __init__(self, qkv, o, gate_up, down, gamma_attn, gamma_mlp):
        self.qkv, self.o, self.gate_up, self.down = qkv, o, gate_up, down
        self.gamma_attn, self.gamma_mlp = gamma_attn, gamma_mlp

    def free(self):
        for w in (self.qkv, self.o, self.gate_up, self.down):
            w.free()


class LayerBuffers:
    """Scratch tensors for up to max_rows token rows of one layer call (reused by every layer)."""

    def __init__(self, max_rows, hidden, ffn, device="cuda"):
        f16, u8 = torch.float16, torch.uint8
        self.hidden, self.ffn = hidden, ffn
        self.xq = torch.empty((max_rows, hidden // 2), dtype=u8, device=device)
        self.sx = torch.empty((max_rows,), dtype=f16, device=device)
        self.qkv = torch.empty((max_rows, 3 * hidden), dtype=f16, device=device)
        self.attn = torch.empty((max_rows, hidden), dtype=f16, device=device)
        self.o = torch.empty((max_rows, hidden), dtype=f16, device=device)
        self.gu = torch.empty((max_rows, 2 * ffn), dtype=f16, device=device)
        self.hq = torch.empty((max_rows, ffn // 2), dtype=u8, device=device)
        self.sh = torch.empty((max_rows,), dtype=f16, device=device)
        # the workspace a linear needs is not monotonic in M (the tile shape changes with M): take the largest
        nbytes = max(B.sqap_workspace_bytes(m, n, k) for m in range(1, max_rows + 1)
                     for (n, k) in ((3 * hidden, hidden), (hidden, hidden), (2 * ffn, hidden), (hidden, ffn)))
        self.ws = torch.zeros((max(nbytes, 256),), dtype=u8, device=device)
        self.iota = torch.arange(max_rows, dtype=torch.int32, device=device)
        self.counter = torch.zeros((1,), dtype=torch.int32, device=device)     # arrival counter of sqap_decode_attention


def layer_forward(w, buf, x, pending, pos, batch, n_heads, head_dim, x_out, d_out, eps=1e-5, rows=None,
                  rotate=False, kv=None, past=0, stream=None, fold_quantizer=False):
    """Runs one layer on M token rows (batch sequences of M / batch tokens each).

    x: residual stream [*, hidden] fp16 (rows picks the M rows when given: the token gather is fused);
    pending: [M, hidden] update not yet added to x, or None; pos: [M] int32 positions.
    x_out [M, hidden] receives the residual stream after the attention block, d_out [M, hidden] the
    feed-forward output still to be added to it (the next call's `pending`).
    kv: this layer's key/value cache of ONE sequence, [capacity, 2 * hidden] fp16 (rotated key | value per
    position), holding `past` positions: the M new rows are appended and attention runs over past + M
    keys (prefill fills the cache with past = 0; a decode step has M = 1).  Needs batch == 1.
    """
    M = pos.numel()
    hidden = buf.hidden
    flags = B.ROTATE_HADAMARD if rotate else 0
    xq, sx, qkv, attn, o = buf.xq[:M], buf.sx[:M], buf.qkv[:M], buf.attn[:M], buf.o[:M]
    gu, hq, sh = buf.gu[:M], buf.hq[:M], buf.sh[:M]
    B.sqap_rmsnorm_quantize_act(x, rows, w.gamma_attn, eps, xq, sx, delta=pending, flags=flags, xsum_out=x_out,
                                stream=stream)
    B.sqap_w4a4_linear(xq, sx, w.qkv, qkv, None, buf.ws, stream=stream)
    one_launch = kv is not None and M == 1 and head_dim % 8 == 0 and head_dim <= 128 and hidden <= 8192
    if kv is None:
        B.sqap_rope(qkv[:, :2 * hidden], pos, 2 * n_heads, head_dim, stream=stream)  # queries and keys in one launch
        B.sqap_attention(qkv[:, :hidden], qkv[:, hidden:2 * hidden], qkv[:, 2 * hidden:], n_heads, head_dim, attn,
                         batch=batch, stream=stream)
    else:
        if batch != 1:
            raise ValueError("a key/value cache belongs to one sequence")
        if one_launch:
            # a decode step: rotation, cache append and attention in one launch.  The quantizer of the next
            # linear can ride along (fold_quantizer: one launch fewer, which pays when the host's launch rate is
            # the limit) but its device-wide arrival costs more GPU time than the separate launch (4.7 against 2.3 us)
            if fold_quantizer:
                B.sqap_decode_attention(qkv, pos, n_heads, head_dim, kv, past, attn, xq, sx, buf.counter, stream=stream)
            else:
                B.sqap_decode_attention(qkv, pos, n_heads, head_dim, kv, past, attn, stream=stream)
        else:
            # rotation and cache append in one launch: rotated key | value rows land in the cache
            B.sqap_rope_append(qkv, pos, n_heads, head_dim, kv[past:past + M], stream=stream)
            B.sqap_attention(qkv[:, :hidden], kv[:past + M, :hidden], kv[:past + M, hidden:], n_heads, head_dim, attn,
                             stream=stream)
    if not (one_launch and fold_quantizer):
        B.sqap_quantize_act(attn, None, xq, sx, stream=stream)
    B.sqap_w4a4_linear(xq, sx, w.o, o, None, buf.ws, stream=stream)
    B.sqap_rmsnorm_quantize_act(x_out, None, w.gamma_mlp, eps, xq, sx, delta=o, xsum_out=x_out, stream=stream)
    B.sqap_w4a4_linear(xq, sx, w.gate_up, gu, None, buf.ws, stream=stream)
    B.sqap_swiglu_quantize_act(gu[:, :buf.ffn], gu[:, buf.ffn:], hq, sh, stream=stream)
    B.sqap_w4a4_linear(hq, sh, w.down, d_out, None, buf.ws, stream=stream)
