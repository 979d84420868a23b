"""ctypes binding of libsqap.so: argument marshalling only.

Every function has the name of the C entry point it wraps (see include/sqap.h)
and takes torch CUDA tensors, which are used purely as device memory; work is
enqueued on torch's current stream unless `stream` is given.  Nothing here
computes: there is no fallback when the library is missing (loading raises).
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SQAP_LIBRARY") or os.path.join(_HERE, "libsqap.so")      # (another build of the library: for A/B runs)

OK, EINVAL, EUNSUPPORTED, EDEVICE, ENOMEM = 0, -1, -2, -3, -4
ROTATE_HADAMARD = 1

EXPORTS = (
    "sqap_last_error", "sqap_version", "sqap_attn_scores", "sqap_attn_scores_batch", "sqap_prune_topk", "sqap_kept_rows",
    "sqap_gather_rows", "sqap_quantize_act", "sqap_quantize_weight", "sqap_weight_pack",
    "sqap_weight_free", "sqap_weight_info", "sqap_workspace_bytes", "sqap_w4a4_linear",
    "sqap_group_create", "sqap_group_run", "sqap_group_free", "sqap_selftest_quotient", "sqap_selftest_dispatch",
    "sqap_prune_rows", "sqap_prune_select", "sqap_channel_scales", "sqap_quantize_act_channelwise",
    "sqap_quantize_weight_folded", "sqap_rmsnorm_quantize_act", "sqap_swiglu_quantize_act", "sqap_rope",
    "sqap_attention", "sqap_residual_add", "sqap_rope_append", "sqap_plan_linear_shares", "sqap_decode_attention", "sqap_group_info", "sqap_init",
    "sqap_set_persistent_kernels", "sqap_attn_scores_workspace_bytes", "sqap_attn_scores_noalloc", "sqap_set_mid_m_kernel", "sqap_decoder_create", "sqap_decoder_step", "sqap_decoder_status",
    "sqap_decoder_set_wait_limit", "sqap_decoder_free",
)


class LinearDesc(ctypes.Structure):
    """Mirror of sqap_linear_desc."""
    _fields_ = [("Xq", ctypes.c_void_p), ("sx", ctypes.c_void_p), ("M", ctypes.c_int32),
                ("W", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("ldy", ctypes.c_int64),
                ("acc_out", ctypes.c_void_p)]


class DecoderLayer(ctypes.Structure):
    """Mirror of sqap_decoder_layer."""
    _fields_ = [("qkv", ctypes.c_void_p), ("o", ctypes.c_void_p), ("gate_up", ctypes.c_void_p), ("down", ctypes.c_void_p),
                ("gamma_attn", ctypes.c_void_p), ("gamma_mlp", ctypes.c_void_p), ("kv", ctypes.c_void_p),
                ("ldkv", ctypes.c_int64)]


class SqapError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("sqap status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libsqap.so is not built: run `python -m paper_2509_09090_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u32, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                                 ctypes.c_size_t)
        L.sqap_last_error.restype = ctypes.c_char_p
        L.sqap_last_error.argtypes = []
        L.sqap_version.restype = ctypes.c_char_p
        L.sqap_version.argtypes = []
        L.sqap_attn_scores.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.sqap_attn_scores_batch.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.sqap_attn_scores_noalloc.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp]
        L.sqap_attn_scores_workspace_bytes.restype = sz
        L.sqap_attn_scores_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.sqap_prune_topk.argtypes = [vp, i32, i32, i32, vp, vp]
        L.sqap_kept_rows.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
        L.sqap_prune_rows.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.sqap_gather_rows.argtypes = [vp, i64, vp, i32, i32, vp, i64, vp]
        L.sqap_prune_select.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, vp]
        L.sqap_channel_scales.argtypes = [vp, i64, vp, i32, i32, u32, vp, i32, vp, vp]
        L.sqap_quantize_act_channelwise.argtypes = [vp, i64, vp, i32, i32, u32, vp, vp, vp, vp]
        L.sqap_quantize_weight_folded.argtypes = [vp, i32, i32, u32, vp, vp, vp, vp]
        L.sqap_quantize_act.argtypes = [vp, i64, vp, i32, i32, u32, vp, vp, vp]
        L.sqap_rmsnorm_quantize_act.argtypes = [vp, i64, vp, i32, i32, vp, vp, ctypes.c_float, u32, vp, vp, vp, vp, vp, vp]
        L.sqap_swiglu_quantize_act.argtypes = [vp, i64, vp, i64, i32, i32, vp, vp, vp, vp, vp]
        L.sqap_rope.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.c_double, vp]
        L.sqap_rope_append.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.c_double, vp, i64, vp]
        L.sqap_attention.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, vp, i64, vp]
        L.sqap_decode_attention.argtypes = [vp, vp, i32, i32, ctypes.c_double, vp, i64, i32, vp, vp, vp, vp, vp]
        L.sqap_residual_add.argtypes = [vp, i64, vp, i64, i32, i32, vp]
        L.sqap_quantize_weight.argtypes = [vp, i32, i32, u32, vp, vp, vp]
        L.sqap_weight_pack.argtypes = [vp, vp, i32, i32, ctypes.POINTER(vp), vp]
        L.sqap_weight_free.argtypes = [vp]
        L.sqap_weight_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(sz)]
        L.sqap_workspace_bytes.restype = sz
        L.sqap_workspace_bytes.argtypes = [i32, i32, i32]
        L.sqap_w4a4_linear.argtypes = [vp, vp, i32, vp, vp, i64, vp, vp, sz, vp]
        L.sqap_group_create.argtypes = [ctypes.POINTER(LinearDesc), i32, ctypes.POINTER(vp)]
        L.sqap_group_run.argtypes = [vp, vp]
        L.sqap_group_free.argtypes = [vp]
        L.sqap_decoder_create.argtypes = [ctypes.POINTER(DecoderLayer), i32, i32, i32, vp, vp, ctypes.c_float,
                                          ctypes.c_double, ctypes.POINTER(vp)]
        L.sqap_decoder_step.argtypes = [vp, vp, vp, i32, vp, vp, vp]
        L.sqap_decoder_status.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), vp]
        L.sqap_decoder_free.argtypes = [vp]
        L.sqap_decoder_set_wait_limit.argtypes = [vp, i64]
        L.sqap_group_info.argtypes = [vp, i32] + [ctypes.POINTER(i32)] * 5
        L.sqap_selftest_quotient.argtypes = [vp, vp]
        L.sqap_init.argtypes = [vp]
        L.sqap_set_persistent_kernels.argtypes = [i32]
        L.sqap_set_mid_m_kernel.argtypes = [i32]
        L.sqap_selftest_dispatch.argtypes = [ctypes.POINTER(u32), vp]
        L.sqap_plan_linear_shares.argtypes = [ctypes.c_int32] * 4 + [ctypes.POINTER(u32), ctypes.POINTER(ctypes.c_double),
                                                                      ctypes.POINTER(ctypes.c_double),
                                                                      ctypes.POINTER(ctypes.c_int32),
                                                                      ctypes.POINTER(ctypes.c_int32)]
        for name in EXPORTS:
            if name not in ("sqap_last_error", "sqap_version", "sqap_workspace_bytes", "sqap_attn_scores_workspace_bytes"):
                getattr(L, name).restype = ctypes.c_int32
        _lib = L
    return _lib


def _check(status):
    if status != OK:
        raise SqapError(status, lib().sqap_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def sqap_init(stream=None):
    """One-time set-up of the current device (synchronises the stream once)."""
    _check(lib().sqap_init(_stream(stream)))


def sqap_set_persistent_kernels(enabled):
    _check(lib().sqap_set_persistent_kernels(1 if enabled else 0))


def sqap_set_mid_m_kernel(which):
    _check(lib().sqap_set_mid_m_kernel(int(which)))


def workspace_error(workspace):
    """Error word a persistent sqap_w4a4_linear launch leaves in its workspace (0: every wait ended).
    Synchronises: reads 8 bytes back from the device."""
    if workspace is None or workspace.numel() * workspace.element_size() < 4008:
        return 0
    return int(workspace.view(torch.uint8)[4000:4008].view(torch.int64).item())


def sqap_version():
    return lib().sqap_version().decode()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def sqap_attn_scores_workspace_bytes(batch, S, H, d, n_vis):
    return int(lib().sqap_attn_scores_workspace_bytes(batch, S, H, d, n_vis))


def sqap_attn_scores(q, k, vis_begin, n_vis, scores_out, workspace=None, stream=None):
    """q [H,d] fp16, k [S,H,d] fp16 -> scores_out [n_vis] fp32.  workspace: device bytes, first 256 zeroed once."""
    S, H, d = k.shape
    _check(lib().sqap_attn_scores(_ptr(q), _ptr(k), S, H, d, vis_begin, n_vis, _ptr(scores_out),
                                  _ptr(workspace), _nbytes(workspace), _stream(stream)))


def sqap_attn_scores_batch(q, k, vis_begin, n_vis, scores_out, workspace=None, stream=None):
    """q [batch,H,d] fp16, k [batch,S,H,d] fp16 -> scores_out [batch,n_vis] fp32."""
    batch, S, H, d = k.shape
    _check(lib().sqap_attn_scores_batch(_ptr(q), _ptr(k), batch, S, H, d, vis_begin, n_vis, _ptr(scores_out),
                                        _ptr(workspace), _nbytes(workspace), _stream(stream)))


def sqap_attn_scores_noalloc(q, k, vis_begin, n_vis, scores_out, stream=None):
    """sqap_attn_scores_batch on the library's built-in scratch array (no workspace, no allocation)."""
    batch, S, H, d = k.shape
    _check(lib().sqap_attn_scores_noalloc(_ptr(q), _ptr(k), batch, S, H, d, vis_begin, n_vis, _ptr(scores_out),
                                          _stream(stream)))


def sqap_prune_topk(scores, keep_k, idx_out, stream=None):
    """scores [batch, n] fp32 -> idx_out [batch, keep_k] int32 (ascending)."""
    batch, n = scores.shape
    _check(lib().sqap_prune_topk(_ptr(scores), batch, n, keep_k, _ptr(idx_out), _stream(stream)))


def sqap_kept_rows(idx, seq_len, vis_begin, n_vis, rows_out, stream=None):
    """idx [batch, keep_k] int32 -> rows_out [batch * (seq_len - n_vis + keep_k)] int32."""
    batch, keep_k = idx.shape
    _check(lib().sqap_kept_rows(_ptr(idx), batch, keep_k, seq_len, vis_begin, n_vis, _ptr(rows_out),
                                _stream(stream)))


def sqap_prune_rows(scores, keep_k, seq_len, vis_begin, idx_out, rows_out, stream=None):
    """Fused sqap_prune_topk + sqap_kept_rows."""
    batch, n = scores.shape
    _check(lib().sqap_prune_rows(_ptr(scores), batch, n, keep_k, seq_len, vis_begin, _ptr(idx_out),
                                 _ptr(rows_out), _stream(stream)))


def sqap_prune_select(scores, grid_w, grid_h, k_attn, keep_total, camera, ring_radius, idx_out, count_out=None,
                      stream=None):
    """K_attn + K_ring + K_fps: scores [batch, grid_w*grid_h] fp32, camera [batch, 26] fp64 or None,
    idx_out [batch, cap] int32 (ascending members, then -1), count_out [batch] int32 or None."""
    batch = scores.shape[0]
    _check(lib().sqap_prune_select(_ptr(scores), batch, grid_w, grid_h, k_attn, keep_total, _ptr(camera),
                                   ring_radius, _ptr(idx_out), idx_out.shape[1], _ptr(count_out), _stream(stream)))


def sqap_gather_rows(X, rows, out, stream=None):
    M, K = rows.numel(), X.shape[1]
    _check(lib().sqap_gather_rows(_ptr(X), X.stride(0), _ptr(rows), M, K, _ptr(out), out.stride(0),
                                  _stream(stream)))


def sqap_quantize_act(X, rows, Xq, sx, flags=0, stream=None):
    """X [S,K] fp16, rows int32 [M] or None -> Xq [M,K/2] u8, sx [M] fp16."""
    K = X.shape[1]
    M = X.shape[0] if rows is None else rows.numel()
    _check(lib().sqap_quantize_act(_ptr(X), X.stride(0), _ptr(rows), M, K, flags, _ptr(Xq), _ptr(sx),
                                   _stream(stream)))


def sqap_quantize_weight(W, Wq, sw, flags=0, stream=None):
    N, K = W.shape
    _check(lib().sqap_quantize_weight(_ptr(W), N, K, flags, _ptr(Wq), _ptr(sw), _stream(stream)))


class Weight:
    """Owns a sqap_weight handle."""

    def __init__(self, handle, N, K):
        self.handle, self.N, self.K = handle, N, K

    def free(self):
        if self.handle:
            _check(lib().sqap_weight_free(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    @property
    def device_bytes(self):
        b = ctypes.c_size_t()
        _check(lib().sqap_weight_info(self.handle, None, None, ctypes.byref(b)))
        return b.value


def sqap_channel_scales(X, rows, amax, scales_out, flags=0, accumulate=False, stream=None):
    """Static per-channel activation scales from calibration rows: X [S,K] fp16 -> scales_out [K] fp16."""
    M = X.shape[0] if rows is None else rows.numel()
    _check(lib().sqap_channel_scales(_ptr(X), X.stride(0), _ptr(rows), M, X.shape[1], flags, _ptr(amax),
                                     1 if accumulate else 0, _ptr(scales_out), _stream(stream)))


def sqap_quantize_act_channelwise(X, rows, col_scales, Xq, sx, flags=0, stream=None):
    M = X.shape[0] if rows is None else rows.numel()
    _check(lib().sqap_quantize_act_channelwise(_ptr(X), X.stride(0), _ptr(rows), M, X.shape[1], flags,
                                               _ptr(col_scales), _ptr(Xq), _ptr(sx), _stream(stream)))


def sqap_quantize_weight_folded(W, col_scales, Wq, sw, flags=0, stream=None):
    N, K = W.shape
    _check(lib().sqap_quantize_weight_folded(_ptr(W), N, K, flags, _ptr(col_scales), _ptr(Wq), _ptr(sw),
                                             _stream(stream)))


def sqap_weight_pack(Wq, sw, stream=None):
    N, half = Wq.shape
    h = ctypes.c_void_p()
    _check(lib().sqap_weight_pack(_ptr(Wq), _ptr(sw), N, 2 * half, ctypes.byref(h), _stream(stream)))
    return Weight(h, N, 2 * half)


def sqap_rmsnorm_quantize_act(X, rows, gamma, eps, Xq, sx, delta=None, flags=0, col_scales=None, xsum_out=None,
                              y_out=None, stream=None):
    """RMSNorm (after an optional residual update) fused into the activation quantizer."""
    K = X.shape[1]
    M = X.shape[0] if rows is None else rows.numel()
    _check(lib().sqap_rmsnorm_quantize_act(_ptr(X), X.stride(0), _ptr(rows), M, K, _ptr(delta), _ptr(gamma), eps,
                                           flags, _ptr(col_scales), _ptr(xsum_out), _ptr(y_out), _ptr(Xq),
                                           _ptr(sx), _stream(stream)))


def sqap_swiglu_quantize_act(G, U, Xq, sx, col_scales=None, h_out=None, stream=None):
    """h = silu(G) * U fused into the activation quantizer; G, U may be column slices of one tensor."""
    M, F = G.shape
    _check(lib().sqap_swiglu_quantize_act(_ptr(G), G.stride(0), _ptr(U), U.stride(0), M, F, _ptr(col_scales),
                                          _ptr(h_out), _ptr(Xq), _ptr(sx), _stream(stream)))


def sqap_rope(X, pos, H, d, base=10000.0, stream=None):
    """X [S, >= H*d] fp16 (row pitch = X.stride(0)), rotated in place at positions pos [S] int32."""
    _check(lib().sqap_rope(_ptr(X), X.stride(0), _ptr(pos), X.shape[0], H, d, base, _stream(stream)))


def sqap_rope_append(QKV, pos, H, d, KV, base=10000.0, stream=None):
    """QKV [S, 3*H*d] fused rows: q rotated in place, rotated k | v written to the cache rows KV [S, 2*H*d]."""
    _check(lib().sqap_rope_append(_ptr(QKV), QKV.stride(0), _ptr(pos), QKV.shape[0], H, d, base, _ptr(KV),
                                  KV.stride(0), _stream(stream)))


def sqap_attention(Q, K, V, H, d, O, batch=1, stream=None):
    """Causal attention; Q, O [batch*Sq, H*d], K, V [batch*Sk, H*d] (row pitches from the strides)."""
    _check(lib().sqap_attention(_ptr(Q), Q.stride(0), _ptr(K), K.stride(0), _ptr(V), V.stride(0), batch,
                                Q.shape[0] // batch, K.shape[0] // batch, H, d, _ptr(O), O.stride(0),
                                _stream(stream)))


def sqap_decode_attention(qkv, pos, H, d, KV, past, O, Xq=None, sx=None, counter=None, base=10000.0, stream=None):
    """One decode step's attention in one launch: qkv [3*H*d] (one token) rotated, key | value appended as
    row `past` of the cache KV [>= past+1, 2*H*d], attention over rows 0..past into O [H*d]; with Xq
    (and sx [1], counter: a zeroed uint32/int32 device word) O is also quantized as by sqap_quantize_act."""
    _check(lib().sqap_decode_attention(_ptr(qkv), _ptr(pos), H, d, base, _ptr(KV), KV.stride(0), past, _ptr(O),
                                       _ptr(Xq), _ptr(sx), _ptr(counter), _stream(stream)))


def sqap_residual_add(X, delta, stream=None):
    M, K = X.shape
    _check(lib().sqap_residual_add(_ptr(X), X.stride(0), _ptr(delta), delta.stride(0), M, K, _stream(stream)))


def sqap_selftest_quotient(counter, stream=None):
    """counter: zeroed int64 device tensor of one element; receives the number of mismatches."""
    _check(lib().sqap_selftest_quotient(_ptr(counter), _stream(stream)))


def sqap_selftest_dispatch(stream=None):
    """XCC id of each of the 256 workgroups of a probe launch (list of int)."""
    table = (ctypes.c_uint32 * 256)()
    _check(lib().sqap_selftest_dispatch(table, _stream(stream)))
    return list(table)


def sqap_plan_linear_shares(M, N, K, blocks_per_xcd=32):
    """Host-only: (bounds[8][33], planned[8], even[8], (tile rows, tile columns)) of the stream-K linear's work split."""
    bounds = (ctypes.c_uint32 * (8 * 33))()
    planned = (ctypes.c_double * 8)()
    even = (ctypes.c_double * 8)()
    bm, bn = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().sqap_plan_linear_shares(M, N, K, blocks_per_xcd, bounds, planned, even, ctypes.byref(bm), ctypes.byref(bn)))
    return [list(bounds[x * 33:(x + 1) * 33]) for x in range(8)], list(planned), list(even), (bm.value, bn.value)


def sqap_workspace_bytes(M, N, K):
    return int(lib().sqap_workspace_bytes(M, N, K))


def sqap_w4a4_linear(Xq, sx, W, Y, acc_out=None, workspace=None, stream=None):
    """Xq [M,K/2] u8, sx [M] fp16, W: Weight -> Y [M,N] fp16 (+ acc_out [M,N] int32)."""
    M = Xq.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sqap_w4a4_linear(_ptr(Xq), _ptr(sx), M, W.handle, _ptr(Y), Y.stride(0), _ptr(acc_out),
                                  _ptr(workspace), ws_bytes, _stream(stream)))


class Group:
    """Owns a sqap_group handle; keeps the tensors it points to alive."""

    def __init__(self, handle, keep):
        self.handle, self._keep = handle, keep

    def run(self, stream=None):
        _check(lib().sqap_group_run(self.handle, _stream(stream)))

    def info(self, compute_units=0):
        """(problems, row groups, wavefronts per row group, wavefronts per workgroup, LDS output slots) of the launch."""
        v = [ctypes.c_int32(0) for _ in range(5)]
        _check(lib().sqap_group_info(self.handle, compute_units, *[ctypes.byref(x) for x in v]))
        return tuple(x.value for x in v)

    def free(self):
        if self.handle:
            _check(lib().sqap_group_free(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def sqap_group_create(problems):
    """problems: list of (Xq, sx, Weight, Y) or (Xq, sx, Weight, Y, acc_out) with M <= 8."""
    n = len(problems)
    arr = (LinearDesc * n)()
    for i, pr in enumerate(problems):
        Xq, sx, W, Y = pr[:4]
        acc = pr[4] if len(pr) > 4 else None
        arr[i].Xq, arr[i].sx, arr[i].M = Xq.data_ptr(), sx.data_ptr(), Xq.shape[0]
        arr[i].W, arr[i].Y, arr[i].ldy = W.handle.value, Y.data_ptr(), Y.stride(0)
        arr[i].acc_out = None if acc is None else acc.data_ptr()
    h = ctypes.c_void_p()
    _check(lib().sqap_group_create(arr, n, ctypes.byref(h)))
    return Group(h, list(problems))


def sqap_group_run(group, stream=None):
    group.run(stream)


class Decoder:
    """Owns a sqap_decoder handle; keeps the tensors and weights it points to alive."""

    def __init__(self, handle, keep):
        self.handle, self._keep = handle, keep

    def step(self, x, pos, past, logits, attn_trace=None, stream=None):
        """x [hidden] fp16, pos [1] int32 (device), past: positions already in the caches, logits [vocab] fp16."""
        _check(lib().sqap_decoder_step(self.handle, _ptr(x), _ptr(pos), past, _ptr(logits), _ptr(attn_trace),
                                       _stream(stream)))

    def status(self, stream=None):
        """Error word of the last step (0: every wait between workgroups ended).  Synchronises the stream."""
        w = ctypes.c_uint64(0)
        _check(lib().sqap_decoder_status(self.handle, ctypes.byref(w), _stream(stream)))
        return w.value

    def set_wait_limit(self, polls):
        """Looks for another workgroup's output before a wait gives up (negative: the default)."""
        _check(lib().sqap_decoder_set_wait_limit(self.handle, int(polls)))

    def free(self):
        if self.handle:
            _check(lib().sqap_decoder_free(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def sqap_decoder_create(layers, n_heads, head_dim, gamma_final, head, eps=1e-5, rope_base=10000.0):
    """layers: list of (qkv, o, gate_up, down: Weight; gamma_attn, gamma_mlp: [hidden] fp16; kv: [capacity, >= 2 hidden] fp16)."""
    n = len(layers)
    arr = (DecoderLayer * n)()
    for i, (qkv, o, gu, dn, g1, g2, kv) in enumerate(layers):
        arr[i].qkv, arr[i].o, arr[i].gate_up, arr[i].down = qkv.handle.value, o.handle.value, gu.handle.value, dn.handle.value
        arr[i].gamma_attn, arr[i].gamma_mlp = g1.data_ptr(), g2.data_ptr()
        arr[i].kv, arr[i].ldkv = kv.data_ptr(), kv.stride(0)
    h = ctypes.c_void_p()
    _check(lib().sqap_decoder_create(arr, n, n_heads, head_dim, _ptr(gamma_final), head.handle, eps, rope_base,
                                     ctypes.byref(h)))
    return Decoder(h, (list(layers), gamma_final, head))
