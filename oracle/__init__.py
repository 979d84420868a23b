"""CPU oracle for the SQAP-VLA hot path: TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes marshalling around ``sqap_oracle.c`` (plain C, written from
the paper, arXiv 2509.09090).  Nothing here is imported by the product package
and nothing here imports it.  Allowed callers: ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg.

Half-precision arrays are ``numpy.float16``; they cross into C as their uint16
bit patterns.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sqap_oracle.c")
_LIB = os.path.join(_HERE, "libsqap_oracle.so")

ROTATE_HADAMARD = 1


def build(force=False):
    """Compile the oracle with the host C compiler (no GPU code involved)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_f16_to_f32.restype = ctypes.c_float
        _lib.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.oracle_f32_to_f16.restype = ctypes.c_uint16
        _lib.oracle_f32_to_f16.argtypes = [ctypes.c_float]
        _lib.oracle_int_gemm.restype = ctypes.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def set_threads(n):
    """Number of OpenMP threads the row loops may use (returns the old value)."""
    omp = ctypes.CDLL("libgomp.so.1")
    old = omp.omp_get_max_threads()
    omp.omp_set_num_threads(int(n))
    return old


def f16_to_f32(bits):
    return float(lib().oracle_f16_to_f32(int(bits)))


def f32_to_f16(x):
    return int(lib().oracle_f32_to_f16(ctypes.c_float(x)))


def prune_topk(scores, keep_k):
    """Eq. 1: indices of the keep_k largest scores of each row, ascending."""
    s = _c(scores, np.float32)
    one = s.ndim == 1
    s2 = s.reshape(1, -1) if one else s
    b, n = s2.shape
    out = np.empty((b, keep_k), dtype=np.int32)
    rc = lib().oracle_prune_topk(_p(s2), b, n, int(keep_k), _p(out))
    if rc != 0:
        raise ValueError("oracle_prune_topk: status %d" % rc)
    return out[0] if one else out


def project_token(Kmat, Rt, xyz, patch_w, patch_h):
    """Eq. 2-3: world point -> token coordinates (t_u, t_v), or None if there is no valid projection."""
    Km, R, p = _c(Kmat, np.float64).reshape(9), _c(Rt, np.float64).reshape(12), _c(xyz, np.float64).reshape(3)
    tu, tv = ctypes.c_int32(0), ctypes.c_int32(0)
    ok = lib().oracle_project_token(_p(Km), _p(R), _p(p), ctypes.c_double(patch_w), ctypes.c_double(patch_h),
                                    ctypes.byref(tu), ctypes.byref(tv))
    return (tu.value, tv.value) if ok else None


def ring(grid_w, grid_h, cu, cv, radius):
    """Eq. 4: membership flags of the Chebyshev ball around token (cu, cv), clipped to the grid."""
    flags = np.zeros(grid_w * grid_h, dtype=np.uint8)
    rc = lib().oracle_ring(int(grid_w), int(grid_h), int(cu), int(cv), int(radius), _p(flags))
    if rc != 0:
        raise ValueError("oracle_ring: status %d" % rc)
    return flags


def fps(grid_w, grid_h, kept, m):
    """Eq. 5: m farthest-point picks (in pick order) given the 0/1 array of tokens already kept."""
    k = np.array(kept, dtype=np.uint8).reshape(grid_w * grid_h).copy()
    picks = np.empty(m, dtype=np.int32)
    rc = lib().oracle_fps(int(grid_w), int(grid_h), _p(k), int(m), _p(picks))
    if rc != 0:
        raise ValueError("oracle_fps: status %d" % rc)
    return picks


def prune_select(scores, grid_w, grid_h, k_attn, keep_total, centre=None, radius=0):
    """K_attn + K_ring + K_fps for one observation: ascending token indices."""
    s = _c(scores, np.float32).reshape(grid_w * grid_h)
    out = np.empty(grid_w * grid_h, dtype=np.int32)
    cu, cv = centre if centre is not None else (0, 0)
    n = lib().oracle_prune_select(_p(s), int(grid_w), int(grid_h), int(k_attn), int(keep_total),
                                  int(centre is not None), int(cu), int(cv), int(radius), _p(out))
    if n < 0:
        raise ValueError("oracle_prune_select: status %d" % n)
    return out[:n].copy()


def kept_rows(idx, seq_len, vis_begin, n_vis):
    """Surviving sequence rows (global over the batch) in original order."""
    i2 = _c(idx, np.int32)
    if i2.ndim == 1:
        i2 = i2.reshape(1, -1)
    b, k = i2.shape
    out = np.empty(b * (seq_len - n_vis + k), dtype=np.int32)
    rc = lib().oracle_kept_rows(_p(i2), b, k, int(seq_len), int(vis_begin), int(n_vis),
                                _p(out))
    if rc != 0:
        raise ValueError("oracle_kept_rows: status %d" % rc)
    return out


def gather_rows(X, rows):
    X = _c(X, np.float16)
    rows = _c(rows, np.int32)
    out = np.empty((rows.size, X.shape[1]), dtype=np.float16)
    lib().oracle_gather_rows(_p(X), ctypes.c_int64(X.shape[1]), _p(rows), rows.size,
                             X.shape[1], _p(out), ctypes.c_int64(X.shape[1]))
    return out


def fwht(v):
    """Eq. 6 rotation of one binary32 vector (copy)."""
    v = np.array(v, dtype=np.float32, copy=True)
    rc = lib().oracle_fwht_f32(_p(v), v.size)
    if rc != 0:
        raise ValueError("oracle_fwht_f32: status %d" % rc)
    return v


def rotate(v):
    """Eq. 6 rotation of one binary32 vector of any length: blocks of the largest power-of-two divisor (copy)."""
    v = np.array(v, dtype=np.float32, copy=True)
    rc = lib().oracle_rotate_f32(_p(v), v.size)
    if rc != 0:
        raise ValueError("oracle_rotate_f32: status %d" % rc)
    return v


def rotation_block(K):
    return int(lib().oracle_rotation_block(int(K)))


def quantize_rows(X, rows=None, rotate=False):
    """Per-row symmetric int4: returns (packed [M,K/2] u8, scale [M] f16, rowsum [M] i32)."""
    X = _c(X, np.float16)
    K = X.shape[1]
    r = None if rows is None else _c(rows, np.int32)
    M = X.shape[0] if r is None else r.size
    q = np.empty((M, K // 2), dtype=np.uint8)
    s = np.empty(M, dtype=np.float16)
    rs = np.empty(M, dtype=np.int32)
    rc = lib().oracle_quantize_rows(_p(X), ctypes.c_int64(K), _p(r), M, K,
                                    1 if rotate else 0, _p(q), _p(s), _p(rs))
    if rc != 0:
        raise ValueError("oracle_quantize_rows: status %d" % rc)
    return q, s, rs


def channel_scales(X, rows=None, rotate=False):
    """Section 3.3, channel-wise activations: static scale per input channel from calibration rows, [K] f16."""
    X = _c(X, np.float16)
    K = X.shape[1]
    r = None if rows is None else _c(rows, np.int32)
    M = X.shape[0] if r is None else r.size
    c = np.empty(K, dtype=np.float16)
    rc = lib().oracle_channel_scales(_p(X), ctypes.c_int64(K), _p(r), M, K, 1 if rotate else 0, _p(c))
    if rc != 0:
        raise ValueError("oracle_channel_scales: status %d" % rc)
    return c


def quantize_rows_channelwise(X, col_scales, rows=None, rotate=False):
    """Codes with one static scale per channel; returns (packed [M,K/2] u8, per-token scale [M] f16 = 1)."""
    X = _c(X, np.float16)
    K = X.shape[1]
    c = _c(col_scales, np.float16)
    assert c.shape == (K,)
    r = None if rows is None else _c(rows, np.int32)
    M = X.shape[0] if r is None else r.size
    q = np.empty((M, K // 2), dtype=np.uint8)
    s = np.empty(M, dtype=np.float16)
    rc = lib().oracle_quantize_rows_channelwise(_p(X), ctypes.c_int64(K), _p(r), M, K, 1 if rotate else 0,
                                                _p(c), _p(q), _p(s))
    if rc != 0:
        raise ValueError("oracle_quantize_rows_channelwise: status %d" % rc)
    return q, s


def quantize_rows_folded(W, col_scales, rotate=False):
    """Weight rows times the activation channel scales, then per-row int4: (packed [N,K/2] u8, scale [N] f16)."""
    W = _c(W, np.float16)
    N, K = W.shape
    c = _c(col_scales, np.float16)
    assert c.shape == (K,)
    q = np.empty((N, K // 2), dtype=np.uint8)
    s = np.empty(N, dtype=np.float16)
    rc = lib().oracle_quantize_rows_folded(_p(W), ctypes.c_int64(K), N, K, 1 if rotate else 0, _p(c), _p(q), _p(s))
    if rc != 0:
        raise ValueError("oracle_quantize_rows_folded: status %d" % rc)
    return q, s


def unpack_int4(Q):
    Q = _c(Q, np.uint8)
    R, half = Q.shape
    out = np.empty((R, 2 * half), dtype=np.int8)
    lib().oracle_unpack_int4(_p(Q), R, 2 * half, _p(out))
    return out


def int_gemm(Xq, Wq):
    """Exact acc[m,n] = sum_k xq[m,k]*wq[n,k]; raises if int32 != int64 anywhere."""
    Xq = _c(Xq, np.uint8)
    Wq = _c(Wq, np.uint8)
    M, half = Xq.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == half
    acc = np.empty((M, N), dtype=np.int32)
    bad = lib().oracle_int_gemm(_p(Xq), _p(Wq), M, N, 2 * half, _p(acc))
    if bad != 0:
        raise ArithmeticError("int32 and int64 accumulators differ (%d)" % bad)
    return acc


def dequant(acc, sx, sw):
    acc = _c(acc, np.int32)
    sx = _c(sx, np.float16)
    sw = _c(sw, np.float16)
    M, N = acc.shape
    Y = np.empty((M, N), dtype=np.float16)
    lib().oracle_dequant(_p(acc), _p(sx), _p(sw), M, N, _p(Y), ctypes.c_int64(N))
    return Y


def w4a4_linear(Xq, sx, Wq, sw):
    """Returns (Y fp16 [M,N], acc int32 [M,N])."""
    acc = int_gemm(Xq, Wq)
    return dequant(acc, sx, sw), acc


def linear_samples(Xq, sx, Wq, sw, ms, ns):
    """acc and Y at chosen (m, n) positions only."""
    Xq = _c(Xq, np.uint8)
    Wq = _c(Wq, np.uint8)
    sx = _c(sx, np.float16)
    sw = _c(sw, np.float16)
    ms = _c(ms, np.int32)
    ns = _c(ns, np.int32)
    acc = np.empty(ms.size, dtype=np.int32)
    y = np.empty(ms.size, dtype=np.float16)
    lib().oracle_linear_samples(_p(Xq), _p(sx), _p(Wq), _p(sw), 2 * Xq.shape[1],
                                _p(ms), _p(ns), ms.size, _p(acc), _p(y))
    return acc, y


def attn_scores(q, k, vis_begin, n_vis):
    """Retention score a_q of the visual span: q [H,d], k [S,H,d] (fp16)."""
    q = _c(q, np.float16)
    k = _c(k, np.float16)
    S, H, d = k.shape
    out = np.empty(n_vis, dtype=np.float32)
    rc = lib().oracle_attn_scores(_p(q), _p(k), S, H, d, int(vis_begin), int(n_vis),
                                  _p(out))
    if rc != 0:
        raise ValueError("oracle_attn_scores: status %d" % rc)
    return out


def rmsnorm_rows(X, gamma, eps, rows=None, delta=None):
    """RMSNorm (with an optional residual update first): returns (x' fp16 [M,K], y fp16 [M,K])."""
    X = _c(X, np.float16)
    gamma = _c(gamma, np.float16)
    K = X.shape[1]
    rows_c = None if rows is None else _c(rows, np.int32)
    M = X.shape[0] if rows is None else len(rows_c)
    delta_c = None if delta is None else _c(delta, np.float16)
    xs = np.empty((M, K), dtype=np.float16)
    y = np.empty((M, K), dtype=np.float16)
    rc = lib().oracle_rmsnorm_rows(_p(X), ctypes.c_int64(X.strides[0] // 2), _p(rows_c), M, K, _p(delta_c),
                                   _p(gamma), ctypes.c_float(eps), _p(xs), _p(y))
    if rc:
        raise ValueError("oracle_rmsnorm_rows: %d" % rc)
    return xs, y


def swiglu(G, U):
    """h = fp16(silu(g) * u), elementwise over [M, F] halves."""
    G = _c(G, np.float16)
    U = _c(U, np.float16)
    M, F = G.shape
    out = np.empty((M, F), dtype=np.float16)
    rc = lib().oracle_swiglu(_p(G), ctypes.c_int64(F), _p(U), ctypes.c_int64(F), M, F, _p(out))
    if rc:
        raise ValueError("oracle_swiglu: %d" % rc)
    return out


def rope(X, pos, base=10000.0):
    """Rotary embedding of [S, H, d] halves at integer positions pos[S]; returns a new array."""
    out = _c(X, np.float16).copy()
    S, H, d = out.shape
    pos = _c(pos, np.int32)
    rc = lib().oracle_rope(_p(out), _p(pos), S, H, d, ctypes.c_double(base))
    if rc:
        raise ValueError("oracle_rope: %d" % rc)
    return out


def attention(Q, K, V):
    """Causal softmax attention: Q [Sq, H, d] (the last Sq positions), K, V [Sk, H, d] -> [Sq, H, d] halves."""
    Q, K, V = _c(Q, np.float16), _c(K, np.float16), _c(V, np.float16)
    Sq, H, d = Q.shape
    Sk = K.shape[0]
    out = np.empty((Sq, H, d), dtype=np.float16)
    rc = lib().oracle_attention(_p(Q), _p(K), _p(V), Sq, Sk, H, d, _p(out))
    if rc:
        raise ValueError("oracle_attention: %d" % rc)
    return out


def residual_add(X, delta):
    out = _c(X, np.float16).copy()
    delta = _c(delta, np.float16)
    M, K = out.shape
    rc = lib().oracle_residual_add(_p(out), _p(delta), M, K)
    if rc:
        raise ValueError("oracle_residual_add: %d" % rc)
    return out


def decoder_layer(x, pending, pos, batch, weights, gamma_attn, gamma_mlp, n_heads, head_dim, eps=1e-5,
                  rotate=False, attn_override=None, past_k=None, past_v=None):
    """One pre-normalisation Llama layer as a chain of the functions above; every stage is returned.

    x [M, hidden] fp16 residual stream, pending [M, hidden] or None, pos [M] positions, batch
    sequences of M / batch rows.  weights: dict name -> (packed int4 [N, K/2], scales [N]) for
    'qkv' (N = 3 hidden), 'o', 'gate_up' (N = 2 ffn), 'down'.  attn_override replaces the attention
    output (lets a test continue from another implementation's result).  past_k, past_v [P, hidden]:
    rotated keys and values of P earlier positions of the (single) sequence, placed in front of the new ones.
    """
    M, hidden = x.shape
    S = M // batch
    st = {}
    st["x1"], y1 = rmsnorm_rows(x, gamma_attn, eps, delta=pending)
    q1, s1, _ = quantize_rows(y1, rotate=rotate)
    st["q1"], st["s1"] = q1, s1
    st["qkv"], _ = w4a4_linear(q1, s1, *weights["qkv"])
    qkv = st["qkv"]
    q = rope(qkv[:, :hidden].reshape(M, n_heads, head_dim), pos)
    k = rope(qkv[:, hidden:2 * hidden].reshape(M, n_heads, head_dim), pos)
    v = np.ascontiguousarray(qkv[:, 2 * hidden:]).reshape(M, n_heads, head_dim)
    st["q_rot"], st["k_rot"] = q.reshape(M, hidden), k.reshape(M, hidden)
    if past_k is not None:
        assert batch == 1
        kk = np.concatenate([_c(past_k, np.float16).reshape(-1, n_heads, head_dim), k])
        vv = np.concatenate([_c(past_v, np.float16).reshape(-1, n_heads, head_dim), v])
        a = attention(q, kk, vv).reshape(M, hidden)
    else:
        a = np.concatenate([attention(q[b * S:(b + 1) * S], k[b * S:(b + 1) * S], v[b * S:(b + 1) * S])
                            for b in range(batch)]).reshape(M, hidden)
    st["attn"] = a
    if attn_override is not None:
        a = attn_override
    q2, s2, _ = quantize_rows(a)
    st["o"], _ = w4a4_linear(q2, s2, *weights["o"])
    st["x2"], y2 = rmsnorm_rows(st["x1"], gamma_mlp, eps, delta=st["o"])
    q3, s3, _ = quantize_rows(y2)
    st["gu"], _ = w4a4_linear(q3, s3, *weights["gate_up"])
    ffn = st["gu"].shape[1] // 2
    h = swiglu(st["gu"][:, :ffn], st["gu"][:, ffn:])
    q4, s4, _ = quantize_rows(h)
    st["hq"], st["sh"] = q4, s4
    st["d"], _ = w4a4_linear(q4, s4, *weights["down"])
    return st
