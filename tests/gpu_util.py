"""Helpers for the GPU parity tests: numpy in, HIP library, numpy out."""
import numpy as np
import torch

from paper_2509_09090_amd import binding as B

DEV = "cuda:0"


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_prune_topk(scores, keep_k):
    s = to_dev(np.atleast_2d(scores).astype(np.float32))
    out = torch.full((s.shape[0], keep_k), -1, dtype=torch.int32, device=DEV)
    B.sqap_prune_topk(s, keep_k, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_kept_rows(idx, seq_len, vis_begin, n_vis):
    i = to_dev(np.atleast_2d(idx).astype(np.int32))
    out = torch.full((i.shape[0] * (seq_len - n_vis + i.shape[1]),), -1, dtype=torch.int32, device=DEV)
    B.sqap_kept_rows(i, seq_len, vis_begin, n_vis, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_gather(X, rows):
    x = to_dev(X)
    r = to_dev(rows.astype(np.int32))
    out = torch.zeros((rows.size, X.shape[1]), dtype=torch.float16, device=DEV)
    B.sqap_gather_rows(x, r, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_quantize(X, rows=None, rotate=False, weight=False):
    x = to_dev(X)
    M = X.shape[0] if rows is None else rows.size
    K = X.shape[1]
    q = torch.zeros((M, K // 2), dtype=torch.uint8, device=DEV)
    s = torch.zeros((M,), dtype=torch.float16, device=DEV)
    flags = B.ROTATE_HADAMARD if rotate else 0
    if weight:
        assert rows is None
        B.sqap_quantize_weight(x, q, s, flags)
    else:
        r = None if rows is None else to_dev(rows.astype(np.int32))
        B.sqap_quantize_act(x, r, q, s, flags)
    torch.cuda.synchronize()
    return q.cpu().numpy(), s.cpu().numpy()


def gpu_linear(Xq, sx, Wq, sw, want_acc=True):
    """Canonical packed operands (numpy) -> (Y fp16, acc int32) through pack + linear."""
    xq, sxd, wq, swd = to_dev(Xq), to_dev(sx), to_dev(Wq), to_dev(sw)
    W = B.sqap_weight_pack(wq, swd)
    M, N, K = Xq.shape[0], Wq.shape[0], 2 * Wq.shape[1]
    Y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    acc = torch.full((M, N), -123456789, dtype=torch.int32, device=DEV) if want_acc else None
    nbytes = B.sqap_workspace_bytes(M, N, K)
    ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=DEV) if nbytes else None
    B.sqap_w4a4_linear(xq, sxd, W, Y, acc, ws)
    torch.cuda.synchronize()
    W.free()
    return Y.cpu().numpy(), (acc.cpu().numpy() if want_acc else None)


def assert_fp16_close(got, ref):
    """Tolerance of the parity gate: |gpu - ref| <= 1e-2 + 1e-3 |ref|; also reports bit equality."""
    g = got.astype(np.float64)
    r = ref.astype(np.float64)
    assert np.all(np.abs(g - r) <= 1e-2 + 1e-3 * np.abs(r)), float(np.abs(g - r).max())
    return int(np.count_nonzero(got.view(np.uint16) != ref.view(np.uint16)))


def score_workspace(batch, S, H, d, n_vis):
    """Zeroed workspace for sqap_attn_scores / sqap_attn_scores_batch (None when the shape needs none)."""
    n = B.sqap_attn_scores_workspace_bytes(batch, S, H, d, n_vis)
    return torch.zeros((n,), dtype=torch.uint8, device=DEV) if n else None
