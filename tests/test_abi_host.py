"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2509_09090_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sqap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sqap_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = B.lib()
    names = _declared()
    assert len(names) >= 13
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_version_and_error_strings():
    assert "gfx950" in B.sqap_version()
    assert isinstance(B.lib().sqap_last_error(), bytes)


def _err():
    return B.lib().sqap_last_error().decode()


def test_prune_topk_validation():
    L = B.lib()
    assert L.sqap_prune_topk(None, 1, 4, 5, None, None) == B.EINVAL and "keep_k" in _err()
    assert L.sqap_prune_topk(None, -1, 4, 1, None, None) == B.EINVAL
    assert L.sqap_prune_topk(None, 1, 4, 2, None, None) == B.EINVAL      # null with work to do
    assert L.sqap_prune_topk(None, 0, 4, 2, None, None) == B.OK          # empty batch
    assert L.sqap_prune_topk(None, 3, 4, 0, None, None) == B.OK          # keep nothing
    one = ctypes.c_void_p(16)
    assert L.sqap_prune_topk(one, 1, 70000, 5, one, None) == B.EUNSUPPORTED


def test_kept_rows_validation():
    L = B.lib()
    assert L.sqap_prune_rows(None, 1, 4, 5, 10, 0, None, None, None) == B.EINVAL    # keep_k > n_vis
    assert L.sqap_prune_rows(None, 1, 4, 2, 10, 8, None, None, None) == B.EINVAL    # span outside
    assert L.sqap_prune_rows(None, 0, 4, 2, 10, 0, None, None, None) == B.OK
    assert L.sqap_kept_rows(None, 1, 5, 10, 0, 4, None, None) == B.EINVAL    # keep_k > n_vis
    assert L.sqap_kept_rows(None, 1, 2, 10, 8, 4, None, None) == B.EINVAL    # span outside
    assert L.sqap_kept_rows(None, 0, 2, 10, 0, 4, None, None) == B.OK


def test_quantize_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    assert L.sqap_quantize_act(p, 5, None, 1, 5, 0, p, p, None) == B.EINVAL and "odd" in _err()
    assert L.sqap_quantize_act(p, 8, None, 1, 16, 0, p, p, None) == B.EINVAL          # ldx < K
    assert L.sqap_quantize_act(p, 16, None, -1, 16, 0, p, p, None) == B.EINVAL
    assert L.sqap_quantize_act(None, 16, None, 1, 16, 0, p, p, None) == B.EINVAL
    assert L.sqap_quantize_act(p, 16, None, 1, 16, 2, p, p, None) == B.EINVAL         # unknown flag
    assert L.sqap_quantize_act(None, 16, None, 0, 16, 0, None, None, None) == B.OK    # M = 0
    assert L.sqap_quantize_act(p, 2056, None, 1, 2056, 1, p, p, None) == B.EUNSUPPORTED   # 2056 = 8 * 257
    assert "multiple of 16" in _err()
    assert L.sqap_quantize_act(p, 12, None, 1, 12, 0, p, p, None) == B.EUNSUPPORTED   # K % 8
    assert L.sqap_quantize_act(p, 32768, None, 1, 32768, 0, p, p, None) == B.EUNSUPPORTED
    assert L.sqap_quantize_act(ctypes.c_void_p(4098), 16, None, 1, 16, 0, p, p, None) == B.EUNSUPPORTED
    assert L.sqap_quantize_weight(p, 4, 7, 0, p, p, None) == B.EINVAL


def test_gather_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    assert L.sqap_gather_rows(p, 8, p, 1, 16, p, 16, None) == B.EINVAL
    assert L.sqap_gather_rows(p, 16, None, 1, 16, p, 16, None) == B.EINVAL
    assert L.sqap_gather_rows(p, 12, p, 1, 12, p, 12, None) == B.EUNSUPPORTED
    assert L.sqap_gather_rows(p, 16, p, 0, 16, p, 16, None) == B.OK


def test_weight_and_linear_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    h = ctypes.c_void_p()
    assert L.sqap_weight_pack(p, p, 0, 32, ctypes.byref(h), None) == B.EINVAL
    assert L.sqap_weight_pack(p, p, 4, 48, ctypes.byref(h), None) == B.EUNSUPPORTED
    assert L.sqap_weight_pack(None, p, 4, 32, ctypes.byref(h), None) == B.EINVAL
    assert h.value is None
    assert L.sqap_weight_free(None) == B.OK
    assert L.sqap_weight_info(None, None, None, None) == B.EINVAL
    assert L.sqap_w4a4_linear(p, p, 1, None, p, 32, None, None, 0, None) == B.EINVAL
    fake = (ctypes.c_uint32 * 32)()          # wrong magic: rejected without a device call
    assert L.sqap_w4a4_linear(p, p, 1, ctypes.cast(fake, ctypes.c_void_p), p, 32, None, None, 0,
                              None) == B.EINVAL
    assert B.sqap_workspace_bytes(0, 10, 32) == 0


def test_attn_scores_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    big = 1 << 30
    assert L.sqap_attn_scores(p, p, 0, 1, 8, 0, 0, p, p, big, None) == B.EINVAL
    assert L.sqap_attn_scores(p, p, 10, 2, 8, 5, 6, p, p, big, None) == B.EINVAL
    assert L.sqap_attn_scores(p, p, 10, 2, 512, 0, 4, p, p, big, None) == B.EUNSUPPORTED
    assert L.sqap_attn_scores(p, p, 10, 2, 8, 0, 0, None, None, 0, None) == B.OK
    assert L.sqap_attn_scores_batch(p, p, -1, 10, 2, 8, 0, 4, p, p, big, None) == B.EINVAL
    assert L.sqap_attn_scores_batch(None, None, 0, 10, 2, 8, 0, 4, None, None, 0, None) == B.OK
    assert L.sqap_attn_scores_batch(p, p, 3, 10, 2, 8, 8, 4, p, p, big, None) == B.EINVAL
    assert L.sqap_attn_scores_batch(p, p, 5000, 10, 2, 8, 0, 4, p, p, big, None) == B.EUNSUPPORTED
    assert L.sqap_attn_scores_batch(p, p, 3, 10, 2, 7, 0, 4, p, p, big, None) == B.EUNSUPPORTED
    # the workspace: 256 bytes of counters per observation + the per-head weights; none for single-workgroup shapes
    assert B.sqap_attn_scores_workspace_bytes(1, 276, 32, 128, 256) == 256 + 4 * 32 * 256
    assert B.sqap_attn_scores_workspace_bytes(16, 276, 32, 128, 256) == 16 * (256 + 4 * 32 * 256)
    assert B.sqap_attn_scores_workspace_bytes(1, 100, 3, 24, 60) == 0          # head size not a power of two
    assert B.sqap_attn_scores_workspace_bytes(1, 5000, 2, 32, 4000) == 0       # logits do not fit LDS
    assert B.sqap_attn_scores_workspace_bytes(0, 276, 32, 128, 256) == 0
    need = B.sqap_attn_scores_workspace_bytes(1, 276, 32, 128, 256)
    assert L.sqap_attn_scores(p, p, 276, 32, 128, 0, 256, p, None, 0, None) == B.EINVAL        # missing
    assert b"workspace" in L.sqap_last_error()
    assert L.sqap_attn_scores(p, p, 276, 32, 128, 0, 256, p, p, need - 1, None) == B.EINVAL    # too small
    assert L.sqap_attn_scores(p, p, 276, 32, 128, 0, 256, p, ctypes.c_void_p(4104), need, None) == B.EINVAL   # misaligned


def test_glue_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    f = ctypes.c_float
    assert L.sqap_rmsnorm_quantize_act(p, 64, None, 2, 64, None, None, f(1e-5), 0, None, None, None, p, p, None) == B.EINVAL
    assert L.sqap_rmsnorm_quantize_act(p, 64, None, 2, 64, None, p, f(-1.0), 0, None, None, None, p, p, None) == B.EINVAL
    assert L.sqap_rmsnorm_quantize_act(p, 64, None, 2, 64, None, p, f(1e-5), 0, None, None, None, None, None, None) == B.EINVAL
    assert L.sqap_rmsnorm_quantize_act(p, 64, None, 2, 60, None, p, f(1e-5), 0, None, None, None, p, p, None) == B.EUNSUPPORTED
    assert L.sqap_rmsnorm_quantize_act(p, 72, None, 2, 72, None, p, f(1e-5), 1, None, None, None, p, p, None) == B.EUNSUPPORTED
    assert L.sqap_rmsnorm_quantize_act(None, 64, None, 0, 64, None, None, f(0.0), 0, None, None, None, None, None, None) == B.OK
    assert L.sqap_swiglu_quantize_act(p, 64, p, 32, 2, 64, None, None, p, p, None) == B.EINVAL
    assert L.sqap_swiglu_quantize_act(p, 64, None, 64, 2, 64, None, None, p, p, None) == B.EINVAL
    assert L.sqap_swiglu_quantize_act(p, 64, ctypes.c_void_p(4100), 64, 2, 64, None, None, p, p, None) == B.EUNSUPPORTED
    assert L.sqap_rope(p, 64, p, 2, 2, 33, ctypes.c_double(1e4), None) == B.EINVAL
    assert L.sqap_rope(p, 32, p, 2, 2, 32, ctypes.c_double(1e4), None) == B.EINVAL
    assert L.sqap_rope(None, 64, None, 0, 2, 32, ctypes.c_double(1e4), None) == B.OK
    assert L.sqap_rope_append(p, 64, p, 2, 2, 32, ctypes.c_double(1e4), p, 128, None) == B.EINVAL      # q|k|v pitch below 3 H d
    assert L.sqap_rope_append(p, 192, p, 2, 2, 32, ctypes.c_double(1e4), p, 64, None) == B.EINVAL      # cache pitch below 2 H d
    assert L.sqap_rope_append(p, 192, p, 2, 2, 32, ctypes.c_double(1e4), None, 128, None) == B.EINVAL
    assert L.sqap_rope_append(None, 192, None, 0, 2, 32, ctypes.c_double(1e4), None, 128, None) == B.OK
    assert L.sqap_attention(p, 64, p, 64, p, 64, 1, 5, 4, 1, 64, p, 64, None) == B.EINVAL
    assert L.sqap_attention(p, 64, p, 64, p, 32, 1, 4, 4, 1, 64, p, 64, None) == B.EINVAL       # pitch below H * d
    assert L.sqap_attention(p, 48, p, 48, p, 48, 1, 4, 4, 1, 48, p, 48, None) == B.EUNSUPPORTED
    assert L.sqap_attention(None, 64, None, 64, None, 64, 2, 0, 4, 1, 64, None, 64, None) == B.OK
    assert L.sqap_attention(p, 64, p, 64, p, 64, -1, 4, 4, 1, 64, p, 64, None) == B.EINVAL
    dbl = ctypes.c_double
    args = lambda **kw: [kw.get(k, v) for k, v in (("QKV", p), ("pos", p), ("H", 2), ("d", 64), ("base", dbl(1e4)), ("KV", p),
                                                    ("ldkv", 256), ("past", 3), ("O", p), ("Xq", None), ("sx", None),
                                                    ("counter", None), ("stream", None))]
    assert L.sqap_decode_attention(*args(H=0)) == B.EINVAL
    assert L.sqap_decode_attention(*args(past=-1)) == B.EINVAL
    assert L.sqap_decode_attention(*args(ldkv=248)) == B.EINVAL                               # pitch below 2 H d
    assert L.sqap_decode_attention(*args(base=dbl(0.0))) == B.EINVAL
    assert L.sqap_decode_attention(*args(O=None)) == B.EINVAL
    assert L.sqap_decode_attention(*args(Xq=p, sx=p)) == B.EINVAL                             # quantizer without its counter
    assert L.sqap_decode_attention(*args(d=60, ldkv=240)) == B.EUNSUPPORTED
    assert L.sqap_decode_attention(*args(d=136, ldkv=544)) == B.EUNSUPPORTED
    assert L.sqap_decode_attention(*args(KV=ctypes.c_void_p(4104))) == B.EUNSUPPORTED
    assert L.sqap_decode_attention(*args(H=128, d=128, ldkv=32768, Xq=p, sx=p, counter=p)) == B.EUNSUPPORTED
    assert L.sqap_residual_add(p, 64, p, 32, 2, 64, None) == B.EINVAL
    assert L.sqap_residual_add(p, 68, p, 68, 2, 68, None) == B.EUNSUPPORTED


def test_group_info_validation():
    L = B.lib()
    v = ctypes.c_int32(0)
    assert L.sqap_group_info(None, 0, ctypes.byref(v), None, None, None, None) == B.EINVAL
    junk = (ctypes.c_uint8 * 64)()
    assert L.sqap_group_info(ctypes.cast(junk, ctypes.c_void_p), 256, None, None, None, None, None) == B.EINVAL
    assert b"group" in L.sqap_last_error()


def test_persistent_switch_is_host_only():
    L = B.lib()
    assert L.sqap_set_persistent_kernels(0) == B.OK
    assert L.sqap_set_persistent_kernels(1) == B.OK


def test_mid_m_switch_is_host_only():
    L = B.lib()
    assert L.sqap_set_mid_m_kernel(0) == B.OK
    assert L.sqap_set_mid_m_kernel(1) == B.OK


def test_decoder_validation():
    """Everything sqap_decoder_* can refuse without a device: null pointers, handles that are not handles."""
    L = B.lib()
    out = ctypes.c_void_p(1)
    junk = (ctypes.c_uint8 * 256)()
    jp = ctypes.cast(junk, ctypes.c_void_p)
    layer = B.DecoderLayer()
    assert L.sqap_decoder_create(None, 1, 4, 64, jp, jp, 1e-5, 10000.0, ctypes.byref(out)) == B.EINVAL
    assert out.value is None                                                       # cleared on failure
    assert L.sqap_decoder_create(ctypes.byref(layer), 1, 4, 64, jp, jp, 1e-5, 10000.0, None) == B.EINVAL
    assert L.sqap_decoder_create(ctypes.byref(layer), 1, 4, 64, jp, jp, -1.0, 10000.0, ctypes.byref(out)) == B.EINVAL
    assert L.sqap_decoder_create(ctypes.byref(layer), 1, 4, 64, jp, jp, 1e-5, 0.0, ctypes.byref(out)) == B.EINVAL
    # the head is not a weight handle (zeroed memory carries no magic)
    assert L.sqap_decoder_create(ctypes.byref(layer), 1, 4, 64, jp, jp, 1e-5, 10000.0, ctypes.byref(out)) == B.EINVAL
    assert "head" in _err()
    word = ctypes.c_uint64(0)
    assert L.sqap_decoder_step(jp, jp, jp, 0, jp, None, None) == B.EINVAL and "decoder handle" in _err()
    assert L.sqap_decoder_step(None, jp, jp, 0, jp, None, None) == B.EINVAL
    assert L.sqap_decoder_status(jp, ctypes.byref(word), None) == B.EINVAL
    assert L.sqap_decoder_set_wait_limit(jp, 0) == B.EINVAL
    assert L.sqap_decoder_free(jp) == B.EINVAL
    assert L.sqap_decoder_free(None) == B.OK


def test_attn_scores_noalloc_validation():
    L = B.lib()
    one = ctypes.c_void_p(16)
    assert L.sqap_attn_scores_noalloc(None, None, 1, 8, 4, 64, 0, 4, None, None) == B.EINVAL
    # beyond the fixed scratch: rejected before anything is launched
    assert L.sqap_attn_scores_noalloc(one, one, 65, 8, 4, 64, 0, 4, one, None) == B.EUNSUPPORTED
    assert L.sqap_attn_scores_noalloc(one, one, 64, 70000, 32, 128, 0, 65536, one, None) == B.EUNSUPPORTED


def test_selftest_dispatch_validation():
    assert B.lib().sqap_selftest_dispatch(None, None) == B.EINVAL


def test_prune_select_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    assert L.sqap_prune_select(p, 1, 16, 16, 300, 128, None, 1, p, 256, None, None) == B.EINVAL      # k_attn > tokens
    assert L.sqap_prune_select(p, 1, 16, 16, 64, 300, None, 1, p, 300, None, None) == B.EINVAL       # total > tokens
    assert L.sqap_prune_select(p, 1, 16, 16, 64, 128, None, 1, p, 100, None, None) == B.EINVAL and "cap" in _err()
    assert L.sqap_prune_select(p, 1, 16, 16, 64, 70, p, 2, p, 70, None, None) == B.EINVAL            # ring may not fit
    assert L.sqap_prune_select(p, 1, 40, 40, 64, 128, None, 1, p, 1600, None, None) == B.EUNSUPPORTED
    assert L.sqap_prune_select(p, 1, 0, 16, 0, 0, None, 1, p, 16, None, None) == B.EINVAL
    assert L.sqap_prune_select(p, 1, 16, 16, 64, 128, None, -1, p, 256, None, None) == B.EINVAL
    assert L.sqap_prune_select(None, 1, 16, 16, 64, 128, None, 1, p, 256, None, None) == B.EINVAL
    assert L.sqap_prune_select(None, 0, 16, 16, 64, 128, None, 1, None, 256, None, None) == B.OK     # empty batch


def test_channelwise_validation():
    L = B.lib()
    p = ctypes.c_void_p(4096)
    assert L.sqap_channel_scales(p, 16, None, 4, 16, 0, None, 0, p, None) == B.EINVAL             # no amax buffer
    assert L.sqap_channel_scales(p, 8, None, 4, 16, 0, p, 0, p, None) == B.EINVAL                 # pitch < K
    assert L.sqap_channel_scales(p, 24, None, 4, 24, 1, p, 0, p, None) == B.EUNSUPPORTED          # rotate, K not 2^n
    assert L.sqap_channel_scales(None, 16, None, 4, 16, 0, p, 0, p, None) == B.EINVAL
    assert L.sqap_quantize_act_channelwise(p, 16, None, 4, 16, 0, None, p, p, None) == B.EINVAL   # no scales
    assert L.sqap_quantize_act_channelwise(p, 16, None, 4, 16, 4, p, p, p, None) == B.EINVAL      # unknown flag
    assert L.sqap_quantize_act_channelwise(p, 16, None, 4, 16, 0, ctypes.c_void_p(4104), p, p, None) == B.EUNSUPPORTED
    assert L.sqap_quantize_act_channelwise(p, 16, None, 0, 16, 0, p, None, None, None) == B.OK    # no rows
    assert L.sqap_quantize_weight_folded(p, 4, 15, 0, p, p, p, None) == B.EINVAL                  # odd K
    assert L.sqap_quantize_weight_folded(p, 4, 16, 0, p, None, p, None) == B.EINVAL
    assert L.sqap_quantize_weight_folded(p, 0, 16, 0, p, None, None, None) == B.OK


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_product_package_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import or load it."""
    pkg = os.path.join(ROOT, "paper_2509_09090_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "sqap_oracle" not in text, f


# ------------------------------------------------------------------ work split of the large-M linear (host logic)
def _play_protocol(bounds, nb, ntile, steps):
    """Walks every workgroup of one XCD through the kernel's visit order; returns (owner of every step,
    partials published, partials waited for)."""
    owner, published, waited = {}, [], []
    for j in range(nb):
        b, e = bounds[j], bounds[j + 1]
        if b >= e:
            continue
        t_first, t_last = b // steps, (e - 1) // steps
        assert 0 <= t_first <= t_last < ntile
        tl = t_last
        seg = lambda tl: (tl * steps, min(max(b - tl * steps, 0), steps), min(max(e - tl * steps, 0), steps))
        tb, s0, s1 = seg(tl)
        if s1 < steps:
            tl -= 1
            if s0 < s1:
                for s in range(s0, s1):
                    assert (t_last, s) not in owner
                    owner[(t_last, s)] = j
                published.append((j, t_last))
        while tl >= t_first:
            tb, s0, s1 = seg(tl)
            if s0 < s1:
                assert s1 == steps
                for s in range(s0, s1):
                    assert (tl, s) not in owner
                    owner[(tl, s)] = j
                if s0 > 0:
                    for jj in range(j):
                        jb, je = bounds[jj], bounds[jj + 1]
                        if jb < je and je > tb and jb < tb + s0:
                            waited.append((jj, tl))
            tl -= 1
    return owner, published, waited


@pytest.mark.parametrize("M,N,K,nb", [(2368, 11008, 4096, 32), (2368, 4096, 11008, 32), (2368, 22016, 4096, 32),
                                      (2560, 11008, 4096, 32), (600, 768, 1024, 32), (513, 544, 640, 32),
                                      (2368, 4096, 4096, 32), (700, 300, 128, 32), (5000, 512, 256, 13),
                                      (1024, 32000, 4096, 32), (2432, 4096, 2048, 7), (736, 256, 12800, 32),
                                      # narrow tiles (a few hundred token rows)
                                      (84, 12288, 4096, 32), (276, 22016, 4096, 32), (148, 11008, 4096, 32),
                                      (199, 4096, 11008, 32), (9, 64, 128, 32), (511, 4096, 4096, 5)])
def test_planned_shares_follow_the_kernel_protocol(M, N, K, nb):
    bounds, planned, even, (bm, bn) = B.sqap_plan_linear_shares(M, N, K, nb)
    assert (bm, bn) == ((256, 256) if M >= 512 else (160 if -(-M // 160) * 160 <= -(-M // 96) * 96 else 96, 128))
    m_tiles, n_tiles, steps = -(-M // bm), -(-N // bn), K // 128
    tiles = m_tiles * n_tiles
    q, r = divmod(tiles, 8)
    for x in range(8):
        ntile = q + (1 if x < r else 0)
        b = bounds[x]
        assert b[0] == 0 and all(b[j] <= b[j + 1] for j in range(32)), b
        assert all(v == ntile * steps for v in b[nb:]), b          # covers the run; unused entries repeat the total
        owner, published, waited = _play_protocol(b, nb, ntile, steps)
        assert len(owner) == ntile * steps                         # every step has exactly one owner
        assert sorted(published) == sorted(waited)                 # every partial is consumed exactly once
        assert len(set(waited)) == len(waited)
        # a workgroup publishes at most one partial (it owns one slot), and a finisher's contributors number < 32
        assert len({j for j, _ in published}) == len(published)
    assert max(planned) <= max(even) + 1e-9                        # never worse than equal step counts, by the model


def test_plan_linear_shares_validation():
    ok = ((ctypes.c_uint32 * 264)(), (ctypes.c_double * 8)(), (ctypes.c_double * 8)(), ctypes.byref(ctypes.c_int32(0)),
          ctypes.byref(ctypes.c_int32(0)))
    L = B.lib()
    assert L.sqap_plan_linear_shares(2368, 4096, 4096, 32, None, *ok[1:]) == B.EINVAL
    assert L.sqap_plan_linear_shares(2368, 4096, 4096, 0, *ok) == B.EINVAL
    assert L.sqap_plan_linear_shares(2368, 4096, 4096, 33, *ok) == B.EINVAL
    assert L.sqap_plan_linear_shares(0, 4096, 4096, 32, *ok) == B.EINVAL
    assert L.sqap_plan_linear_shares(8, 4096, 4096, 32, *ok) == B.EUNSUPPORTED
    assert L.sqap_plan_linear_shares(2368, 4096, 4000, 32, *ok) == B.EUNSUPPORTED


def test_planned_shares_random_shapes():
    """The same walk over seeded random shapes (small, so that many fit in the time budget)."""
    import random
    rnd = random.Random(2024)
    for _ in range(150):
        M = rnd.choice([9, 84, 148, 276, 511, 512, 513, 544, 600, 736, 768, 1000, 1025, 2368, 4096, rnd.randint(9, 6000)])
        N = rnd.choice([32, 256, 300, 768, 4096, 11008, rnd.randint(1, 20000)])
        K = 128 * rnd.choice([1, 2, 3, 5, 8, 32, 86, rnd.randint(1, 100)])
        nb = rnd.choice([32, 32, 32, 1, 2, 7, 13, 31])
        bounds, planned, even, (bm, bn) = B.sqap_plan_linear_shares(M, N, K, nb)
        m_tiles, n_tiles, steps = -(-M // bm), -(-N // bn), K // 128
        q, r = divmod(m_tiles * n_tiles, 8)
        for x in range(8):
            ntile = q + (1 if x < r else 0)
            b = bounds[x]
            assert b[0] == 0 and all(b[j] <= b[j + 1] for j in range(32)), (M, N, K, nb, b)
            assert all(v == ntile * steps for v in b[nb:]), (M, N, K, nb, b)
            owner, published, waited = _play_protocol(b, nb, ntile, steps)
            assert len(owner) == ntile * steps, (M, N, K, nb)
            assert sorted(published) == sorted(waited), (M, N, K, nb)
            assert len({j for j, _ in published}) == len(published), (M, N, K, nb)
        assert max(planned) <= max(even) + 1e-9, (M, N, K, nb)
