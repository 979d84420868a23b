"""Pins for the CPU oracle: it is checked against things other than itself
(library routines, closed forms, brute force, fixed values) so that a dropped
term, a wrong sign or index, or a transposed operand fails here.  No GPU."""
import itertools
import os

import numpy as np
import pytest
import scipy.linalg
import scipy.special

from paper_2509_09090_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ------------------------------------------------------------------ half
def test_f16_to_f32_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_golden_cases(oracle):
    with open(os.path.join(GOLDEN, "half_rounding_cases.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, b = line.split()[:2]
            x = np.array([int(a, 16)], dtype=np.uint32).view(np.float32)[0]
            assert oracle.f32_to_f16(float(x)) == int(b, 16), line


def test_f32_to_f16_matches_numpy(oracle):
    rng = np.random.default_rng(1)
    # random bit patterns around the half range plus every half value +- 1 float ulp
    xs = [rng.standard_normal(20000).astype(np.float32) * np.float32(s)
          for s in (1e-7, 1e-5, 1e-3, 1.0, 300.0, 40000.0)]
    h = np.arange(0x7c00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = ((h[:-1].astype(np.float64) + h[1:].astype(np.float64)) / 2).astype(np.float32)
    xs += [h, -h, mids, np.nextafter(mids, np.float32(np.inf)),
           np.nextafter(mids, np.float32(-np.inf))]
    x = np.concatenate(xs)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ top-k
def _library_topk(s, k):
    """Stable library sort on descending score: ties keep the lower index first,
    NaN sorts last."""
    order = np.argsort(-s.astype(np.float64), kind="stable")
    return np.sort(order[:k]).astype(np.int32)


def _rank_brute(s, k):
    """Brute force from the definition of the total order (O(n^2))."""
    n = len(s)
    kept = []
    for i in range(n):
        ahead = 0
        for j in range(n):
            if j == i:
                continue
            si, sj = s[i], s[j]
            if np.isnan(sj):
                before = np.isnan(si) and j < i
            elif np.isnan(si):
                before = True
            else:
                before = sj > si or (sj == si and j < i)
            ahead += bool(before)
        if ahead < k:
            kept.append(i)
    return np.array(kept, dtype=np.int32)


@pytest.mark.parametrize("n,k", [(1, 0), (1, 1), (7, 3), (64, 32), (256, 128), (256, 64),
                                 (256, 0), (256, 256), (255, 254), (300, 1), (1000, 17)])
def test_topk_random_vs_stable_sort(oracle, n, k):
    rng = np.random.default_rng(n * 1000 + k)
    s = rng.random((5, n), dtype=np.float32)
    got = oracle.prune_topk(s, k)
    assert got.shape == (5, k)
    for b in range(5):
        assert np.array_equal(got[b], _library_topk(s[b], k))


def test_topk_adversarial(oracle):
    n = 64
    cases = {
        "all_equal": np.full(n, 0.5, np.float32),
        "two_valued": np.tile(np.array([1.0, 0.0], np.float32), n // 2),
        "descending": np.linspace(1, 0, n).astype(np.float32),
        "ascending": np.linspace(0, 1, n).astype(np.float32),
        "dups_at_cut": np.repeat(np.arange(n // 4, dtype=np.float32), 4),
        "signed_zero": np.array([0.0, -0.0] * (n // 2), np.float32),
        "with_nan": np.where(np.arange(n) % 5 == 0, np.nan, np.arange(n) % 7).astype(np.float32),
        "all_nan": np.full(n, np.nan, np.float32),
        "infs": np.array([np.inf, -np.inf, 1.0, np.inf] * (n // 4), np.float32),
        "negatives": -np.arange(n, dtype=np.float32),
    }
    for name, s in cases.items():
        for k in (0, 1, 2, 31, 32, 33, n - 1, n):
            got = oracle.prune_topk(s, k)
            assert np.array_equal(got, _library_topk(s, k)), (name, k)
            assert np.array_equal(got, _rank_brute(s, k)), (name, k)


def test_topk_invariants(oracle):
    rng = np.random.default_rng(3)
    s = np.round(rng.random((8, 256)) * 20).astype(np.float32) / 20   # many duplicates
    k = 100
    got = oracle.prune_topk(s, k)
    for b in range(8):
        idx = got[b]
        assert len(idx) == k and np.all(np.diff(idx) > 0)
        dropped = np.setdiff1d(np.arange(256), idx)
        assert s[b, idx].min() >= s[b, dropped].max()
        cut = s[b, idx].min()
        kept_at_cut = idx[s[b, idx] == cut]
        dropped_at_cut = dropped[s[b, dropped] == cut]
        if len(dropped_at_cut):
            assert kept_at_cut.max() < dropped_at_cut.min()


def test_topk_all_equal_keeps_prefix(oracle):
    assert np.array_equal(oracle.prune_topk(np.zeros(10, np.float32), 4), np.arange(4))


def test_topk_rejects_keep_above_n(oracle):
    with pytest.raises(ValueError):
        oracle.prune_topk(np.zeros(4, np.float32), 5)


# ------------------------------------------------------------------ ring, FPS, final set (Eq. 2-5)
def _fixture_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield [int(v) for v in line.split()]


def test_ring_counts_match_the_hand_counted_fixture(oracle):
    for cx, cy, R, count in _fixture_rows("chebyshev_ball_counts.txt"):
        assert int(oracle.ring(16, 16, cx, cy, R).sum()) == count, (cx, cy, R)


def test_ring_membership_is_the_chebyshev_ball(oracle):
    """Every cell, against max(|du|, |dv|) written with numpy broadcasting; non-square grids and
    centres outside the grid included (a transposed grid or an L1/L2 ball fails here)."""
    for gw, gh, cu, cv, R in [(16, 16, 5, 9, 3), (7, 3, 6, 0, 2), (3, 7, 0, 6, 2), (16, 16, -2, 4, 3),
                              (16, 16, 20, 20, 5), (4, 4, 1, 1, 0), (5, 9, 2, 4, 50)]:
        u, v = np.meshgrid(np.arange(gw), np.arange(gh))              # row-major: index = v * gw + u
        want = (np.maximum(np.abs(u - cu), np.abs(v - cv)) <= R).astype(np.uint8).reshape(-1)
        assert np.array_equal(oracle.ring(gw, gh, cu, cv, R), want), (gw, gh, cu, cv, R)
    # a diagonal neighbour is in the radius-1 ball (it is not in the L1 ball)
    assert oracle.ring(16, 16, 8, 8, 1)[9 * 16 + 9] == 1


def test_fps_hand_worked_sequence(oracle):
    rows = list(_fixture_rows("fps_4x4_worked.txt"))
    kept = np.zeros(16, np.uint8)
    kept[0] = 1
    picks = oracle.fps(4, 4, kept, len(rows))
    assert [int(p) for p in picks] == [r[1] for r in rows]


def _fps_numpy(gw, gh, kept, m):
    """Independent statement of farthest point sampling: a running minimum-distance array
    updated after every pick (the oracle recomputes all minima from scratch instead)."""
    n = gw * gh
    xy = np.stack([np.arange(n) % gw, np.arange(n) // gw], axis=1).astype(np.int64)
    kept = kept.astype(bool).copy()
    big = np.iinfo(np.int64).max
    mind = np.full(n, big)
    for s in np.flatnonzero(kept):
        mind = np.minimum(mind, ((xy - xy[s]) ** 2).sum(axis=1))
    picks = []
    for _ in range(m):
        cand = np.where(kept, -1, mind)
        best = int(np.argmax(cand))                 # argmax returns the first (lowest) index among equals
        picks.append(best)
        kept[best] = True
        mind = np.minimum(mind, ((xy - xy[best]) ** 2).sum(axis=1))
    return picks


def test_fps_vs_running_minimum_formulation(oracle):
    rng = np.random.default_rng(5)
    for gw, gh in [(4, 4), (8, 8), (5, 3), (3, 6), (16, 16), (1, 9)]:
        n = gw * gh
        for trial in range(4):
            kept = (rng.random(n) < (0.0, 0.1, 0.3, 0.6)[trial]).astype(np.uint8)
            free = int(n - kept.sum())
            for m in sorted({0, 1, free // 2, free}):
                got = [int(p) for p in oracle.fps(gw, gh, kept, m)]
                assert got == _fps_numpy(gw, gh, kept, m), (gw, gh, trial, m)


def test_fps_each_pick_maximises_the_distance_to_the_kept_set(oracle):
    """The defining property, checked pick by pick with brute-force distances."""
    rng = np.random.default_rng(6)
    gw, gh = 6, 5
    n = gw * gh
    kept = np.zeros(n, bool)
    kept[rng.choice(n, 4, replace=False)] = True
    picks = oracle.fps(gw, gh, kept.astype(np.uint8), 10)
    assert len(set(int(p) for p in picks)) == 10 and not kept[picks].any()
    cur = kept.copy()
    for p in picks:
        dist = {c: min((c % gw - s % gw) ** 2 + (c // gw - s // gw) ** 2 for s in np.flatnonzero(cur))
                for c in np.flatnonzero(~cur)}
        top = max(dist.values())
        assert dist[int(p)] == top and int(p) == min(c for c, d in dist.items() if d == top)
        cur[p] = True


def test_fps_from_an_empty_set_starts_at_token_zero_and_rejects_too_many(oracle):
    assert [int(p) for p in oracle.fps(4, 4, np.zeros(16, np.uint8), 2)] == [0, 15]
    with pytest.raises(ValueError):
        oracle.fps(2, 2, np.array([1, 1, 1, 0], np.uint8), 2)


def test_projection_closed_forms(oracle):
    """Eq. 2-3 on cases whose answer is known without multiplying matrices by machine."""
    Kmat = np.array([[100.0, 0, 112], [0, 100, 112], [0, 0, 1]])
    ident = np.hstack([np.eye(3), np.zeros((3, 1))])
    # pinhole, identity pose: u = fx x/z + cx, v = fy y/z + cy
    assert oracle.project_token(Kmat, ident, [1, 2, 4], 14, 14) == ((25 + 112) // 14, (50 + 112) // 14)
    # the optical axis lands on the principal point, patch (8, 8) of a 16 x 16 grid of 14-pixel patches
    assert oracle.project_token(Kmat, ident, [0, 0, 3], 14, 14) == (8, 8)
    # a quarter turn about the optical axis takes (x, y, z) to (-y, x, z)
    rot = np.hstack([np.array([[0.0, -1, 0], [1, 0, 0], [0, 0, 1]]), np.zeros((3, 1))])
    assert oracle.project_token(Kmat, rot, [1, 2, 4], 14, 14) == ((-50 + 112) // 14, (25 + 112) // 14)
    # a translation adds to the camera-frame point before the division
    tr = np.hstack([np.eye(3), np.array([[0.5], [0.0], [1.0]])])
    assert oracle.project_token(Kmat, tr, [1, 2, 4], 14, 14) == (int(np.floor((100 * 1.5 / 5 + 112) / 14)),
                                                                  int(np.floor((100 * 2 / 5 + 112) / 14)))
    # unequal patch sizes, and floor (not truncation) left of / above the image
    assert oracle.project_token(Kmat, ident, [1, 2, 4], 7, 28) == ((25 + 112) // 7, (50 + 112) // 28)
    assert oracle.project_token(np.array([[100.0, 0, 0], [0, 100, 0], [0, 0, 1]]), ident, [-0.01, -3, 2], 14, 14) \
        == (-1, -11)
    # behind or on the camera plane: no token
    assert oracle.project_token(Kmat, ident, [1, 2, -4], 14, 14) is None
    assert oracle.project_token(Kmat, ident, [1, 2, 0], 14, 14) is None


def test_projection_matches_homogeneous_matrix_product(oracle):
    rng = np.random.default_rng(8)
    for _ in range(200):
        Kmat = np.array([[rng.uniform(50, 400), 0, rng.uniform(50, 200)], [0, rng.uniform(50, 400), rng.uniform(50, 200)],
                         [0, 0, 1]])
        q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
        Rt = np.hstack([q, rng.standard_normal((3, 1))])
        p = rng.standard_normal(3) * 2
        h = Kmat @ Rt @ np.append(p, 1.0)
        got = oracle.project_token(Kmat, Rt, p, 14.0, 14.0)
        if h[2] <= 0:
            assert got is None
            continue
        u, v = h[0] / h[2] / 14.0, h[1] / h[2] / 14.0
        if min(abs(u - round(u)), abs(v - round(v))) < 1e-9:       # too close to a patch border to call
            continue
        assert got == (int(np.floor(u)), int(np.floor(v)))


def test_final_set_is_the_union_with_the_quota_filled_by_fps(oracle):
    rng = np.random.default_rng(9)
    for gw, gh, k_attn, total, centre, R in [(16, 16, 64, 128, (5, 9), 2), (16, 16, 0, 40, (0, 0), 1),
                                             (16, 16, 100, 128, None, 0), (8, 8, 10, 30, (7, 7), 3),
                                             (16, 16, 128, 128, (8, 8), 1), (6, 4, 5, 24, (2, 2), 1)]:
        n = gw * gh
        s = rng.random(n).astype(np.float32)
        attn = _library_topk(s, k_attn)
        kept = np.zeros(n, np.uint8)
        kept[attn] = 1
        if centre is not None:
            u, v = np.meshgrid(np.arange(gw), np.arange(gh))
            kept |= (np.maximum(np.abs(u - centre[0]), np.abs(v - centre[1])) <= R).astype(np.uint8).reshape(-1)
        base = int(kept.sum())
        m = max(0, total - base)
        want = set(np.flatnonzero(kept)) | set(_fps_numpy(gw, gh, kept, m))
        got = oracle.prune_select(s, gw, gh, k_attn, total, centre, R)
        assert list(got) == sorted(want)
        assert len(got) == max(total, base)            # the union is never cut; the quota only adds


def test_final_set_special_cases(oracle):
    s = np.linspace(1, 0, 256).astype(np.float32)
    # no ring, no quota left: exactly Eq. 1
    assert np.array_equal(oracle.prune_select(s, 16, 16, 128, 128), np.arange(128))
    # ring overlapping the attention set is not counted twice
    got = oracle.prune_select(s, 16, 16, 16, 16, (0, 0), 1)            # ring {0,1,16,17}; 0 and 1 already in the top row
    assert list(got) == list(range(16)) + [16, 17]
    # everything kept
    assert np.array_equal(oracle.prune_select(s, 16, 16, 0, 256), np.arange(256))
    with pytest.raises(ValueError):
        oracle.prune_select(s, 16, 16, 257, 128)


# ------------------------------------------------------------------ rows / gather
def test_kept_rows_and_gather(oracle):
    rng = np.random.default_rng(4)
    B, S, v0, nv, k = 3, 30, 4, 16, 5
    idx = np.stack([np.sort(rng.choice(nv, k, replace=False)) for _ in range(B)]).astype(np.int32)
    rows = oracle.kept_rows(idx, S, v0, nv)
    assert rows.size == B * (S - nv + k)
    assert np.all(np.diff(rows) > 0)                      # original order kept
    for b in range(B):
        mine = rows[(rows >= b * S) & (rows < (b + 1) * S)] - b * S
        text = np.concatenate([np.arange(0, v0), np.arange(v0 + nv, S)])
        want = np.sort(np.concatenate([text, idx[b] + v0]))
        assert np.array_equal(mine, want)
    X = rng.standard_normal((B * S, 12)).astype(np.float16)
    out = oracle.gather_rows(X, rows)
    assert np.array_equal(out.view(np.uint16), X[rows].view(np.uint16))


# ------------------------------------------------------------------ Hadamard
def test_sylvester_fixture_is_what_scipy_builds():
    H = np.loadtxt(os.path.join(GOLDEN, "sylvester_h8.txt"))
    assert np.array_equal(H, scipy.linalg.hadamard(8))


def test_fwht_matches_fixture_matrix(oracle):
    H = np.loadtxt(os.path.join(GOLDEN, "sylvester_h8.txt"))
    rng = np.random.default_rng(5)
    x = rng.standard_normal(8)
    got = oracle.fwht(x)
    assert np.allclose(got, H @ x.astype(np.float32).astype(np.float64) / np.sqrt(8), atol=1e-6)


@pytest.mark.parametrize("K", [1, 2, 4, 16, 64, 512, 4096])
def test_fwht_vs_dense_product(oracle, K):
    rng = np.random.default_rng(K)
    x = rng.standard_normal(K).astype(np.float32)
    want = scipy.linalg.hadamard(K).astype(np.float64) @ x.astype(np.float64) / np.sqrt(K)
    got = oracle.fwht(x)
    assert np.allclose(got, want, atol=2e-5 * np.sqrt(np.log2(K) + 1))
    # involution (H/sqrt K is symmetric orthogonal) and Parseval
    assert np.allclose(oracle.fwht(got), x, atol=1e-4)
    assert np.isclose(np.linalg.norm(got.astype(np.float64)), np.linalg.norm(x.astype(np.float64)),
                      rtol=1e-5)


def test_fwht_unit_vectors(oracle):
    K = 64
    H = scipy.linalg.hadamard(K)
    for j in (0, 1, 5, 63):
        e = np.zeros(K, np.float32)
        e[j] = 1
        assert np.array_equal(oracle.fwht(e), (H[:, j] / 8.0).astype(np.float32))


def test_fwht_rejects_non_power_of_two(oracle):
    with pytest.raises(ValueError):
        oracle.fwht(np.zeros(12, np.float32))


def test_rotation_of_other_lengths_is_block_diagonal(oracle):
    """Lengths that are not a power of two: one orthonormal Sylvester block per aligned run of B channels, B the
    largest power of two dividing K; the whole matrix for a power of two."""
    assert [oracle.rotation_block(K) for K in (4096, 11008, 1536, 2056, 96, 7)] == [4096, 256, 512, 8, 32, 1]
    rng = np.random.default_rng(31)
    v = rng.standard_normal(512).astype(np.float32)
    assert np.array_equal(oracle.rotate(v).view(np.uint32), oracle.fwht(v).view(np.uint32))
    for K in (96, 192, 1536):
        B = oracle.rotation_block(K)
        v = (rng.standard_normal(K) * 3).astype(np.float32)
        dense = scipy.linalg.block_diag(*([scipy.linalg.hadamard(B) / np.sqrt(B)] * (K // B)))
        want = dense @ v.astype(np.float64)
        got = oracle.rotate(v).astype(np.float64)
        assert np.all(np.abs(got - want) <= 1e-5 * np.abs(v).max() * np.log2(B))
        assert abs(np.linalg.norm(got) - np.linalg.norm(v.astype(np.float64))) <= 1e-5 * np.linalg.norm(v)   # orthonormal
        # an impulse stays inside its block
        e = np.zeros(K, np.float32)
        e[B + 3] = 1.0
        out = oracle.rotate(e)
        assert np.all(out[:B] == 0) and np.all(out[2 * B:] == 0) and np.all(np.abs(out[B:2 * B]) == np.float32(1 / np.sqrt(B)))
    # Eq. 6: rotating the weight rows and the activation row leaves the product unchanged
    K, N = 192, 7
    W = rng.standard_normal((N, K)).astype(np.float32)
    x = rng.standard_normal(K).astype(np.float32)
    Wr = np.stack([oracle.rotate(w) for w in W]).astype(np.float64)
    assert np.allclose(Wr @ oracle.rotate(x).astype(np.float64), W.astype(np.float64) @ x.astype(np.float64), atol=1e-4)
    # the quantizer takes such rows, and refuses blocks too small to rotate in registers (B < 16)
    X = (rng.standard_normal((3, 192))).astype(np.float16)
    q, s, _ = oracle.quantize_rows(X, rotate=True)
    vr = oracle.rotate(X[1].astype(np.float32))
    assert s[1] == np.float16(np.abs(vr).max() / np.float32(7.0))
    with pytest.raises(ValueError):
        oracle.quantize_rows(np.zeros((1, 2056), np.float16), rotate=True)


def test_rotation_leaves_the_linear_unchanged(oracle):
    """Eq. 6: (W H^T)(H x) = W x with the orthonormal H."""
    rng = np.random.default_rng(6)
    K, N = 256, 8
    x = rng.standard_normal(K).astype(np.float32)
    W = rng.standard_normal((N, K)).astype(np.float32)
    xr = oracle.fwht(x).astype(np.float64)
    Wr = np.stack([oracle.fwht(W[n]) for n in range(N)]).astype(np.float64)
    assert np.allclose(Wr @ xr, W.astype(np.float64) @ x.astype(np.float64), atol=1e-3)


# ------------------------------------------------------------------ quantizer
def _codes(oracle, q):
    return oracle.unpack_int4(q).astype(np.int32)


def test_unpack_layout_low_nibble_first(oracle):
    q = np.array([[0x21, 0xF8, 0x7F]], dtype=np.uint8)
    assert np.array_equal(oracle.unpack_int4(q), [[1, 2, -8, -1, -1, 7]])


def test_quantizer_error_bound_and_range(oracle):
    X, _ = wl.activations(64, 512, 4, 20.0, np.random.default_rng(7))
    q, s, rs = oracle.quantize_rows(X)
    c = _codes(oracle, q)
    sf = s.astype(np.float64)[:, None]
    err = np.abs(c * sf - X.astype(np.float64))
    assert np.all(err <= sf / 2 * (1 + 1e-6))
    assert c.min() >= -7 and c.max() <= 7
    amax_pos = np.argmax(np.abs(X.astype(np.float32)), axis=1)
    assert np.all(np.abs(c[np.arange(64), amax_pos]) == 7)
    assert np.array_equal(rs, c.sum(axis=1))
    # the scale is the half nearest to amax/7
    amax = np.abs(X.astype(np.float32)).max(axis=1)
    assert np.array_equal(s.view(np.uint16), (amax / np.float32(7)).astype(np.float16).view(np.uint16))


def test_quantizer_clamp_reaches_minus_eight_only_below_the_normal_scales(oracle):
    """Code -8 exists in the format but the divisor 7 never asks for it; it appears only where the scale has
    too few bits: amax = 10 * 2^-24 gives the scale 2^-24 (10/7 rounds to one subnormal unit), v / s = -10."""
    u = 2.0 ** -24
    X = np.array([[-10 * u, 10 * u, -7 * u, 3 * u]], dtype=np.float16)
    q, s, _ = oracle.quantize_rows(X)
    assert s.view(np.uint16)[0] == 1
    assert list(oracle.unpack_int4(q)[0]) == [-8, 7, -7, 3]
    # in the normal range of scales the most negative code is -7
    rng = np.random.default_rng(17)
    Xn = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-6, 6, (64, 1)))).astype(np.float16)
    assert oracle.unpack_int4(oracle.quantize_rows(Xn)[0]).min() == -7


def test_quantizer_sign_symmetry_and_power_of_two_scaling(oracle):
    X, _ = wl.activations(16, 128, 2, 20.0, np.random.default_rng(8))
    q, s, _ = oracle.quantize_rows(X)
    qn, sn, _ = oracle.quantize_rows(-X)
    assert np.array_equal(_codes(oracle, qn), -_codes(oracle, q))
    assert np.array_equal(sn, s)
    for p in (-4, 3):                       # stays in the normal half range
        Xs = (X.astype(np.float32) * np.float32(2.0 ** p)).astype(np.float16)
        qs, ss, _ = oracle.quantize_rows(Xs)
        assert np.array_equal(_codes(oracle, qs), _codes(oracle, q))
        assert np.array_equal(ss.astype(np.float32), s.astype(np.float32) * np.float32(2.0 ** p))


def test_quantizer_every_finite_half_as_a_row(oracle):
    """Rows (x, 0) for every finite half x: error bound, +-7 mapping, symmetry."""
    bits = np.arange(0x7c00, dtype=np.uint16)
    x = bits.view(np.float16)
    X = np.stack([x, np.zeros_like(x)], axis=1)
    q, s, _ = oracle.quantize_rows(X)
    c = _codes(oracle, q)
    assert np.all(c[:, 1] == 0)
    sf = s.astype(np.float64)
    assert np.all(sf > 0)
    normal_scale = sf >= 2.0 ** -14
    assert np.all(c[normal_scale, 0] == 7)
    err = np.abs(c[:, 0] * sf - x.astype(np.float64))
    assert np.all(err[normal_scale] <= sf[normal_scale] / 2)
    # below the normal range the scale has few bits; the code is then clamped at 7
    assert np.all((c[:, 0] >= 0) & (c[:, 0] <= 7))
    assert c[0, 0] == 0 and bits[0] == 0 and s.view(np.uint16)[0] == 1   # all-zero row
    qn, sn, _ = oracle.quantize_rows(-X)
    # (the clamp range [-8, 7] is not symmetric, so only where no clamp bites)
    assert np.array_equal(_codes(oracle, qn)[normal_scale], -c[normal_scale])
    assert np.array_equal(sn, s)
    assert _codes(oracle, qn).min() >= -8


def test_quantizer_pairs_of_halves(oracle):
    """Rows (x, y) for sampled pairs: the smaller element obeys the error bound."""
    rng = np.random.default_rng(9)
    b = rng.integers(0x0400, 0x7bff, size=(20000, 2)).astype(np.uint16)
    b |= (rng.integers(0, 2, size=b.shape).astype(np.uint16) << 15)
    X = b.view(np.float16)
    q, s, _ = oracle.quantize_rows(X)
    c = _codes(oracle, q)
    sf = s.astype(np.float64)[:, None]
    ok = sf[:, 0] >= 2.0 ** -14
    err = np.abs(c * sf - X.astype(np.float64))
    assert np.all(err[ok] <= sf[ok] / 2 * (1 + 1e-6))
    assert np.all(np.abs(c).max(axis=1)[ok] == 7)


def test_quantizer_half_way_cases_round_to_even(oracle):
    # scale exactly 1 (amax 7): 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, -3.5 -> -4, 6.5 -> 6
    X = np.array([[7, 0.5, 1.5, 2.5, -3.5, 6.5, -0.5, 4.5]], dtype=np.float16)
    q, s, _ = oracle.quantize_rows(X)
    assert float(s[0]) == 1.0
    assert np.array_equal(_codes(oracle, q), [[7, 0, 2, 2, -4, 6, 0, 4]])


def test_quantizer_rows_argument_is_a_gather(oracle):
    X, _ = wl.activations(40, 64, 1, 20.0, np.random.default_rng(10))
    rows = np.array([5, 3, 39, 0, 5], dtype=np.int32)
    q1, s1, r1 = oracle.quantize_rows(X, rows=rows)
    q2, s2, r2 = oracle.quantize_rows(X[rows])
    assert np.array_equal(q1, q2) and np.array_equal(s1, s2) and np.array_equal(r1, r2)


def test_rotation_reduces_quantisation_error_on_outlier_channels(oracle):
    """Section 3.3: rotating spreads the outlier energy, so int4 error falls."""
    X, _ = wl.activations(32, 1024, 10, 30.0, np.random.default_rng(11))
    xf = X.astype(np.float64)
    q0, s0, _ = oracle.quantize_rows(X)
    e0 = np.linalg.norm(_codes(oracle, q0) * s0.astype(np.float64)[:, None] - xf)
    q1, s1, _ = oracle.quantize_rows(X, rotate=True)
    xr = np.stack([oracle.fwht(X[i].astype(np.float32)) for i in range(32)]).astype(np.float64)
    e1 = np.linalg.norm(_codes(oracle, q1) * s1.astype(np.float64)[:, None] - xr)
    assert e1 < 0.6 * e0        # norms are equal (orthonormal H), so errors compare directly
    with pytest.raises(ValueError):
        oracle.quantize_rows(X[:, :1000], rotate=True)


# ------------------------------------------------------------------ channel-wise activations (Section 3.3)
def test_channel_scales_are_the_column_maxima(oracle):
    """numpy's own half conversion and column reduction; a row-wise (per-token) maximum fails here."""
    rng = np.random.default_rng(21)
    X = (rng.standard_normal((37, 64)) * rng.uniform(0.01, 50, 64)).astype(np.float16)
    X[:, 5] = 0                                            # an all-zero channel gets the smallest scale
    want = (np.abs(X.astype(np.float32)).max(axis=0) / np.float32(7)).astype(np.float16)
    want[5] = np.float16(2.0 ** -24)
    assert np.array_equal(oracle.channel_scales(X).view(np.uint16), want.view(np.uint16))
    rows = np.array([3, 3, 20, 7], np.int32)
    want_r = (np.abs(X[rows].astype(np.float32)).max(axis=0) / np.float32(7)).astype(np.float16)
    want_r[5] = np.float16(2.0 ** -24)
    assert np.array_equal(oracle.channel_scales(X, rows=rows).view(np.uint16), want_r.view(np.uint16))


def test_channelwise_codes_error_bound_and_unit_token_scale(oracle):
    rng = np.random.default_rng(22)
    X, _ = wl.activations(64, 256, 3, 30.0, rng)
    c = oracle.channel_scales(X)
    q, s = oracle.quantize_rows_channelwise(X, c)
    assert np.all(s.view(np.uint16) == 0x3c00)             # the linear's epilogue multiplies by exactly 1
    codes = oracle.unpack_int4(q).astype(np.float64)
    assert codes.min() >= -7 and codes.max() <= 7          # calibration rows never reach the clamp
    cf = c.astype(np.float64)
    assert np.all(np.abs(codes * cf - X.astype(np.float64)) <= cf / 2 * (1 + 1e-3))
    # every channel uses its range: the largest |code| of each column is 7 (6 only through the half rounding of c)
    assert np.all(np.abs(codes).max(axis=0) >= 6)


def test_channelwise_by_python_loops(oracle):
    X = np.array([[1.0, -2.0, 0.5, 100.0], [0.25, 7.0, -0.5, -50.0]], np.float16)
    c = np.array([0.5, 1.0, 0.125, 16.0], np.float16)
    want = [[2, -2, 4, 6], [0, 7, -4, -3]]       # 1/.5, -2/1, .5/.125, 100/16=6.25->6 ; .25/.5=.5->0 (even), 7, -4, -3.125->-3
    q, _ = oracle.quantize_rows_channelwise(X, c)
    assert oracle.unpack_int4(q).tolist() == want
    # out-of-calibration values are clamped, not wrapped
    q2, _ = oracle.quantize_rows_channelwise(np.array([[9.0, -20.0, 3.0, 0.0]], np.float16), c)
    assert oracle.unpack_int4(q2).tolist() == [[7, -8, 7, 0]]


def test_folding_power_of_two_scales_changes_only_the_weight_scale(oracle):
    """c_k = 2^-3 for every k: W * c is exact, the codes cannot change and the row scale is divided by 8."""
    rng = np.random.default_rng(23)
    W = wl.weights(24, 128, rng)
    c = np.full(128, 0.125, np.float16)
    q0, s0, _ = oracle.quantize_rows(W)
    q1, s1 = oracle.quantize_rows_folded(W, c)
    assert np.array_equal(q0, q1)
    assert np.array_equal(s1.astype(np.float32) * 8, s0.astype(np.float32))
    # a single large channel scale pulls that column's codes up and the others down
    c2 = c.copy()
    c2[7] = 8.0
    q2, _ = oracle.quantize_rows_folded(W, c2)
    codes0, codes2 = oracle.unpack_int4(q0).astype(int), oracle.unpack_int4(q2).astype(int)
    assert np.abs(codes2[:, 7]).sum() > np.abs(codes0[:, 7]).sum()
    assert np.abs(np.delete(codes2, 7, axis=1)).sum() < np.abs(np.delete(codes0, 7, axis=1)).sum()


def test_channelwise_linear_reproduces_the_fp_linear_and_beats_per_token_on_outliers(oracle):
    """y = x W^T with x ~ c q and c folded into W.  On activations with a few huge channels the per-token
    quantizer zeroes the ordinary channels (the failure Section 3.3 describes); the channel-wise one does not.
    A missing or doubled fold, or scales applied along the wrong axis, breaks the first assertion."""
    rng = np.random.default_rng(24)
    M, K, N = 48, 512, 40
    X, ch = wl.activations(M, K, 5, 30.0, rng)
    W = wl.weights(N, K, rng)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    c = oracle.channel_scales(X)
    xq, sx1 = oracle.quantize_rows_channelwise(X, c)
    wq, sw = oracle.quantize_rows_folded(W, c)
    y_cw, _ = oracle.w4a4_linear(xq, sx1, wq, sw)
    xq_t, sx_t, _ = oracle.quantize_rows(X)
    wq_t, sw_t, _ = oracle.quantize_rows(W)
    y_tok, _ = oracle.w4a4_linear(xq_t, sx_t, wq_t, sw_t)
    err = lambda y: np.linalg.norm(y.astype(np.float64) - ref) / np.linalg.norm(ref)
    # the outlier channels carry most of the output energy and both quantizers resolve them; what is left is
    # the ordinary channels, which only the channel-wise activations keep
    keep = np.ones(K, bool)
    keep[ch] = False
    ref_ord = X[:, keep].astype(np.float64) @ W[:, keep].astype(np.float64).T
    codes_cw = oracle.unpack_int4(xq).astype(np.float64) * c.astype(np.float64)
    codes_tok = oracle.unpack_int4(xq_t).astype(np.float64) * sx_t.astype(np.float64)[:, None]
    act_err = lambda xh: np.linalg.norm(xh[:, keep] - X[:, keep].astype(np.float64)) / np.linalg.norm(X[:, keep])
    assert err(y_cw) < 0.35
    assert act_err(codes_cw) < 0.2 < 0.9 < act_err(codes_tok)
    assert np.linalg.norm(ref_ord) > 0


# ------------------------------------------------------------------ GEMM + epilogue
def test_int_gemm_vs_numpy_int64(oracle):
    rng = np.random.default_rng(12)
    M, N, K = 13, 21, 96
    Xq = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    Wq = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    acc = oracle.int_gemm(Xq, Wq)
    want = oracle.unpack_int4(Xq).astype(np.int64) @ oracle.unpack_int4(Wq).astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64), want)
    # not symmetric in its operands: a transposed read would fail here
    assert acc.shape == (M, N)


def test_int_gemm_hand_cases(oracle):
    K = 64
    p7 = np.full((1, K // 2), 0x77, np.uint8)          # all +7
    m7 = np.full((1, K // 2), 0x99, np.uint8)          # all -7
    m8 = np.full((1, K // 2), 0x88, np.uint8)          # all -8
    assert oracle.int_gemm(p7, m7)[0, 0] == -49 * K
    assert oracle.int_gemm(m8, m8)[0, 0] == 64 * K
    # W picks single codes: row n has a 1 at k = n only
    W = np.zeros((4, K // 2), np.uint8)
    for n in range(4):
        W[n, n // 2] = 1 << (4 * (n % 2))
    X = np.zeros((1, K // 2), np.uint8)
    X[0, 0] = 0x2F          # k0 = -1, k1 = 2
    X[0, 1] = 0x93          # k2 = 3, k3 = -7
    assert np.array_equal(oracle.int_gemm(X, W), [[-1, 2, 3, -7]])


def test_dequant_against_numpy_half_conversion(oracle):
    rng = np.random.default_rng(13)
    M, N = 9, 33
    acc = rng.integers(-700000, 700000, size=(M, N)).astype(np.int32)
    sx = (rng.random(M) * 3 + 0.01).astype(np.float16)
    sw = (rng.random(N) * 0.02 + 1e-4).astype(np.float16)
    Y = oracle.dequant(acc, sx, sw)
    with np.errstate(over="ignore"):
        want = ((acc.astype(np.float32) * sx.astype(np.float32)[:, None])
                * sw.astype(np.float32)[None, :]).astype(np.float16)
    assert np.array_equal(Y.view(np.uint16), want.view(np.uint16))


def test_linear_samples_agree_with_full_product(oracle):
    rng = np.random.default_rng(14)
    M, N, K = 10, 12, 64
    Xq = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    Wq = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    sx = (rng.random(M) + 0.1).astype(np.float16)
    sw = (rng.random(N) * 0.01 + 1e-3).astype(np.float16)
    want_acc = oracle.unpack_int4(Xq).astype(np.int64) @ oracle.unpack_int4(Wq).astype(np.int64).T
    ms, ns = np.meshgrid(np.arange(M), np.arange(N), indexing="ij")
    acc, y = oracle.linear_samples(Xq, sx, Wq, sw, ms.ravel(), ns.ravel())
    assert np.array_equal(acc.reshape(M, N), want_acc)
    Y, _ = oracle.w4a4_linear(Xq, sx, Wq, sw)
    assert np.array_equal(y.reshape(M, N).view(np.uint16), Y.view(np.uint16))


def test_w4a4_linear_approximates_the_fp_linear(oracle):
    """End to end on configuration 0: the W4A4 output tracks the fp32 linear, and
    tracks it better once the rotation of Eq. 6 is applied to both operands."""
    c = wl.toy_config()
    X, W = c["X"], c["W"]
    ref = X.astype(np.float64) @ W.astype(np.float64).T

    def run(rotate):
        if rotate:
            Wr = np.stack([oracle.fwht(W[n].astype(np.float32)) for n in range(W.shape[0])])
            Wq, sw, _ = oracle.quantize_rows(Wr.astype(np.float16))
        else:
            Wq, sw, _ = oracle.quantize_rows(W)
        Xq, sx, _ = oracle.quantize_rows(X, rotate=rotate)
        Y, _ = oracle.w4a4_linear(Xq, sx, Wq, sw)
        return np.linalg.norm(Y.astype(np.float64) - ref) / np.linalg.norm(ref)

    e_plain, e_rot = run(False), run(True)
    assert e_plain < 1.0
    assert e_rot < 0.35 and e_rot < e_plain


# ------------------------------------------------------------------ score
def test_attn_scores_vs_library_softmax(oracle):
    rng = np.random.default_rng(15)
    S, H, d, v0, nv = 37, 4, 16, 3, 20
    q, k = wl.query_and_keys(S, H, d, rng)
    got = oracle.attn_scores(q, k, v0, nv)
    logits = np.einsum("hd,shd->hs", q.astype(np.float64), k.astype(np.float64)) / np.sqrt(d)
    p = scipy.special.softmax(logits, axis=1)
    assert np.allclose(got, p[:, v0:v0 + nv].mean(axis=0), rtol=1e-6, atol=1e-9)
    full = oracle.attn_scores(q, k, 0, S)
    assert np.isclose(full.sum(), 1.0, atol=1e-6)


def test_attn_scores_uniform_and_shift_invariance(oracle):
    S, H, d = 10, 2, 8
    q = np.ones((H, d), np.float16)
    k = np.ones((S, H, d), np.float16)
    assert np.allclose(oracle.attn_scores(q, k, 0, S), 1.0 / S)
    rng = np.random.default_rng(16)
    q, k = wl.query_and_keys(S, H, d, rng)
    q = np.round(q * 4) / 4
    k = np.round(k * 4) / 4
    base = oracle.attn_scores(q, k, 2, 5)
    # adding one vector to every key adds a per-head constant to all logits
    shifted = oracle.attn_scores(q, (k + np.float16(0.5)).astype(np.float16), 2, 5)
    assert np.allclose(base, shifted, rtol=1e-5)


# ------------------------------------------------------------------ brute force, tiny
def test_tiny_linear_by_python_loops(oracle):
    rng = np.random.default_rng(17)
    M, N, K = 3, 4, 8
    X = (rng.standard_normal((M, K)) * 2).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    Xq, sx, _ = oracle.quantize_rows(X)
    Wq, sw, _ = oracle.quantize_rows(W)
    xc, wc = _codes(oracle, Xq), _codes(oracle, Wq)
    Y, acc = oracle.w4a4_linear(Xq, sx, Wq, sw)
    for m, n in itertools.product(range(M), range(N)):
        s = sum(int(xc[m, k]) * int(wc[n, k]) for k in range(K))
        assert acc[m, n] == s
        approx = s * float(sx[m]) * float(sw[n])
        assert abs(float(Y[m, n]) - approx) <= 1e-3 * abs(approx) + 1e-7


# ------------------------------------------------------------------ decoder glue
def _exact_inv_rms(row_f16, eps):
    """1/sqrt(mean square + eps) from exact rational arithmetic on the half values."""
    from fractions import Fraction
    S = sum(Fraction(float(v)) ** 2 for v in row_f16)          # a half converts to Fraction exactly
    Sd = float(S)                                              # correctly rounded to binary64
    return np.float32(1.0 / np.sqrt(Sd / len(row_f16) + float(np.float32(eps))))


def test_rmsnorm_constant_row_and_unit_rms(oracle):
    K = 96
    for c in (0.5, -3.0, 100.0, 6.1e-5):
        X = np.full((1, K), c, dtype=np.float16)
        _, y = oracle.rmsnorm_rows(X, np.ones(K, np.float16), 0.0)
        assert np.all(y == np.float16(np.sign(c))), c              # x / |x|
    # eps equal to the mean square halves the normalised power: x / sqrt(2 x^2) = 1 / sqrt(2)
    for c in (0.5, -0.03125, 16.0):
        X = np.full((1, K), c, dtype=np.float16)
        _, y = oracle.rmsnorm_rows(X, np.ones(K, np.float16), c * c)
        assert np.all(y == np.float16(np.sign(c) * np.sqrt(0.5))), c
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((7, 512)) * 3).astype(np.float16)
    _, y = oracle.rmsnorm_rows(X, np.ones(512, np.float16), 0.0)
    rms = np.sqrt((y.astype(np.float64) ** 2).mean(axis=1))
    assert np.all(np.abs(rms - 1.0) < 1e-3)                        # only the rounding to half is left
    gamma = (1 + 0.2 * rng.standard_normal(512)).astype(np.float16)
    _, yg = oracle.rmsnorm_rows(X, gamma, 1e-5)
    x = X.astype(np.float64)
    ref = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5) * gamma.astype(np.float64)
    assert np.all(np.abs(yg.astype(np.float64) - ref) <= 2.0 ** -11 * np.abs(ref) + 1e-7 + 2e-7 * np.abs(ref))


def test_rmsnorm_power_of_two_scaling_changes_nothing(oracle):
    rng = np.random.default_rng(6)
    X = rng.standard_normal((5, 200)).astype(np.float16)
    gamma = (1 + 0.1 * rng.standard_normal(200)).astype(np.float16)
    _, y0 = oracle.rmsnorm_rows(X, gamma, 0.0)
    for j in (-3, 2, 5):
        Xs = (X.astype(np.float32) * np.float32(2.0 ** j)).astype(np.float16)
        assert np.array_equal(Xs.astype(np.float32), X.astype(np.float32) * np.float32(2.0 ** j))  # exact scaling
        _, y = oracle.rmsnorm_rows(Xs, gamma, 0.0)
        assert np.array_equal(y.view(np.uint16), y0.view(np.uint16)), j


def test_rmsnorm_sum_of_squares_is_exact(oracle):
    """Rows whose squares span 80 binary orders: any floating-point running sum loses the small terms."""
    K = 4096
    rows = []
    r = np.full(K, 2.0 ** -24, dtype=np.float16)               # smallest subnormal everywhere ...
    r[7] = np.float16(65504.0)                                 # ... and the largest half once
    rows.append(r)
    r = np.full(K, 2.0 ** -14, dtype=np.float16)
    r[::5] = np.float16(1.0009765625)
    rows.append(r)
    rng = np.random.default_rng(7)
    r = (rng.standard_normal(K) * np.exp(rng.uniform(-15, 8, K))).astype(np.float16)
    rows.append(np.clip(r, -60000, 60000).astype(np.float16))
    X = np.stack(rows)
    gamma = np.ones(K, np.float16)
    for eps in (0.0, 1e-6, 1e-12):
        _, y = oracle.rmsnorm_rows(X, gamma, eps)
        for i in range(X.shape[0]):
            inv = _exact_inv_rms(X[i], eps)
            want = (X[i].astype(np.float32) * inv).astype(np.float16)     # gamma = 1: second product is exact
            assert np.array_equal(y[i].view(np.uint16), want.view(np.uint16)), (i, eps)
    # the tiny terms matter: with eps = 0 the row of 2^-24 alone normalises to 1
    _, y = oracle.rmsnorm_rows(np.full((1, K), 2.0 ** -24, np.float16), gamma, 0.0)
    assert np.all(y == np.float16(1.0))


def test_rmsnorm_gather_and_residual_update(oracle):
    rng = np.random.default_rng(8)
    X = rng.standard_normal((9, 64)).astype(np.float16)
    D = rng.standard_normal((4, 64)).astype(np.float16)
    gamma = (1 + 0.1 * rng.standard_normal(64)).astype(np.float16)
    rows = np.array([8, 0, 3, 3], np.int32)
    xs, y = oracle.rmsnorm_rows(X, gamma, 1e-5, rows=rows, delta=D)
    want_x = (X[rows].astype(np.float32) + D.astype(np.float32)).astype(np.float16)    # numpy's own conversions
    assert np.array_equal(xs.view(np.uint16), want_x.view(np.uint16))
    assert np.array_equal(oracle.residual_add(X[rows], D).view(np.uint16), want_x.view(np.uint16))
    _, y2 = oracle.rmsnorm_rows(want_x, gamma, 1e-5)
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))
    with pytest.raises(ValueError):
        oracle.rmsnorm_rows(np.array([[np.inf, 1.0]], np.float16), np.ones(2, np.float16), 0.0)


def test_swiglu_against_high_precision_and_identities(oracle):
    import decimal
    decimal.getcontext().prec = 50
    gs = np.array([0.0, 1.0, -1.0, 0.5, 3.140625, -2.71875, 8.0, -8.0, 11.0, -17.0, 6.1e-5, -6.1e-5, 60000.0, -60000.0,
                   30.0, -30.0], dtype=np.float16)
    one = np.ones_like(gs)
    h = oracle.swiglu(gs[None, :], one[None, :])[0]
    for g, got in zip(gs, h):
        gd = decimal.Decimal(float(g))
        true = gd / (1 + (-gd).exp())
        want = np.float16(np.float32(float(true)))               # silu to float, product with 1, to half
        assert got.view(np.uint16) == want.view(np.uint16) or abs(float(got) - float(true)) <= 2.0 ** -11 * abs(float(true)) + 2.0 ** -25, g
    assert h[0] == 0 and float(h[12]) == 60000.0 and float(h[13]) == 0.0       # silu(0) = 0, silu(+big) = big, silu(-big) = -0
    rng = np.random.default_rng(9)
    G = (rng.standard_normal((3, 500)) * 4).astype(np.float16)
    U = (rng.standard_normal((3, 500)) * 2).astype(np.float16)
    H = oracle.swiglu(G, U).astype(np.float64)
    ref = scipy.special.expit(G.astype(np.float64)) * G.astype(np.float64) * U.astype(np.float64)   # library logistic
    assert np.all(np.abs(H - ref) <= 2.0 ** -11 * np.abs(ref) + 1e-7 + 3e-7 * np.abs(ref))
    # silu(g) - silu(-g) = g: the u factor and the sign of the exponent are where a slip would show
    plus = oracle.swiglu(G, np.ones_like(G)).astype(np.float64)
    minus = oracle.swiglu(-G, np.ones_like(G)).astype(np.float64)
    assert np.all(np.abs(plus - minus - G.astype(np.float64)) <= 2.0 ** -9 * np.maximum(np.abs(G.astype(np.float64)), 1e-3))
    # operands are not swapped: silu acts on the first argument only
    assert not np.array_equal(oracle.swiglu(G, U), oracle.swiglu(U, G))
    h1, h2 = oracle.swiglu(G, U).astype(np.float32), oracle.swiglu(G, 2 * U).astype(np.float32)
    normal = np.abs(h1) >= 2.0 ** -13                            # doubling is exact away from the subnormal halves
    assert np.array_equal(h2[normal], 2 * h1[normal])


def test_rope_is_a_rotation_by_position_times_frequency(oracle):
    rng = np.random.default_rng(10)
    S, H, d, base = 11, 3, 16, 10000.0
    X = rng.standard_normal((S, H, d)).astype(np.float16)
    pos = np.array([0, 1, 2, 3, 5, 8, 13, 21, 34, 147, 275], np.int32)
    Y = oracle.rope(X, pos, base).astype(np.float64)
    assert np.array_equal(Y[0], X[0].astype(np.float64))                       # position 0: identity
    z = X[..., :d // 2].astype(np.float64) + 1j * X[..., d // 2:].astype(np.float64)
    freq = base ** (-np.arange(d // 2) * 2.0 / d)
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])             # complex multiplication
    want = np.concatenate([zr.real, zr.imag], axis=-1)
    assert np.all(np.abs(Y - want) <= 2.0 ** -11 * np.abs(want) + 1e-6)
    # the defining property: rotated dot products depend on the position difference only
    q = rng.standard_normal((1, 1, d)).astype(np.float16)
    k = rng.standard_normal((1, 1, d)).astype(np.float16)
    dots = []
    for (m, n) in ((3, 1), (10, 8), (102, 100)):
        qm = oracle.rope(q, np.array([m], np.int32), base).astype(np.float64).ravel()
        kn = oracle.rope(k, np.array([n], np.int32), base).astype(np.float64).ravel()
        dots.append(qm @ kn)
    assert np.ptp(dots) < 2e-2 * max(1.0, abs(dots[0]))


def test_attention_closed_forms_and_matrix_form(oracle):
    rng = np.random.default_rng(11)
    S, H, d = 13, 2, 8
    V = rng.standard_normal((S, H, d)).astype(np.float16)
    K = rng.standard_normal((S, H, d)).astype(np.float16)
    # zero queries: uniform weights over the keys up to and including the query's own position
    O = oracle.attention(np.zeros((S, H, d), np.float16), K, V).astype(np.float64)
    run = np.cumsum(V.astype(np.float64), axis=0) / np.arange(1, S + 1)[:, None, None]
    assert np.all(np.abs(O - run) <= 2.0 ** -11 * np.abs(run) + 1e-7)
    assert np.array_equal(O[0], V[0].astype(np.float64))                       # a single key: its value
    # a query that singles out one key returns that key's value
    Kb = np.zeros((S, H, d), np.float16)
    Kb[:, :, 0] = np.arange(S)[:, None]                                        # key t has first coordinate t
    Qb = np.zeros((S, H, d), np.float16)
    Qb[:, :, 0] = 200.0                                                        # prefers the largest visible t = s
    O = oracle.attention(Qb, Kb, V)
    assert np.array_equal(O.view(np.uint16), V.view(np.uint16))
    # matrix formulation with library routines
    Q = rng.standard_normal((S, H, d)).astype(np.float16)
    L = np.einsum("shi,thi->hst", Q.astype(np.float64), K.astype(np.float64)) / np.sqrt(d)
    L = np.where(np.tril(np.ones((S, S), bool))[None], L, -np.inf)
    P = scipy.special.softmax(L, axis=-1)
    want = np.einsum("hst,thi->shi", P, V.astype(np.float64))
    got = oracle.attention(Q, K, V).astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -11 * np.abs(want) + 1e-7)
    # fewer queries than keys: they are the last positions, so the result is the tail of the square case
    tail = oracle.attention(Q[-3:], K, V)
    assert np.array_equal(tail.view(np.uint16), oracle.attention(Q, K, V)[-3:].view(np.uint16))
    assert np.all(np.abs(tail.astype(np.float64) - want[-3:]) <= 2.0 ** -11 * np.abs(want[-3:]) + 1e-7)
    with pytest.raises(ValueError):
        oracle.attention(Q, K[:5], V[:5])


def test_decoder_layer_composition_follows_a_float_layer(oracle):
    """The chain of stages against a binary64 layer with the dequantized weights and no activation
    quantization: 4-bit activations leave about 10 % (attention block) and 35 % (feed-forward output)
    relative error; a swapped gate/up, a missing rotation or a missing residual leave much more."""
    rng = np.random.default_rng(3)
    hidden, H, d, F, batch, S = 256, 4, 64, 512, 2, 19
    M = batch * S
    x = rng.standard_normal((M, hidden)).astype(np.float16)
    pend = (0.5 * rng.standard_normal((M, hidden))).astype(np.float16)
    pos = np.tile(np.arange(S), batch).astype(np.int32)
    ws, wd = {}, {}
    for name, (N, K) in dict(qkv=(3 * hidden, hidden), o=(hidden, hidden), gate_up=(2 * F, hidden), down=(hidden, F)).items():
        W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float16)
        q, s, _ = oracle.quantize_rows(W)
        ws[name] = (q, s)
        wd[name] = oracle.unpack_int4(q).astype(np.float64) * s.astype(np.float64)[:, None]
    g1 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
    g2 = (1 + 0.1 * rng.standard_normal(hidden)).astype(np.float16)
    st = oracle.decoder_layer(x, pend, pos, batch, ws, g1, g2, H, d)

    def rms(v, g):
        return v / np.sqrt((v * v).mean(axis=1, keepdims=True) + 1e-5) * g.astype(np.float64)

    X = x.astype(np.float64) + pend.astype(np.float64)
    qkv = rms(X, g1) @ wd["qkv"].T
    q, k, v = [qkv[:, i * hidden:(i + 1) * hidden].reshape(M, H, d) for i in range(3)]
    freq = 10000.0 ** (-np.arange(d // 2) * 2.0 / d)

    def rot(t):
        z = (t[..., :d // 2] + 1j * t[..., d // 2:]) * np.exp(1j * pos[:, None, None] * freq)
        return np.concatenate([z.real, z.imag], axis=-1)

    q, k = rot(q), rot(k)
    out = np.zeros((M, H, d))
    for b in range(batch):
        sl = slice(b * S, (b + 1) * S)
        L = np.einsum("shi,thi->hst", q[sl], k[sl]) / np.sqrt(d)
        L = np.where(np.tril(np.ones((S, S), bool))[None], L, -np.inf)
        out[sl] = np.einsum("hst,thi->shi", scipy.special.softmax(L, axis=-1), v[sl])
    X2 = X + out.reshape(M, hidden) @ wd["o"].T
    gu = rms(X2, g2) @ wd["gate_up"].T
    dd = (gu[:, :F] * scipy.special.expit(gu[:, :F]) * gu[:, F:]) @ wd["down"].T
    e_x2 = np.linalg.norm(st["x2"].astype(np.float64) - X2) / np.linalg.norm(X2)
    e_d = np.linalg.norm(st["d"].astype(np.float64) - dd) / np.linalg.norm(dd)
    assert e_x2 < 0.15 and e_d < 0.5, (e_x2, e_d)
