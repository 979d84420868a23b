"""Seeded synthetic inputs for the W4A4 + token-pruning hot path.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no quantizer, no top-k, no GEMM) and imports neither the
HIP binding nor the CPU oracle.  Both sides of every parity test receive the
bytes produced here.

The paper evaluates on a robot-manipulation simulator with trained CogACT
weights; neither is available, so these inputs reproduce only the *shape* of
that workload: a Llama-2-7B-shaped decoder (hidden 4096, FFN 11008, vocab
32000), 256 visual + 20 text tokens per observation, activations that are
standard normal except for a small fixed set of outlier channels (the
structure described in Section 3.3 / Fig. 4a of the paper), weights N(0, 0.02)
and uniform retention scores.
"""
import numpy as np

BASE_SEED = 20250909

HIDDEN = 4096
FFN = 11008
VOCAB = 32000
N_LAYERS = 32
N_HEADS = 32
HEAD_DIM = 128
N_VISUAL = 256
N_TEXT = 20
SEQ_LEN = N_VISUAL + N_TEXT

# tensor ids used to key the generator
T_SCORES, T_X, T_W, T_Q, T_KCACHE, T_CAMERA = 0, 1, 2, 3, 4, 5

# name -> (N = out features, K = in features) of one decoder layer's linears
LAYER_LINEARS = (
    ("q", HIDDEN, HIDDEN),
    ("k", HIDDEN, HIDDEN),
    ("v", HIDDEN, HIDDEN),
    ("o", HIDDEN, HIDDEN),
    ("gate", FFN, HIDDEN),
    ("up", FFN, HIDDEN),
    ("down", HIDDEN, FFN),
)
LM_HEAD = ("lm_head", VOCAB, HIDDEN)


def rng_for(cfg, layer, tensor, extra=0, seed=BASE_SEED):
    """Counter-based generator keyed by (seed, config, layer, tensor, extra)."""
    ss = np.random.SeedSequence([int(seed), int(cfg), int(layer), int(tensor), int(extra)])
    return np.random.Generator(np.random.Philox(ss))


def outlier_channels(K, n_outliers, rng):
    """Sorted, distinct channel numbers that carry the large activations."""
    return np.sort(rng.choice(K, size=n_outliers, replace=False)).astype(np.int64)


def activations(M, K, n_outliers, outlier_scale, rng):
    """[M,K] fp16: N(0,1), with the same n_outliers channels of every row scaled up."""
    ch = outlier_channels(K, n_outliers, rng)
    x = rng.standard_normal((M, K), dtype=np.float32)
    x[:, ch] *= np.float32(outlier_scale)
    return x.astype(np.float16), ch


def weights(N, K, rng, std=0.02):
    """[N,K] fp16 ~ N(0, std)."""
    w = rng.standard_normal((N, K), dtype=np.float32)
    w *= np.float32(std)
    return w.astype(np.float16)


def scores(batch, n_tokens, rng):
    """[batch, n_tokens] fp32 ~ U(0,1)."""
    return rng.random((batch, n_tokens), dtype=np.float32)


def cameras(batch, grid_w, grid_h, patch, rng):
    """[batch, 26] fp64 camera records for the robot-aware ring: intrinsics K (3x3), extrinsics [R|t]
    (3x4), a world point, patch width and height.  A pinhole camera looking at a point whose image
    falls on or near the grid_w x grid_h patch grid; about one record in eight has the point behind
    the camera.  Only data: the projection itself is done by whoever consumes the record."""
    out = np.empty((batch, 26), dtype=np.float64)
    W, H = grid_w * patch, grid_h * patch
    for b in range(batch):
        f = rng.uniform(0.8, 1.6) * W
        Kmat = np.array([[f, 0.0, W / 2 + rng.uniform(-4, 4)], [0.0, f * rng.uniform(0.95, 1.05), H / 2 + rng.uniform(-4, 4)],
                         [0.0, 0.0, 1.0]])
        q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
        if np.linalg.det(q) < 0:
            q[:, 0] = -q[:, 0]
        t = rng.standard_normal(3)
        depth = rng.uniform(0.5, 2.0) * (-1.0 if rng.random() < 0.125 else 1.0)
        cam = np.array([rng.uniform(-0.6, 0.6) * depth * W / f, rng.uniform(-0.6, 0.6) * depth * H / f, depth])
        world = q.T @ (cam - t)                 # so that R world + t lands where intended (up to rounding)
        out[b, 0:9] = Kmat.reshape(-1)
        out[b, 9:21] = np.hstack([q, t.reshape(3, 1)]).reshape(-1)
        out[b, 21:24] = world
        out[b, 24:26] = patch
    return out


def query_and_keys(S, H, d, rng):
    """q [H,d] and key cache [S,H,d], fp16 ~ N(0,1)."""
    q = rng.standard_normal((H, d), dtype=np.float32).astype(np.float16)
    k = rng.standard_normal((S, H, d), dtype=np.float32).astype(np.float16)
    return q, k


def n_outliers_for(K, frac=0.01):
    return int(round(frac * K))


# The five workload configurations.  M is the number of rows that reach the
# linears after pruning: batch * (keep_k + n_text).
CONFIGS = {
    0: dict(name="toy", batch=1, n_visual=64, n_text=0, keep_k=32, K=512, N=512,
            n_outliers=4, outlier_scale=20.0),
    1: dict(name="one_layer_M148", batch=1, n_visual=N_VISUAL, n_text=N_TEXT, keep_k=128,
            outlier_frac=0.01, outlier_scale=30.0),
    2: dict(name="stack32_M276_M84", batch=1, n_visual=N_VISUAL, n_text=N_TEXT, keep_k=64,
            prune_after_layer=2, outlier_frac=0.01, outlier_scale=30.0),
    3: dict(name="batched_prefill_M2368", batch=16, n_visual=N_VISUAL, n_text=N_TEXT,
            keep_k=128, outlier_frac=0.01, outlier_scale=30.0),
    4: dict(name="decode_M1to8", batch_sizes=(1, 2, 4, 8), steps=7, kv_prefix=148,
            outlier_frac=0.01, outlier_scale=30.0),
}


def toy_config(seed=BASE_SEED):
    """Configuration 0: 64 tokens x K=512, 4 outlier channels x20, W 512x512, keep 32."""
    c = CONFIGS[0]
    X, ch = activations(c["n_visual"], c["K"], c["n_outliers"], c["outlier_scale"],
                        rng_for(0, 0, T_X, seed=seed))
    W = weights(c["N"], c["K"], rng_for(0, 0, T_W, seed=seed))
    s = scores(1, c["n_visual"], rng_for(0, 0, T_SCORES, seed=seed))
    return dict(X=X, W=W, scores=s, keep_k=c["keep_k"], outlier_channels=ch)


def layer_weight(cfg, layer, linear_index, seed=BASE_SEED):
    """fp16 weight of one linear of one decoder layer (index into LAYER_LINEARS; 7 = lm_head)."""
    name, N, K = LM_HEAD if linear_index == 7 else LAYER_LINEARS[linear_index]
    return weights(N, K, rng_for(cfg, layer, T_W, linear_index, seed=seed))


def layer_input(cfg, layer, linear_index, rows, seed=BASE_SEED, outlier_frac=0.01,
                outlier_scale=30.0):
    """fp16 input [rows, K] of one linear, with round(frac*K) outlier channels."""
    name, N, K = LM_HEAD if linear_index == 7 else LAYER_LINEARS[linear_index]
    X, _ = activations(rows, K, n_outliers_for(K, outlier_frac), outlier_scale,
                       rng_for(cfg, layer, T_X, linear_index, seed=seed))
    return X
