"""Seeded synthetic inputs for the NVFP4 hot path (numpy only).

Shapes, distributions and structure follow the five benchmark configurations:
activations with a few outlier channels, small-variance weights and gradients,
and a KV cache with per-head scales.  They stand in for activations, weights,
gradients and KV tensors of the paper's 5B video DiT, which are not available.
This module holds no arithmetic of the method: it only draws numbers and
rounds them to bf16 bit patterns (uint16), which both the CPU oracle and the
HIP library consume.
"""
import numpy as np

D_MODEL = 3072
D_FFN = 14336
TOKENS_INFER = 3520
TOKENS_TRAIN = 17600
KV_TOKENS, KV_HEADS, KV_DIM = 18480, 24, 128


def to_bf16_bits(x_f32):
    """float32 array -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x_f32, dtype=np.float32).view(np.uint32)
    rnd = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rnd) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _rng(seed, tensor_id):
    return np.random.default_rng([seed, tensor_id])


def normal(shape, std, seed, tensor_id):
    g = _rng(seed, tensor_id)
    x = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bf16_bits(x)


def activation_with_outliers(rows, K, seed, tensor_id, frac=0.01, gain=20.0):
    """N(0,1) with round(frac*K) seeded K-channels multiplied by `gain`."""
    g = _rng(seed, tensor_id)
    x = g.standard_normal((rows, K), dtype=np.float32)
    n_out = int(frac * K + 0.5)
    ch = g.permutation(K)[:n_out]
    x[:, ch] *= np.float32(gain)
    return to_bf16_bits(x)


def kv_tensor(T, H, d, seed, tensor_id):
    """N(0,1) times a per-head scale drawn from U(0.5, 4); returns [T, H, d]."""
    g = _rng(seed, tensor_id)
    s = g.uniform(0.5, 4.0, size=H).astype(np.float32)
    x = g.standard_normal((T, H, d), dtype=np.float32)
    x *= s[None, :, None]
    return to_bf16_bits(x)


def config1(seed=0):
    """Tiny W4A4 check: A[128,256], W[256,256] ~ N(0,1)."""
    return {"A": normal((128, 256), 1.0, seed, 0), "W": normal((256, 256), 1.0, seed, 1)}


def config2(seed=1, M=TOKENS_INFER):
    """Single DiT projection: A[M,3072] with outlier channels, W[3072,3072] ~ N(0,0.02)."""
    return {"A": activation_with_outliers(M, D_MODEL, seed, 0),
            "W": normal((D_MODEL, D_MODEL), 0.02, seed, 1)}


def config3(seed=2, M=TOKENS_INFER, d_model=D_MODEL, d_ffn=D_FFN):
    """DiT FFN pair: A[M,d_model] -> W1[d_ffn,d_model] -> GELU -> W2[d_model,d_ffn]."""
    return {"A": activation_with_outliers(M, d_model, seed, 0),
            "W1": normal((d_ffn, d_model), 0.02, seed, 1),
            "W2": normal((d_model, d_ffn), 0.02, seed, 2)}


def config4(seed=3, T=KV_TOKENS, H=KV_HEADS, d=KV_DIM):
    """KV cache: K and V [T,H,d] with per-head scales."""
    return {"K": kv_tensor(T, H, d, seed, 0), "V": kv_tensor(T, H, d, seed, 1)}


def config5(seed=4, M=TOKENS_TRAIN, d_model=D_MODEL, d_ffn=D_FFN):
    """Training triplet: X[M,d_model] (outliers), W[d_ffn,d_model], dY[M,d_ffn] ~ N(0,1e-3)."""
    return {"X": activation_with_outliers(M, d_model, seed, 0),
            "W": normal((d_ffn, d_model), 0.02, seed, 1),
            "dY": normal((M, d_ffn), 1e-3, seed, 2)}
