"""Shared test helpers: tiny seeded bf16 inputs and independent numpy references."""
import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rand_qkv(rng, H, G, L, d=128, scale=1.0):
    q = f32_to_bf16_bits(rng.standard_normal((H, d)).astype(np.float32) * scale)
    K = f32_to_bf16_bits(rng.standard_normal((G, L, d)).astype(np.float32) * scale)
    V = f32_to_bf16_bits(rng.standard_normal((G, L, d)).astype(np.float32) * scale)
    return q, K, V


def dense_attention_f64(q, K, V, tokens=None, sm_scale=None):
    """softmax(q K^T * sm_scale) V with numpy matmuls in float64, GQA by repetition."""
    qf, Kf, Vf = bits_to_f64(q), bits_to_f64(K), bits_to_f64(V)
    H, d = qf.shape
    G = Kf.shape[0]
    g = H // G
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    out = np.zeros((H, d))
    for h in range(H):
        Kh, Vh = Kf[h // g], Vf[h // g]
        if tokens is not None:
            Kh, Vh = Kh[tokens], Vh[tokens]
        w = (Kh @ qf[h]) * sm_scale
        w = np.exp(w - w.max())
        out[h] = (w / w.sum()) @ Vh
    return out
