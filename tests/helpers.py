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


def host_view(inp, layer_pos, b):
    """Logical (q[H,d], K[G,L,d], V[G,L,d]) bf16 bit patterns of sequence b for the oracle."""
    import oracle
    from paper_2508_07101_amd.workloads import bf16_bits
    lay = inp.layers[layer_pos]
    L = inp.seq_lens_host[b]
    q = bf16_bits(lay.q[b])
    if inp.block_table is None:
        return q, bf16_bits(lay.k[b, :, :L]), bf16_bits(lay.v[b, :, :L])
    bt = inp.block_table[b].cpu().numpy()
    n = (L + inp.workload.page_size - 1) // inp.workload.page_size
    pages = torch_unique_pages(bt[:n])
    # copy only this sequence's pages to the host, then let the oracle resolve the table
    import numpy as np
    import torch
    sel = torch.as_tensor(pages, device=lay.k.device, dtype=torch.long)
    remap = {int(p): i for i, p in enumerate(pages)}
    bt_local = np.array([remap[int(p)] for p in bt[:n]], dtype=np.int32)
    kp, vp = bf16_bits(lay.k[sel]), bf16_bits(lay.v[sel])
    return q, oracle.resolve_paged(kp, bt_local, L), oracle.resolve_paged(vp, bt_local, L)


def torch_unique_pages(bt_row):
    seen, out = set(), []
    for p in bt_row:
        if int(p) not in seen:
            seen.add(int(p))
            out.append(int(p))
    return out


def assert_close_bf16(got_bits, want_bits, what=""):
    """|got - want| <= 2e-2 + 1e-2 |want| elementwise on bf16 outputs (the stated tolerance)."""
    g, w = bits_to_f64(got_bits), bits_to_f64(want_bits)
    err = np.abs(g - w)
    tol = 2e-2 + 1e-2 * np.abs(w)
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.4g}"
