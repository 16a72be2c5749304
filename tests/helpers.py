"""Shared test utilities: independent brute-force references written with numpy
(used to pin the oracle) and small conversions.  None of this is used by the
product or by the oracle."""
import numpy as np


def bf16_round(x):
    """fp32/fp64 array -> bf16 bit patterns (uint16), round to nearest even."""
    f = np.ascontiguousarray(x, np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def bf16_to_f64(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rand_bf16(rng, shape, scale=1.0):
    return bf16_round(rng.standard_normal(shape) * scale)


def brute_attention(q, k, v, q_start, scale, mask=None, group=1):
    """Textbook masked softmax attention with an explicit [C][n_k] 0/1 mask per head.
    q: [C][Hq][D], k/v: [n_k][Hkv][D] as fp64.  mask: [Hq][C][n_k] or None (causal)."""
    C, Hq, D = q.shape
    n_k = q_start + C
    out = np.zeros((Hq, C, D)); lse = np.full((Hq, C), -np.inf)
    for h in range(Hq):
        g = h // group
        logits = scale * (q[:, h, :] @ k[:n_k, g, :].T)          # [C][n_k]
        causal = np.arange(n_k)[None, :] <= (q_start + np.arange(C))[:, None]
        m = causal if mask is None else (causal & (mask[h] != 0))
        for i in range(C):
            sel = np.nonzero(m[i])[0]
            if sel.size == 0:
                continue
            x = logits[i, sel]
            e = np.exp(x - x.max())
            out[h, i] = (e / e.sum()) @ v[sel, g, :]
            lse[h, i] = x.max() + np.log(e.sum())
    return out, lse
