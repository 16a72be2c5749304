"""Seeded synthetic Q/K/V for the vertical-slash prefill workloads.

This module holds NO arithmetic of the method (no softmax, no scoring, no
selection): it only manufactures the bytes that both the HIP library and the CPU
oracle are fed.  The bytes it returns ARE the input; neither side regenerates
them.  Everything is a pure function of (base seed, config, tensor id, element
index) through a counter-based integer hash, so any slice of any tensor can be
produced on its own, on the CPU or on the GPU (torch is used as an array
library only).

Recipe (stands in for the post-RoPE Q/K/V of an LLM layer at the shapes of the
Qwen2.5-1M models, section 2 table: 7B = 28 query / 4 KV heads, 14B = 40 / 8):
  1. Q, K, V i.i.d. N(0,1)  (hash -> two uniforms -> Box-Muller, fp32).
  2. optional heavy tail: each (key position, kv head) is scaled with
     probability 0.05 by exp(z), z ~ N(0,1)  (workload "14b_1m").
  3. RoPE, base 1e7 (the final base frequency of the long-context training
     stages), half-split pairing (d with d + D/2), absolute positions, on Q and K.
  4. "sinks": n_sink distinct key positions per KV head get + a_g * u added,
     and every query gets + u, with u a seeded unit vector (per KV head).
     This plants vertical lines; no slash structure is planted.
  5. one rounding to bf16 (round to nearest even).
Extra, not one of the five configurations ("7b_1m_local"): before RoPE a shared seeded
vector (per KV head, length local_mag) is added to every query and key, so that q_i . k_j
gains a term that depends only on i - j and decays slowly with it -- slash lines that
cluster at small offsets, as the attention maps of trained models show them.
Extra ("7b_1m_dca"): the positions fed to RoPE are those of Dual Chunk Attention (section
5.1) with chunk length c = dca_chunk and local window dca_window: a key at position j is
rotated at j mod c; the queries come in three rotations, at i mod c (intra-chunk), at
(i mod c) + c (successive-chunk: against a key of the chunk before, the difference is the true
distance i - j) and at the constant c + dca_window - 1 (inter-chunk: no relative position
exceeds what one chunk plus the window has seen).  Only the positions differ; which rotation
meets which key is decided by the library and the oracle, not here.  The selection of such a
workload takes rotations of its own (make_q_dca_select: continuous relative positions).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace

import torch

BASE_SEED = 0x250115383
_M32 = 0xFFFFFFFF

# tensor ids (sub-streams)
_T_Q, _T_K, _T_V, _T_U, _T_SINKPOS, _T_TAILP, _T_TAILZ, _T_SINKCNT = range(8)


@dataclass(frozen=True)
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_ctx: int                 # total tokens prefilled
    chunk: int                 # C
    last_q: int = 64
    vertical_budget: int = 0
    slash_budget: int = 0
    keep_first_cols: int = 1
    keep_local_band: int = 64
    n_sink: int = 0            # sink key positions per KV head (max when ranged)
    n_sink_min: int = -1       # >=0: per-KV-head count drawn uniformly in [min, n_sink]
    sink_mag: float = 3.0      # a_g = sink_mag * 2**(g % 4) when sink_mag_per_head
    sink_mag_per_head: bool = False
    heavy_tail: bool = False
    local_mag: float = 0.0     # > 0: planted slash structure (see the module docstring)
    dca_chunk: int = 0         # > 0: Dual Chunk Attention positions (see the module docstring)
    dca_window: int = 0
    rope_theta: float = 1.0e7
    config_id: int = 0
    seed: int = BASE_SEED
    dense: bool = False        # every column and diagonal selected

    @property
    def n_chunks(self) -> int:
        return (self.n_ctx + self.chunk - 1) // self.chunk

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


# The five benchmark configurations (tiny, dense 64K, 128K, 1M at the 7B shape, 1M at the 14B shape).
WORKLOADS = {
    "tiny_4k": Workload("tiny_4k", 4, 1, 64, 4096, 1024, vertical_budget=128, slash_budget=256,
                        n_sink=16, config_id=0),
    "dense_7b_64k": Workload("dense_7b_64k", 28, 4, 128, 65536, 32768, n_sink=0, config_id=1,
                             dense=True),
    "7b_128k": Workload("7b_128k", 28, 4, 128, 131072, 32768, vertical_budget=1000,
                        slash_budget=6096, n_sink=256, sink_mag_per_head=True, config_id=2),
    "7b_1m": Workload("7b_1m", 28, 4, 128, 1048576, 32768, vertical_budget=1000,
                      slash_budget=6096, n_sink=256, sink_mag_per_head=True, config_id=3),
    "14b_1m": Workload("14b_1m", 40, 8, 128, 1048576, 32768, vertical_budget=2000,
                       slash_budget=8192, n_sink=512, n_sink_min=32, sink_mag_per_head=True,
                       heavy_tail=True, config_id=4),
    # extra: the 7B configuration with planted, clustered slash lines (not one of the five)
    "7b_1m_local": Workload("7b_1m_local", 28, 4, 128, 1048576, 32768, vertical_budget=1000,
                            slash_budget=6096, n_sink=256, sink_mag_per_head=True, local_mag=8.0, config_id=5),
    # extra: the 7B configuration with Dual Chunk Attention positions (chunks of 256K tokens, four of
    # them in 1M; the local window is not given in the paper, 8192 is this recipe's choice)
    "7b_1m_dca": Workload("7b_1m_dca", 28, 4, 128, 1048576, 32768, vertical_budget=1000,
                          slash_budget=6096, n_sink=256, sink_mag_per_head=True, dca_chunk=262144,
                          dca_window=8192, config_id=6),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields changed (reduced test sizes)."""
    return replace(w, **kw)


# ---------------------------------------------------------------------------
# counter-based hash: (key, 64-bit counter) -> 32 uniform bits, on int64 tensors
# ---------------------------------------------------------------------------
def _mix32(x: torch.Tensor) -> torch.Tensor:
    # an avalanche finaliser on 32-bit words carried in int64 lanes
    x = x & _M32
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def _key(seed: int, config_id: int, tensor_id: int, stream: int) -> int:
    k = (seed ^ (config_id * 0x9E3779B1) ^ (tensor_id * 0x85EBCA77) ^ (stream * 0xC2B2AE3D)) & 0xFFFFFFFFFFFFFFFF
    return k


def _hash_u32(idx: torch.Tensor, key: int) -> torch.Tensor:
    """idx: int64 counters (>=0).  Returns int64 values in [0, 2^32)."""
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    k0, k1 = key & _M32, (key >> 32) & _M32
    h = _mix32(lo ^ k0)
    h = _mix32(h + ((hi ^ k1) * 0x27D4EB2F & _M32) + 0x165667B1)
    return h


def _uniform(idx: torch.Tensor, key: int) -> torch.Tensor:
    """(0,1] uniforms in fp32 from 24 hash bits."""
    return ((_hash_u32(idx, key) >> 8).to(torch.float32) + 1.0) * (1.0 / 16777216.0)


def _normal(idx: torch.Tensor, key: int) -> torch.Tensor:
    u1 = _uniform(idx * 2, key)
    u2 = _uniform(idx * 2 + 1, key)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _counters(t0: int, t1: int, n_heads: int, d: int, device) -> torch.Tensor:
    t = torch.arange(t0, t1, dtype=torch.int64, device=device).view(-1, 1, 1)
    h = torch.arange(n_heads, dtype=torch.int64, device=device).view(1, -1, 1)
    e = torch.arange(d, dtype=torch.int64, device=device).view(1, 1, -1)
    return (t * n_heads + h) * d + e


def _rope(x: torch.Tensor, t0, theta: float) -> torch.Tensor:
    """Half-split rotary embedding (fp64 angles) at absolute positions t0, t0 + 1, ... when t0 is
    an int, or at the positions given by an int64 tensor [n]."""
    n, _, d = x.shape
    half = d // 2
    if isinstance(t0, torch.Tensor):
        pos = t0.to(torch.float64).view(-1, 1, 1)
    else:
        pos = torch.arange(t0, t0 + n, dtype=torch.float64, device=x.device).view(-1, 1, 1)
    inv = theta ** (-torch.arange(half, dtype=torch.float64, device=x.device) * 2.0 / d)
    ang = pos * inv.view(1, 1, -1)
    c, s = torch.cos(ang).to(torch.float32), torch.sin(ang).to(torch.float32)
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * c - b * s, a * s + b * c], dim=-1)


def unit_vectors(w: Workload, device="cpu") -> torch.Tensor:
    """u[g]: one seeded unit vector per KV head, fp32 [Hkv][D]."""
    idx = torch.arange(w.n_kv_heads * w.head_dim, dtype=torch.int64, device=device)
    u = _normal(idx, _key(w.seed, w.config_id, _T_U, 0)).view(w.n_kv_heads, w.head_dim)
    return u / u.norm(dim=-1, keepdim=True)


def local_vectors(w: Workload, device="cpu") -> torch.Tensor:
    """One seeded unit vector per KV head for the planted slash structure, fp32 [Hkv][D]."""
    idx = torch.arange(w.n_kv_heads * w.head_dim, dtype=torch.int64, device=device)
    u = _normal(idx, _key(w.seed, w.config_id, _T_U, 1)).view(w.n_kv_heads, w.head_dim)
    return u / u.norm(dim=-1, keepdim=True)


def sink_counts(w: Workload) -> list[int]:
    if w.n_sink_min < 0:
        return [w.n_sink] * w.n_kv_heads
    idx = torch.arange(w.n_kv_heads, dtype=torch.int64)
    r = _hash_u32(idx, _key(w.seed, w.config_id, _T_SINKCNT, 0))
    span = w.n_sink - w.n_sink_min + 1
    return [int(w.n_sink_min + (int(x) % span)) for x in r]


def sink_positions(w: Workload) -> list[torch.Tensor]:
    """Per KV head: sorted distinct key positions in [0, n_ctx) (CPU int64)."""
    out = []
    for g, cnt in enumerate(sink_counts(w)):
        cnt = min(cnt, w.n_ctx)
        if cnt == 0:
            out.append(torch.zeros(0, dtype=torch.int64))
            continue
        # draw 4x candidates, keep the first cnt distinct ones in draw order
        idx = torch.arange(4 * cnt + 64, dtype=torch.int64)
        cand = _hash_u32(idx, _key(w.seed, w.config_id, _T_SINKPOS, g)) % w.n_ctx
        seen, keep = set(), []
        for c in cand.tolist():
            if c not in seen:
                seen.add(c); keep.append(c)
                if len(keep) == cnt:
                    break
        out.append(torch.tensor(sorted(keep), dtype=torch.int64))
    return out


def sink_magnitudes(w: Workload) -> list[float]:
    return [w.sink_mag * (2.0 ** (g % 4) if w.sink_mag_per_head else 1.0) for g in range(w.n_kv_heads)]


def _to_bf16(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16)


def _make_q_at(w: Workload, t0: int, t1: int, positions, device) -> torch.Tensor:
    x = _normal(_counters(t0, t1, w.n_q_heads, w.head_dim, device), _key(w.seed, w.config_id, _T_Q, 0))
    g_of_h = torch.arange(w.n_q_heads, device=device) // (w.n_q_heads // w.n_kv_heads)
    if w.local_mag > 0:
        x = x + w.local_mag * local_vectors(w, device)[g_of_h].unsqueeze(0)
    x = _rope(x, positions, w.rope_theta)
    if w.n_sink > 0:
        x = x + unit_vectors(w, device)[g_of_h].unsqueeze(0)
    return _to_bf16(x)


def make_q(w: Workload, t0: int, t1: int, device="cpu") -> torch.Tensor:
    """Queries of tokens t0..t1-1: bf16 [t1-t0][Hq][D] (with DCA positions: the intra-chunk rotation)."""
    if w.dca_chunk > 0:
        return make_q_dca(w, t0, t1, device)[0]
    return _make_q_at(w, t0, t1, t0, device)


def dca_positions(i, chunk: int, window: int):
    """RoPE positions of Dual Chunk Attention for token indices i (an int64 tensor): the key position and
    the query's position under the intra-chunk, successive-chunk and inter-chunk pattern (section 5.1, DCA
    paragraph: distances inside a chunk and inside the local window are kept, every other pair sees the
    largest position c + w - 1 against the key's position in its own chunk)."""
    m = i % chunk
    return m, m, m + chunk, torch.full_like(i, chunk + window - 1)


def dca_select_positions(i, chunk: int, window: int):
    """The same for the SELECTION of critical tokens (section 5.2, "Integrating with DCA": relative
    positions that stay as consistent as possible along a diagonal): the successive-chunk position
    (i mod c) + c serves every pair of adjacent chunks, so their relative position is the true distance,
    and the inter-chunk position moves with the query, (i mod c) + c + w - 1, so that along a diagonal it
    is constant within a pair of chunks.  With c = 5 and c + w - 1 = 7 this gives the diagonal lists that
    the caption of the section's figure prints (tests/golden/dca_diagonal_lists.txt).  Returns
    (key, intra, successive, inter, window to select with = 2c: all of the chunk before the query's)."""
    m = i % chunk
    return m, m, m + chunk, m + chunk + window - 1, 2 * chunk


def make_q_dca(w: Workload, t0: int, t1: int, device="cpu"):
    """The three rotations of the queries of tokens t0..t1-1 under Dual Chunk Attention:
    (intra-chunk, successive-chunk, inter-chunk), each bf16 [t1-t0][Hq][D]."""
    assert w.dca_chunk > 0
    i = torch.arange(t0, t1, dtype=torch.int64, device=device)
    _, intra, succ, inter = dca_positions(i, w.dca_chunk, w.dca_window)
    return (_make_q_at(w, t0, t1, intra, device), _make_q_at(w, t0, t1, succ, device),
            _make_q_at(w, t0, t1, inter, device))


def make_q_dca_select(w: Workload, t0: int, t1: int, device="cpu"):
    """The rotations the SELECTION of a Dual Chunk Attention workload uses for the successive-chunk
    and the inter-chunk pattern, and the (chunk, window) that go with them: (q_succ, q_inter, c, 2c);
    see dca_select_positions.  The intra-chunk rotation is shared with the attention, which keeps
    DCA's own positions."""
    assert w.dca_chunk > 0
    i = torch.arange(t0, t1, dtype=torch.int64, device=device)
    _, _, succ, inter, win = dca_select_positions(i, w.dca_chunk, w.dca_window)
    return (_make_q_at(w, t0, t1, succ, device), _make_q_at(w, t0, t1, inter, device), w.dca_chunk, win)


def _make_kv_slab(w: Workload, t0: int, t1: int, device, sinks, mags, u):
    kc = _counters(t0, t1, w.n_kv_heads, w.head_dim, device)
    k = _normal(kc, _key(w.seed, w.config_id, _T_K, 0))
    v = _normal(kc, _key(w.seed, w.config_id, _T_V, 0))
    if w.heavy_tail:
        th = _counters(t0, t1, w.n_kv_heads, 1, device)
        pick = _uniform(th, _key(w.seed, w.config_id, _T_TAILP, 0)) <= 0.05
        z = _normal(th, _key(w.seed, w.config_id, _T_TAILZ, 0))
        k = k * torch.where(pick, torch.exp(z), torch.ones_like(z))
    if w.local_mag > 0:
        k = k + w.local_mag * local_vectors(w, device).unsqueeze(0)
    if w.dca_chunk > 0:
        k = _rope(k, torch.arange(t0, t1, dtype=torch.int64, device=device) % w.dca_chunk, w.rope_theta)
    else:
        k = _rope(k, t0, w.rope_theta)
    for g in range(w.n_kv_heads):
        pos = sinks[g]
        pos = pos[(pos >= t0) & (pos < t1)].to(device) - t0
        if pos.numel():
            k[pos, g, :] += mags[g] * u[g]
    return _to_bf16(k), _to_bf16(v)


def make_kv(w: Workload, n_tokens: int | None = None, device="cpu", slab: int = 1 << 16):
    """Key/value cache of tokens 0..n_tokens-1: two bf16 [n_tokens][Hkv][D] tensors."""
    n = w.n_ctx if n_tokens is None else n_tokens
    K = torch.empty((n, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=device)
    V = torch.empty_like(K)
    sinks, mags, u = sink_positions(w), sink_magnitudes(w), unit_vectors(w, device)
    for t0 in range(0, n, slab):
        t1 = min(n, t0 + slab)
        K[t0:t1], V[t0:t1] = _make_kv_slab(w, t0, t1, device, sinks, mags, u)
    return K, V


def as_u16(x: torch.Tensor):
    """bf16 tensor -> numpy uint16 bit patterns on the host (what the oracle reads)."""
    import numpy as np
    return x.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
