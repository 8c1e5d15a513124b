"""Seeded synthetic workloads (numpy only, no torch, none of the method's arithmetic).

These generators are the one piece shared by the GPU tests / benchmark and the
CPU oracle's callers: they draw the random tensors, cast them to the storage
type and lay cache rows out in pages.  They compute nothing of TPLA itself.

Stand-ins for the paper's decode workloads (MoE-removed DeepSeek-V3 and
Kimi-K2 at "maximum batch per context length", Sec. 5.4.1): the head counts
and cache widths are the paper's, everything else is drawn from the seed.

Storage arrays: float32 for "f32"; uint16 bit patterns for "bf16" (rounded to
nearest even from the float32 draw).  `as_f64` gives their exact values.
Draw order per config seed s:
    default_rng([s, 0]): W_UK, W_UV, q_nope, q_pe, heavy-channel indices,
                         sign diagonal, sequence lengths, page permutation
    default_rng([s, 1000 + b]): latent rows then k_pe rows of sequence b
"""
from dataclasses import dataclass, replace
import math

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d_c: int
    g: int
    d_r: int
    d_n: int
    d_v: int
    dtype: str = "bf16"            # "f32" | "bf16"
    page_tokens: int = 64
    seed: int = 0
    context: int = 0               # uniform length, or 0 when ragged
    ragged: tuple = ()             # (min_len, max_len): log-uniform lengths
    transform: str = "identity"    # "identity" | "hadamard"
    permute_pages: bool = False
    pool_slack: float = 0.0        # extra pool pages (fraction), NaN-filled
    heavy_channels: int = 0        # latent columns multiplied by 10
    weight_std: float = 0.02
    unit_variance_rows: bool = False   # tiny config: every tensor / sqrt(last dim)
    rms_prefill: bool = False      # cache written through the RMSNorm cache-write call
    d_model: int = 7168            # width of the block output (DeepSeek-V3 / Kimi-K2 hidden size)

    @property
    def dl(self):
        return self.d_c // self.g

    @property
    def sm_scale(self):
        return 1.0 / math.sqrt(self.d_n + self.d_r)


# The five configurations of the benchmark definition.
CONFIGS = {
    "tiny": Workload("tiny", B=1, H=4, d_c=64, g=2, d_r=16, d_n=32, d_v=32, dtype="f32", seed=0,
                     context=128, unit_variance_rows=True),
    "dsv3_4k": Workload("dsv3_4k", B=16, H=64, d_c=512, g=2, d_r=64, d_n=128, d_v=128, seed=2, context=4096),
    "dsv3_32k": Workload("dsv3_32k", B=32, H=64, d_c=512, g=2, d_r=64, d_n=128, d_v=128, seed=3,
                         context=32768, transform="hadamard"),
    "kimi_32k": Workload("kimi_32k", B=64, H=32, d_c=512, g=2, d_r=64, d_n=128, d_v=128, seed=4,
                         context=32768, heavy_channels=8),
    "ragged_g4": Workload("ragged_g4", B=128, H=64, d_c=512, g=4, d_r=64, d_n=128, d_v=128, seed=5,
                          ragged=(1024, 131072), permute_pages=True, pool_slack=0.05,
                          transform="hadamard", rms_prefill=True),
}


def scaled(w, **kw):
    """A smaller copy of a configuration (same widths unless overridden)."""
    return replace(w, **kw)


# ---------------------------------------------------------------- storage
def f32_to_bf16_bits(x):
    """float32 array -> uint16 bfloat16 bit patterns, round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def to_storage(x, dtype):
    x32 = np.asarray(x, dtype=np.float32)
    return x32 if dtype == "f32" else f32_to_bf16_bits(x32)


def as_f64(stored, dtype):
    """Exact float64 values of a storage array."""
    if dtype == "f32":
        return np.asarray(stored, dtype=np.float32).astype(np.float64)
    u = np.asarray(stored, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def nan_fill(shape, dtype):
    if dtype == "f32":
        return np.full(shape, np.nan, dtype=np.float32)
    return np.full(shape, 0x7FC0, dtype=np.uint16)


# ---------------------------------------------------------------- draws
def _rng(w, stream):
    return np.random.default_rng([w.seed, stream])


def draw_model_side(w):
    """Weights, queries, heavy-channel indices, sign diagonal, lengths, page order.
    Returns a dict of storage arrays / integer arrays."""
    r = _rng(w, 0)
    W_UK = r.standard_normal((w.H, w.d_n, w.d_c))
    W_UV = r.standard_normal((w.H, w.d_c, w.d_v))
    q_nope = r.standard_normal((w.B, w.H, w.d_n))
    q_pe = r.standard_normal((w.B, w.H, w.d_r))
    if w.unit_variance_rows:
        W_UK /= math.sqrt(w.d_c); W_UV /= math.sqrt(w.d_v)
        q_nope /= math.sqrt(w.d_n); q_pe /= math.sqrt(w.d_r)
    else:
        W_UK *= w.weight_std; W_UV *= w.weight_std
    heavy = np.sort(r.choice(w.d_c, size=w.heavy_channels, replace=False)) if w.heavy_channels else np.zeros(0, dtype=np.int64)
    signs = r.choice(np.array([-1.0, 1.0]), size=w.d_c).astype(np.float32)
    if w.ragged:
        lo, hi = w.ragged
        lens = np.floor(np.exp(r.uniform(math.log(lo), math.log(hi), size=w.B))).astype(np.int64)
    else:
        lens = np.full(w.B, w.context, dtype=np.int64)
    pages_per_seq = (lens + w.page_tokens - 1) // w.page_tokens
    n_used = int(pages_per_seq.sum())
    n_pool = n_used + int(math.ceil(n_used * w.pool_slack))
    order = r.permutation(n_pool) if w.permute_pages else np.arange(n_pool)
    max_pages = max(1, int(pages_per_seq.max()))
    block_table = np.zeros((w.B, max_pages), dtype=np.int32)
    k = 0
    for b in range(w.B):
        n = int(pages_per_seq[b])
        block_table[b, :n] = order[k:k + n]
        k += n
    return {
        "W_UK": to_storage(W_UK, w.dtype), "W_UV": to_storage(W_UV, w.dtype),
        "q_nope": to_storage(q_nope, w.dtype), "q_pe": to_storage(q_pe, w.dtype),
        "heavy": heavy, "signs": signs, "seq_lens": lens.astype(np.int32),
        "block_table": block_table, "n_pool_pages": max(1, n_pool), "max_pages": max_pages,
    }


def draw_output_weight(w):
    """W_O [H d_v, d_model] for the output-projection stage (own stream: 500)."""
    r = _rng(w, 500)
    W = r.standard_normal((w.H * w.d_v, w.d_model), dtype=np.float32) * np.float32(w.weight_std)
    return to_storage(W, w.dtype)


def draw_sequence(w, b, L, heavy=None, width=None):
    """Cache-side draws of sequence b: latent rows [L, width or d_c] and k_pe rows
    [L, d_r] as storage arrays.  With rms_prefill the latent rows are the raw
    (un-normalised) latents, each token with its own scale."""
    r = _rng(w, 1000 + b)
    dc = w.d_c if width is None else width
    c = r.standard_normal((L, dc), dtype=np.float32)
    k = r.standard_normal((L, w.d_r), dtype=np.float32)
    if w.unit_variance_rows:
        c /= np.float32(math.sqrt(dc)); k /= np.float32(math.sqrt(w.d_r))
    if heavy is not None and len(heavy):
        c[:, heavy] *= np.float32(10.0)
    if w.rms_prefill:
        c *= np.exp(r.uniform(-1.0, 1.0, size=(L, 1))).astype(np.float32)
    return to_storage(c, w.dtype), to_storage(k, w.dtype)


def draw_anisotropic_latents(seed, n, d, decay=6.0, offset=0.25):
    """Calibration-style latents [n, d] (float32): independent normal components
    whose standard deviations fall geometrically by exp(-decay) from first to
    last, turned by a random rotation and shifted by a constant -- so the
    covariance has a distinct, known-shaped spectrum and a non-zero mean."""
    r = np.random.default_rng([seed, 900])
    rot = np.linalg.qr(r.standard_normal((d, d)))[0]
    scales = np.exp(-decay * np.arange(d) / d)
    return ((r.standard_normal((n, d)) * scales) @ rot.T + offset).astype(np.float32)


# ---------------------------------------------------------------- paging
def place_rows(pool, page_ids, rows):
    """Writes rows [L, width] of one sequence into pool [P, page_tokens, width]
    at the pages listed for it (pure indexing)."""
    pt = pool.shape[1]
    L = rows.shape[0]
    t = np.arange(L)
    pool[np.asarray(page_ids)[t // pt], t % pt] = rows


def slot_mapping(page_ids, L, page_tokens):
    """Flat pool slot (page * page_tokens + offset) of tokens 0..L-1."""
    t = np.arange(L)
    return (np.asarray(page_ids, dtype=np.int64)[t // page_tokens] * page_tokens + t % page_tokens).astype(np.int32)


def algorithmic_bytes_per_shard(w, seq_lens):
    """Cache bytes one shard's decode must read: sum(L_b) * (d_c/g + d_r) * sizeof."""
    esz = 4 if w.dtype == "f32" else 2
    return int(np.sum(seq_lens)) * (w.dl + w.d_r) * esz
