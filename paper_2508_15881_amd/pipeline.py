"""Device buffers and call sequencing for one TPLA decode layer-step.

Only marshalling: torch allocates device memory and provides the stream;
every arithmetic step runs inside libtpla (see include/tpla.h).
"""
import math

import numpy as np
import torch

from . import binding as B


def torch_dtype(dtype):
    return torch.float32 if dtype in ("f32", B.TPLA_F32) else torch.bfloat16


def to_device(stored, dtype, device="cuda"):
    """Storage array (float32, or uint16 bf16 bit patterns) -> device tensor."""
    a = np.ascontiguousarray(stored)
    if dtype == "f32":
        return torch.from_numpy(a).to(device)
    return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)


def from_device_bits(t):
    """Device tensor -> storage array (float32, or uint16 bit patterns for bf16)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def make_shape(w):
    """TplaShape of a workloads.Workload."""
    return B.TplaShape(w.B, w.H, w.d_c, w.g, w.d_r, w.d_n, w.d_v, w.page_tokens,
                       B.TPLA_F32 if w.dtype == "f32" else B.TPLA_BF16, w.sm_scale)


class DecodeStep:
    """Buffers for absorb -> g x decode_shard -> combine on one GPU."""

    def __init__(self, shape, max_pages_per_seq, n_splits=0, device="cuda", d_model=0):
        self.shape = shape
        self.max_pages = int(max_pages_per_seq)
        self.n_splits = int(n_splits)
        st = torch.float32 if shape.dtype == B.TPLA_F32 else torch.bfloat16
        g, Bn, H, dl = shape.g, shape.B, shape.H, shape.d_c // shape.g
        self.q_lat = torch.empty((g, Bn, H, dl), dtype=st, device=device)
        self.o_lat = torch.empty((g, Bn, H, dl), dtype=torch.float32, device=device)
        self.lse = torch.empty((g, Bn, H), dtype=torch.float32, device=device)
        self.o = torch.empty((Bn, H, shape.d_v), dtype=torch.float32, device=device)
        self.ws_bytes = max(B.tpla_workspace_bytes(shape, self.max_pages, self.n_splits),
                            B.tpla_workspace_bytes_all(shape, self.max_pages, self.n_splits))
        if self.ws_bytes == 0:
            raise B.TplaError(-2, B.tpla_last_error())
        # with a block output width the workspace also serves the output projection's partial tiles
        self.d_model = int(d_model)
        if self.d_model > 0:
            self.ws_bytes = max(self.ws_bytes, B.tpla_attention_block_workspace_bytes(shape, self.max_pages, self.n_splits, self.d_model))
            self.out = torch.empty((Bn, self.d_model), dtype=st, device=device)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)

    def absorb(self, q_nope, W_UK_t, mu=None):
        B.tpla_absorb_query(self.shape, q_nope, W_UK_t, mu, self.q_lat)

    def decode(self, i, q_pe, shard_pool, block_table, seq_lens):
        B.tpla_decode_shard(self.shape, self.q_lat[i], q_pe, shard_pool, block_table, self.max_pages,
                            seq_lens, self.n_splits, self.workspace, self.ws_bytes,
                            self.o_lat[i], self.lse[i])

    def decode_all(self, q_pe, shard_pools, block_table, seq_lens):
        """All g slices in one launch."""
        B.tpla_decode_shards(self.shape, self.q_lat, q_pe, shard_pools, block_table, self.max_pages,
                             seq_lens, self.n_splits, self.workspace, self.ws_bytes, self.o_lat, self.lse)

    def combine(self, W_UV_t):
        B.tpla_combine_shards(self.shape, self.o_lat, W_UV_t, self.o)

    def decode_all_combine(self, q_pe, shard_pools, block_table, seq_lens, W_UV_t):
        """All g slices in one launch, then the split merge and the combine as one kernel."""
        B.tpla_decode_shards_combine(self.shape, self.q_lat, q_pe, shard_pools, block_table, self.max_pages,
                                     seq_lens, self.n_splits, self.workspace, self.ws_bytes, W_UV_t, self.o,
                                     self.o_lat, self.lse)

    def decode_all_project(self, q_pe, shard_pools, block_table, seq_lens, W_UV_t, W_O):
        """All g slices in one launch, merge + combine, then the block's output projection: one call.
        self.out [B, d_model] is written in the storage type (bf16 for bf16 shapes)."""
        B.tpla_decode_shards_project(self.shape, self.q_lat, q_pe, shard_pools, block_table, self.max_pages, seq_lens,
                                     self.n_splits, self.workspace, self.ws_bytes, W_UV_t, W_O, self.d_model, self.out,
                                     self.shape.dtype, self.o, self.o_lat, self.lse)

    def run(self, q_nope, q_pe, W_UK_t, W_UV_t, shard_pools, block_table, seq_lens, mu=None, fused=True):
        """One decode layer-step.  fused: all slices in one decode launch with the merge and
        the combine behind it as one kernel (how one GPU runs the whole step); otherwise one
        tpla_decode_shard call per slice (one device's share at a time), then the combine."""
        self.absorb(q_nope, W_UK_t, mu)
        if fused:
            self.decode_all_combine(q_pe, shard_pools, block_table, seq_lens, W_UV_t)
        else:
            for i in range(self.shape.g):
                self.decode(i, q_pe, shard_pools[i], block_table, seq_lens)
            self.combine(W_UV_t)
        return self.o


    def capture(self, q_nope, q_pe, W_UK_t, W_UV_t, shard_pools, block_table, seq_lens, mu=None, fused=True):
        """The layer-step as a HIP graph (torch.cuda.CUDAGraph): one eager run first (kernel
        attributes are set on first use), then the capture.  Replaying it reads the same input
        tensors and writes self.o, self.o_lat, self.lse; the library allocates nothing and records
        no memset, so the step is capturable as it is.  tpla_profile_enable must be off."""
        self.run(q_nope, q_pe, W_UK_t, W_UV_t, shard_pools, block_table, seq_lens, mu, fused)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(q_nope, q_pe, W_UK_t, W_UV_t, shard_pools, block_table, seq_lens, mu, fused)
        return graph


def transform_weights(shape, mode, signs, U, W_UK, W_UV):
    """W_UK [H,d_n,d_c] -> W_UK U (last axis); W_UV [H,d_c,d_v] -> U^T W_UV (middle axis)."""
    W_UK_t = torch.empty_like(W_UK)
    W_UV_t = torch.empty_like(W_UV)
    H, d_n, d_c = W_UK.shape
    B.tpla_transform_latent(shape, mode, 0, signs, U, W_UK, W_UK_t, H * d_n, 1)
    B.tpla_transform_latent(shape, mode, 0, signs, U, W_UV, W_UV_t, H, W_UV.shape[2])
    return W_UK_t, W_UV_t


def pca_calibrate(shape, mla_pool, page_ids, page_fill, n_rows, device="cuda"):
    """PCA basis of the latents in the listed pages: second moments on the GPU
    (tpla_latent_moments), eigen-decomposition on the host (tpla_pca_basis).
    n_rows = number of valid rows (all page_fill entries, or pages x page_tokens).
    Returns (U float32 device tensor [d_c, d_c], eigenvalues, variance fractions of the g slices)."""
    n_pages = int(page_ids.numel()) if page_ids is not None else int(mla_pool.shape[0])
    ws_b = B.tpla_latent_moments_workspace_bytes(shape, n_pages)
    ws = torch.empty(max(ws_b, 16), dtype=torch.uint8, device=device)
    s = torch.empty(shape.d_c, dtype=torch.float64, device=device)
    G = torch.empty((shape.d_c, shape.d_c), dtype=torch.float64, device=device)
    B.tpla_latent_moments(shape, mla_pool, page_ids, page_fill, n_pages, ws, ws_b, s, G)
    torch.cuda.synchronize()
    U, eig, frac = B.tpla_pca_basis(shape.d_c, shape.g, int(n_rows), s.cpu().numpy(), G.cpu().numpy())
    return torch.from_numpy(U).to(device), eig, frac
