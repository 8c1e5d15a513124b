// Orthogonal reparameterisation kernels (Sec. 4.1 / 4.3 of the paper) and the
// MLA-style cache write.
//   * transform_axis_kernel: shape-agnostic, one workgroup per vector, LDS.
//   * transform_paged_fwht_kernel: streaming cache pass on the vector ALU -- one
//     row per group of d_c/8 lanes, 8 elements per lane, Walsh-Hadamard
//     butterflies in registers (strides 1,2,4) and across lanes (strides
//     8..d_c/2).  Runs the identity (slicing-only) pass, float storage and the
//     widths the matrix-core pass (transform_mfma.hip) does not take.
//   * transform_paged_generic_kernel: identity / dense U / wide rows.
#include "tpla_internal.h"

namespace tpla {

// ---------------------------------------------------------------------------
// In-LDS transform of one vector x[0..d) (float), result left in x.
// mode identity: nothing.  Hadamard: natural-order butterflies, 1/sqrt(d),
// sign diagonal before (forward) or after (inverse).  Dense: y = x U or x U^T.
// `tmp` is a second d-float buffer.  All threads of the block must call.
__device__ void transform_vector_lds(float* x, float* tmp, int d, const TransformArgs& t) {
  const int tid = threadIdx.x, nt = blockDim.x;
  if (t.mode == TPLA_U_IDENTITY) return;
  if (t.mode == TPLA_U_HADAMARD) {
    if (t.signs && !t.inverse) {
      for (int i = tid; i < d; i += nt) x[i] *= t.signs[i];
      __syncthreads();
    }
    for (int h = 1; h < d; h <<= 1) {
      for (int i = tid; i < d / 2; i += nt) {
        const int lo = ((i / h) * 2 * h) + (i % h), hi = lo + h;
        const float u = x[lo], v = x[hi];
        x[lo] = u + v;
        x[hi] = u - v;
      }
      __syncthreads();
    }
    const float sc = 1.0f / sqrtf((float)d);
    for (int i = tid; i < d; i += nt) {
      float v = x[i] * sc;
      if (t.signs && t.inverse) v *= t.signs[i];
      x[i] = v;
    }
    __syncthreads();
    return;
  }
  // dense
  for (int j = tid; j < d; j += nt) {
    float s = 0.f;
    if (!t.inverse)
      for (int k = 0; k < d; ++k) s = fmaf(x[k], t.U[(size_t)k * d + j], s);
    else
      for (int k = 0; k < d; ++k) s = fmaf(x[k], t.U[(size_t)j * d + k], s);
    tmp[j] = s;
  }
  __syncthreads();
  for (int j = tid; j < d; j += nt) x[j] = tmp[j];
  __syncthreads();
}

template <typename T>
__global__ void __launch_bounds__(256) transform_axis_kernel(TransformArgs t, const T* __restrict__ src,
                                                             T* __restrict__ dst, int64_t n_inner) {
  extern __shared__ float smem[];
  const int d = t.d_c;
  float* x = smem;
  float* tmp = smem + d;
  const int64_t o = blockIdx.x / n_inner, i = blockIdx.x % n_inner;
  const T* s = src + (size_t)o * d * n_inner + i;
  T* q = dst + (size_t)o * d * n_inner + i;
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[k] = load_as_f32(s + (size_t)k * n_inner);
  __syncthreads();
  transform_vector_lds(x, tmp, d, t);
  for (int k = threadIdx.x; k < d; k += blockDim.x) store_from_f32(q + (size_t)k * n_inner, x[k]);
}

int launch_transform_axis(const TransformArgs& t, const void* src, void* dst, int64_t n_outer,
                          int64_t n_inner, hipStream_t st) {
  const size_t smem = 2u * (size_t)t.d_c * sizeof(float);
  const dim3 grid((unsigned)(n_outer * n_inner));
  if (t.dtype == TPLA_F32)
    hipLaunchKernelGGL(transform_axis_kernel<float>, grid, dim3(256), smem, st, t,
                       static_cast<const float*>(src), static_cast<float*>(dst), n_inner);
  else
    hipLaunchKernelGGL(transform_axis_kernel<bf16_t>, grid, dim3(256), smem, st, t,
                       static_cast<const bf16_t*>(src), static_cast<bf16_t*>(dst), n_inner);
  return check_launch("transform_axis_kernel");
}

// ---------------------------------------------------------------------------
// Streaming pass over MLA pages: row = [latent d_c | k_pe d_r].  LPR = d_c/8
// lanes cooperate on one row (LPR a power of two <= 64).  After the transform
// lane l holds elements 8l..8l+7 of c U, which belong to slice (8l)/dl.
// Value of lane (l ^ M) without going through LDS: DPP for M < 16, the
// row / half swaps of gfx950 above that.
template <int M>
__device__ __forceinline__ float lane_xor(float v, int lane) {
  const int x = __float_as_int(v);
  if constexpr (M == 1) return __int_as_float(__builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  if constexpr (M == 2) return __int_as_float(__builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  if constexpr (M == 4) {
    // rotations by 4 and 12 inside a row of 16: one of them is lane l + 4, the other l - 4
    const int a = __builtin_amdgcn_update_dpp(x, x, 0x124, 0xF, 0xF, false);   // row_ror:4  -> lane (l - 4) & 15
    const int b = __builtin_amdgcn_update_dpp(x, x, 0x12C, 0xF, 0xF, false);   // row_ror:12 -> lane (l + 4) & 15
    return __int_as_float((lane & 4) ? a : b);
  }
  if constexpr (M == 8) return __int_as_float(__builtin_amdgcn_update_dpp(x, x, 0x128, 0xF, 0xF, false));  // row_ror:8
  if constexpr (M == 16) {
    // swaps rows 1,3 of the first operand with rows 0,2 of the second
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)x, false, false);
    return __int_as_float((int)((lane & 16) ? r[0] : r[1]));
  }
  if constexpr (M == 32) {
    // swaps the upper half of the first operand with the lower half of the second
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return __int_as_float((int)((lane & 32) ? r[0] : r[1]));
  }
  return v;
}

constexpr int FWHT_ROWS_MAX = 4;
template <int M>
__device__ __forceinline__ void fwht_lane_stage(Vec8* x, int n_rows_here, int l, int lane, int lpr) {
  if (M >= lpr) return;
  const float sg = (l & M) ? -1.0f : 1.0f;
#pragma unroll
  for (int r = 0; r < FWHT_ROWS_MAX; ++r)
    if (r < n_rows_here)
#pragma unroll
    for (int i = 0; i < 8; ++i) x[r].v[i] = fmaf(x[r].v[i], sg, lane_xor<M>(x[r].v[i], lane));
}

constexpr int FWHT_ROWS = FWHT_ROWS_MAX;   // rows per lane group: their loads and butterflies are independent
template <typename T, bool HADAMARD>
__global__ void __launch_bounds__(256) transform_paged_fwht_kernel(
    TransformArgs t, const T* __restrict__ mla_pool, ShardPools pools, const int32_t* __restrict__ page_ids,
    int64_t n_rows, int page_tokens, int d_r, int g) {
  const int d_c = t.d_c, dl = d_c / g;
  const int lpr = d_c / 8;
  const int rows_per_block = (256 / lpr) * FWHT_ROWS;
  const int sub = threadIdx.x / lpr, l = threadIdx.x % lpr;
  // 32-bit row arithmetic (n_rows < 2^31 is checked by the caller); one
  // division per lane group, the following rows step through the page
  const unsigned row0 = blockIdx.x * (unsigned)rows_per_block + (unsigned)sub * FWHT_ROWS;
  const unsigned last = (unsigned)(n_rows - 1);
  const unsigned base_row = min(row0, last);
  const unsigned pg0 = base_row / (unsigned)page_tokens;
  const unsigned slot0 = base_row - pg0 * (unsigned)page_tokens;
  // rows past the end redo the last row (same values to the same place), so
  // every lane takes part in the lane exchanges
  size_t in_row[FWHT_ROWS], out_row[FWHT_ROWS];
  Vec8 x[FWHT_ROWS], kpe[FWHT_ROWS];
  const bool has_kpe = 8 * l < d_r;          // d_r <= d_c for this kernel: one piece per lane at most
#pragma unroll
  for (int r = 0; r < FWHT_ROWS; ++r) {
    unsigned pg = pg0, slot = slot0;
    if (row0 + r <= last) {
      slot += r;
      if (slot >= (unsigned)page_tokens) { slot -= page_tokens; pg += 1; }   // FWHT_ROWS <= page_tokens
    }
    const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
    const size_t tok = page * page_tokens + slot;
    in_row[r] = tok * (size_t)(d_c + d_r);
    out_row[r] = tok * (size_t)(dl + d_r);
    x[r] = load8(mla_pool + in_row[r] + 8 * l);
    if (has_kpe) kpe[r] = load8(mla_pool + in_row[r] + d_c + 8 * l);
  }
  if (HADAMARD) {
    if (t.signs) {
      float sg[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) sg[i] = t.signs[8 * l + i];
#pragma unroll
      for (int r = 0; r < FWHT_ROWS; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) x[r].v[i] *= sg[i];
    }
    // strides 1, 2, 4 inside the lane
#pragma unroll
    for (int r = 0; r < FWHT_ROWS; ++r)
#pragma unroll
      for (int h = 1; h < 8; h <<= 1)
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (!(i & h)) {
            const float u = x[r].v[i], v = x[r].v[i | h];
            x[r].v[i] = u + v;
            x[r].v[i | h] = u - v;
          }
    // strides 8 .. d_c/2 across lanes: partner lane l ^ m, new = partner + (upper ? -own : own)
    const int lane = threadIdx.x & 63;
    fwht_lane_stage<1>(x, FWHT_ROWS, l, lane, lpr);
    fwht_lane_stage<2>(x, FWHT_ROWS, l, lane, lpr);
    fwht_lane_stage<4>(x, FWHT_ROWS, l, lane, lpr);
    fwht_lane_stage<8>(x, FWHT_ROWS, l, lane, lpr);
    fwht_lane_stage<16>(x, FWHT_ROWS, l, lane, lpr);
    fwht_lane_stage<32>(x, FWHT_ROWS, l, lane, lpr);
    const float sc = 1.0f / sqrtf((float)d_c);
#pragma unroll
    for (int r = 0; r < FWHT_ROWS; ++r)
#pragma unroll
      for (int i = 0; i < 8; ++i) x[r].v[i] *= sc;
  }
  const int col = 8 * l;
  const int shard = col / dl;
#pragma unroll
  for (int r = 0; r < FWHT_ROWS; ++r) {
    if (row0 + r > last) break;
    store8(static_cast<T*>(pools.p[shard]) + out_row[r] + (col - shard * dl), x[r]);
    // replicate the RoPE key on every slice
    if (has_kpe)
      for (int i = 0; i < g; ++i) store8(static_cast<T*>(pools.p[i]) + out_row[r] + dl + 8 * l, kpe[r]);
  }
}

// Any mode / width: one workgroup per row through LDS.
template <typename T>
__global__ void __launch_bounds__(256) transform_paged_generic_kernel(
    TransformArgs t, const T* __restrict__ mla_pool, ShardPools pools, const int32_t* __restrict__ page_ids,
    int page_tokens, int d_r, int g) {
  extern __shared__ float smem[];
  const int d_c = t.d_c, dl = d_c / g;
  float* x = smem;
  float* tmp = smem + d_c;
  const int64_t row = blockIdx.x;
  const int64_t pg = row / page_tokens;
  const int slot = (int)(row % page_tokens);
  const int64_t page = page_ids ? (int64_t)page_ids[pg] : pg;
  const T* in = mla_pool + ((size_t)page * page_tokens + slot) * (size_t)(d_c + d_r);
  const size_t out_row = ((size_t)page * page_tokens + slot) * (size_t)(dl + d_r);
  for (int k = threadIdx.x; k < d_c; k += blockDim.x) x[k] = load_as_f32(in + k);
  __syncthreads();
  transform_vector_lds(x, tmp, d_c, t);
  for (int k = threadIdx.x; k < d_c; k += blockDim.x) {
    const int shard = k / dl;
    store_from_f32(static_cast<T*>(pools.p[shard]) + out_row + (k - shard * dl), x[k]);
  }
  for (int k = threadIdx.x; k < d_r; k += blockDim.x) {
    const T v = in[d_c + k];
    for (int i = 0; i < g; ++i) static_cast<T*>(pools.p[i])[out_row + dl + k] = v;
  }
}

template <typename T>
static int launch_paged_t(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                          const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                          hipStream_t st) {
  const int64_t n_rows = n_pages * sh.page_tokens;
  const int lpr = sh.d_c / 8;
  const bool pow2 = (sh.d_c & (sh.d_c - 1)) == 0;
  const bool fast = pow2 && lpr >= 1 && lpr <= 64 && sh.d_r <= sh.d_c && sh.page_tokens >= FWHT_ROWS &&
                    (t.mode == TPLA_U_HADAMARD || t.mode == TPLA_U_IDENTITY);
  const T* in = static_cast<const T*>(mla_pool);
  if (fast) {
    const int rows_per_block = (256 / lpr) * FWHT_ROWS;
    const dim3 grid((unsigned)((n_rows + rows_per_block - 1) / rows_per_block));
    if (t.mode == TPLA_U_HADAMARD)
      hipLaunchKernelGGL((transform_paged_fwht_kernel<T, true>), grid, dim3(256), 0, st, t, in, pools,
                         page_ids, n_rows, sh.page_tokens, sh.d_r, sh.g);
    else
      hipLaunchKernelGGL((transform_paged_fwht_kernel<T, false>), grid, dim3(256), 0, st, t, in, pools,
                         page_ids, n_rows, sh.page_tokens, sh.d_r, sh.g);
    return check_launch("transform_paged_fwht_kernel");
  }
  const size_t smem = 2u * (size_t)sh.d_c * sizeof(float);
  hipLaunchKernelGGL(transform_paged_generic_kernel<T>, dim3((unsigned)n_rows), dim3(256), smem, st, t,
                     in, pools, page_ids, sh.page_tokens, sh.d_r, sh.g);
  return check_launch("transform_paged_generic_kernel");
}

int launch_transform_paged(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                           const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                           hipStream_t st) {
  if (transform_paged_mfma_supported(t, sh, n_pages))
    return launch_transform_paged_mfma(t, sh, mla_pool, pools, page_ids, n_pages, st);
  if (transform_paged_dense_mfma_supported(t, sh, n_pages))
    return launch_transform_paged_dense_mfma(t, sh, mla_pool, pools, page_ids, n_pages, st);
  if (sh.dtype == TPLA_F32) return launch_paged_t<float>(t, sh, mla_pool, pools, page_ids, n_pages, st);
  return launch_paged_t<bf16_t>(t, sh, mla_pool, pools, page_ids, n_pages, st);
}

// ---------------------------------------------------------------------------
// MLA-style cache write: one wave per token.
template <typename T>
__global__ void __launch_bounds__(256) write_mla_cache_kernel(const T* __restrict__ c_raw,
                                                              const T* __restrict__ k_pe,
                                                              const int32_t* __restrict__ slot_mapping,
                                                              int64_t n_tok, float rms_eps, T* __restrict__ pool,
                                                              int d_c, int d_r) {
  const int lane = threadIdx.x & 63;
  const int64_t tkn = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tkn >= n_tok) return;
  const int slot = slot_mapping[tkn];
  if (slot < 0) return;
  const T* c = c_raw + (size_t)tkn * d_c;
  T* out = pool + (size_t)slot * (size_t)(d_c + d_r);
  float scale = 1.0f;
  if (rms_eps >= 0.f) {
    float ss = 0.f;
    for (int k = lane; k < d_c; k += 64) {
      const float v = load_as_f32(c + k);
      ss = fmaf(v, v, ss);
    }
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) ss += __shfl_xor(ss, m);
    scale = 1.0f / sqrtf(ss / (float)d_c + rms_eps);
  }
  for (int k = lane; k < d_c; k += 64) store_from_f32(out + k, load_as_f32(c + k) * scale);
  for (int k = lane; k < d_r; k += 64) out[d_c + k] = k_pe[(size_t)tkn * d_r + k];
}

int launch_write_mla_cache(const tpla_shape_t& sh, const void* c_raw, const void* k_pe,
                           const int32_t* slot_mapping, int64_t T, float rms_eps, void* mla_pool,
                           hipStream_t st) {
  const dim3 grid((unsigned)((T + 3) / 4));
  if (sh.dtype == TPLA_F32)
    hipLaunchKernelGGL(write_mla_cache_kernel<float>, grid, dim3(256), 0, st,
                       static_cast<const float*>(c_raw), static_cast<const float*>(k_pe), slot_mapping, T,
                       rms_eps, static_cast<float*>(mla_pool), sh.d_c, sh.d_r);
  else
    hipLaunchKernelGGL(write_mla_cache_kernel<bf16_t>, grid, dim3(256), 0, st,
                       static_cast<const bf16_t*>(c_raw), static_cast<const bf16_t*>(k_pe), slot_mapping, T,
                       rms_eps, static_cast<bf16_t*>(mla_pool), sh.d_c, sh.d_r);
  return check_launch("write_mla_cache_kernel");
}

// ---------------------------------------------------------------------------
// Decode-token append with per-slice RMSNorm: one wave per (sequence, slice).
template <typename T>
__global__ void __launch_bounds__(64) append_token_sliced_kernel(const T* __restrict__ c_t,
                                                                 const T* __restrict__ k_pe,
                                                                 MuFactors alpha, float rms_eps,
                                                                 const int32_t* __restrict__ slots,
                                                                 ShardPools pools, int d_c, int d_r, int g) {
  const int b = blockIdx.x, i = blockIdx.y, lane = threadIdx.x;
  const int slot = slots[b];
  if (slot < 0) return;
  const int dl = d_c / g;
  const T* x = c_t + (size_t)b * d_c + (size_t)i * dl;
  float ss = 0.f;
  for (int k = lane; k < dl; k += 64) {
    const float v = load_as_f32(x + k);
    ss = fmaf(v, v, ss);
  }
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) ss += __shfl_xor(ss, m);
  const float scale = 1.0f / sqrtf(alpha.v[i] * ss / (float)d_c + rms_eps);
  T* out = static_cast<T*>(pools.p[i]) + (size_t)slot * (size_t)(dl + d_r);
  for (int k = lane; k < dl; k += 64) store_from_f32(out + k, load_as_f32(x + k) * scale);
  for (int k = lane; k < d_r; k += 64) out[dl + k] = k_pe[(size_t)b * d_r + k];
}

int launch_append_token_sliced(const tpla_shape_t& sh, const void* c_t, const void* k_pe,
                               const MuFactors& alpha, float rms_eps, const int32_t* slots,
                               const ShardPools& pools, hipStream_t st) {
  const dim3 grid((unsigned)sh.B, (unsigned)sh.g);
  if (sh.dtype == TPLA_F32)
    hipLaunchKernelGGL(append_token_sliced_kernel<float>, grid, dim3(64), 0, st, static_cast<const float*>(c_t),
                       static_cast<const float*>(k_pe), alpha, rms_eps, slots, pools, sh.d_c, sh.d_r, sh.g);
  else
    hipLaunchKernelGGL(append_token_sliced_kernel<bf16_t>, grid, dim3(64), 0, st, static_cast<const bf16_t*>(c_t),
                       static_cast<const bf16_t*>(k_pe), alpha, rms_eps, slots, pools, sh.d_c, sh.d_r, sh.g);
  return check_launch("append_token_sliced_kernel");
}

}  // namespace tpla
