// Orthogonal reparameterisation kernels (Sec. 4.1 / 4.3 of the paper) and the
// MLA-style cache write.
//   * transform_axis_kernel: shape-agnostic, one workgroup per vector, LDS.
//   * transform_paged_fwht_kernel: the streaming cache pass -- one row per
//     group of d_c/8 lanes, 8 elements per lane, Walsh-Hadamard butterflies in
//     registers (strides 1,2,4) and across lanes (strides 8..d_c/2).
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
template <typename T, bool HADAMARD>
__global__ void __launch_bounds__(256) transform_paged_fwht_kernel(
    TransformArgs t, const T* __restrict__ mla_pool, ShardPools pools, const int32_t* __restrict__ page_ids,
    int64_t n_rows, int page_tokens, int d_r, int g) {
  const int d_c = t.d_c, dl = d_c / g;
  const int lpr = d_c / 8;
  const int rows_per_block = 256 / lpr;
  const int sub = threadIdx.x / lpr, l = threadIdx.x % lpr;
  const int64_t row = (int64_t)blockIdx.x * rows_per_block + sub;
  if (row >= n_rows) return;
  const int64_t pg = row / page_tokens;
  const int slot = (int)(row % page_tokens);
  const int64_t page = page_ids ? (int64_t)page_ids[pg] : pg;
  const size_t in_row = ((size_t)page * page_tokens + slot) * (size_t)(d_c + d_r);
  const size_t out_row = ((size_t)page * page_tokens + slot) * (size_t)(dl + d_r);

  Vec8 x = load8(mla_pool + in_row + 8 * l);
  if (HADAMARD) {
    if (t.signs) {
#pragma unroll
      for (int i = 0; i < 8; ++i) x.v[i] *= t.signs[8 * l + i];
    }
    // strides 1, 2, 4 inside the lane
#pragma unroll
    for (int h = 1; h < 8; h <<= 1)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (!(i & h)) {
          const float u = x.v[i], v = x.v[i | h];
          x.v[i] = u + v;
          x.v[i | h] = u - v;
        }
    // strides 8 .. d_c/2 across lanes: partner lane l ^ m
    for (int m = 1; m < lpr; m <<= 1) {
      const bool upper = (l & m) != 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float other = __shfl_xor(x.v[i], m);
        x.v[i] = upper ? (other - x.v[i]) : (x.v[i] + other);
      }
    }
    const float sc = 1.0f / sqrtf((float)d_c);
#pragma unroll
    for (int i = 0; i < 8; ++i) x.v[i] *= sc;
  }
  const int col = 8 * l;
  const int shard = col / dl;
  store8(static_cast<T*>(pools.p[shard]) + out_row + (col - shard * dl), x);
  // replicate the RoPE key on every slice
  for (int c = 8 * l; c < d_r; c += 8 * lpr) {
    const Vec8 k = load8(mla_pool + in_row + d_c + c);
    for (int i = 0; i < g; ++i) store8(static_cast<T*>(pools.p[i]) + out_row + dl + c, k);
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
  const bool fast = pow2 && lpr >= 1 && lpr <= 64 && (t.mode == TPLA_U_HADAMARD || t.mode == TPLA_U_IDENTITY);
  const T* in = static_cast<const T*>(mla_pool);
  if (fast) {
    const int rows_per_block = 256 / lpr;
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

}  // namespace tpla
