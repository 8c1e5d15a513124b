// The two small per-head contractions around the shard decode:
//   absorb  : q_lat[i,b,h,:] = mu_i * (q_nope[b,h,:] @ W_UK_t[h])[slice i]     (Sec. 3.3, 4, 4.2)
//   combine : o[b,h,:] = sum_i o_lat[i,b,h,:] @ W_UV_t[h, slice i, :]          (Sec. 4, sum = all-reduce)
// Both read each weight element once per chunk of BT sequences; the weights
// (a few MB) dominate their traffic.
#include "tpla_internal.h"

namespace tpla {

constexpr int BT = 16;   // sequences per register tile

// grid (H, ceil(d_c / 256), ceil(B / BT)); thread = one latent column.
template <typename T>
__global__ void __launch_bounds__(256) absorb_query_kernel(const T* __restrict__ q_nope,
                                                           const T* __restrict__ W, MuFactors mu,
                                                           T* __restrict__ q_lat, int B, int H, int d_n,
                                                           int d_c, int g) {
  extern __shared__ float qs[];   // [BT][d_n]
  const int h = blockIdx.x;
  const int col = blockIdx.y * 256 + threadIdx.x;
  const int b0 = blockIdx.z * BT;
  const int nb = min(BT, B - b0);
  for (int i = threadIdx.x; i < BT * d_n; i += 256) {
    const int bb = i / d_n, n = i % d_n;
    qs[i] = (bb < nb) ? load_as_f32(q_nope + ((size_t)(b0 + bb) * H + h) * d_n + n) : 0.f;
  }
  __syncthreads();
  if (col >= d_c) return;
  float acc[BT];
#pragma unroll
  for (int bb = 0; bb < BT; ++bb) acc[bb] = 0.f;
  const T* w = W + (size_t)h * d_n * d_c + col;
  for (int n = 0; n < d_n; ++n) {
    const float wv = load_as_f32(w + (size_t)n * d_c);
#pragma unroll
    for (int bb = 0; bb < BT; ++bb) acc[bb] = fmaf(qs[bb * d_n + n], wv, acc[bb]);
  }
  const int dl = d_c / g;
  const int i = col / dl, c = col - i * dl;
  const float m = mu.v[i];
#pragma unroll
  for (int bb = 0; bb < BT; ++bb)
    if (bb < nb) store_from_f32(q_lat + (((size_t)i * B + (b0 + bb)) * H + h) * dl + c, acc[bb] * m);
}


// Vectorised variant: workgroup = (head, 256-column slab, 8 sequences).
// Thread (cg, ng): 8 consecutive latent columns, query rows ng, ng+8, ...
// (a 32-lane half-wave reads one 512-byte piece of a weight row), 8x8
// accumulators; the 8 row groups are summed with one shuffle and one pass
// through LDS.
constexpr int AB = 8;   // sequences per workgroup
template <typename T>
__global__ void __launch_bounds__(256) absorb_query_vec_kernel(const T* __restrict__ q_nope,
                                                               const T* __restrict__ W, MuFactors mu,
                                                               T* __restrict__ q_lat, int B, int H, int d_n,
                                                               int d_c, int g) {
  extern __shared__ float sm[];          // [AB][d_n] queries, then [4][AB][256] partial sums
  float* qs = sm;
  float* red = sm + AB * d_n;
  const int h = blockIdx.x;
  const int col0 = blockIdx.y * 256;
  const int b0 = blockIdx.z * AB;
  const int nb = min(AB, B - b0);
  const int tid = threadIdx.x, cg = tid & 31, ng = tid >> 5, wave = tid >> 6;
  for (int i = tid; i < AB * d_n; i += 256) {
    const int bb = i / d_n, n = i % d_n;
    qs[i] = (bb < nb) ? load_as_f32(q_nope + ((size_t)(b0 + bb) * H + h) * d_n + n) : 0.f;
  }
  __syncthreads();
  const int col = col0 + cg * 8;
  float acc[AB][8];
#pragma unroll
  for (int bb = 0; bb < AB; ++bb)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[bb][c] = 0.f;
  if (col < d_c) {
    const T* w = W + (size_t)h * d_n * d_c + col;
    for (int n = ng; n < d_n; n += 8) {
      const Vec8 wv = load8_cached(w + (size_t)n * d_c);
#pragma unroll
      for (int bb = 0; bb < AB; ++bb) {
        const float qv = qs[bb * d_n + n];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[bb][c] = fmaf(qv, wv.v[c], acc[bb][c]);
      }
    }
  }
  // the two row groups of a wave, then the four waves
#pragma unroll
  for (int bb = 0; bb < AB; ++bb)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[bb][c] += __shfl_xor(acc[bb][c], 32);
  if ((tid & 32) == 0) {
#pragma unroll
    for (int bb = 0; bb < AB; ++bb)
#pragma unroll
      for (int c = 0; c < 8; ++c) red[(wave * AB + bb) * 256 + cg * 8 + c] = acc[bb][c];
  }
  __syncthreads();
  // thread -> (sequence bb, column group): 8 x 32 outputs of 8 columns
  const int bb = tid >> 5;
  if (bb < nb && col < d_c) {
    Vec8 r;
#pragma unroll
    for (int c = 0; c < 8; ++c)
      r.v[c] = red[(0 * AB + bb) * 256 + cg * 8 + c] + red[(1 * AB + bb) * 256 + cg * 8 + c] +
               red[(2 * AB + bb) * 256 + cg * 8 + c] + red[(3 * AB + bb) * 256 + cg * 8 + c];
    const int dl = d_c / g;
    const int i = col / dl, c0 = col - i * dl;       // 8 columns never straddle a slice (dl % 8 == 0)
    const float m = mu.v[i];
#pragma unroll
    for (int c = 0; c < 8; ++c) r.v[c] *= m;
    T* dst = q_lat + (((size_t)i * B + (b0 + bb)) * H + h) * dl + c0;
    if (sizeof(T) == 2) {
      u32x4 raw;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        raw[c] = (unsigned)f32_to_bf16_bits(r.v[2 * c]) | ((unsigned)f32_to_bf16_bits(r.v[2 * c + 1]) << 16);
      *reinterpret_cast<u32x4*>(dst) = raw;
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) store_from_f32(dst + c, r.v[c]);
    }
  }
}

int launch_absorb_query(const tpla_shape_t& sh, const void* q_nope, const void* W_UK_t,
                        const MuFactors& mu, void* q_lat, hipStream_t st) {
  {
    const size_t vsm = ((size_t)AB * sh.d_n + 4u * AB * 256) * sizeof(float);
    const dim3 vgrid((unsigned)sh.H, (unsigned)((sh.d_c + 255) / 256), (unsigned)((sh.B + AB - 1) / AB));
    if (vsm <= 64 * 1024 && vgrid.y <= 65535 && vgrid.z <= 65535) {
      if (sh.dtype == TPLA_F32)
        hipLaunchKernelGGL(absorb_query_vec_kernel<float>, vgrid, dim3(256), vsm, st,
                           static_cast<const float*>(q_nope), static_cast<const float*>(W_UK_t), mu,
                           static_cast<float*>(q_lat), sh.B, sh.H, sh.d_n, sh.d_c, sh.g);
      else
        hipLaunchKernelGGL(absorb_query_vec_kernel<bf16_t>, vgrid, dim3(256), vsm, st,
                           static_cast<const bf16_t*>(q_nope), static_cast<const bf16_t*>(W_UK_t), mu,
                           static_cast<bf16_t*>(q_lat), sh.B, sh.H, sh.d_n, sh.d_c, sh.g);
      return check_launch("absorb_query_vec_kernel");
    }
  }
  const size_t smem = (size_t)BT * sh.d_n * sizeof(float);
  if (smem > 64 * 1024) return fail(TPLA_ERR_UNSUPPORTED, "d_n=%d too wide", sh.d_n);
  const dim3 grid((unsigned)sh.H, (unsigned)((sh.d_c + 255) / 256), (unsigned)((sh.B + BT - 1) / BT));
  if (grid.x > 65535 * 32768u || grid.y > 65535 || grid.z > 65535)
    return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  if (sh.dtype == TPLA_F32)
    hipLaunchKernelGGL(absorb_query_kernel<float>, grid, dim3(256), smem, st,
                       static_cast<const float*>(q_nope), static_cast<const float*>(W_UK_t), mu,
                       static_cast<float*>(q_lat), sh.B, sh.H, sh.d_n, sh.d_c, sh.g);
  else
    hipLaunchKernelGGL(absorb_query_kernel<bf16_t>, grid, dim3(256), smem, st,
                       static_cast<const bf16_t*>(q_nope), static_cast<const bf16_t*>(W_UK_t), mu,
                       static_cast<bf16_t*>(q_lat), sh.B, sh.H, sh.d_n, sh.d_c, sh.g);
  return check_launch("absorb_query_kernel");
}

// grid (H, ceil(d_v / 128), ceil(B / BT)); thread = one value column.
// The latent axis is walked in chunks of CK staged through LDS.
constexpr int CK = 128;
template <typename T, typename OT>
__global__ void __launch_bounds__(128) combine_shards_kernel(const float* __restrict__ o_lat,
                                                             const T* __restrict__ W,
                                                             OT* __restrict__ o, int B, int H, int d_c,
                                                             int d_v, int g) {
  __shared__ float os[BT][CK];
  const int h = blockIdx.x;
  const int col = blockIdx.y * 128 + threadIdx.x;
  const int b0 = blockIdx.z * BT;
  const int nb = min(BT, B - b0);
  const int dl = d_c / g;
  float acc[BT];
#pragma unroll
  for (int bb = 0; bb < BT; ++bb) acc[bb] = 0.f;
  for (int k0 = 0; k0 < d_c; k0 += CK) {
    const int kn = min(CK, d_c - k0);
    __syncthreads();
    for (int i = threadIdx.x; i < BT * CK; i += 128) {
      const int bb = i / CK, k = i % CK;
      float v = 0.f;
      if (bb < nb && k < kn) {
        const int kk = k0 + k;
        const int sl = kk / dl, c = kk - sl * dl;
        v = o_lat[(((size_t)sl * B + (b0 + bb)) * H + h) * dl + c];
      }
      os[bb][k] = v;
    }
    __syncthreads();
    if (col < d_v) {
      const T* w = W + ((size_t)h * d_c + k0) * d_v + col;
      for (int k = 0; k < kn; ++k) {
        const float wv = load_as_f32(w + (size_t)k * d_v);
#pragma unroll
        for (int bb = 0; bb < BT; ++bb) acc[bb] = fmaf(os[bb][k], wv, acc[bb]);
      }
    }
  }
  if (col < d_v)
#pragma unroll
    for (int bb = 0; bb < BT; ++bb)
      if (bb < nb) store_from_f32(o + ((size_t)(b0 + bb) * H + h) * d_v + col, acc[bb]);
}


// Vectorised variant (d_v a multiple of 8): workgroup = (head, 128-column
// slab, 8 sequences).  Thread (cg, kg): 8 consecutive value columns, latent
// rows kg, kg+16, ... (16 lanes read one 256-byte piece of a weight row).
template <typename T, typename OT>
__global__ void __launch_bounds__(256) combine_shards_vec_kernel(const float* __restrict__ o_lat,
                                                                 const T* __restrict__ W,
                                                                 OT* __restrict__ o, int B, int H,
                                                                 int d_c, int d_v, int g) {
  extern __shared__ float sm[];          // [AB][d_c] latent outputs, then [4][AB][128] partial sums
  float* os = sm;
  float* red = sm + AB * d_c;
  const int h = blockIdx.x;
  const int col0 = blockIdx.y * 128;
  const int b0 = blockIdx.z * AB;
  const int nb = min(AB, B - b0);
  const int dl = d_c / g;
  const int tid = threadIdx.x, cg = tid & 15, kg = tid >> 4, wave = tid >> 6;
  for (int i = tid; i < AB * d_c; i += 256) {
    const int bb = i / d_c, k = i % d_c;
    float v = 0.f;
    if (bb < nb) {
      const int sl = k / dl, c = k - sl * dl;
      v = o_lat[(((size_t)sl * B + (b0 + bb)) * H + h) * dl + c];
    }
    os[i] = v;
  }
  __syncthreads();
  const int col = col0 + cg * 8;
  float acc[AB][8];
#pragma unroll
  for (int bb = 0; bb < AB; ++bb)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[bb][c] = 0.f;
  if (col < d_v) {
    const T* w = W + (size_t)h * d_c * d_v + col;
    for (int k = kg; k < d_c; k += 16) {
      const Vec8 wv = load8_cached(w + (size_t)k * d_v);
#pragma unroll
      for (int bb = 0; bb < AB; ++bb) {
        const float ov = os[bb * d_c + k];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[bb][c] = fmaf(ov, wv.v[c], acc[bb][c]);
      }
    }
  }
#pragma unroll
  for (int bb = 0; bb < AB; ++bb)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float v = acc[bb][c];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[bb][c] = v;
    }
  if ((tid & 48) == 0) {
#pragma unroll
    for (int bb = 0; bb < AB; ++bb)
#pragma unroll
      for (int c = 0; c < 8; ++c) red[(wave * AB + bb) * 128 + cg * 8 + c] = acc[bb][c];
  }
  __syncthreads();
  // thread -> (sequence, 4 columns): 8 x 128 outputs
  const int bb = tid >> 5, c4 = (tid & 31) * 4;
  if (bb < nb) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int cc = c4 + c;
      if (col0 + cc < d_v)
        store_from_f32(o + ((size_t)(b0 + bb) * H + h) * d_v + col0 + cc,
                       red[(0 * AB + bb) * 128 + cc] + red[(1 * AB + bb) * 128 + cc] +
                           red[(2 * AB + bb) * 128 + cc] + red[(3 * AB + bb) * 128 + cc]);
    }
  }
}

template <typename OT>
static int launch_combine_shards_to(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, OT* o,
                                    hipStream_t st) {
  if (sh.d_v % 8 == 0) {
    const size_t vsm = ((size_t)AB * sh.d_c + 4u * AB * 128) * sizeof(float);
    const dim3 vgrid((unsigned)sh.H, (unsigned)((sh.d_v + 127) / 128), (unsigned)((sh.B + AB - 1) / AB));
    if (vsm <= 64 * 1024 && vgrid.y <= 65535 && vgrid.z <= 65535) {
      if (sh.dtype == TPLA_F32)
        hipLaunchKernelGGL((combine_shards_vec_kernel<float, OT>), vgrid, dim3(256), vsm, st, o_lat,
                           static_cast<const float*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
      else
        hipLaunchKernelGGL((combine_shards_vec_kernel<bf16_t, OT>), vgrid, dim3(256), vsm, st, o_lat,
                           static_cast<const bf16_t*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
      return check_launch("combine_shards_vec_kernel");
    }
  }
  const dim3 grid((unsigned)sh.H, (unsigned)((sh.d_v + 127) / 128), (unsigned)((sh.B + BT - 1) / BT));
  if (grid.y > 65535 || grid.z > 65535) return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  if (sh.dtype == TPLA_F32)
    hipLaunchKernelGGL((combine_shards_kernel<float, OT>), grid, dim3(128), 0, st, o_lat,
                       static_cast<const float*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  else
    hipLaunchKernelGGL((combine_shards_kernel<bf16_t, OT>), grid, dim3(128), 0, st, o_lat,
                       static_cast<const bf16_t*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  return check_launch("combine_shards_kernel");
}

int launch_combine_shards(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, void* o, int o_dtype,
                          hipStream_t st) {
  if (o_dtype == TPLA_BF16) return launch_combine_shards_to(sh, o_lat, W_UV_t, static_cast<bf16_t*>(o), st);
  return launch_combine_shards_to(sh, o_lat, W_UV_t, static_cast<float*>(o), st);
}

}  // namespace tpla
