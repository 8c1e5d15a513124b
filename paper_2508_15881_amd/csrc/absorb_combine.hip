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

int launch_absorb_query(const tpla_shape_t& sh, const void* q_nope, const void* W_UK_t,
                        const MuFactors& mu, void* q_lat, hipStream_t st) {
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
template <typename T>
__global__ void __launch_bounds__(128) combine_shards_kernel(const float* __restrict__ o_lat,
                                                             const T* __restrict__ W,
                                                             float* __restrict__ o, int B, int H, int d_c,
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
      if (bb < nb) o[((size_t)(b0 + bb) * H + h) * d_v + col] = acc[bb];
}

int launch_combine_shards(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, float* o,
                          hipStream_t st) {
  const dim3 grid((unsigned)sh.H, (unsigned)((sh.d_v + 127) / 128), (unsigned)((sh.B + BT - 1) / BT));
  if (grid.y > 65535 || grid.z > 65535) return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  if (sh.dtype == TPLA_F32)
    hipLaunchKernelGGL(combine_shards_kernel<float>, grid, dim3(128), 0, st, o_lat,
                       static_cast<const float*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  else
    hipLaunchKernelGGL(combine_shards_kernel<bf16_t>, grid, dim3(128), 0, st, o_lat,
                       static_cast<const bf16_t*>(W_UV_t), o, sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  return check_launch("combine_shards_kernel");
}

}  // namespace tpla
