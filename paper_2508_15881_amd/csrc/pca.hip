// PCA calibration (Sec. 4.3.2 of the paper): the second moments of cached
// latents on the GPU, the eigen-decomposition of their covariance on the host.
//   * latent_gram_mfma_kernel: G = sum_r x_r^T x_r and s = sum_r x_r over paged
//     bf16 rows, 128 x 128 blocks of the upper triangle on the matrix cores.
//     The contraction runs over rows, so both MFMA operands are columns of the
//     staged tile, fetched with transposing LDS reads.
//   * latent_gram_generic_kernel: any storage type / width (plain FMA).
//   * latent_moments_reduce_kernel: sums the per-split partials in double, in
//     split order (deterministic), and mirrors the triangle.
//   * pca_basis_host: covariance = G/n - m m^T, Householder tridiagonalisation
//     and implicit QR steps in double, eigenvalues sorted descending; the variance fractions of the g
//     slices (the alpha, beta of Sec. 4.3.2).
#include "tpla_internal.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

namespace tpla {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int GB = 128;                  // block edge of the Gram matrix
constexpr int GT = 32;                   // rows per staged tile (one MFMA k-step)
constexpr int GPITCH = GB * 2 + 32;      // bytes per staged row of a slab: rows of a 4-row group 8 banks apart

__host__ __device__ inline int gram_blocks(int nbk) { return nbk * (nbk + 1) / 2; }

// 4 rows x 16 columns of bf16 -> lane i of the 16-lane group gets column i of the 4 rows.
__device__ __forceinline__ bf16x4 lds_tr(const char* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(const_cast<char*>(p)));
  return __builtin_bit_cast(bf16x4, v);
}

// grid: (blocks of the upper triangle, splits).  Split sp takes pages
// [sp * pages_per_split, ...).  part_gram[sp][blk][128][128], part_sum[sp][d_c]
// (column sums written by the diagonal blocks).
__global__ void __launch_bounds__(256) latent_gram_mfma_kernel(
    const bf16_t* __restrict__ mla_pool, const int32_t* __restrict__ page_ids, const int32_t* __restrict__ page_fill,
    int n_pages, int pages_per_split, int page_tokens, int d_c, int d_r, float* __restrict__ part_gram,
    float* __restrict__ part_sum) {
  __shared__ __attribute__((aligned(16))) char tile[2][GT * GPITCH];     // slab i, slab j
  __shared__ float red[16][GB];
  const int nbk = d_c / GB;
  int blk = blockIdx.x, bi = 0;
  while (blk >= nbk - bi) { blk -= nbk - bi; ++bi; }     // row bi of the triangle holds nbk - bi blocks
  const int bj = bi + blk;
  const int sp = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 15, hi = lane >> 4;
  const int wi = wave >> 1, wj = wave & 1;
  const int in_pitch = d_c + d_r;
  // staging: thread t fetches pieces t and t + 256 of a slab tile: rows t/16 and t/16 + 16, 8 columns at 8 (t%16)
  const int st_row = tid >> 4, st_col = (tid & 15) * 8;
  // transposing reads: rows 4 hi + lo/4 (+16), columns 4 (lo%4) of a 16-column block
  const int tr_off = (4 * hi + (lo >> 2)) * GPITCH + 8 * (lo & 3);

  f32x4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
  float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int pg_begin = sp * pages_per_split;
  const int pg_end = min(n_pages, pg_begin + pages_per_split);
  const int tiles_per_page = (page_tokens + GT - 1) / GT;
  for (int pg = pg_begin; pg < pg_end; ++pg) {
    const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
    const int fill = page_fill ? min(page_fill[pg], page_tokens) : page_tokens;
    const bf16_t* base = mla_pool + page * (size_t)page_tokens * in_pitch;
    for (int t = 0; t < tiles_per_page; ++t) {
      if (t * GT >= fill) break;                       // uniform: nothing valid left in this page
      u32x4 vi[2], vj[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int r = t * GT + st_row + 16 * u;
        const bool ok = r < fill;
        const bf16_t* row = base + (size_t)(ok ? r : 0) * in_pitch;
        vi[u] = *reinterpret_cast<const u32x4*>(row + GB * bi + st_col);
        vj[u] = *reinterpret_cast<const u32x4*>(row + GB * bj + st_col);
        if (!ok) { vi[u] = u32x4{0u, 0u, 0u, 0u}; vj[u] = u32x4{0u, 0u, 0u, 0u}; }
      }
      if (bi == bj) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            csum[2 * e] += __uint_as_float(vi[u][e] << 16);
            csum[2 * e + 1] += __uint_as_float(vi[u][e] & 0xFFFF0000u);
          }
      }
      __syncthreads();                                 // the previous tile has been consumed
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        *reinterpret_cast<u32x4*>(tile[0] + (st_row + 16 * u) * GPITCH + st_col * 2) = vi[u];
        *reinterpret_cast<u32x4*>(tile[1] + (st_row + 16 * u) * GPITCH + st_col * 2) = vj[u];
      }
      __syncthreads();
      bf16x8 fa[4], fb[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const char* pa = tile[0] + tr_off + (64 * wi + 16 * m) * 2;
        const char* pb = tile[1] + tr_off + (64 * wj + 16 * m) * 2;
        const bf16x4 a0 = lds_tr(pa), a1 = lds_tr(pa + 16 * GPITCH);
        const bf16x4 b0 = lds_tr(pb), b1 = lds_tr(pb + 16 * GPITCH);
        fa[m] = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        fb[m] = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
  }

  // partial block: lane holds column 64 wj + 16 b + lo, rows 64 wi + 16 a + 4 hi + e
  float* out = part_gram + ((size_t)sp * gram_blocks(nbk) + blockIdx.x) * (GB * GB);
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        out[(64 * wi + 16 * a + 4 * hi + e) * GB + 64 * wj + 16 * b + lo] = acc[a][b][e];
  if (bi == bj) {
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) red[st_row][st_col + e] = csum[e];
    __syncthreads();
    if (tid < GB) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s += red[r][tid];
      part_sum[(size_t)sp * d_c + GB * bi + tid] = s;
    }
  }
}

// Any storage / width: thread (i, j >= i) of a 16 x 16 patch, rows of split sp.
// part_gram[sp][d_c][d_c] (upper triangle), part_sum[sp][d_c].
template <typename T>
__global__ void __launch_bounds__(256) latent_gram_generic_kernel(
    const T* __restrict__ mla_pool, const int32_t* __restrict__ page_ids, const int32_t* __restrict__ page_fill,
    int n_pages, int pages_per_split, int page_tokens, int d_c, int d_r, float* __restrict__ part_gram,
    float* __restrict__ part_sum) {
  const int i = blockIdx.x * 16 + threadIdx.x / 16, j = blockIdx.y * 16 + threadIdx.x % 16;
  const int sp = blockIdx.z;
  if (blockIdx.y < blockIdx.x) return;                  // below the diagonal: mirrored by the reduction
  const bool live = i < d_c && j < d_c;
  const int in_pitch = d_c + d_r;
  float g = 0.f, s = 0.f;
  const int pg_end = min(n_pages, (sp + 1) * pages_per_split);
  for (int pg = sp * pages_per_split; pg < pg_end; ++pg) {
    const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
    const int fill = page_fill ? min(page_fill[pg], page_tokens) : page_tokens;
    const T* base = mla_pool + page * (size_t)page_tokens * in_pitch;
    if (live)
      for (int r = 0; r < fill; ++r) {
        const float xi = load_as_f32(base + (size_t)r * in_pitch + i), xj = load_as_f32(base + (size_t)r * in_pitch + j);
        g = fmaf(xi, xj, g);
        s += xj;
      }
  }
  if (!live) return;
  part_gram[((size_t)sp * d_c + i) * d_c + j] = g;
  if (i == j) part_sum[(size_t)sp * d_c + j] = s;
}

// blocked != 0: partials are 128 x 128 blocks of the upper triangle; else full matrices.
__global__ void __launch_bounds__(256) latent_moments_reduce_kernel(
    const float* __restrict__ part_gram, const float* __restrict__ part_sum, int n_splits, int d_c, int blocked,
    double* __restrict__ sum, double* __restrict__ gram) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= d_c * d_c) return;
  const int i = idx / d_c, j = idx % d_c;
  if (j < i) return;
  double g = 0.0;
  if (blocked) {
    const int nbk = d_c / GB, bi = i / GB, bj = j / GB;
    const int blk = bi * nbk - bi * (bi - 1) / 2 + (bj - bi);
    const size_t stride = (size_t)gram_blocks(nbk) * (GB * GB);
    const float* p = part_gram + (size_t)blk * (GB * GB) + (i % GB) * GB + (j % GB);
    for (int sp = 0; sp < n_splits; ++sp) g += (double)p[sp * stride];
  } else {
    const float* p = part_gram + (size_t)i * d_c + j;
    for (int sp = 0; sp < n_splits; ++sp) g += (double)p[(size_t)sp * d_c * d_c];
  }
  gram[(size_t)i * d_c + j] = g;
  gram[(size_t)j * d_c + i] = g;
  if (i == j) {
    double s = 0.0;
    for (int sp = 0; sp < n_splits; ++sp) s += (double)part_sum[(size_t)sp * d_c + j];
    sum[j] = s;
  }
}

static bool gram_mfma_supported(const tpla_shape_t& sh) {
  return sh.dtype == TPLA_BF16 && sh.d_c % GB == 0 && sh.d_c <= 1024 && sh.d_r % 8 == 0;
}

int latent_moments_splits(const tpla_shape_t& sh, int64_t n_pages) {
  // enough workgroups for two per CU, rows per split bounded so float partials stay accurate
  const int blocks = gram_mfma_supported(sh) ? gram_blocks(sh.d_c / GB) : ((sh.d_c + 15) / 16) * ((sh.d_c + 15) / 16);
  int64_t s = (2 * (int64_t)device_cu_count() + blocks - 1) / blocks;
  const int64_t by_rows = (n_pages * sh.page_tokens + 16383) / 16384;
  s = std::max<int64_t>(s, by_rows);
  s = std::min<int64_t>(s, std::min<int64_t>(n_pages, 1024));
  return (int)std::max<int64_t>(s, 1);
}

size_t latent_moments_workspace(const tpla_shape_t& sh, int64_t n_pages) {
  const size_t S = (size_t)latent_moments_splits(sh, n_pages);
  const size_t per = gram_mfma_supported(sh) ? (size_t)gram_blocks(sh.d_c / GB) * GB * GB : (size_t)sh.d_c * sh.d_c;
  return S * (per + sh.d_c) * sizeof(float);
}

int launch_latent_moments(const tpla_shape_t& sh, const void* mla_pool, const int32_t* page_ids,
                          const int32_t* page_fill, int64_t n_pages, float* workspace, double* sum, double* gram,
                          hipStream_t st) {
  const int S = latent_moments_splits(sh, n_pages);
  const int pps = (int)((n_pages + S - 1) / S);
  const bool mfma = gram_mfma_supported(sh);
  const size_t per = mfma ? (size_t)gram_blocks(sh.d_c / GB) * GB * GB : (size_t)sh.d_c * sh.d_c;
  float* part_gram = workspace;
  float* part_sum = workspace + (size_t)S * per;
  if (mfma) {
    hipLaunchKernelGGL(latent_gram_mfma_kernel, dim3(gram_blocks(sh.d_c / GB), S), dim3(256), 0, st,
                       static_cast<const bf16_t*>(mla_pool), page_ids, page_fill, (int)n_pages, pps, sh.page_tokens,
                       sh.d_c, sh.d_r, part_gram, part_sum);
  } else {
    const dim3 grid((sh.d_c + 15) / 16, (sh.d_c + 15) / 16, S);
    if (sh.dtype == TPLA_F32)
      hipLaunchKernelGGL(latent_gram_generic_kernel<float>, grid, dim3(256), 0, st, static_cast<const float*>(mla_pool),
                         page_ids, page_fill, (int)n_pages, pps, sh.page_tokens, sh.d_c, sh.d_r, part_gram, part_sum);
    else
      hipLaunchKernelGGL(latent_gram_generic_kernel<bf16_t>, grid, dim3(256), 0, st,
                         static_cast<const bf16_t*>(mla_pool), page_ids, page_fill, (int)n_pages, pps, sh.page_tokens,
                         sh.d_c, sh.d_r, part_gram, part_sum);
  }
  int rc = check_launch("latent_gram kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(latent_moments_reduce_kernel, dim3((sh.d_c * sh.d_c + 255) / 256), dim3(256), 0, st, part_gram,
                     part_sum, S, sh.d_c, mfma ? 1 : 0, sum, gram);
  return check_launch("latent_moments_reduce_kernel");
}

// ---------------------------------------------------------------------------
// Host: eigen-decomposition of the symmetric covariance in two textbook steps:
// Householder reflections bring A to tridiagonal form T = Q^T A Q, then
// implicit QR steps with Wilkinson's shift diagonalise T.  A is d x d row-major
// (overwritten); V gets the eigenvectors as ROWS (every rotation and reflection
// then works on contiguous rows); lam gets the eigenvalues, unsorted.  Returns
// false if the QR iteration does not converge.
static bool symmetric_eigen(std::vector<double>& A, std::vector<double>& V, std::vector<double>& lam, int d) {
  std::vector<double> off((size_t)std::max(d, 1), 0.0), v((size_t)d), p((size_t)d), u((size_t)d);
  std::fill(V.begin(), V.end(), 0.0);
  for (int i = 0; i < d; ++i) V[(size_t)i * d + i] = 1.0;
  // ---- tridiagonal form: step k clears row/column k beyond its first off-diagonal entry ----
  for (int k = 0; k + 2 < d; ++k) {
    const int m = d - k - 1;                       // size of the trailing block, indices k+1 .. d-1
    const double* x = &A[(size_t)k * d + k + 1];   // row k right of the diagonal (= column k below it)
    double norm2 = 0.0;
    for (int i = 0; i < m; ++i) norm2 += x[i] * x[i];
    double tail2 = norm2 - x[0] * x[0];
    if (tail2 <= 0.0) {                            // already tridiagonal here
      off[k] = x[0];
      continue;
    }
    const double sigma = std::sqrt(norm2);
    const double alpha = x[0] > 0.0 ? -sigma : sigma;          // the entry that replaces x
    for (int i = 0; i < m; ++i) v[i] = x[i];
    v[0] -= alpha;
    const double vnorm2 = tail2 + v[0] * v[0];
    const double beta = 2.0 / vnorm2;                          // H = I - beta v v^T
    // trailing block B <- H B H = B - v w^T - w v^T with p = beta B v, w = p - (beta/2)(v.p) v
    double vp = 0.0;
    for (int i = 0; i < m; ++i) {
      const double* Bi = &A[(size_t)(k + 1 + i) * d + k + 1];
      double acc = 0.0;
      for (int j = 0; j < m; ++j) acc += Bi[j] * v[j];
      p[i] = beta * acc;
      vp += v[i] * p[i];
    }
    const double half = 0.5 * beta * vp;
    for (int i = 0; i < m; ++i) p[i] -= half * v[i];           // p is w from here on
    for (int i = 0; i < m; ++i) {
      double* Bi = &A[(size_t)(k + 1 + i) * d + k + 1];
      const double vi = v[i], wi = p[i];
      for (int j = 0; j < m; ++j) Bi[j] -= vi * p[j] + wi * v[j];
    }
    off[k] = alpha;
    // V = Q^T: rows k+1.. of V <- H (rows k+1.. of V)
    std::fill(u.begin(), u.end(), 0.0);
    for (int i = 0; i < m; ++i) {
      const double* Vi = &V[(size_t)(k + 1 + i) * d];
      const double vi = v[i];
      for (int j = 0; j < d; ++j) u[j] += vi * Vi[j];
    }
    for (int i = 0; i < m; ++i) {
      double* Vi = &V[(size_t)(k + 1 + i) * d];
      const double bv = beta * v[i];
      for (int j = 0; j < d; ++j) Vi[j] -= bv * u[j];
    }
  }
  for (int i = 0; i < d; ++i) lam[i] = A[(size_t)i * d + i];
  if (d >= 2) off[d - 2] = A[(size_t)(d - 2) * d + d - 1];
  // ---- QR steps on the unreduced block [lo, hi] at the bottom, deflating as off-diagonals vanish ----
  const double eps = 2.220446049250313e-16;
  int hi = d - 1;
  long budget = 60L * d;
  while (hi > 0) {
    if (std::fabs(off[hi - 1]) <= eps * (std::fabs(lam[hi - 1]) + std::fabs(lam[hi]))) {
      off[hi - 1] = 0.0;
      --hi;
      continue;
    }
    if (--budget < 0) return false;
    int lo = hi - 1;
    while (lo > 0 && std::fabs(off[lo - 1]) > eps * (std::fabs(lam[lo - 1]) + std::fabs(lam[lo]))) --lo;
    if (lo > 0) off[lo - 1] = 0.0;
    // Wilkinson's shift: the eigenvalue of the last 2 x 2 block closer to its last entry
    const double delta = 0.5 * (lam[hi - 1] - lam[hi]), b = off[hi - 1];
    const double mu = lam[hi] - b * b / (delta + (delta >= 0.0 ? 1.0 : -1.0) * std::hypot(delta, b));
    double x = lam[lo] - mu, z = off[lo];
    for (int k = lo; k < hi; ++k) {
      // rotation in the (k, k+1) plane that sends (x, z) to (r, 0); T <- G^T T G chases the bulge down
      const double r = std::hypot(x, z);
      const double c = r != 0.0 ? x / r : 1.0, sn = r != 0.0 ? -z / r : 0.0;
      if (k > lo) off[k - 1] = r;
      const double a = lam[k], e = off[k], cc = lam[k + 1];
      lam[k] = a * c * c - 2.0 * e * c * sn + cc * sn * sn;
      lam[k + 1] = a * sn * sn + 2.0 * e * c * sn + cc * c * c;
      off[k] = (a - cc) * c * sn + e * (c * c - sn * sn);
      x = off[k];
      if (k + 1 < hi) {
        z = -sn * off[k + 1];
        off[k + 1] *= c;
      }
      double* Vk = &V[(size_t)k * d];
      double* Vk1 = &V[(size_t)(k + 1) * d];
      for (int j = 0; j < d; ++j) {
        const double p0 = Vk[j], p1 = Vk1[j];
        Vk[j] = c * p0 - sn * p1;
        Vk1[j] = sn * p0 + c * p1;
      }
    }
  }
  return true;
}

int pca_basis_host(int d, int g, double n_rows, const double* sum, const double* gram, float* U, double* eig,
                   double* frac) {
  std::vector<double> A((size_t)d * d), V((size_t)d * d);
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < d; ++j)
      A[(size_t)i * d + j] = gram[(size_t)i * d + j] / n_rows - (sum[i] / n_rows) * (sum[j] / n_rows);
  for (int i = 0; i < d; ++i)                            // exact symmetry whatever the caller passed
    for (int j = i + 1; j < d; ++j) A[(size_t)j * d + i] = A[(size_t)i * d + j] = 0.5 * (A[(size_t)i * d + j] + A[(size_t)j * d + i]);
  std::vector<double> lam((size_t)d);
  if (!symmetric_eigen(A, V, lam, d)) return fail(TPLA_ERR_UNSUPPORTED, "the QR iteration did not converge");
  std::vector<int> order(d);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return lam[a] > lam[b]; });
  double total = 0.0;
  for (int k = 0; k < d; ++k) {
    const int src = order[k];
    eig[k] = lam[src];
    total += eig[k];
    // sign convention: the largest-magnitude component of every eigenvector is positive
    int big = 0;
    for (int i = 1; i < d; ++i)
      if (std::fabs(V[(size_t)src * d + i]) > std::fabs(V[(size_t)src * d + big])) big = i;
    const double sg = V[(size_t)src * d + big] < 0.0 ? -1.0 : 1.0;
    for (int i = 0; i < d; ++i) U[(size_t)i * d + k] = (float)(sg * V[(size_t)src * d + i]);   // column k
  }
  const int dl = d / g;
  for (int i = 0; i < g; ++i) {
    double part = 0.0;
    for (int k = i * dl; k < (i + 1) * dl; ++k) part += eig[k];
    frac[i] = total != 0.0 ? part / total : 1.0 / g;
  }
  return TPLA_OK;
}

}  // namespace tpla
