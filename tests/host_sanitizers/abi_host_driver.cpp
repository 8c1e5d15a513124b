// Host-side exerciser of libtpla's C ABI for a build with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (no GPU work: every call either
// fails validation before a launch or runs on the host).  It walks the argument
// checks of every entry point with fake, aligned device addresses, the page-table
// validator on in-range and out-of-range tables, and the host eigen-solver of the
// PCA basis on matrices whose decomposition is known.  Exit status 0 = every
// expectation held and no sanitizer report was raised (reports abort).
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "tpla.h"
#include "tpla_internal.h"   // the plan arithmetic shared by the split kernel and the merge kernels

static int g_failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      fprintf(stderr, "%s:%d: expectation failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, \
              tpla_last_error());                                           \
      ++g_failures;                                                         \
    }                                                                       \
  } while (0)

static tpla_shape_t shape(int B = 2, int H = 64, int d_c = 512, int g = 2) {
  tpla_shape_t s;
  s.B = B; s.H = H; s.d_c = d_c; s.g = g; s.d_r = 64; s.d_n = 128; s.d_v = 128;
  s.page_tokens = 64; s.dtype = TPLA_BF16; s.sm_scale = 0.07f;
  return s;
}

// x_{n+1} = x_n * 6364136223846793005 + 1442695040888963407, top bits -> (-1, 1)
static double lcg(uint64_t& st) {
  st = st * 6364136223846793005ULL + 1442695040888963407ULL;
  return (double)(st >> 11) / 4503599627370496.0 - 1.0;
}

static void* const A = (void*)(uintptr_t)4096;        // aligned, never dereferenced
static void* const A2 = (void*)(uintptr_t)(4096 + 2); // misaligned

static void argument_checks() {
  tpla_shape_t s = shape();
  float* Af = (float*)A;
  const int32_t* Ai = (const int32_t*)A;
  // decode: one slice, all slices, with the combine, without a workspace
  EXPECT(tpla_decode_shard(&s, NULL, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_decode_shard(&s, A, A, A, Ai, 0, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_decode_shard(&s, A2, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_ALIGN);
  EXPECT(tpla_decode_shard(&s, A, A, A, Ai, 4, Ai, 2, A, 16, Af, NULL, NULL) == TPLA_ERR_WORKSPACE);
  EXPECT(tpla_decode_shard(NULL, A, A, A, Ai, 4, Ai, 2, A, 16, Af, NULL, NULL) == TPLA_ERR_NULL);
  tpla_shape_t bad = shape(); bad.dtype = 7;
  EXPECT(tpla_decode_shard(&bad, A, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_DTYPE);
  bad = shape(2, 64, 512, 3);
  EXPECT(tpla_decode_shard(&bad, A, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  bad = shape(2, 64, 1024, 16);
  EXPECT(tpla_decode_shard(&bad, A, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  bad = shape(); bad.sm_scale = NAN;
  EXPECT(tpla_decode_shard(&bad, A, A, A, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  const void* pools[TPLA_MAX_G] = {A, A};
  const void* pools_hole[TPLA_MAX_G] = {A, NULL};
  EXPECT(tpla_decode_shards(&s, A, A, pools_hole, Ai, 4, Ai, 0, A, (size_t)1 << 30, Af, NULL, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_decode_shards(&s, A, A, pools, Ai, 4, Ai, 3, A, 16, Af, NULL, NULL) == TPLA_ERR_WORKSPACE);
  EXPECT(tpla_decode_shards(&s, A, A, pools, Ai, 2147483647, Ai, 3, A, 16, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_decode_shards_combine(&s, A, A, pools, Ai, 4, Ai, 0, A, (size_t)1 << 30, NULL, Af, Af, NULL, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_decode_shards_combine(&s, A, A, pools, Ai, 4, Ai, 0, A, (size_t)1 << 30, A2, Af, Af, NULL, NULL) == TPLA_ERR_ALIGN);
  EXPECT(tpla_decode_shards_combine(&s, A, A, pools, Ai, 4, Ai, 2, A, 16, A, Af, Af, NULL, NULL) == TPLA_ERR_WORKSPACE);
  tpla_shape_t big = shape(32);
  EXPECT(tpla_decode_shards_combine_static(&big, A, A, pools, Ai, 2048, Ai, 1024, A, Af, Af, NULL, NULL) == TPLA_ERR_WORKSPACE);
  EXPECT(tpla_decode_shards_combine_static(&s, A, A, pools, Ai, 0, Ai, 0, A, Af, Af, NULL, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_decode_shards_combine_static(&s, A, A, pools, Ai, 4, Ai, 0, NULL, Af, Af, NULL, NULL) == TPLA_ERR_NULL);
  // workspace sizes: plain arithmetic on the plan
  EXPECT(tpla_workspace_bytes(&s, 512, 1) == (size_t)2 * 64 * (256 + 2) * 4);
  EXPECT(tpla_workspace_bytes(&s, 512, 8) == (size_t)8 * 2 * 64 * (256 + 2) * 4);
  EXPECT(tpla_workspace_bytes(&s, 4, 100) == (size_t)4 * 2 * 64 * (256 + 2) * 4);
  EXPECT(tpla_workspace_bytes(&s, 512, 0) > 0 && tpla_workspace_bytes_all(&s, 512, 0) >= tpla_workspace_bytes(&s, 512, 0));
  EXPECT(tpla_workspace_bytes(&s, 0, 0) == 0 && tpla_workspace_bytes_all(&s, 4, -1) == 0);
  // absorb, combine, transforms, cache writes
  const float mu_bad[TPLA_MAX_G] = {1.0f, INFINITY};
  EXPECT(tpla_absorb_query(&s, NULL, A, NULL, A, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_absorb_query(&s, A, A2, NULL, A, NULL) == TPLA_ERR_ALIGN);
  EXPECT(tpla_absorb_query(&s, A, A, mu_bad, A, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_combine_shards(&s, Af, NULL, Af, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_transform_latent(&s, 9, 0, NULL, NULL, A, A, 4, 1, NULL) == TPLA_ERR_SHAPE);
  bad = shape(2, 64, 96, 2);
  EXPECT(tpla_transform_latent(&bad, TPLA_U_HADAMARD, 0, NULL, NULL, A, A, 4, 1, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_transform_latent(&s, TPLA_U_DENSE, 0, NULL, NULL, A, A, 4, 1, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_transform_latent(&s, TPLA_U_IDENTITY, 0, NULL, NULL, A, A, 0, 1, NULL) == TPLA_OK);
  void* wpools[TPLA_MAX_G] = {A, A};
  void* wpools_mis[TPLA_MAX_G] = {A, A2};
  EXPECT(tpla_transform_latent_paged(&s, TPLA_U_IDENTITY, NULL, NULL, A, wpools_mis, NULL, 3, NULL) == TPLA_ERR_ALIGN);
  EXPECT(tpla_transform_latent_paged(&s, TPLA_U_IDENTITY, NULL, NULL, A, wpools, NULL, -1, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_transform_latent_paged(&s, TPLA_U_IDENTITY, NULL, NULL, A, wpools, NULL, 0, NULL) == TPLA_OK);
  EXPECT(tpla_write_mla_cache(&s, A, A, NULL, 5, 1e-6f, A, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_write_mla_cache(&s, A, A, Ai, -5, 1e-6f, A, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_write_mla_cache(&s, A, A, Ai, 0, 1e-6f, A, NULL) == TPLA_OK);
  const float alpha_bad[TPLA_MAX_G] = {2.0f, -1.0f};
  EXPECT(tpla_append_token_sliced(&s, A, A, alpha_bad, 1e-6f, Ai, wpools, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_append_token_sliced(&s, A, A, NULL, -1.0f, Ai, wpools, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_append_token_sliced(&s, A, A, NULL, 1e-6f, Ai, wpools_mis, NULL) == TPLA_ERR_ALIGN);
  // output projection, PCA moments, prefill
  EXPECT(tpla_output_projection(&s, Af, NULL, 64, A, (size_t)1 << 20, Af, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_output_projection(&s, Af, A, 0, A, (size_t)1 << 20, Af, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_latent_moments_workspace_bytes(&s, 0) == 0 && tpla_latent_moments_workspace_bytes(&s, 40) > 0);
  EXPECT(tpla_latent_moments(&s, A, NULL, NULL, 4, A, 16, (double*)A, (double*)A, NULL) == TPLA_ERR_WORKSPACE);
  EXPECT(tpla_latent_moments(&s, A, NULL, NULL, 0, A, (size_t)1 << 30, (double*)A, (double*)A, NULL) == TPLA_ERR_SHAPE);
  EXPECT(tpla_prefill_workspace_bytes(&s, 100) == (size_t)100 * 64 * 256 * 2);
  EXPECT(tpla_prefill_attention(&s, A, A, A, A, A, A, NULL, 8, 8, A, (size_t)1 << 30, Af, NULL) == TPLA_ERR_NULL);
  EXPECT(tpla_prefill_attention(&s, A, A, A, A, A, A, Ai, 8, 8, A, 64, Af, NULL) == TPLA_ERR_WORKSPACE);
  bad = shape(); bad.d_n = 64;
  EXPECT(tpla_prefill_attention(&bad, A, A, A, A, A, A, Ai, 8, 8, A, (size_t)1 << 30, Af, NULL) == TPLA_ERR_UNSUPPORTED);
  // measurement aids
  float ms[4]; int32_t n = -1;
  EXPECT(tpla_profile_enable(-1) == TPLA_ERR_SHAPE);
  EXPECT(tpla_profile_collect(ms, -3, &n) == TPLA_ERR_SHAPE);
  EXPECT(tpla_profile_collect(ms, 4, &n) == TPLA_OK && n == 0);
  EXPECT(tpla_stream_read(NULL, 100, A, NULL) == TPLA_ERR_NULL);
  EXPECT(strlen(tpla_last_error()) > 0 && tpla_version() >= 100);
}

static void block_table_checks() {
  tpla_shape_t s = shape(3);
  // exactly-sized heap arrays: a read past a row or past the lengths is a sanitizer report
  std::vector<int32_t> bt = {0, 1, 2, 3, 4, 5, 0, 0, 6, 0, 0, 0};
  std::vector<int32_t> ln = {200, 65, 1};
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, ln.data(), 7, 0) == TPLA_OK);
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, ln.data(), 7, 1) == TPLA_OK);
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, ln.data(), 6, 0) == TPLA_ERR_SHAPE);
  EXPECT(strstr(tpla_last_error(), "block_table[2][0]=6") != NULL);
  std::vector<int32_t> full = {256, 256, 256};             // every row used to its last entry
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, full.data(), 7, 0) == TPLA_OK);
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, full.data(), 7, 1) == TPLA_ERR_SHAPE);   // page 0 repeats
  std::vector<int32_t> over = {257, 65, 1};
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, over.data(), 7, 0) == TPLA_ERR_SHAPE);
  std::vector<int32_t> neg = {200, -1, 1};
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, neg.data(), 7, 0) == TPLA_ERR_SHAPE);
  std::vector<int32_t> huge_id = bt; huge_id[0] = 2147483647;
  EXPECT(tpla_validate_block_table(&s, huge_id.data(), 4, ln.data(), 7, 1) == TPLA_ERR_SHAPE);
  std::vector<int32_t> neg_id = bt; neg_id[5] = -2147483647 - 1;
  EXPECT(tpla_validate_block_table(&s, neg_id.data(), 4, ln.data(), 7, 1) == TPLA_ERR_SHAPE);
  EXPECT(tpla_validate_block_table(&s, NULL, 4, ln.data(), 7, 0) == TPLA_ERR_NULL);
  EXPECT(tpla_validate_block_table(&s, bt.data(), 4, ln.data(), 0, 0) == TPLA_ERR_SHAPE);
}


// The decomposition of C: U orthonormal, U^T C U = diag(eig) descending, fractions sum to 1.
static void check_basis(int d, int g, const std::vector<double>& C, double n_rows_scale, const char* what) {
  std::vector<double> sum((size_t)d, 0.0), gram((size_t)d * d), eig((size_t)d), frac((size_t)g);
  std::vector<float> U((size_t)d * d);
  for (size_t i = 0; i < gram.size(); ++i) gram[i] = C[i] * n_rows_scale;
  const int rc = tpla_pca_basis(d, g, (int64_t)n_rows_scale, sum.data(), gram.data(), U.data(), eig.data(), frac.data());
  EXPECT(rc == TPLA_OK);
  if (rc != TPLA_OK) return;
  double worst_orth = 0.0, worst_diag = 0.0, cmax = 0.0, fs = 0.0;
  for (double c : C) cmax = fmax(cmax, fabs(c));
  for (int i = 0; i + 1 < d; ++i) EXPECT(eig[i] >= eig[i + 1]);
  std::vector<double> CU((size_t)d * d, 0.0);
  for (int i = 0; i < d; ++i)
    for (int k = 0; k < d; ++k) {
      const double c = C[(size_t)i * d + k];
      for (int j = 0; j < d; ++j) CU[(size_t)i * d + j] += c * U[(size_t)k * d + j];
    }
  for (int a = 0; a < d; ++a)
    for (int b = 0; b < d; ++b) {
      double dot = 0.0, q = 0.0;
      for (int i = 0; i < d; ++i) {
        dot += (double)U[(size_t)i * d + a] * U[(size_t)i * d + b];
        q += (double)U[(size_t)i * d + a] * CU[(size_t)i * d + b];
      }
      worst_orth = fmax(worst_orth, fabs(dot - (a == b ? 1.0 : 0.0)));
      worst_diag = fmax(worst_diag, fabs(q - (a == b ? eig[a] : 0.0)));
    }
  for (double f : frac) fs += f;
  if (!(worst_orth <= 1e-5 && worst_diag <= 1e-5 * cmax && fabs(fs - 1.0) <= 1e-12)) {
    fprintf(stderr, "%s: orthogonality %.3g, off-diagonal %.3g (scale %.3g), fractions %.17g\n", what, worst_orth,
            worst_diag, cmax, fs);
    ++g_failures;
  }
}

static void pca_checks() {
  uint64_t st = 12345;
  for (int d : {1, 2, 7, 64, 160}) {
    // C = X^T X / m from a random m x d matrix with column scales 1 .. 1/d
    const int m = 3 * d + 1;
    std::vector<double> X((size_t)m * d), C((size_t)d * d, 0.0);
    for (int r = 0; r < m; ++r)
      for (int j = 0; j < d; ++j) X[(size_t)r * d + j] = lcg(st) / (1.0 + j);
    for (int r = 0; r < m; ++r)
      for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j) C[(size_t)i * d + j] += X[(size_t)r * d + i] * X[(size_t)r * d + j] / m;
    check_basis(d, (d % 2 == 0) ? 2 : 1, C, 1000.0, "random covariance");
  }
  {  // repeated eigenvalues and an exactly diagonal input
    const int d = 12;
    std::vector<double> C((size_t)d * d, 0.0);
    for (int i = 0; i < d; ++i) C[(size_t)i * d + i] = (i % 3 == 0) ? 5.0 : 2.0;
    check_basis(d, 4, C, 10.0, "diagonal with repeated values");
    std::vector<double> Z((size_t)d * d, 0.0);
    check_basis(d, 3, Z, 10.0, "zero matrix");
  }
  std::vector<double> z(16, 0.0);
  std::vector<float> zf(16, 0.f);
  EXPECT(tpla_pca_basis(4, 3, 10, z.data(), z.data(), zf.data(), z.data(), z.data()) == TPLA_ERR_SHAPE);
  EXPECT(tpla_pca_basis(4, 2, 0, z.data(), z.data(), zf.data(), z.data(), z.data()) == TPLA_ERR_SHAPE);
  EXPECT(tpla_pca_basis(4, 2, 10, NULL, z.data(), zf.data(), z.data(), z.data()) == TPLA_ERR_NULL);
}

// Balanced plan: range w of W is [plan_start(w), plan_start(w + 1)) of the T pages of all sequences laid
// end to end, with equal or round-weighted shares.  The split kernel derives its work items with
// balanced_item, the merge kernels find the slots of a sequence with balanced_owner /
// balanced_range_meets: for every (T, W, weights, lengths) both sides must name the same (workgroup,
// sequence) pairs, every page exactly once.
static void plan_checks() {
  uint64_t st = 99;
  const int Ws[] = {1, 2, 3, 7, 16, 40, 256, 512, 768};
  const int wts[][4] = {{1, 1, 1, 1}, {135, 121, 128, 128}, {149, 131, 106, 128}, {128, 128, 128, 128}, {3, 1, 1, 7}};
  const int cus[] = {256, 8, 5};
  const int wxs[][2] = {{1, 1}, {128, 118}, {100, 131}};
  for (const auto& wx : wxs)
  for (const auto& wt : wts)
    for (int n_cus : cus)
      for (int W : Ws)
        for (int trial = 0; trial < 12; ++trial) {
          tpla::BalancedPlan p;
          p.W = W;
          p.n_cus = n_cus;
          for (int r = 0; r < 4; ++r) p.wt[r] = wt[r];
          p.wx[0] = wx[0];
          p.wx[1] = wx[1];
          const int n_seq = 1 + (int)((lcg(st) + 1.0) * 6.0);
          std::vector<int> pages((size_t)n_seq), excl((size_t)n_seq);
          int T = 0;
          for (int v = 0; v < n_seq; ++v) {
            // short batches (T < W: empty ranges), empty sequences, and long ones
            const double u = lcg(st);
            pages[v] = u < -0.6 ? 0 : (trial % 3 == 0 ? (int)((u + 1.0) * 3.0) : (int)((u + 1.0) * 0.8 * W));
            excl[v] = T;
            T += pages[v];
          }
          if (T == 0) continue;
          EXPECT(tpla::plan_start(p, T, 0) == 0 && tpla::plan_start(p, T, W) == T);
          for (int w = 0; w < W; ++w) {
            EXPECT(tpla::plan_start(p, T, w) <= tpla::plan_start(p, T, w + 1));
            EXPECT(tpla::plan_start(p, T, w) == (int)((long long)T * tpla::plan_cum(p, w) / tpla::plan_cum(p, W)));
            int r0 = -1, r1 = -1;
            tpla::plan_range(p, T, w, &r0, &r1);                         // what a workgroup computes for itself
            EXPECT(r0 == tpla::plan_start(p, T, w) && r1 == tpla::plan_start(p, T, w + 1));
          }
          if (wt[0] == wt[1] && wt[1] == wt[2] && wt[2] == wt[3] && wx[0] == wx[1])      // equal weights: the plain equal shares
            for (int w = 0; w <= W; ++w) EXPECT(tpla::plan_start(p, T, w) == (int)((long long)w * T / W));
          for (int c = 0; c < T; ++c) {
            const int w = tpla::balanced_owner(p, c, T);
            EXPECT(w >= 0 && w < W && tpla::plan_start(p, T, w) <= c && c < tpla::plan_start(p, T, w + 1));
          }
          std::vector<int> covered((size_t)T, 0);
          for (int v = 0; v < n_seq; ++v) {
            int n_items = 0, w_first = -1, w_last = -1;
            for (int w = 0; w < W; ++w) {
              const int start = tpla::plan_start(p, T, w), end = tpla::plan_start(p, T, w + 1);
              int p0 = -1, p1 = -1;
              const bool item = pages[v] > 0 && tpla::balanced_item(start, end, excl[v], pages[v], &p0, &p1);
              EXPECT(item == (pages[v] > 0 && tpla::balanced_range_meets(p, w, T, excl[v], excl[v] + pages[v])));
              if (!item) continue;
              EXPECT(0 <= p0 && p0 < p1 && p1 <= pages[v]);
              for (int q = p0; q < p1; ++q) ++covered[(size_t)(excl[v] + q)];
              if (w_first < 0) w_first = w;
              w_last = w;
              ++n_items;
            }
            if (pages[v] > 0) {
              // what the merge computes: first and last owner of the sequence's pages
              EXPECT(w_first == tpla::balanced_owner(p, excl[v], T));
              EXPECT(w_last == tpla::balanced_owner(p, excl[v] + pages[v] - 1, T));
              EXPECT(n_items >= 1 && n_items <= w_last - w_first + 1);
              if (!tpla::plan_sparse(p, T)) EXPECT(n_items == w_last - w_first + 1);   // no empty range in between
            } else {
              EXPECT(n_items == 0);
            }
          }
          for (int c = 0; c < T; ++c) EXPECT(covered[(size_t)c] == 1);
        }
  // the weighted plans of the library's own launches leave no range empty (the merge relies on it:
  // it only looks for empty ranges when there are fewer pages than ranges)
  const int full[][8] = {{512, 256, 135, 121, 128, 128, 128, 128}, {768, 256, 140, 129, 115, 128, 128, 128},
                         {768, 256, 149, 131, 106, 128, 128, 113}, {512, 256, 128, 128, 128, 128, 128, 123},
                         {512, 256, 128, 128, 128, 128, 128, 115}, {256, 256, 128, 128, 128, 128, 128, 123}};
  for (const auto& f : full) {
    tpla::BalancedPlan p;
    p.W = f[0];
    p.n_cus = f[1];
    for (int r = 0; r < 4; ++r) p.wt[r] = f[2 + r];
    p.wx[0] = f[6];
    p.wx[1] = f[7];
    for (int T : {32 * f[0], 32 * f[0] + 17, 100000, 2000000})
      for (int w = 0; w < p.W; ++w) EXPECT(tpla::plan_start(p, T, w) < tpla::plan_start(p, T, w + 1));
    // owners at the edges of every range for page counts on both sides of the 32-bit path's limit
    // (T W < 2^31) and far beyond it
    for (int T : {4194303, 4194304, 4194305, 2796202, 2796203, 123456789, 2000000000})
      for (int w = 0; w < p.W; ++w) {
        const int lo = tpla::plan_start(p, T, w), hi = tpla::plan_start(p, T, w + 1);
        EXPECT(lo < hi);
        EXPECT(lo == (int)((long long)T * tpla::plan_cum(p, w) / tpla::plan_cum(p, p.W)));
        EXPECT(tpla::balanced_owner(p, lo, T) == w && tpla::balanced_owner(p, hi - 1, T) == w);
        EXPECT(tpla::balanced_owner(p, lo + (hi - lo) / 2, T) == w);
      }
  }
  // the same with equal weights (the 32-bit path and its fallback)
  for (int W : {1, 3, 256, 512, 768}) {
    tpla::BalancedPlan p;
    p.W = W;
    p.n_cus = 256;
    for (int r = 0; r < 4; ++r) p.wt[r] = 128;
    p.wx[0] = p.wx[1] = 128;
    for (long long T64 : {2147483647LL / W - 1, 2147483647LL / W, 2147483647LL / W + 1, 2147483647LL / W + 2, 2000000000LL}) {
      if (T64 > 2147483647LL) continue;
      const int T = (int)T64;
      for (int w = 0; w < W; ++w) {
        const int lo = tpla::plan_start(p, T, w), hi = tpla::plan_start(p, T, w + 1);
        EXPECT(lo == (int)((long long)w * T / W) && lo < hi);
        int r0 = -1, r1 = -1;
        tpla::plan_range(p, T, w, &r0, &r1);
        EXPECT(r0 == lo && r1 == hi);
        EXPECT(tpla::balanced_owner(p, lo, T) == w && tpla::balanced_owner(p, hi - 1, T) == w);
      }
    }
  }
}

int main() {
  plan_checks();
  argument_checks();
  block_table_checks();
  pca_checks();
  if (g_failures) {
    fprintf(stderr, "%d expectation(s) failed\n", g_failures);
    return 1;
  }
  printf("abi_host_driver: all expectations held\n");
  return 0;
}
