// Internal declarations shared by the translation units of libtpla.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "tpla.h"

namespace tpla {

// Records the message returned by tpla_last_error() and hands back `code`.
int fail(int code, const char* fmt, ...);
// Checks hipGetLastError() after a launch.
int check_launch(const char* what);
// Number of compute units of the current device (cached per device).
int device_cu_count();

typedef __bf16 bf16_t;

// Split plan of the decode: the sequence axis of every sequence is cut into
// chunks of pages_per_split pages; chunk s of sequence b is non-empty when
// s * pages_per_split < ceil(seq_lens[b] / page_tokens).
// Balanced mode instead lays all pages end to end and gives each of n_wg
// workgroups an equal range (see decode_mfma_balanced_kernel).
struct SplitPlan {
  int32_t balanced;
  int32_t n_wg;              // balanced: workgroups; partial slots = n_wg + n_shards * B
  int32_t n_splits;          // static
  int32_t pages_per_split;   // static
  int32_t round_wt[4];       // balanced: weight of the ranges of each placement round
  int32_t xcc_wt[2];         // balanced: weight of the ranges of even / odd workgroups
};
SplitPlan plan_splits(const tpla_shape_t& sh, int32_t n_shards, int32_t max_pages_per_seq, int32_t n_splits_req);

// Balanced plan.  The T pages of all (slice, sequence) pairs are laid end to end and cut into W
// ranges, one per workgroup; range w is [plan_start(w), plan_start(w + 1)).  Ranges are weighted by
// the placement round of their workgroup (round = w / n_cus; the hardware fills every compute unit
// once before it places a second workgroup on any) and by the parity of its position in the round
// (workgroups go to the eight XCCs in turn and n_cus is a multiple of 8 on the hardware, so this is the
// parity of the XCC): the weight of range w is wt[w / n_cus] * wx[(w % n_cus) & 1].
// All weights equal = ranges [w T / W, (w + 1) T / W).
struct BalancedPlan {
  int32_t W;        // ranges = workgroups
  int32_t n_cus;    // workgroups per placement round
  int32_t wt[4];    // weight of a range of round min(r, 3); positive
  int32_t wx[2];    // weight of a range at an even / odd position of its round; positive
};
// Sum of the weights of ranges 0 .. w-1.
__host__ __device__ __forceinline__ long long plan_cum(const BalancedPlan& p, int w) {
  long long c = 0;
  int r = 0, left = w;
  const long long pair = (long long)p.wx[0] + p.wx[1];
  while (r < 3 && left > p.n_cus) {
    c += ((long long)(p.n_cus / 2) * pair + (long long)(p.n_cus & 1) * p.wx[0]) * p.wt[r];
    left -= p.n_cus;
    ++r;
  }
  return c + ((long long)(left / 2) * pair + (long long)(left & 1) * p.wx[0]) * p.wt[r];
}
// First page of range w, 0 <= w <= W (T pages in all; T * total weight stays below 2^62).
// total = plan_cum(p, p.W), for callers that need several ranges.
__host__ __device__ __forceinline__ int plan_start(const BalancedPlan& p, long long T, int w, long long total) {
  return (int)(T * plan_cum(p, w) / total);
}
__host__ __device__ __forceinline__ int plan_start(const BalancedPlan& p, long long T, int w) {
  return plan_start(p, T, w, plan_cum(p, p.W));
}
__host__ __device__ __forceinline__ bool plan_equal_weights(const BalancedPlan& p) {
  return p.wt[0] == p.wt[1] && p.wt[1] == p.wt[2] && p.wt[2] == p.wt[3] && p.wx[0] == p.wx[1];
}
// Range w as [*start, *end) = [plan_start(w), plan_start(w + 1)), 0 <= w < W: equal ranges of not too many
// pages in 32-bit arithmetic (every workgroup of the split kernel begins with this).
__host__ __device__ __forceinline__ void plan_range(const BalancedPlan& p, int T, int w, int* start, int* end) {
  if (plan_equal_weights(p) && (long long)T * p.W < 2147483647LL) {
    *start = (int)((unsigned)w * (unsigned)T / (unsigned)p.W);
    *end = (int)(((unsigned)w + 1u) * (unsigned)T / (unsigned)p.W);
    return;
  }
  const long long total = plan_cum(p, p.W);
  *start = plan_start(p, T, w, total);
  *end = plan_start(p, T, w + 1, total);
}
// The range that holds page c, 0 <= c < T.
__host__ __device__ __forceinline__ int balanced_owner(const BalancedPlan& p, int c, int T) {
  if (plan_equal_weights(p) && (long long)T * p.W < 2147483647LL) {
    // equal ranges [w T / W, (w + 1) T / W): the owner of c is the last w with w T / W <= c, in 32-bit arithmetic
    const unsigned w = (((unsigned)c + 1u) * (unsigned)p.W + (unsigned)T - 1u) / (unsigned)T - 1u;
    return (int)w;
  }
  // First guess from the inverse of the piecewise linear cumulative weight (with the mean of the two
  // parity weights) in floating point, then steps to the exact range with the test
  //   plan_start(w) <= c   <=>   T cum(w) < (c + 1) total
  // which needs no division (a 64-bit integer division costs the GPU a hundred instructions; the
  // guess only decides how many steps follow, the result is exact either way).
  const long long total = plan_cum(p, p.W);
  const double pair = (double)p.wx[0] + (double)p.wx[1];
  double x = (double)c * (double)total / (double)T;
  int r = 0, base = 0;
  while (r < 3 && base + p.n_cus < p.W) {
    const double round_weight = (double)(plan_cum(p, base + p.n_cus) - plan_cum(p, base));
    if (x < round_weight) break;
    x -= round_weight;
    base += p.n_cus;
    ++r;
  }
  int w = base + (int)(2.0 * x / ((double)p.wt[r] * pair));
  if (w > p.W - 1) w = p.W - 1;
  if (w < 0) w = 0;
  const long long bound = ((long long)c + 1) * total;
  while (w + 1 < p.W && (long long)T * plan_cum(p, w + 1) < bound) ++w;
  while (w > 0 && !((long long)T * plan_cum(p, w) < bound)) --w;
  return w;
}
// Whether some range of the plan may be empty (fewer pages than ranges; with weights, fewer than
// about 1.1 per range): the merge then has to test every range between a sequence's first and last.
__host__ __device__ __forceinline__ bool plan_sparse(const BalancedPlan& p, long long T) {
  int m = p.wt[0];
  for (int r = 1; r < 4; ++r) m = p.wt[r] < m ? p.wt[r] : m;
  const int mx = p.wx[0] < p.wx[1] ? p.wx[0] : p.wx[1];
  return T * m * mx < plan_cum(p, p.W);
}
// Whether range w meets the pages [c0, c1) (only in doubt when plan_sparse()).
__host__ __device__ __forceinline__ bool balanced_range_meets(const BalancedPlan& p, int w, int T, int c0, int c1) {
  const int lo = plan_start(p, T, w), hi = plan_start(p, T, w + 1);
  return (lo > c0 ? lo : c0) < (hi < c1 ? hi : c1);
}
// The work item of a workgroup that owns the pages [start, end) in a sequence whose n pages begin at
// page e of the laid-out order: its pages [*p0, *p1) counted inside the sequence.  False when the two
// ranges share no page (also for an empty workgroup range that lies inside the sequence).
__host__ __device__ __forceinline__ bool balanced_item(int start, int end, int e, int n, int* p0, int* p1) {
  const int lo = start > e ? start : e, hi = end < e + n ? end : e + n;
  *p0 = lo - e;
  *p1 = hi - e;
  return lo < hi;
}

// Partial results of one (slice, sequence, split): acc [n_shards, B, S, H, dl]
// floats, then ml [n_shards, B, S, H, 2] floats (running max in log2 units, sum of weights).
// Several latent slices can share one launch: slice i uses q_lat[i], pools[i],
// the common q_pe / page table / lengths, and row i of every output.
struct DecodeArgs {
  const void* q_lat;     // [n_shards, B, H, dl]
  const void* q_pe;      // [B, H, d_r]
  const void* pools[TPLA_MAX_G];   // each [P, page_tokens, dl + d_r]
  const int32_t* block_table;
  const int32_t* seq_lens;
  float* part_acc;
  float* part_ml;
  float* o_lat;          // [n_shards, B, H, dl]
  float* lse;            // [n_shards, B, H] or nullptr
  int32_t n_shards;
  int32_t B, H, dl, d_r, page_tokens, max_pages;
  int32_t n_splits, pages_per_split;
  int32_t balanced, n_wg;
  BalancedPlan geom;     // balanced: ranges and their weights (geom.W == n_wg)
  // balanced, written by workgroup 0 of the split kernel for the merge (n_v = n_shards * B entries each):
  // [0, n_v) first page of every (slice, sequence) in the laid-out order; [n_v] total pages T;
  // [n_v + 1, 2 n_v + 1) the range that owns its first page; [2 n_v + 1, 3 n_v + 1) how many ranges from
  // there to the owner of its last page (0 for an empty sequence); [3 n_v + 1] plan_sparse(T)
  int32_t* plan;
  float scale_log2;      // sm_scale * log2(e)
};

// True when the MFMA kernel covers this shape (bf16 only).
bool decode_mfma_supported(const tpla_shape_t& sh);
// Workgroups of the matrix-core kernel for this shape that fit on one compute
// unit (0 = unknown).
int decode_mfma_blocks_per_cu(const tpla_shape_t& sh);
// Range weights by placement round (wt) and by even / odd position in the round (wx) for a launch that
// puts per_cu workgroups of the matrix-core kernel on every compute unit.
void decode_mfma_round_weights(const tpla_shape_t& sh, int per_cu, int32_t wt[4], int32_t wx[2]);
// ev_start / ev_stop (both or neither): events that receive the kernel's begin and end times.
int launch_decode_mfma(const DecodeArgs& a, hipStream_t st, hipEvent_t ev_start = nullptr,
                       hipEvent_t ev_stop = nullptr);
// Length of sequence b as every decode kernel uses it: clipped to what its block-table row can
// address, so a length that disagrees with max_pages_per_seq gives wrong numbers, never a read
// past the table.
__device__ __forceinline__ int seq_len_clipped(const DecodeArgs& a, int b) {
  const long long cap = (long long)a.max_pages * a.page_tokens;
  const long long L = a.seq_lens[b];
  return (int)(L < 0 ? 0 : (L > cap ? cap : L));
}

int launch_decode_generic(const DecodeArgs& a, int dtype, hipStream_t st);
int launch_decode_merge(const DecodeArgs& a, hipStream_t st);

struct TransformArgs {
  int32_t d_c, dtype, mode, inverse;
  const float* signs;
  const float* U;
};
int launch_transform_axis(const TransformArgs& t, const void* src, void* dst, int64_t n_outer,
                          int64_t n_inner, hipStream_t st);
struct ShardPools {
  void* p[TPLA_MAX_G];
};
int launch_transform_paged(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                           const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                           hipStream_t st);
// Matrix-core Hadamard pass (bf16, d_c 256 / 512): see transform_mfma.hip.
bool transform_paged_mfma_supported(const TransformArgs& t, const tpla_shape_t& sh, int64_t n_pages);
int launch_transform_paged_mfma(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                                const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                                hipStream_t st);
bool transform_paged_dense_mfma_supported(const TransformArgs& t, const tpla_shape_t& sh, int64_t n_pages);
int launch_transform_paged_dense_mfma(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                                      const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                                      hipStream_t st);
int launch_write_mla_cache(const tpla_shape_t& sh, const void* c_raw, const void* k_pe,
                           const int32_t* slot_mapping, int64_t T, float rms_eps, void* mla_pool,
                           hipStream_t st);

int launch_append_token_sliced(const tpla_shape_t& sh, const void* c_t, const void* k_pe,
                               const struct MuFactors& alpha, float rms_eps, const int32_t* slots,
                               const ShardPools& pools, hipStream_t st);

// Output projection (after the combine): out = x @ W_O.
int output_projection_ksplit(const tpla_shape_t& sh, int D);
size_t output_projection_scratch_floats(const tpla_shape_t& sh, int D, int out_dtype);
int launch_output_projection(const tpla_shape_t& sh, const float* x, const void* W_O, int D, float* part,
                             void* out, int out_dtype, hipStream_t st);

// Prefill (un-absorbed MLA, causal, packed sequences): see prefill_mfma.hip.
bool prefill_mfma_supported(const tpla_shape_t& sh);
int launch_prefill_attention(const tpla_shape_t& sh, const void* q_nope, const void* q_pe, const void* c,
                             const void* k_pe, const void* W_UK, const void* W_UV, const int32_t* cu_seqlens,
                             int T, int max_seq_len, void* kv_workspace, float* o, hipStream_t st);

int launch_stream_read(const void* buf, size_t bytes, void* sink, hipStream_t st);

// PCA calibration: see pca.hip.
int latent_moments_splits(const tpla_shape_t& sh, int64_t n_pages);
size_t latent_moments_workspace(const tpla_shape_t& sh, int64_t n_pages);
int launch_latent_moments(const tpla_shape_t& sh, const void* mla_pool, const int32_t* page_ids,
                          const int32_t* page_fill, int64_t n_pages, float* workspace, double* sum, double* gram,
                          hipStream_t st);
int pca_basis_host(int d, int g, double n_rows, const double* sum, const double* gram, float* U, double* eig,
                   double* frac);

struct MuFactors {
  float v[TPLA_MAX_G];
};
int launch_absorb_query(const tpla_shape_t& sh, const void* q_nope, const void* W_UK_t,
                        const MuFactors& mu, void* q_lat, hipStream_t st);
int launch_combine_shards(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, void* o, int o_dtype,
                          hipStream_t st);
// Matrix-core variants (bf16 weights, widths that tile): see absorb_combine_mfma.hip.
bool absorb_mfma_supported(const tpla_shape_t& sh);
int launch_absorb_query_mfma(const tpla_shape_t& sh, const void* q_nope, const void* W_UK_t,
                             const MuFactors& mu, void* q_lat, hipStream_t st);
bool combine_mfma_supported(const tpla_shape_t& sh);
int launch_combine_shards_mfma(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, void* o, int o_dtype,
                               hipStream_t st);
// Split merge fused with the combine: reads the decode's partial results, writes o_lat, lse and o.
bool merge_combine_mfma_supported(const tpla_shape_t& sh);
int launch_merge_combine_mfma(const DecodeArgs& a, const tpla_shape_t& sh, const void* W_UV_t, void* o, int o_dtype,
                              hipStream_t st);

// ---- small device helpers -------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return (float)x; }
__device__ __forceinline__ float load_as_f32(const float* p) { return *p; }
__device__ __forceinline__ float load_as_f32(const bf16_t* p) { return (float)*p; }
__device__ __forceinline__ void store_from_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_from_f32(bf16_t* p, float v) { *p = (bf16_t)v; }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 8 consecutive elements of a row, as floats.
struct Vec8 {
  float v[8];
};
__device__ __forceinline__ Vec8 load8(const bf16_t* p) {
  const u32x4 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  Vec8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.v[2 * i] = __uint_as_float(raw[i] << 16);
    r.v[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
  return r;
}
__device__ __forceinline__ Vec8 load8(const float* p) {
  const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  const u32x4 b = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p) + 1);
  Vec8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.v[i] = __uint_as_float(a[i]);
    r.v[4 + i] = __uint_as_float(b[i]);
  }
  return r;
}
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(unsigned short, (bf16_t)f);
}
__device__ __forceinline__ void store8(bf16_t* p, const Vec8& r) {
  u32x4 raw;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    raw[i] = (unsigned)f32_to_bf16_bits(r.v[2 * i]) | ((unsigned)f32_to_bf16_bits(r.v[2 * i + 1]) << 16);
  __builtin_nontemporal_store(raw, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store8(float* p, const Vec8& r) {
  u32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = __float_as_uint(r.v[i]);
    b[i] = __float_as_uint(r.v[4 + i]);
  }
  __builtin_nontemporal_store(a, reinterpret_cast<u32x4*>(p));
  __builtin_nontemporal_store(b, reinterpret_cast<u32x4*>(p) + 1);
}

// Plain (cached) variant of load8 for operands that are re-read.
__device__ __forceinline__ Vec8 load8_cached(const bf16_t* p) {
  const u32x4 raw = *reinterpret_cast<const u32x4*>(p);
  Vec8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.v[2 * i] = __uint_as_float(raw[i] << 16);
    r.v[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
  return r;
}
__device__ __forceinline__ Vec8 load8_cached(const float* p) {
  const u32x4 a = *reinterpret_cast<const u32x4*>(p);
  const u32x4 b = *(reinterpret_cast<const u32x4*>(p) + 1);
  Vec8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    r.v[i] = __uint_as_float(a[i]);
    r.v[4 + i] = __uint_as_float(b[i]);
  }
  return r;
}

}  // namespace tpla
