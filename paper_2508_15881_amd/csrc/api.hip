// C ABI entry points of libtpla: argument validation, split planning and
// dispatch to the kernels.  No kernel is launched when validation fails.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <math.h>
#include "tpla_internal.h"
#include <mutex>
#include <vector>

namespace tpla {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TPLA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return TPLA_OK;
}

int device_cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// ---- optional event bracketing of the split kernel -------------------------
struct ProfileState {
  hipEvent_t* ev = nullptr;   // 2 * cap events
  int cap = 0;
  int used = 0;
};
static thread_local ProfileState g_prof;

static void profile_mark(hipStream_t st, bool start) {
  if (g_prof.cap == 0 || g_prof.used >= g_prof.cap) return;
  (void)hipEventRecord(g_prof.ev[2 * g_prof.used + (start ? 0 : 1)], st);
  if (!start) ++g_prof.used;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_dtype(const tpla_shape_t* sh) {
  if (!sh) return fail(TPLA_ERR_NULL, "shape is NULL");
  if (sh->dtype != TPLA_F32 && sh->dtype != TPLA_BF16)
    return fail(TPLA_ERR_DTYPE, "dtype %d is neither TPLA_F32 nor TPLA_BF16", sh->dtype);
  return TPLA_OK;
}

// Full consistency check of the attention geometry.
static int check_shape(const tpla_shape_t* sh) {
  int rc = check_dtype(sh);
  if (rc) return rc;
  if (sh->B < 1 || sh->H < 1 || sh->d_c < 1 || sh->g < 1 || sh->d_r < 1 || sh->d_n < 1 ||
      sh->d_v < 1 || sh->page_tokens < 1)
    return fail(TPLA_ERR_SHAPE, "every dimension must be positive (B=%d H=%d d_c=%d g=%d d_r=%d d_n=%d d_v=%d page_tokens=%d)",
                sh->B, sh->H, sh->d_c, sh->g, sh->d_r, sh->d_n, sh->d_v, sh->page_tokens);
  if (sh->g > TPLA_MAX_G) return fail(TPLA_ERR_SHAPE, "g=%d exceeds TPLA_MAX_G=%d", sh->g, TPLA_MAX_G);
  if (sh->d_c % sh->g) return fail(TPLA_ERR_SHAPE, "d_c=%d is not divisible by g=%d", sh->d_c, sh->g);
  const int dl = sh->d_c / sh->g;
  if (dl % 8 || sh->d_r % 8)
    return fail(TPLA_ERR_SHAPE, "d_c/g=%d and d_r=%d must be multiples of 8 (16-byte row pieces)", dl, sh->d_r);
  if (!(sh->sm_scale > 0.0f) || !isfinite(sh->sm_scale))
    return fail(TPLA_ERR_SHAPE, "sm_scale must be positive and finite");
  return TPLA_OK;
}

SplitPlan plan_splits(const tpla_shape_t& sh, int32_t n_shards, int32_t max_pages, int32_t n_splits_req) {
  SplitPlan p;
  p.balanced = 0;
  p.n_wg = 0;
  for (int r = 0; r < 4; ++r) p.round_wt[r] = 1;
  p.xcc_wt[0] = p.xcc_wt[1] = 1;
  int32_t n = n_splits_req;
  if (n <= 0 && sh.dtype == TPLA_BF16 && decode_mfma_supported(sh)) {
    // Automatic plan of the matrix-core kernel: exactly as many workgroups as
    // the chip holds at once, each taking an equal share of all pages.
    int per_cu = decode_mfma_blocks_per_cu(sh);
    if (per_cu <= 0) per_cu = 2;
    int n_wg = device_cu_count() * per_cu;
    if (n_wg > 1024) n_wg = 1024;     // the merge handles at most 1024 partial results per sequence
    const long long most = (long long)n_shards * sh.B * max_pages;
    // Small batches: a workgroup's fixed costs (queries, first tiles, partial result) want at least
    // 8 pages behind them, but never fewer workgroups than compute units (measured at 16 x 4096
    // tokens: 256 workgroups of 8 pages 26 us, 512 of 4 pages 31 us, 128 of 16 pages 38 us).
    const int cus = device_cu_count();
    if (most / 8 < n_wg) n_wg = most / 8 > cus ? (int)(most / 8) : (cus < n_wg ? cus : n_wg);
    if (n_wg > most) n_wg = (int)most;
    // A full launch of long ranges: the workgroup placed first on a compute unit runs ahead of the
    // ones placed after it, so the ranges are sized by placement round for all to end together.
    if (n_wg == cus * per_cu && cus % 8 == 0 && most / n_wg >= 32) decode_mfma_round_weights(sh, per_cu, p.round_wt, p.xcc_wt);
    p.balanced = 1;
    p.n_wg = n_wg;
    p.n_splits = 1;
    p.pages_per_split = max_pages;
    return p;
  }
  if (n <= 0) {
    // Static chunks sized so that one round of workgroups covers the batch
    // when sequences are equally long; at least 4 pages per chunk.
    const int slots = device_cu_count() * 4;
    n = slots / (sh.B * n_shards);
    const int32_t cap = (max_pages + 3) / 4;
    if (n > cap) n = cap;
    if (n > 1024) n = 1024;
    if (n < 1) n = 1;
  }
  if (n > max_pages) n = max_pages;
  if (n < 1) n = 1;
  p.pages_per_split = (max_pages + n - 1) / n;
  p.n_splits = (max_pages + p.pages_per_split - 1) / p.pages_per_split;
  return p;
}

// Partial-result slots of a plan, and the workspace: acc [slots, H, dl] floats,
// (reference, sum) [slots, H, 2] floats, then (balanced) the plan table the split kernel leaves for the merge.
static size_t plan_slots(const tpla_shape_t& sh, int n_shards, const SplitPlan& p) {
  return p.balanced ? (size_t)p.n_wg + (size_t)n_shards * sh.B : (size_t)n_shards * sh.B * p.n_splits;
}
static size_t workspace_for(const tpla_shape_t& sh, int n_shards, const SplitPlan& p) {
  const size_t dl = (size_t)(sh.d_c / sh.g);
  size_t bytes = plan_slots(sh, n_shards, p) * sh.H * (dl + 2) * sizeof(float);
  if (p.balanced) bytes += ((3 * (size_t)n_shards * sh.B + 2) * sizeof(int32_t) + 15) / 16 * 16;
  return bytes;
}

// Validation, planning and launches shared by the one-slice and the
// all-slices entry points.  With W_UV_t and o given (all slices only) the
// combine follows, fused with the split merge where the shape allows.
static int decode_common(const tpla_shape_t* shape, int n_shards, const void* q_lat, const void* q_pe,
                         const void* const* pools, const int32_t* block_table, int32_t max_pages_per_seq,
                         const int32_t* seq_lens, int32_t n_splits, void* workspace,
                         size_t workspace_bytes, float* o_lat, float* lse, void* stream,
                         const void* W_UV_t = nullptr, void* o = nullptr, int o_dtype = TPLA_F32) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q_lat || !q_pe || !pools || !block_table || !seq_lens || !workspace || !o_lat)
    return fail(TPLA_ERR_NULL, "a required pointer is NULL");
  if (!aligned16(W_UV_t) || !aligned16(o)) return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (max_pages_per_seq < 1 || n_splits < 0)
    return fail(TPLA_ERR_SHAPE, "max_pages_per_seq=%d n_splits=%d", max_pages_per_seq, n_splits);
  if ((int64_t)max_pages_per_seq * shape->page_tokens > (int64_t)2147483647)
    return fail(TPLA_ERR_SHAPE, "max_pages_per_seq * page_tokens overflows int32");
  for (int i = 0; i < n_shards; ++i) {
    if (!pools[i]) return fail(TPLA_ERR_NULL, "cache pool %d is NULL", i);
    if (!aligned16(pools[i])) return fail(TPLA_ERR_ALIGN, "cache pool %d is not 16-byte aligned", i);
  }
  if (!aligned16(q_lat) || !aligned16(q_pe) || !aligned16(block_table) || !aligned16(seq_lens) ||
      !aligned16(workspace) || !aligned16(o_lat) || !aligned16(lse))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  const SplitPlan plan = plan_splits(*shape, n_shards, max_pages_per_seq, n_splits);
  const size_t need = workspace_for(*shape, n_shards, plan);
  if (workspace_bytes < need)
    return fail(TPLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  if (plan.n_splits > 1024)
    return fail(TPLA_ERR_UNSUPPORTED, "n_splits=%d above 1024", plan.n_splits);
  if ((int64_t)n_shards * shape->B * plan.n_splits > (int64_t)2147483647 / 4 ||
      (int64_t)n_shards * shape->B * max_pages_per_seq > (int64_t)2147483647 / 2)
    return fail(TPLA_ERR_UNSUPPORTED, "n_shards * B * n_splits (or * max_pages_per_seq) too large");

  DecodeArgs a;
  const int dl = shape->d_c / shape->g;
  a.q_lat = q_lat;
  a.q_pe = q_pe;
  for (int i = 0; i < TPLA_MAX_G; ++i) a.pools[i] = i < n_shards ? pools[i] : nullptr;
  a.block_table = block_table;
  a.seq_lens = seq_lens;
  a.part_acc = static_cast<float*>(workspace);
  const size_t slots = plan_slots(*shape, n_shards, plan);
  a.part_ml = a.part_acc + slots * shape->H * dl;
  a.plan = reinterpret_cast<int32_t*>(a.part_ml + slots * shape->H * 2);
  a.balanced = plan.balanced;
  a.n_wg = plan.n_wg;
  a.geom.W = plan.n_wg;
  a.geom.n_cus = device_cu_count();
  for (int r = 0; r < 4; ++r) a.geom.wt[r] = plan.round_wt[r];
  a.geom.wx[0] = plan.xcc_wt[0];
  a.geom.wx[1] = plan.xcc_wt[1];
  a.o_lat = o_lat;
  a.lse = lse;
  a.n_shards = n_shards;
  a.B = shape->B;
  a.H = shape->H;
  a.dl = dl;
  a.d_r = shape->d_r;
  a.page_tokens = shape->page_tokens;
  a.max_pages = max_pages_per_seq;
  a.n_splits = plan.n_splits;
  a.pages_per_split = plan.pages_per_split;
  a.scale_log2 = shape->sm_scale * 1.4426950408889634f;

  hipStream_t st = (hipStream_t)stream;
  if (shape->dtype == TPLA_BF16 && decode_mfma_supported(*shape)) {
    // recording: the event pair is attached to the kernel's dispatch and takes its begin and end times
    const bool rec = g_prof.cap > 0 && g_prof.used < g_prof.cap;
    rc = launch_decode_mfma(a, st, rec ? g_prof.ev[2 * g_prof.used] : nullptr,
                            rec ? g_prof.ev[2 * g_prof.used + 1] : nullptr);
    if (rec && rc == TPLA_OK) ++g_prof.used;
  } else {
    profile_mark(st, true);
    rc = launch_decode_generic(a, shape->dtype, st);
    profile_mark(st, false);
  }
  if (rc) return rc;
  if (!W_UV_t) return launch_decode_merge(a, st);
  if (merge_combine_mfma_supported(*shape)) return launch_merge_combine_mfma(a, *shape, W_UV_t, o, o_dtype, st);
  rc = launch_decode_merge(a, st);
  if (rc) return rc;
  if (combine_mfma_supported(*shape)) return launch_combine_shards_mfma(*shape, o_lat, W_UV_t, o, o_dtype, st);
  return launch_combine_shards(*shape, o_lat, W_UV_t, o, o_dtype, st);
}

// ---- scratch of the entry point that takes no workspace ---------------------
// The partial results of tpla_decode_shards_combine_static live in this array
// instead of a caller's buffer.  Every device the library runs on holds its own
// copy at its own address; host code never uses the array's name as an address
// but the per-device pointer that hipGetSymbolAddress returned.
static __device__ __align__(256) unsigned char scratch[TPLA_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {nullptr};   // per device, filled on the first call there

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return fail(TPLA_ERR_HIP, "no current device (or a device index above 63)");
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return fail(TPLA_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TPLA_OK;
}

}  // namespace tpla

using namespace tpla;

extern "C" {
#pragma GCC visibility push(default)

const char* tpla_last_error(void) { return g_err; }

int tpla_version(void) { return 100; }

int tpla_transform_latent(const tpla_shape_t* shape, int mode, int inverse, const float* signs,
                          const float* U, const void* src, void* dst, int64_t n_outer,
                          int64_t n_inner, void* stream) {
  int rc = check_dtype(shape);
  if (rc) return rc;
  if (!src || !dst) return fail(TPLA_ERR_NULL, "src/dst is NULL");
  if (shape->d_c < 1 || n_outer < 0 || n_inner < 1)
    return fail(TPLA_ERR_SHAPE, "d_c=%d n_outer=%lld n_inner=%lld", shape->d_c, (long long)n_outer, (long long)n_inner);
  if (mode != TPLA_U_IDENTITY && mode != TPLA_U_HADAMARD && mode != TPLA_U_DENSE)
    return fail(TPLA_ERR_SHAPE, "unknown transform mode %d", mode);
  if (mode == TPLA_U_HADAMARD && (shape->d_c & (shape->d_c - 1)))
    return fail(TPLA_ERR_SHAPE, "Hadamard transform needs a power-of-two d_c, got %d", shape->d_c);
  if (mode == TPLA_U_DENSE && !U) return fail(TPLA_ERR_NULL, "dense mode needs U");
  if (shape->d_c > 8192) return fail(TPLA_ERR_UNSUPPORTED, "d_c=%d above 8192", shape->d_c);
  if (!aligned16(src) || !aligned16(dst) || !aligned16(signs) || !aligned16(U))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (n_outer == 0) return TPLA_OK;
  if (n_outer * n_inner > (int64_t)2147483647)
    return fail(TPLA_ERR_UNSUPPORTED, "n_outer*n_inner above 2^31-1");
  TransformArgs t{shape->d_c, shape->dtype, mode, inverse ? 1 : 0, signs, U};
  return launch_transform_axis(t, src, dst, n_outer, n_inner, (hipStream_t)stream);
}

int tpla_transform_latent_paged(const tpla_shape_t* shape, int mode, const float* signs,
                                const float* U, const void* mla_pool, void* const* shard_pools,
                                const int32_t* page_ids, int64_t n_pages, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!mla_pool || !shard_pools) return fail(TPLA_ERR_NULL, "mla_pool/shard_pools is NULL");
  if (mode != TPLA_U_IDENTITY && mode != TPLA_U_HADAMARD && mode != TPLA_U_DENSE)
    return fail(TPLA_ERR_SHAPE, "unknown transform mode %d", mode);
  if (mode == TPLA_U_HADAMARD && (shape->d_c & (shape->d_c - 1)))
    return fail(TPLA_ERR_SHAPE, "Hadamard transform needs a power-of-two d_c, got %d", shape->d_c);
  if (mode == TPLA_U_DENSE && !U) return fail(TPLA_ERR_NULL, "dense mode needs U");
  if (shape->d_c > 8192) return fail(TPLA_ERR_UNSUPPORTED, "d_c=%d above 8192", shape->d_c);
  if (shape->d_c % 8) return fail(TPLA_ERR_SHAPE, "d_c must be a multiple of 8");
  if (n_pages < 0 || n_pages * shape->page_tokens > (int64_t)2147483647)
    return fail(TPLA_ERR_SHAPE, "n_pages=%lld out of range", (long long)n_pages);
  ShardPools pools;
  for (int i = 0; i < TPLA_MAX_G; ++i) pools.p[i] = nullptr;
  for (int i = 0; i < shape->g; ++i) {
    if (!shard_pools[i]) return fail(TPLA_ERR_NULL, "shard_pools[%d] is NULL", i);
    if (!aligned16(shard_pools[i])) return fail(TPLA_ERR_ALIGN, "shard_pools[%d] not 16-byte aligned", i);
    pools.p[i] = shard_pools[i];
  }
  if (!aligned16(mla_pool) || !aligned16(page_ids) || !aligned16(signs) || !aligned16(U))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (n_pages == 0) return TPLA_OK;
  TransformArgs t{shape->d_c, shape->dtype, mode, 0, signs, U};
  return launch_transform_paged(t, *shape, mla_pool, pools, page_ids, n_pages, (hipStream_t)stream);
}

int tpla_write_mla_cache(const tpla_shape_t* shape, const void* c_raw, const void* k_pe,
                         const int32_t* slot_mapping, int64_t T, float rms_eps, void* mla_pool,
                         void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!c_raw || !k_pe || !slot_mapping || !mla_pool) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (T < 0 || T > (int64_t)2147483647) return fail(TPLA_ERR_SHAPE, "T=%lld out of range", (long long)T);
  if (shape->d_c % 8) return fail(TPLA_ERR_SHAPE, "d_c must be a multiple of 8");
  if (!aligned16(c_raw) || !aligned16(k_pe) || !aligned16(slot_mapping) || !aligned16(mla_pool))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (isnan(rms_eps)) return fail(TPLA_ERR_SHAPE, "rms_eps is NaN");
  if (T == 0) return TPLA_OK;
  return launch_write_mla_cache(*shape, c_raw, k_pe, slot_mapping, T, rms_eps, mla_pool,
                                (hipStream_t)stream);
}

int tpla_append_token_sliced(const tpla_shape_t* shape, const void* c_t, const void* k_pe,
                             const float* alpha, float rms_eps, const int32_t* slots,
                             void* const* shard_pools, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!c_t || !k_pe || !slots || !shard_pools) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (!(rms_eps >= 0.0f) || !isfinite(rms_eps)) return fail(TPLA_ERR_SHAPE, "rms_eps must be finite and >= 0");
  ShardPools pools;
  for (int i = 0; i < TPLA_MAX_G; ++i) pools.p[i] = nullptr;
  MuFactors a;
  for (int i = 0; i < TPLA_MAX_G; ++i) a.v[i] = (float)shape->g;
  for (int i = 0; i < shape->g; ++i) {
    if (!shard_pools[i]) return fail(TPLA_ERR_NULL, "shard_pools[%d] is NULL", i);
    if (!aligned16(shard_pools[i])) return fail(TPLA_ERR_ALIGN, "shard_pools[%d] not 16-byte aligned", i);
    pools.p[i] = shard_pools[i];
    if (alpha) {
      if (!(alpha[i] > 0.0f) || !isfinite(alpha[i])) return fail(TPLA_ERR_SHAPE, "alpha[%d] must be positive", i);
      a.v[i] = alpha[i];
    }
  }
  if (!aligned16(c_t) || !aligned16(k_pe) || !aligned16(slots))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (shape->B > 2147483647 / 2 || shape->g > 65535) return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  return launch_append_token_sliced(*shape, c_t, k_pe, a, rms_eps, slots, pools, (hipStream_t)stream);
}

int tpla_absorb_query(const tpla_shape_t* shape, const void* q_nope, const void* W_UK_t,
                      const float* mu, void* q_lat, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q_nope || !W_UK_t || !q_lat) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (!aligned16(q_nope) || !aligned16(W_UK_t) || !aligned16(q_lat))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  MuFactors m;
  for (int i = 0; i < TPLA_MAX_G; ++i) m.v[i] = 1.0f;
  if (mu)
    for (int i = 0; i < shape->g; ++i) {
      if (!isfinite(mu[i])) return fail(TPLA_ERR_SHAPE, "mu[%d] is not finite", i);
      m.v[i] = mu[i];
    }
  if (absorb_mfma_supported(*shape))
    return launch_absorb_query_mfma(*shape, q_nope, W_UK_t, m, q_lat, (hipStream_t)stream);
  return launch_absorb_query(*shape, q_nope, W_UK_t, m, q_lat, (hipStream_t)stream);
}

size_t tpla_workspace_bytes(const tpla_shape_t* shape, int32_t max_pages_per_seq, int32_t n_splits) {
  if (check_shape(shape) != TPLA_OK) return 0;
  if (max_pages_per_seq < 1 || n_splits < 0) {
    fail(TPLA_ERR_SHAPE, "max_pages_per_seq=%d n_splits=%d", max_pages_per_seq, n_splits);
    return 0;
  }
  return workspace_for(*shape, 1, plan_splits(*shape, 1, max_pages_per_seq, n_splits));
}

size_t tpla_workspace_bytes_all(const tpla_shape_t* shape, int32_t max_pages_per_seq, int32_t n_splits) {
  if (check_shape(shape) != TPLA_OK) return 0;
  if (max_pages_per_seq < 1 || n_splits < 0) {
    fail(TPLA_ERR_SHAPE, "max_pages_per_seq=%d n_splits=%d", max_pages_per_seq, n_splits);
    return 0;
  }
  return workspace_for(*shape, shape->g, plan_splits(*shape, shape->g, max_pages_per_seq, n_splits));
}

int tpla_decode_shard(const tpla_shape_t* shape, const void* q_lat_i, const void* q_pe,
                      const void* shard_pool, const int32_t* block_table,
                      int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                      void* workspace, size_t workspace_bytes, float* o_lat_i, float* lse_i,
                      void* stream) {
  const void* pools[1] = {shard_pool};
  if (shape && !shard_pool) return fail(TPLA_ERR_NULL, "a required pointer is NULL");
  return decode_common(shape, 1, q_lat_i, q_pe, pools, block_table, max_pages_per_seq, seq_lens, n_splits,
                       workspace, workspace_bytes, o_lat_i, lse_i, stream);
}

int tpla_decode_shards(const tpla_shape_t* shape, const void* q_lat, const void* q_pe,
                       const void* const* shard_pools, const int32_t* block_table,
                       int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                       void* workspace, size_t workspace_bytes, float* o_lat, float* lse,
                       void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  return decode_common(shape, shape->g, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                       n_splits, workspace, workspace_bytes, o_lat, lse, stream);
}

int tpla_decode_shards_combine(const tpla_shape_t* shape, const void* q_lat, const void* q_pe,
                               const void* const* shard_pools, const int32_t* block_table,
                               int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                               void* workspace, size_t workspace_bytes, const void* W_UV_t, float* o,
                               float* o_lat, float* lse, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!W_UV_t || !o) return fail(TPLA_ERR_NULL, "W_UV_t/o is NULL");
  return decode_common(shape, shape->g, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                       n_splits, workspace, workspace_bytes, o_lat, lse, stream, W_UV_t, o);
}

int tpla_decode_shards_combine_static(const tpla_shape_t* shape, const void* q_lat, const void* q_pe,
                                      const void* const* shard_pools, const int32_t* block_table,
                                      int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                                      const void* W_UV_t, float* o, float* o_lat, float* lse, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!W_UV_t || !o) return fail(TPLA_ERR_NULL, "W_UV_t/o is NULL");
  if (max_pages_per_seq < 1 || n_splits < 0)
    return fail(TPLA_ERR_SHAPE, "max_pages_per_seq=%d n_splits=%d", max_pages_per_seq, n_splits);
  const size_t need = workspace_for(*shape, shape->g, plan_splits(*shape, shape->g, max_pages_per_seq, n_splits));
  if (need > (size_t)TPLA_STATIC_SCRATCH_BYTES)
    return fail(TPLA_ERR_WORKSPACE,
                "this call needs %zu bytes of partial results, the built-in scratch holds %zu: use "
                "tpla_decode_shards_combine with a workspace of the caller",
                need, (size_t)TPLA_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  return decode_common(shape, shape->g, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                       n_splits, ws, (size_t)TPLA_STATIC_SCRATCH_BYTES, o_lat, lse, stream, W_UV_t, o);
}

static int check_out_dtype(int32_t d) {
  if (d != TPLA_F32 && d != TPLA_BF16) return fail(TPLA_ERR_DTYPE, "output dtype %d is neither TPLA_F32 nor TPLA_BF16", d);
  return TPLA_OK;
}

int tpla_combine_shards_to(const tpla_shape_t* shape, const float* o_lat, const void* W_UV_t, void* o,
                           int32_t o_dtype, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_out_dtype(o_dtype))) return rc;
  if (!o_lat || !W_UV_t || !o) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (!aligned16(o_lat) || !aligned16(W_UV_t) || !aligned16(o))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if (combine_mfma_supported(*shape))
    return launch_combine_shards_mfma(*shape, o_lat, W_UV_t, o, o_dtype, (hipStream_t)stream);
  return launch_combine_shards(*shape, o_lat, W_UV_t, o, o_dtype, (hipStream_t)stream);
}

int tpla_combine_shards(const tpla_shape_t* shape, const float* o_lat, const void* W_UV_t, float* o,
                        void* stream) {
  return tpla_combine_shards_to(shape, o_lat, W_UV_t, o, TPLA_F32, stream);
}

int tpla_decode_shards_combine_to(const tpla_shape_t* shape, const void* q_lat, const void* q_pe,
                                  const void* const* shard_pools, const int32_t* block_table,
                                  int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                                  void* workspace, size_t workspace_bytes, const void* W_UV_t, void* o,
                                  int32_t o_dtype, float* o_lat, float* lse, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_out_dtype(o_dtype))) return rc;
  if (!W_UV_t || !o) return fail(TPLA_ERR_NULL, "W_UV_t/o is NULL");
  return decode_common(shape, shape->g, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                       n_splits, workspace, workspace_bytes, o_lat, lse, stream, W_UV_t, o, o_dtype);
}

size_t tpla_output_projection_workspace_bytes(const tpla_shape_t* shape, int32_t D) {
  if (check_shape(shape) != TPLA_OK || D < 1) return 0;
  // sized for either output type (a bf16 output always passes through float partial tiles)
  return output_projection_scratch_floats(*shape, D, TPLA_BF16) * sizeof(float);
}

static int output_projection_common(const tpla_shape_t* shape, const float* o, const void* W_O, int32_t D,
                                    void* workspace, size_t workspace_bytes, void* out, int32_t out_dtype,
                                    void* stream) {
  if (!o || !W_O || !out) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (D < 1) return fail(TPLA_ERR_SHAPE, "D=%d", D);
  if ((long long)shape->H * shape->d_v > 2147483647LL || (long long)shape->B * D > 2147483647LL)
    return fail(TPLA_ERR_UNSUPPORTED, "H*d_v or B*D above 2^31-1");
  if (!aligned16(o) || !aligned16(W_O) || !aligned16(out) || !aligned16(workspace))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  const size_t need = output_projection_scratch_floats(*shape, D, out_dtype) * sizeof(float);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(TPLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  if ((D + 255) / 256 > 2147483647 / 2 || shape->B > 65535) return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  return launch_output_projection(*shape, o, W_O, D, static_cast<float*>(workspace), out, out_dtype,
                                  (hipStream_t)stream);
}

int tpla_output_projection_to(const tpla_shape_t* shape, const float* o, const void* W_O, int32_t D,
                              void* workspace, size_t workspace_bytes, void* out, int32_t out_dtype, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_out_dtype(out_dtype))) return rc;
  return output_projection_common(shape, o, W_O, D, workspace, workspace_bytes, out, out_dtype, stream);
}

int tpla_output_projection(const tpla_shape_t* shape, const float* o, const void* W_O, int32_t D,
                           void* workspace, size_t workspace_bytes, float* out, void* stream) {
  return tpla_output_projection_to(shape, o, W_O, D, workspace, workspace_bytes, out, TPLA_F32, stream);
}

size_t tpla_attention_block_workspace_bytes(const tpla_shape_t* shape, int32_t max_pages_per_seq, int32_t n_splits,
                                            int32_t D) {
  const size_t a = tpla_workspace_bytes_all(shape, max_pages_per_seq, n_splits);
  if (a == 0 || D < 1) return 0;
  const size_t b = tpla_output_projection_workspace_bytes(shape, D);
  return a > b ? a : b;
}

int tpla_decode_shards_project(const tpla_shape_t* shape, const void* q_lat, const void* q_pe,
                               const void* const* shard_pools, const int32_t* block_table,
                               int32_t max_pages_per_seq, const int32_t* seq_lens, int32_t n_splits,
                               void* workspace, size_t workspace_bytes, const void* W_UV_t, const void* W_O,
                               int32_t D, void* out, int32_t out_dtype, float* o, float* o_lat, float* lse,
                               void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_out_dtype(out_dtype))) return rc;
  if (!W_UV_t || !o || !W_O || !out) return fail(TPLA_ERR_NULL, "W_UV_t/W_O/o/out is NULL");
  if (D < 1) return fail(TPLA_ERR_SHAPE, "D=%d", D);
  // every check of the projection before the first launch: the partial results of the decode and the
  // partial tiles of the projection use the workspace one after the other
  const size_t need = output_projection_scratch_floats(*shape, D, out_dtype) * sizeof(float);
  if (workspace_bytes < need)
    return fail(TPLA_ERR_WORKSPACE, "workspace has %zu bytes, the projection needs %zu", workspace_bytes, need);
  if (!aligned16(W_O) || !aligned16(out)) return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  if ((long long)shape->H * shape->d_v > 2147483647LL || (long long)shape->B * D > 2147483647LL ||
      (D + 255) / 256 > 2147483647 / 2 || shape->B > 65535)
    return fail(TPLA_ERR_UNSUPPORTED, "H*d_v, B*D or the grid too large");
  rc = decode_common(shape, shape->g, q_lat, q_pe, shard_pools, block_table, max_pages_per_seq, seq_lens,
                     n_splits, workspace, workspace_bytes, o_lat, lse, stream, W_UV_t, o, TPLA_F32);
  if (rc) return rc;
  return output_projection_common(shape, o, W_O, D, workspace, workspace_bytes, out, out_dtype, stream);
}

size_t tpla_prefill_workspace_bytes(const tpla_shape_t* shape, int64_t T) {
  if (check_shape(shape) != TPLA_OK || T < 1) return 0;
  return (size_t)T * shape->H * (shape->d_n + shape->d_v) * 2;
}

int tpla_prefill_attention(const tpla_shape_t* shape, const void* q_nope, const void* q_pe, const void* c,
                           const void* k_pe, const void* W_UK, const void* W_UV, const int32_t* cu_seqlens,
                           int64_t T, int32_t max_seq_len, void* workspace, size_t workspace_bytes, float* o,
                           void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q_nope || !q_pe || !c || !k_pe || !W_UK || !W_UV || !cu_seqlens || !o)
    return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (T < 1 || max_seq_len < 1) return fail(TPLA_ERR_SHAPE, "T=%lld max_seq_len=%d", (long long)T, max_seq_len);
  if (!prefill_mfma_supported(*shape))
    return fail(TPLA_ERR_UNSUPPORTED, "prefill needs bf16, d_n = d_v = 128, d_r = 64, d_c a multiple of 128 up to 512");
  if (T * shape->H >= ((int64_t)1 << 31) / 2 || shape->B > 65535 || shape->H > 65535)
    return fail(TPLA_ERR_UNSUPPORTED, "T*H, B or H too large for this kernel");
  if (!aligned16(q_nope) || !aligned16(q_pe) || !aligned16(c) || !aligned16(k_pe) || !aligned16(W_UK) ||
      !aligned16(W_UV) || !aligned16(workspace) || !aligned16(o))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  const size_t need = tpla_prefill_workspace_bytes(shape, T);
  if (!workspace || workspace_bytes < need)
    return fail(TPLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  return launch_prefill_attention(*shape, q_nope, q_pe, c, k_pe, W_UK, W_UV, cu_seqlens, (int)T, max_seq_len,
                                  workspace, o, (hipStream_t)stream);
}

size_t tpla_latent_moments_workspace_bytes(const tpla_shape_t* shape, int64_t n_pages) {
  if (check_shape(shape) != TPLA_OK || n_pages < 1) return 0;
  return latent_moments_workspace(*shape, n_pages);
}

int tpla_latent_moments(const tpla_shape_t* shape, const void* mla_pool, const int32_t* page_ids,
                        const int32_t* page_fill, int64_t n_pages, void* workspace, size_t workspace_bytes,
                        double* sum, double* gram, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!mla_pool || !sum || !gram) return fail(TPLA_ERR_NULL, "a tensor pointer is NULL");
  if (n_pages < 1) return fail(TPLA_ERR_SHAPE, "n_pages=%lld", (long long)n_pages);
  if (n_pages * shape->page_tokens >= ((int64_t)1 << 31)) return fail(TPLA_ERR_UNSUPPORTED, "more than 2^31-1 rows");
  if (!aligned16(mla_pool) || !aligned16(workspace) || !aligned16(sum) || !aligned16(gram))
    return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  const size_t need = latent_moments_workspace(*shape, n_pages);
  if (!workspace || workspace_bytes < need)
    return fail(TPLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace ? workspace_bytes : (size_t)0, need);
  return launch_latent_moments(*shape, mla_pool, page_ids, page_fill, n_pages, static_cast<float*>(workspace), sum,
                               gram, (hipStream_t)stream);
}

int tpla_pca_basis(int32_t d_c, int32_t g, int64_t n_rows, const double* sum, const double* gram, float* U,
                   double* eig, double* frac) {
  if (!sum || !gram || !U || !eig || !frac) return fail(TPLA_ERR_NULL, "a pointer is NULL");
  if (d_c < 1 || d_c > 4096 || g < 1 || g > TPLA_MAX_G || d_c % g != 0 || n_rows < 1)
    return fail(TPLA_ERR_SHAPE, "d_c=%d g=%d n_rows=%lld", d_c, g, (long long)n_rows);
  return pca_basis_host(d_c, g, (double)n_rows, sum, gram, U, eig, frac);
}

int tpla_profile_enable(int32_t max_records) {
  if (max_records < 0 || max_records > (1 << 20)) return fail(TPLA_ERR_SHAPE, "max_records=%d", max_records);
  if (g_prof.ev) {
    for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    g_prof = ProfileState();
  }
  if (max_records == 0) return TPLA_OK;
  g_prof.ev = new hipEvent_t[2 * (size_t)max_records];
  for (int i = 0; i < 2 * max_records; ++i) {
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
      delete[] g_prof.ev;
      g_prof = ProfileState();
      return fail(TPLA_ERR_HIP, "hipEventCreate failed");
    }
  }
  g_prof.cap = max_records;
  return TPLA_OK;
}

int tpla_profile_collect(float* ms, int32_t capacity, int32_t* n_records) {
  if (!ms || !n_records) return fail(TPLA_ERR_NULL, "ms/n_records is NULL");
  if (capacity < 0) return fail(TPLA_ERR_SHAPE, "capacity=%d", capacity);
  int n = g_prof.used < capacity ? g_prof.used : capacity;
  for (int i = 0; i < n; ++i) {
    if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms[i], g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess)
      return fail(TPLA_ERR_HIP, "event %d could not be read", i);
  }
  *n_records = n;
  g_prof.used = 0;
  return TPLA_OK;
}

int tpla_stream_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink) return fail(TPLA_ERR_NULL, "buf/sink is NULL");
  if (!aligned16(buf) || !aligned16(sink)) return fail(TPLA_ERR_ALIGN, "pointers must be 16-byte aligned");
  return launch_stream_read(buf, bytes, sink, (hipStream_t)stream);
}

int tpla_validate_block_table(const tpla_shape_t* shape, const int32_t* block_table, int32_t max_pages_per_seq,
                              const int32_t* seq_lens, int64_t n_pool_pages, int forbid_shared) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!block_table || !seq_lens) return fail(TPLA_ERR_NULL, "block_table/seq_lens is NULL");
  if (max_pages_per_seq < 1 || n_pool_pages < 1)
    return fail(TPLA_ERR_SHAPE, "max_pages_per_seq=%d n_pool_pages=%lld", max_pages_per_seq, (long long)n_pool_pages);
  const int64_t cap = (int64_t)max_pages_per_seq * shape->page_tokens;
  std::vector<bool> used;
  if (forbid_shared) used.assign((size_t)n_pool_pages, false);
  for (int b = 0; b < shape->B; ++b) {
    const int64_t L = seq_lens[b];
    if (L < 0 || L > cap)
      return fail(TPLA_ERR_SHAPE, "seq_lens[%d]=%lld outside [0, %lld]", b, (long long)L, (long long)cap);
    const int64_t n = (L + shape->page_tokens - 1) / shape->page_tokens;
    for (int64_t j = 0; j < n; ++j) {
      const int64_t id = block_table[(int64_t)b * max_pages_per_seq + j];
      if (id < 0 || id >= n_pool_pages)
        return fail(TPLA_ERR_SHAPE, "block_table[%d][%lld]=%lld outside the pool of %lld pages", b, (long long)j,
                    (long long)id, (long long)n_pool_pages);
      if (forbid_shared) {
        if (used[(size_t)id])
          return fail(TPLA_ERR_SHAPE, "page %lld is used twice (again at block_table[%d][%lld])", (long long)id, b,
                      (long long)j);
        used[(size_t)id] = true;
      }
    }
  }
  return TPLA_OK;
}

#pragma GCC visibility pop
}  // extern "C"
