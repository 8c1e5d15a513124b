/*
 * libtpla -- shard-local latent-attention decode for Tensor-Parallel Latent
 * Attention (TPLA, arXiv 2508.15881) on AMD MI355X (gfx950).
 *
 * C ABI.  Conventions shared by every entry point:
 *   - Tensor arguments are DEVICE pointers owned by the caller unless the
 *     comment says "host".  The library never frees or keeps them.  All
 *     tensors are dense, row-major, innermost index last.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued on it and the call returns without synchronising.
 *   - Element type: shape->dtype selects the storage type of caches, queries
 *     and weights: TPLA_F32 (float storage, float arithmetic) or TPLA_BF16
 *     (bfloat16 storage, float accumulation).  Softmax statistics, latent
 *     outputs and final outputs are always float.
 *   - Return value: TPLA_OK (0) or a negative TPLA_ERR_* code, and
 *     tpla_last_error() (thread-local, static storage, never NULL) describes
 *     the failure.  When argument validation fails nothing has been launched;
 *     TPLA_ERR_HIP (the runtime refused a launch or a kernel attribute) can
 *     come after earlier kernels of the same call were enqueued, and the
 *     outputs are then undefined.  Argument validation only
 *     looks at the host-visible values; page ids and sequence lengths that
 *     live in device memory are trusted (seq_lens[b] <= max_pages_per_seq *
 *     page_tokens, page ids inside the pool).
 *   - Every base pointer must be 16-byte aligned (TPLA_ERR_ALIGN).
 *
 * Symbols follow the paper: d_c latent width (4 d_h), d_r RoPE width, d_n /
 * d_v per-head no-RoPE query / value width, H query heads handled by this
 * device (Sec. 4.4: h_q / (k/g)), g number of latent slices, U the
 * orthogonal reparameterisation (Sec. 4.1), mu the per-slice score factors
 * of the softmax slicing condition (Sec. 4.2).
 */
#ifndef TPLA_H_
#define TPLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TPLA_OK 0
#define TPLA_ERR_NULL (-1)        /* a required pointer is NULL                      */
#define TPLA_ERR_SHAPE (-2)       /* a dimension is non-positive or inconsistent     */
#define TPLA_ERR_ALIGN (-3)       /* a base pointer is not 16-byte aligned           */
#define TPLA_ERR_WORKSPACE (-4)   /* workspace smaller than tpla_workspace_bytes()   */
#define TPLA_ERR_DTYPE (-5)       /* shape->dtype is not TPLA_F32 / TPLA_BF16        */
#define TPLA_ERR_HIP (-6)         /* the HIP runtime refused a launch                */
#define TPLA_ERR_UNSUPPORTED (-7) /* valid request this build has no kernel for      */

#define TPLA_F32 0
#define TPLA_BF16 1

#define TPLA_U_IDENTITY 0 /* U = I                                                  */
#define TPLA_U_HADAMARD 1 /* U = diag(signs) H_{d_c} / sqrt(d_c), Sec. 4.3.1        */
#define TPLA_U_DENSE 2    /* U given as a dense matrix (e.g. PCA, Sec. 4.3.2)       */

#define TPLA_MAX_G 8 /* largest supported number of latent slices */

typedef struct tpla_shape {
  int32_t B;           /* sequences in the decode batch                              */
  int32_t H;           /* query heads handled here                                   */
  int32_t d_c;         /* full latent width                                          */
  int32_t g;           /* latent slices; slice i = columns [i d_c/g, (i+1) d_c/g)    */
  int32_t d_r;         /* RoPE key / query width (replicated on every slice)         */
  int32_t d_n;         /* per-head no-RoPE query width                               */
  int32_t d_v;         /* per-head value width                                       */
  int32_t page_tokens; /* tokens per cache page                                      */
  int32_t dtype;       /* TPLA_F32 or TPLA_BF16                                      */
  float sm_scale;      /* softmax scale, 1/sqrt(d_n + d_r) in Sec. 3.3               */
} tpla_shape_t;

/* Description of the last error on the calling thread ("" if none). */
const char* tpla_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int tpla_version(void);

/*
 * Orthogonal reparameterisation along one axis (Sec. 4.1: W_new = U^T W and
 * c_new = c U; Sec. 4.3 for the choice of U).
 * src and dst are [n_outer, d_c, n_inner] tensors of shape->dtype elements
 * (dst may equal src).  For every (o, i):
 *     inverse = 0:  dst[o, j, i] = sum_k src[o, k, i] * U[k, j]      (x U)
 *     inverse = 1:  dst[o, j, i] = sum_k src[o, k, i] * U[j, k]      (x U^T)
 * so cache rows and W_UK[h] ([.., d_c], n_inner = 1) and W_UV[h]
 * ([d_c, d_v], n_inner = d_v) all use inverse = 0.
 * mode = TPLA_U_IDENTITY: copy.  TPLA_U_HADAMARD: signs is NULL (all +1) or
 * d_c floats of +-1; d_c must be a power of two.  TPLA_U_DENSE: U is
 * [d_c, d_c] floats.  Arithmetic is float; one rounding on the way out.
 * Only shape->d_c and shape->dtype are read.
 */
int tpla_transform_latent(const tpla_shape_t* shape, int mode, int inverse,
                          const float* signs, const float* U,
                          const void* src, void* dst,
                          int64_t n_outer, int64_t n_inner, void* stream);

/*
 * Cache form of the reparameterisation (Sec. 4.1) plus the slicing of Sec. 4
 * and the replication of the RoPE key of Sec. 4.2.  Reads MLA-style pages
 * mla_pool [P, page_tokens, d_c + d_r] (row = latent then k_pe) and writes,
 * for every listed page and every slice i, shard_pools[i]
 * [P, page_tokens, d_c/g + d_r] with row = (c U)[i d_c/g : (i+1) d_c/g] then
 * k_pe, at the same page id.  shard_pools is a HOST array of g device
 * pointers.  page_ids: n_pages int32 page ids on the device, or NULL for
 * pages 0..n_pages-1.  Every slot of a listed page is processed.
 */
int tpla_transform_latent_paged(const tpla_shape_t* shape, int mode,
                                const float* signs, const float* U,
                                const void* mla_pool, void* const* shard_pools,
                                const int32_t* page_ids, int64_t n_pages, void* stream);

/*
 * MLA-style cache write (Sec. 3.3; norm weight absorbed as in Sec. 4.1):
 * for token t < T, pool row slot_mapping[t] (= page * page_tokens + offset)
 * of mla_pool [P, page_tokens, d_c + d_r] becomes
 *     [ c_raw[t] / sqrt(mean(c_raw[t]^2) + rms_eps)  ||  k_pe[t] ].
 * rms_eps < 0 stores c_raw unnormalised.  c_raw [T, d_c], k_pe [T, d_r] in
 * shape->dtype; slot_mapping int32 [T]; a negative slot skips the token.
 */
int tpla_write_mla_cache(const tpla_shape_t* shape, const void* c_raw, const void* k_pe,
                         const int32_t* slot_mapping, int64_t T, float rms_eps,
                         void* mla_pool, void* stream);

/*
 * Decode-token cache append with the RMSNorm taken per slice (Sec. 4.1,
 * RMSNorm slicing condition; alpha = 2 for a Hadamard basis and g = 2,
 * Sec. 4.3.1): device i only holds slice x_i = c_t[b, i d_c/g : (i+1) d_c/g]
 * of the new token's latent (U basis) and replaces the global mean square by
 * alpha[i] * |x_i|^2 / d_c:
 *     row slots[b] of shard_pools[i] = [ x_i / sqrt(alpha[i] |x_i|^2 / d_c + rms_eps)  ||  k_pe[b] ]
 * c_t [B, d_c], k_pe [B, d_r] in shape->dtype; alpha: HOST array of g floats
 * or NULL for all equal to g (balanced slices); slots int32 [B], row index
 * page * page_tokens + offset, negative = skip; shard_pools: HOST array of g
 * device pointers, each [P, page_tokens, d_c/g + d_r].
 */
int tpla_append_token_sliced(const tpla_shape_t* shape, const void* c_t, const void* k_pe,
                             const float* alpha, float rms_eps, const int32_t* slots,
                             void* const* shard_pools, void* stream);

/*
 * Absorbed query (Sec. 3.3) cut into slices (Sec. 4) with the factor of the
 * softmax slicing condition folded in (Sec. 4.2):
 *     q_lat[i, b, h, :] = mu[i] * (q_nope[b, h, :] @ W_UK_t[h])[i d_c/g : (i+1) d_c/g]
 * q_nope [B, H, d_n], W_UK_t [H, d_n, d_c] (already in the U basis),
 * q_lat [g, B, H, d_c/g], all shape->dtype.  mu: HOST array of g floats or
 * NULL for all ones.
 */
int tpla_absorb_query(const tpla_shape_t* shape, const void* q_nope, const void* W_UK_t,
                      const float* mu, void* q_lat, void* stream);

/*
 * Bytes of scratch tpla_decode_shard needs for the given split count
 * (n_splits = 0 asks for the count the library would choose by itself).
 * Returns 0 on invalid arguments.
 */
size_t tpla_workspace_bytes(const tpla_shape_t* shape, int32_t max_pages_per_seq, int32_t n_splits);

/*
 * One device's attention over its latent slice (Sec. 4, per-device softmax
 * equation; RoPE key replicated, Sec. 4.2).  For every sequence b and head h,
 * with row_t = pool row of token t of sequence b (latent slice, then k_pe):
 *     s_t      = sm_scale * (q_lat_i[b,h] . row_t[:d_c/g] + q_pe[b,h] . row_t[d_c/g:])
 *     p        = softmax over t in [0, seq_lens[b])
 *     o_lat_i[b,h,:] = sum_t p_t * row_t[:d_c/g]        lse_i[b,h] = log sum_t exp(s_t)
 * Token t of sequence b lives in page block_table[b, t / page_tokens], slot
 * t % page_tokens of shard_pool [P, page_tokens, d_c/g + d_r].  Slots at or
 * beyond seq_lens[b] are never read.  seq_lens[b] = 0 gives o = 0, lse = -inf.
 * The sequence axis is processed in n_splits independent chunks per sequence
 * (0 = library's choice) whose partial results go through `workspace` and are
 * merged in a fixed order: for fixed arguments the result is bit-reproducible.
 * q_lat_i [B,H,d_c/g], q_pe [B,H,d_r] in shape->dtype; block_table int32
 * [B, max_pages_per_seq]; seq_lens int32 [B]; o_lat_i float [B,H,d_c/g];
 * lse_i float [B,H] or NULL.
 * A length below 0 or beyond max_pages_per_seq * page_tokens is clipped to that range by the kernels
 * (the result is then that of the clipped length; the block table is never read past its row).
 */
int tpla_decode_shard(const tpla_shape_t* shape,
                      const void* q_lat_i, const void* q_pe, const void* shard_pool,
                      const int32_t* block_table, int32_t max_pages_per_seq,
                      const int32_t* seq_lens, int32_t n_splits,
                      void* workspace, size_t workspace_bytes,
                      float* o_lat_i, float* lse_i, void* stream);

/*
 * All g slices in one launch: the same computation as g calls of
 * tpla_decode_shard (slice i: q_lat[i], shard_pools[i] -> o_lat[i], lse[i];
 * q_pe, block_table and seq_lens are shared, Sec. 4.2), which is how one GPU
 * stands in for the g devices of Sec. 4 -- the chunks of all slices fill the
 * chip together, so each can be longer and fewer partial results are
 * written.  q_lat [g,B,H,d_c/g]; shard_pools: HOST array of g device
 * pointers; o_lat float [g,B,H,d_c/g]; lse float [g,B,H] or NULL; workspace
 * of tpla_workspace_bytes_all() bytes.  Results are bit-reproducible for
 * fixed arguments; they may differ from tpla_decode_shard's in the last bits
 * because the automatic split count differs.
 */
size_t tpla_workspace_bytes_all(const tpla_shape_t* shape, int32_t max_pages_per_seq, int32_t n_splits);
int tpla_decode_shards(const tpla_shape_t* shape,
                       const void* q_lat, const void* q_pe, const void* const* shard_pools,
                       const int32_t* block_table, int32_t max_pages_per_seq,
                       const int32_t* seq_lens, int32_t n_splits,
                       void* workspace, size_t workspace_bytes,
                       float* o_lat, float* lse, void* stream);

/*
 * Value up-projection of every slice and the sum over slices that the
 * all-reduce of Sec. 4 performs (W_UV kept separate from W_O, Sec. 3.3):
 *     o[b, h, :] = sum_i o_lat[i, b, h, :] @ W_UV_t[h, i d_c/g : (i+1) d_c/g, :]
 * o_lat float [g, B, H, d_c/g]; W_UV_t [H, d_c, d_v] in shape->dtype (U
 * basis); o float [B, H, d_v].
 */
int tpla_combine_shards(const tpla_shape_t* shape, const float* o_lat, const void* W_UV_t,
                        float* o, void* stream);
/* The same with the output type chosen by the caller: o is float (o_dtype = TPLA_F32) or bfloat16
 * (TPLA_BF16, one rounding to nearest even of the float result) [B, H, d_v]. */
int tpla_combine_shards_to(const tpla_shape_t* shape, const float* o_lat, const void* W_UV_t,
                           void* o, int32_t o_dtype, void* stream);

/*
 * tpla_decode_shards followed by tpla_combine_shards as one call (the
 * per-slice attention, the value up-projection and the sum over slices of
 * Sec. 4, Eq. for O_i and the all-reduce after W^{VO}_i with W_UV kept out of
 * W_O, Sec. 3.3): the merge of the sequence chunks and the combine run as one
 * kernel where the shape allows (bf16, d_v a multiple of 128, d_c of 512,
 * d_c/g of 128), as two otherwise.  Arguments as in those two calls; o_lat
 * float [g,B,H,d_c/g] is required and written (the merged per-slice outputs),
 * lse float [g,B,H] or NULL, o float [B,H,d_v].  Same workspace size as
 * tpla_decode_shards.  Results are bit-reproducible for fixed arguments and
 * agree with the two separate calls up to the rounding order of the merge.
 */
int tpla_decode_shards_combine(const tpla_shape_t* shape,
                               const void* q_lat, const void* q_pe, const void* const* shard_pools,
                               const int32_t* block_table, int32_t max_pages_per_seq,
                               const int32_t* seq_lens, int32_t n_splits,
                               void* workspace, size_t workspace_bytes,
                               const void* W_UV_t, float* o,
                               float* o_lat, float* lse, void* stream);

/* tpla_decode_shards_combine with o written as float (o_dtype = TPLA_F32) or bfloat16 (TPLA_BF16). */
int tpla_decode_shards_combine_to(const tpla_shape_t* shape,
                                  const void* q_lat, const void* q_pe, const void* const* shard_pools,
                                  const int32_t* block_table, int32_t max_pages_per_seq,
                                  const int32_t* seq_lens, int32_t n_splits,
                                  void* workspace, size_t workspace_bytes,
                                  const void* W_UV_t, void* o, int32_t o_dtype,
                                  float* o_lat, float* lse, void* stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): tpla_decode_shards_combine with the partial results of the
 * sequence chunks kept in a device array built into the library instead of a
 * caller's workspace.  Same arguments otherwise, same kernels, same plan, hence
 * the same bits as tpla_decode_shards_combine.  The call allocates and frees
 * nothing.  The array is TPLA_STATIC_SCRATCH_BYTES large on every GPU the
 * library runs on and stays until the process ends; a call that would need
 * more (tpla_workspace_bytes_all() tells) returns TPLA_ERR_WORKSPACE and
 * launches nothing.  All calls on one GPU share that GPU's array: calls that
 * overlap there (two streams, two threads) race; calls on one stream do not.
 * Nothing in the array has to be cleared between calls: every partial result a
 * call reads, it has written before.
 */
#define TPLA_STATIC_SCRATCH_BYTES (64u << 20)
int tpla_decode_shards_combine_static(const tpla_shape_t* shape,
                                      const void* q_lat, const void* q_pe, const void* const* shard_pools,
                                      const int32_t* block_table, int32_t max_pages_per_seq,
                                      const int32_t* seq_lens, int32_t n_splits,
                                      const void* W_UV_t, float* o,
                                      float* o_lat, float* lse, void* stream);

/*
 * Output projection of the attention block (Sec. 3.3: O~ = O W^O with the
 * value up-projection kept out of W^O; Sec. 4: the quantity the devices
 * all-reduce): out[b, :] = o[b, :, :] flattened to H d_v  @  W_O.
 * o float [B, H, d_v] (the result of tpla_combine_shards); W_O [H d_v, D] in
 * shape->dtype, row-major; out float [B, D].  workspace: scratch of
 * tpla_output_projection_workspace_bytes() bytes (may be 0 -> NULL allowed).
 * The k axis is split over workgroups and summed in a fixed order.
 */
size_t tpla_output_projection_workspace_bytes(const tpla_shape_t* shape, int32_t D);
int tpla_output_projection(const tpla_shape_t* shape, const float* o, const void* W_O, int32_t D,
                           void* workspace, size_t workspace_bytes, float* out, void* stream);
/* The same with out [B, D] written as float (out_dtype = TPLA_F32) or bfloat16 (TPLA_BF16). */
int tpla_output_projection_to(const tpla_shape_t* shape, const float* o, const void* W_O, int32_t D,
                              void* workspace, size_t workspace_bytes, void* out, int32_t out_dtype, void* stream);

/*
 * The attention block's output from the cache in one call (Sec. 4: O~_i = O_i W^{VO}_i summed over
 * the devices, with W^{VO} kept as its two factors W_UV and W_O, Sec. 3.3): tpla_decode_shards_combine
 * followed by tpla_output_projection_to,
 *     out[b, :] = ( sum_i o_lat[i, b, :, :] @ W_UV_t[:, slice i, :] ) flattened to H d_v  @  W_O.
 * Arguments as in those calls.  o float [B, H, d_v], o_lat float [g, B, H, d_c/g] are required and
 * written (the intermediate results); lse float [g, B, H] or NULL; out [B, D] in out_dtype.  One
 * workspace of tpla_attention_block_workspace_bytes() bytes serves the decode's partial results and then
 * the projection's partial tiles.  Every argument check of both stages runs before the first launch.
 * Bit-reproducible for fixed arguments; the same bits as the two calls made one after the other.
 */
size_t tpla_attention_block_workspace_bytes(const tpla_shape_t* shape, int32_t max_pages_per_seq,
                                            int32_t n_splits, int32_t D);
int tpla_decode_shards_project(const tpla_shape_t* shape,
                               const void* q_lat, const void* q_pe, const void* const* shard_pools,
                               const int32_t* block_table, int32_t max_pages_per_seq,
                               const int32_t* seq_lens, int32_t n_splits,
                               void* workspace, size_t workspace_bytes,
                               const void* W_UV_t, const void* W_O, int32_t D,
                               void* out, int32_t out_dtype,
                               float* o, float* o_lat, float* lse, void* stream);

/*
 * Prefill attention with MLA in its un-absorbed form (Sec. 4.5: the prefill
 * phase keeps MLA, heads split over devices; Sec. 3.3: per-head keys
 * k = W_UK[h] c and values v = c W_UV[h], the RoPE key shared by all heads).
 * The T tokens of shape->B sequences are packed; cu_seqlens int32 [B + 1]
 * (device, cu_seqlens[0] = 0, non-decreasing, cu_seqlens[B] = T) gives their
 * row ranges; token t attends to the tokens of its own sequence up to and
 * including itself.  q_nope [T, H, d_n], q_pe [T, H, d_r], c [T, d_c] (the
 * normalised latent, as cached), k_pe [T, d_r], W_UK [H, d_n, d_c],
 * W_UV [H, d_c, d_v] in shape->dtype (original basis: no U); o float
 * [T, H, d_v].  max_seq_len: an upper bound of the longest sequence (queries
 * beyond it are not computed).  Row ranges are clipped to [0, T) by the kernel.  workspace:
 * tpla_prefill_workspace_bytes() bytes (the projected keys and values, bf16).
 * shape->g, page_tokens are not used.  Implemented for bf16 with d_n = d_v =
 * 128, d_r = 64, d_c a multiple of 128 up to 512 (TPLA_ERR_UNSUPPORTED
 * otherwise).  The latent rows are what tpla_write_mla_cache stores.
 */
size_t tpla_prefill_workspace_bytes(const tpla_shape_t* shape, int64_t T);
int tpla_prefill_attention(const tpla_shape_t* shape, const void* q_nope, const void* q_pe, const void* c,
                           const void* k_pe, const void* W_UK, const void* W_UV, const int32_t* cu_seqlens,
                           int64_t T, int32_t max_seq_len, void* workspace, size_t workspace_bytes, float* o,
                           void* stream);

/*
 * PCA calibration, step 1 (Sec. 4.3.2: the covariance of collected latents,
 * position features excluded): second moments of the latent part of cached
 * rows.  mla_pool as in tpla_transform_latent_paged; page_ids int32 [n_pages]
 * (NULL = pages 0..n_pages-1); page_fill int32 [n_pages], the number of valid
 * tokens at the start of each listed page (NULL = every page full; the rest of
 * a page is never read, so it may hold anything).  Writes, as DEVICE doubles,
 * sum[d_c] = sum_r x_r and gram[d_c * d_c] = sum_r x_r^T x_r (row-major,
 * symmetric, both triangles).  Products accumulate in float inside a split of
 * at most 16384 rows, splits are added in double in a fixed order.
 * workspace: tpla_latent_moments_workspace_bytes() bytes of device scratch.
 * n_pages * page_tokens must be below 2^31.
 */
size_t tpla_latent_moments_workspace_bytes(const tpla_shape_t* shape, int64_t n_pages);
int tpla_latent_moments(const tpla_shape_t* shape, const void* mla_pool, const int32_t* page_ids,
                        const int32_t* page_fill, int64_t n_pages, void* workspace, size_t workspace_bytes,
                        double* sum, double* gram, void* stream);

/*
 * PCA calibration, step 2 (Sec. 4.3.2), on the HOST and synchronous: all
 * pointers are host memory.  From the moments of n_rows latents forms the
 * covariance gram/n - mean mean^T, diagonalises it (Householder tridiagonal form,
 * then implicit QR steps, in double) and writes U float [d_c, d_c] row-major whose COLUMN k is the
 * eigenvector of the k-th largest eigenvalue (sign: its largest component is
 * positive) -- the dense U of tpla_transform_latent --, eig double [d_c]
 * descending, and frac double [g]: the share of the total variance in each
 * contiguous slice of d_c/g components (alpha, beta of Sec. 4.3.2 for g = 2).
 * d_c must be a multiple of g.  Returns TPLA_ERR_UNSUPPORTED if the iteration
 * does not converge.
 */
int tpla_pca_basis(int32_t d_c, int32_t g, int64_t n_rows, const double* sum, const double* gram, float* U,
                   double* eig, double* frac);

/*
 * Measurement aid for the split kernel of tpla_decode_shard (the pass over
 * the cache of Sec. 4.5's memory-bound decode).  After
 * tpla_profile_enable(n) with n > 0, each decode call (tpla_decode_shard,
 * tpla_decode_shards, tpla_decode_shards_combine) on this thread times that
 * kernel -- not the merge that follows it -- with a pair of HIP events on the
 * call's stream, for at most n calls: the matrix-core kernel is launched with
 * the events attached to its dispatch, so they hold its own begin and end
 * times; the generic kernel is bracketed by two recorded events.
 * tpla_profile_collect waits for the recorded events, writes the elapsed
 * milliseconds of each bracketed kernel to the HOST array ms (capacity
 * entries), stores the count in *n_records and starts over.
 * tpla_profile_enable(0) switches the recording off and frees the events.
 */
int tpla_profile_enable(int32_t max_records);
int tpla_profile_collect(float* ms, int32_t capacity, int32_t* n_records);

/*
 * Measurement aid for the memory-bound decode of Sec. 4.5: reads the first
 * bytes - bytes % 20480 bytes of the DEVICE buffer buf once, with 128-bit
 * streaming loads and nothing else, so that a caller can time what the box
 * delivers to a pure reader and set the decode kernel's rate against it.
 * sink: 4 writable device bytes (never written in practice).
 */
int tpla_stream_read(const void* buf, size_t bytes, void* sink, void* stream);

/*
 * Host-side check of the paging inputs of the decode calls, for callers that
 * want one before a launch (the kernels trust the page ids: an id outside the
 * pool is an access outside the pool).  HOST pointers: block_table int32
 * [B, max_pages_per_seq], seq_lens int32 [B].  Checks 0 <= seq_lens[b] <=
 * max_pages_per_seq * page_tokens, that the ids of the pages a sequence uses
 * (the first ceil(seq_lens[b] / page_tokens) of its row) lie in
 * [0, n_pool_pages), and that no page is used twice (by two sequences or
 * twice by one): a shared page is legal for reading, so this last check only
 * runs with forbid_shared != 0.  Returns TPLA_OK or TPLA_ERR_SHAPE with the
 * first offending entry named by tpla_last_error().  Synchronous, no GPU work.
 */
int tpla_validate_block_table(const tpla_shape_t* shape, const int32_t* block_table,
                              int32_t max_pages_per_seq, const int32_t* seq_lens,
                              int64_t n_pool_pages, int forbid_shared);

#ifdef __cplusplus
}
#endif
#endif /* TPLA_H_ */
