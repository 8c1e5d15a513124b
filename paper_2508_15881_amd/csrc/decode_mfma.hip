// bf16 shard decode on the matrix cores (gfx950).
//
// One workgroup = one (sequence, split).  It walks its pages in tiles of TOK
// tokens.  A tile (TOK rows of d_c/g + d_r bf16, contiguous inside a page)
// is fetched with 128-bit loads into registers one tile ahead, then written
// to LDS, where all heads share it.  Wave w owns heads [16w, 16w+16):
//   S^T[tok, head] = K[tok, :] . Q[head, :]      MFMA 16x16x32, M = tokens, N = heads
//   online softmax per head (one head per lane column, 16-lane DPP-free
//   layout: a lane only ever sees its own head)
//   O^T[dim, head] += V^T[dim, tok] . P^T[tok, head]   M = latent dims, N = heads
// The latent prefix of a row is both key and value, so the same LDS tile is
// read row-wise for the scores and through the transposing LDS read for the
// output.  The S^T accumulator layout is already the B-operand layout of the
// second product once the token order inside a 32-token step is permuted
// identically for V^T, so P never leaves registers.
#include "tpla_internal.h"

namespace tpla {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define TPLA_LDS(p) ((__attribute__((address_space(3))) s16x4*)(p))

constexpr int PAGE_TOKENS = 64;
constexpr float LAZY = 8.0f;   // log2 units: the softmax reference lags the running maximum by at most this

// 16-byte pieces of a tile are stored at a swizzled position so that both
// the row-wise reads (16 tokens x 16 B at one column) and the transposing
// reads (16 tokens x 32 B at one column) spread over all LDS banks: piece c
// of token `tok` lives at piece index tok * RC + (c ^ ((tok >> 1) & 7)).
__device__ __forceinline__ int swz(int tok, int c, int RC) { return tok * RC + (c ^ ((tok >> 1) & 7)); }

template <int DL, int DR, int NW, int TOK>
__global__ void __launch_bounds__(NW * 64) decode_mfma_kernel(DecodeArgs a) {
  constexpr int RC = (DL + DR) / 8;      // 16-byte pieces per row
  constexpr int KS = (DL + DR) / 32;     // k-steps of the score product
  constexpr int DB = DL / 16;            // 16-wide blocks of latent dims
  constexpr int TB = TOK / 16;           // 16-token blocks per tile
  constexpr int S2 = TOK / 32;           // 32-token k-steps of the output product
  constexpr int NT = NW * 64;
  constexpr int TC = TOK * RC;           // pieces per tile
  constexpr int CPT = (TC + NT - 1) / NT;
  constexpr int TPP = PAGE_TOKENS / TOK; // tiles per page
  static_assert(RC % 8 == 0, "row must be a multiple of 64 elements");
  static_assert(TOK % 32 == 0 && PAGE_TOKENS % TOK == 0, "tile size");

  extern __shared__ u32x4 smem[];        // 2 tiles

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j16 = lane & 15, q4 = lane >> 4;
  const int b = blockIdx.x / a.n_splits, s = blockIdx.x % a.n_splits;
  const int L = a.seq_lens[b];
  const int n_pages = (L + PAGE_TOKENS - 1) / PAGE_TOKENS;
  const int p0 = s * a.pages_per_split;
  if (p0 >= n_pages) return;
  int p1 = p0 + a.pages_per_split;
  if (p1 > n_pages) p1 = n_pages;
  const int t_begin = p0 * PAGE_TOKENS;
  const int t_end = min(p1 * PAGE_TOKENS, L);
  const int ntiles = (t_end - t_begin + TOK - 1) / TOK;
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  const u32x4* pool = static_cast<const u32x4*>(a.pool);

  // ---- staging bookkeeping: piece x = tid + j*NT of a tile -----------------
  int st_tok[CPT], st_slot[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int x = tid + j * NT;
    const int tok = x / RC, c = x % RC;
    st_tok[j] = (x < TC) ? tok : TOK;    // TOK = never valid
    st_slot[j] = swz(tok, c, RC);
  }
  u32x4 pre[CPT];
  auto fetch = [&](int t) {
    const int T = p0 * TPP + t;
    const int page = bt[T / TPP];
    const u32x4* src = pool + (size_t)page * (PAGE_TOKENS * RC) + (size_t)(T % TPP) * TC + tid;
    const int valid = t_end - (t_begin + t * TOK);   // rows >= valid are not read
    if (valid >= TOK) {
#pragma unroll
      for (int j = 0; j < CPT; ++j)
        if ((j + 1) * NT <= TC || st_tok[j] < TOK) pre[j] = __builtin_nontemporal_load(src + j * NT);
    } else {
#pragma unroll
      for (int j = 0; j < CPT; ++j) {
        if (st_tok[j] < valid)
          pre[j] = __builtin_nontemporal_load(src + j * NT);
        else
          pre[j] = u32x4{0u, 0u, 0u, 0u};
      }
    }
  };

  // ---- this wave's 16 heads of the query, as B operands --------------------
  const int head = wave * 16 + j16;
  bf16x8 qreg[KS];
  {
    const bf16_t* ql = static_cast<const bf16_t*>(a.q_lat) + ((size_t)b * a.H + head) * DL;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q_pe) + ((size_t)b * a.H + head) * DR;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 32 + q4 * 8;
      qreg[ks] = (k0 < DL) ? *reinterpret_cast<const bf16x8*>(ql + k0)
                           : *reinterpret_cast<const bf16x8*>(qp + (k0 - DL));
    }
  }

  // ---- per-lane LDS byte offsets -------------------------------------------
  // score product: token 16*tb + j16, piece 4*ks + q4
  const int xk = (j16 >> 1) & 7;
  int k_off[2];
  k_off[0] = (j16 * RC + ((q4) ^ xk)) * 16;
  k_off[1] = (j16 * RC + ((4 | q4) ^ xk)) * 16;
  // output product: token 4*q4 + (j16>>2) (+16), dims 16*db + 4*(j16&3) .. +4
  const int v_tok = 4 * q4 + (j16 >> 2);
  const int xv = (v_tok >> 1) & 7;
  const int cb = (j16 & 3) >> 1;
  int v_off[4];
#pragma unroll
  for (int d = 0; d < 4; ++d) v_off[d] = (v_tok * RC + (((d << 1) | cb) ^ xv)) * 16 + (j16 & 1) * 8;

  f32x4 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  fetch(0);
  for (int t = 0; t < ntiles; ++t) {
    u32x4* buf = smem + (t & 1) * TC;
#pragma unroll
    for (int j = 0; j < CPT; ++j)
      if (st_tok[j] < TOK) buf[st_slot[j]] = pre[j];
    if (t + 1 < ntiles) fetch(t + 1);
    __syncthreads();
    const char* tile = reinterpret_cast<const char*>(buf);

    // ---- scores ------------------------------------------------------------
    f32x4 sacc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) sacc[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
            tile + k_off[ks & 1] + (ks >> 1) * 128 + tb * (16 * RC * 16));
        sacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qreg[ks], sacc[tb], 0, 0, 0);
      }
    }

    // ---- online softmax (lane = one head; tokens 16*tb + 4*q4 + i) ----------
    // The reference m_run of the exponentials is only moved when some score
    // exceeds it by more than LAZY (weights stay <= 2^LAZY, harmless in
    // float), so the accumulator rescale is off the common path.
    const int valid = t_end - (t_begin + t * TOK);
    if (valid < TOK) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (16 * tb + 4 * q4 + i >= valid) sacc[tb][i] = -INFINITY;
    }
    float mx = sacc[0][0];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = fmaxf(mx, sacc[tb][i]);
    mx *= a.scale_log2;
    if (__any(mx > m_run + LAZY)) {
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int d = 0; d < DB; ++d) acc[d] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[tb][i], a.scale_log2, -m_run));
        sacc[tb][i] = p;
        psum += p;
      }
    l_run += psum;

    // ---- output: O^T += V^T P^T ----------------------------------------------
#pragma unroll
    for (int s2 = 0; s2 < S2; ++s2) {
      bf16x8 pb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pb[i] = (bf16_t)sacc[2 * s2][i];
        pb[4 + i] = (bf16_t)sacc[2 * s2 + 1][i];
      }
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        const char* pa = tile + v_off[d & 3] + (d >> 2) * 128 + s2 * (32 * RC * 16);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TPLA_LDS(pa));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TPLA_LDS(pa + 16 * RC * 16));
        const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v8), pb, acc[d], 0, 0, 0);
      }
    }
    // the next iteration writes the other buffer; the barrier at its top
    // orders these reads before the write after that one
  }

  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  const size_t item = ((size_t)b * a.n_splits + s) * a.H + head;
  float* pacc = a.part_acc + item * DL + 4 * q4;
#pragma unroll
  for (int d = 0; d < DB; ++d) *reinterpret_cast<f32x4*>(pacc + 16 * d) = acc[d];
  if (q4 == 0) {
    a.part_ml[item * 2 + 0] = m_run;
    a.part_ml[item * 2 + 1] = l_tot;
  }
}

bool decode_mfma_supported(const tpla_shape_t& sh) {
  if (sh.dtype != TPLA_BF16 || sh.page_tokens != PAGE_TOKENS || sh.d_r != 64) return false;
  const int dl = sh.d_c / sh.g;
  if (dl != 128 && dl != 256 && dl != 512) return false;
  return sh.H == 16 || sh.H == 32 || sh.H == 64 || sh.H == 128;
}

// Kernel entry, its LDS size and how many of its workgroups fit on one
// compute unit (0 when the runtime cannot tell, e.g. without a device).
struct KernelInfo {
  void (*fn)(DecodeArgs) = nullptr;
  size_t smem = 0;
  int threads = 0;
  int blocks_per_cu = 0;
  bool ready = false;
};

template <int DL, int NW>
static int kernel_info(KernelInfo** out) {
  constexpr int TOK = 32;
  static KernelInfo info;
  if (!info.ready) {
    info.fn = decode_mfma_kernel<DL, 64, NW, TOK>;
    info.smem = 2u * TOK * ((DL + 64) / 8) * 16;
    info.threads = NW * 64;
    // dynamic LDS above the 64 KiB default needs opting in
    if (info.smem > 64 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(info.fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)info.smem) != hipSuccess) {
      (void)hipGetLastError();
      return fail(TPLA_ERR_HIP, "cannot raise the dynamic LDS limit to %zu", info.smem);
    }
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(info.fn), info.threads,
                                                     info.smem) != hipSuccess) {
      (void)hipGetLastError();
      n = 0;
    }
    info.blocks_per_cu = n;
    info.ready = true;
  }
  *out = &info;
  return TPLA_OK;
}

template <int DL>
static int kernel_info_dl(int H, KernelInfo** out) {
  switch (H) {
    case 16: return kernel_info<DL, 1>(out);
    case 32: return kernel_info<DL, 2>(out);
    case 64: return kernel_info<DL, 4>(out);
    case 128: return kernel_info<DL, 8>(out);
  }
  return fail(TPLA_ERR_UNSUPPORTED, "H=%d", H);
}

static int kernel_info_for(int dl, int H, KernelInfo** out) {
  switch (dl) {
    case 128: return kernel_info_dl<128>(H, out);
    case 256: return kernel_info_dl<256>(H, out);
    case 512: return kernel_info_dl<512>(H, out);
  }
  return fail(TPLA_ERR_UNSUPPORTED, "d_c/g=%d", dl);
}

int decode_mfma_blocks_per_cu(const tpla_shape_t& sh) {
  KernelInfo* k = nullptr;
  if (kernel_info_for(sh.d_c / sh.g, sh.H, &k) != TPLA_OK) return 0;
  return k->blocks_per_cu;
}

int launch_decode_mfma(const DecodeArgs& a, hipStream_t st) {
  KernelInfo* k = nullptr;
  const int rc = kernel_info_for(a.dl, a.H, &k);
  if (rc) return rc;
  hipLaunchKernelGGL(k->fn, dim3((unsigned)(a.B * a.n_splits)), dim3(k->threads), k->smem, st, a);
  return check_launch("decode_mfma_kernel");
}

}  // namespace tpla
