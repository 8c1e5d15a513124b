// Matrix-core versions of the two per-head contractions around the decode
// (bf16 weights): absorb  q_lat = mu * (q_nope @ W_UK')   (Sec. 3.3 / 4 / 4.2)
//                 combine o = sum_i o_lat_i @ W_UV'[slice i]   (Sec. 4)
// Both are X[b, k] @ W[k, j] per head with W row-major (j contiguous), while
// the MFMA B operand wants 8 consecutive k per lane: the weight slab goes
// through LDS and comes back through the transposing read, which hands lane j
// the 4 rows of column j.  The float o_lat is split into bf16 hi + lo parts
// (two MFMAs) so the combine keeps float accuracy.
#include "lds_tile.h"

namespace tpla {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define TPLA_LDS4(p) ((__attribute__((address_space(3))) s16x4*)(p))

// LDS slab [rows][16 * PPR bytes] of 16-byte pieces; piece p of row r sits at
// p ^ wswz(r).  A transposing read touches rows {0..3, 8..11, 16..19, 24..27}
// (+4) of a 32-row step at one 32-byte column: wswz spreads those 16 rows
// over the 8 bank groups, two rows each.
__device__ __forceinline__ int wswz(int r) { return ((r & 3) | (((r >> 3) & 1) << 2)) << 1; }

// Same for 8-piece (128-byte) rows, where the row parity already selects the
// bank half: the remaining two bits come from row bits 1 and 3.
__device__ __forceinline__ int wswz8(int r) { return (((r >> 1) & 1) | (((r >> 3) & 1) << 1)) << 1; }

// B fragment (32 k-rows x 16 columns) of MFMA 16x16x32 from the slab.
// rows k0..k0+31, 16-byte piece pair (2*cb, 2*cb+1) of a PPR-piece row.
template <int PPR>
__device__ __forceinline__ bf16x8 read_b_frag(const char* slab, int k0, int cb, int j16, int q4) {
  const int r0 = k0 + 8 * q4 + (j16 >> 2);
  const int p = 2 * cb + ((j16 & 3) >> 1);
  const int byte = (j16 & 1) * 8;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      TPLA_LDS4(slab + (r0 * PPR + (p ^ wswz(r0))) * 16 + byte));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      TPLA_LDS4(slab + ((r0 + 4) * PPR + (p ^ wswz(r0 + 4))) * 16 + byte));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// ---------------------------------------------------------------------------
// absorb: grid (H, d_c / 128, Z); 4 waves, wave w owns columns 32w..32w+31 of the
// slab; LDS slab = W_UK'[h][0..d_n)[c0..c0+128).  A workgroup walks over blocks of 16
// sequences, one dependent load per block, so batches of more than 32 sequences are
// dealt over Z workgroups per (head, column block), each staging the slab for itself
// (32 KB from L2): block mb goes to z = mb mod Z.
constexpr int AQ_COLS = 128;
__global__ void __launch_bounds__(256) absorb_query_mfma_kernel(const bf16_t* __restrict__ q_nope,
                                                                const bf16_t* __restrict__ W, MuFactors mu,
                                                                bf16_t* __restrict__ q_lat, int B, int H,
                                                                int d_n, int d_c, int g) {
  extern __shared__ u32x4 slab4[];
  char* slab = reinterpret_cast<char*>(slab4);
  constexpr int PPR = AQ_COLS / 8;   // 16 pieces per row
  const int h = blockIdx.x, c0 = blockIdx.y * AQ_COLS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j16 = lane & 15, q4 = lane >> 4;
  const bf16_t* Wh = W + (size_t)h * d_n * d_c + c0;
  // the slab goes straight into LDS: instruction k fills pieces [64k, 64k + 64), the swizzle is
  // applied to the address each lane fetches from
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  for (int k = wave_s; k < d_n * PPR / 64; k += 4) {
    const int x = k * 64 + lane, r = x / PPR, p = (x % PPR) ^ wswz(r);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Wh + (size_t)r * d_c + 8 * p),
                                     (__attribute__((address_space(3))) void*)(slab + k * 1024), 16, 0, 0);
  }
  const int dl = d_c / g;
  const int KS = d_n / 32;
  constexpr int KS_MAX = 8;                    // d_n <= 256
  const int n_mb = (B + 15) / 16;
  // the first block's query rows are on their way while the slab lands
  bf16x8 av[KS_MAX];
  auto load_rows = [&](int mb) {
    const int b = 16 * mb + j16;
    const bf16_t* qrow = q_nope + ((size_t)min(b, B - 1) * H + h) * d_n + 8 * q4;
#pragma unroll
    for (int ks = 0; ks < KS_MAX; ++ks)
      if (ks < KS) av[ks] = *reinterpret_cast<const bf16x8*>(qrow + 32 * ks);
  };
  const int mb0 = blockIdx.z, mb_step = gridDim.z;
  load_rows(mb0);                              // mb0 < n_mb by the launch
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int mb = mb0; mb < n_mb; mb += mb_step) {
    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int ks = 0; ks < KS_MAX; ++ks) {
      if (ks < KS) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const bf16x8 bf = read_b_frag<PPR>(slab, 32 * ks, 2 * wave + cb, j16, q4);
          acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ks], bf, acc[cb], 0, 0, 0);
        }
      }
    }
    if (mb + mb_step < n_mb) load_rows(mb + mb_step);     // under this block's stores
    // acc[cb][i]: sequence 16 mb + 4 q4 + i, column c0 + 32 wave + 16 cb + j16
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const int col = c0 + 32 * wave + 16 * cb + j16;
      const int sl = col / dl, c = col - sl * dl;
      const float m = mu.v[sl];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int bb = 16 * mb + 4 * q4 + i;
        if (bb < B) q_lat[(((size_t)sl * B + bb) * H + h) * dl + c] = (bf16_t)(acc[cb][i] * m);
      }
    }
  }
}

bool absorb_mfma_supported(const tpla_shape_t& sh) {
  return sh.dtype == TPLA_BF16 && sh.d_n % 32 == 0 && sh.d_n <= 256 && sh.d_c % AQ_COLS == 0 &&
         (sh.d_c / sh.g) % 16 == 0 && sh.d_c / AQ_COLS <= 65535;
}

int launch_absorb_query_mfma(const tpla_shape_t& sh, const void* q_nope, const void* W_UK_t,
                             const MuFactors& mu, void* q_lat, hipStream_t st) {
  const size_t smem = (size_t)sh.d_n * AQ_COLS * 2;
  const int n_mb = (sh.B + 15) / 16;
  const int Z = n_mb <= 2 ? 1 : (n_mb + 1) / 2 < 8 ? (n_mb + 1) / 2 : 8;   // two blocks per workgroup, at most 8 deep
  hipLaunchKernelGGL(absorb_query_mfma_kernel, dim3((unsigned)sh.H, (unsigned)(sh.d_c / AQ_COLS), (unsigned)Z), dim3(256),
                     smem, st, static_cast<const bf16_t*>(q_nope), static_cast<const bf16_t*>(W_UK_t), mu,
                     static_cast<bf16_t*>(q_lat), sh.B, sh.H, sh.d_n, sh.d_c, sh.g);
  return check_launch("absorb_query_mfma_kernel");
}

// ---------------------------------------------------------------------------
// combine: grid (H, d_v / 64).  The latent axis is walked in chunks of CK_ROWS
// rows staged in LDS; inside a chunk wave w owns rows 128w..128w+127 (so every
// o_lat element is fetched and split into hi/lo by exactly one wave) and all
// 64 columns; the four waves' partial sums meet in LDS at the end.
constexpr int CB_COLS = 64;
constexpr int CK_ROWS = 512;
template <typename OT>
__global__ void __launch_bounds__(256) combine_shards_mfma_kernel(const float* __restrict__ o_lat,
                                                                  const bf16_t* __restrict__ W,
                                                                  OT* __restrict__ o, int B, int H,
                                                                  int d_c, int d_v, int g) {
  extern __shared__ u32x4 slab4[];
  char* slab = reinterpret_cast<char*>(slab4);
  constexpr int PPR = CB_COLS / 8;   // 8 pieces per row
  constexpr int WK = CK_ROWS / 4;    // rows per wave and chunk
  const int h = blockIdx.x, c0 = blockIdx.y * CB_COLS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j16 = lane & 15, q4 = lane >> 4;
  const int dl = d_c / g;
  const int n_mb = (B + 15) / 16;
  for (int mb0 = 0; mb0 < n_mb; mb0 += 2) {
    f32x4 acc[2][4];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) acc[m][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < d_c; kc += CK_ROWS) {
      // this lane's o_lat pieces of the chunk: issued before the weights are staged
      float4 xa[WK / 32][2][2];
#pragma unroll
      for (int ks = 0; ks < WK / 32; ++ks) {
        const int k = kc + WK * wave + 32 * ks + 8 * q4;
        const int sl = k / dl, c = k - sl * dl;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          const int b = min(16 * (mb0 + m) + j16, B - 1);
          const float* src = o_lat + (((size_t)sl * B + b) * H + h) * dl + c;
          xa[ks][m][0] = *reinterpret_cast<const float4*>(src);
          xa[ks][m][1] = *reinterpret_cast<const float4*>(src + 4);
        }
      }
      __syncthreads();
      const bf16_t* Wh = W + ((size_t)h * d_c + kc) * d_v + c0;
      for (int x = tid; x < CK_ROWS * PPR; x += 256) {
        const int r = x / PPR, p = x % PPR;
        slab4[r * PPR + (p ^ wswz8(r))] = *reinterpret_cast<const u32x4*>(Wh + (size_t)r * d_v + 8 * p);
      }
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < WK / 32; ++ks) {
        bf16x8 ah[2], al[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          const float xs[8] = {xa[ks][m][0].x, xa[ks][m][0].y, xa[ks][m][0].z, xa[ks][m][0].w,
                               xa[ks][m][1].x, xa[ks][m][1].y, xa[ks][m][1].z, xa[ks][m][1].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const bf16_t hi16 = (bf16_t)xs[e];
            ah[m][e] = hi16;
            al[m][e] = (bf16_t)(xs[e] - (float)hi16);
          }
        }
        const int r0 = WK * wave + 32 * ks + 8 * q4 + (j16 >> 2);
        const int byte = (j16 & 1) * 8;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
          const int p = 2 * cb + ((j16 & 3) >> 1);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              TPLA_LDS4(slab + (r0 * PPR + (p ^ wswz8(r0))) * 16 + byte));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              TPLA_LDS4(slab + ((r0 + 4) * PPR + (p ^ wswz8(r0 + 4))) * 16 + byte));
          const s16x8 v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 bf = __builtin_bit_cast(bf16x8, v8);
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            acc[m][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[m], bf, acc[m][cb], 0, 0, 0);
            acc[m][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[m], bf, acc[m][cb], 0, 0, 0);
          }
        }
      }
    }
    // sum the four waves' partial tiles through LDS; wave w finishes column block w
    __syncthreads();
    f32x4* red = reinterpret_cast<f32x4*>(slab);     // [wave][m][cb][lane]
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) red[((wave * 2 + m) * 4 + cb) * 64 + lane] = acc[m][cb];
    __syncthreads();
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      f32x4 t = red[((0 * 2 + m) * 4 + wave) * 64 + lane];
#pragma unroll
      for (int w2 = 1; w2 < 4; ++w2) t += red[((w2 * 2 + m) * 4 + wave) * 64 + lane];
      // t[i]: sequence 16 (mb0 + m) + 4 q4 + i, column c0 + 16 wave + j16
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int bb = 16 * (mb0 + m) + 4 * q4 + i;
        if (bb < B) store_from_f32(o + ((size_t)bb * H + h) * d_v + c0 + 16 * wave + j16, t[i]);
      }
    }
  }
}

bool combine_mfma_supported(const tpla_shape_t& sh) {
  return sh.dtype == TPLA_BF16 && sh.d_v % CB_COLS == 0 && sh.d_c % CK_ROWS == 0 && (sh.d_c / sh.g) % 32 == 0 &&
         sh.d_v / CB_COLS <= 65535;
}

int launch_combine_shards_mfma(const tpla_shape_t& sh, const float* o_lat, const void* W_UV_t, void* o, int o_dtype,
                               hipStream_t st) {
  const size_t smem = (size_t)CK_ROWS * CB_COLS * 2;
  const dim3 grid((unsigned)sh.H, (unsigned)(sh.d_v / CB_COLS));
  if (o_dtype == TPLA_BF16)
    hipLaunchKernelGGL(combine_shards_mfma_kernel<bf16_t>, grid, dim3(256), smem, st, o_lat,
                       static_cast<const bf16_t*>(W_UV_t), static_cast<bf16_t*>(o), sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  else
    hipLaunchKernelGGL(combine_shards_mfma_kernel<float>, grid, dim3(256), smem, st, o_lat,
                       static_cast<const bf16_t*>(W_UV_t), static_cast<float*>(o), sh.B, sh.H, sh.d_c, sh.d_v, sh.g);
  return check_launch("combine_shards_mfma_kernel");
}

// ---------------------------------------------------------------------------
// Split merge and combine in one kernel: the decode's partial results go
// straight into  o = sum_i o_lat_i @ W_UV'[slice i]  without a pass through
// memory and a launch in between.  Grid (H, ceil(B / 16), d_v / 128): a
// workgroup of 8 waves owns one head, 16 (or 8) sequences and 128 output columns.
// Its weight slab W_UV'[h][512 rows][128 columns] is fetched straight into
// LDS while the lanes merge: lane (j16, q4) of wave w owns sequence j16 and
// latent rows 64 w + 32 ks + 8 q4 .. +8 of the chunk (one slice per wave, as
// d_c / g is a multiple of 64).  The slots of its (slice, sequence) are taken
// 16 at a time: the four lanes of a sequence fetch four (reference, sum)
// pairs each, agree on the reference through two shuffles, rescale what they
// have so far (nothing, unless a sequence has more than 16 slots) and add
// their 16 columns of the 16 partial rows in slot order, eight rows in
// flight.  The merged values are written out as o_lat / lse on the way and
// then feed the MFMAs as bf16 hi + lo parts, as in the combine kernel above.
constexpr int MC_ROWS = 512;
constexpr int MC_COLS = 128;
constexpr int MC_NW = 8;
constexpr int MC_AHEAD = 8;      // partial rows in flight per lane

template <typename OT>
__global__ void __launch_bounds__(MC_NW * 64) merge_combine_mfma_kernel(DecodeArgs a, const bf16_t* __restrict__ W,
                                                                        OT* __restrict__ o, int d_c, int d_v,
                                                                        int spw) {
  extern __shared__ u32x4 slab4[];
  char* slab = reinterpret_cast<char*>(slab4);
  constexpr int PPR = MC_COLS / 8;     // 16 pieces per row
  constexpr int NCB = MC_COLS / 16;    // 8 column blocks, all owned by every wave
  constexpr int WK = MC_ROWS / MC_NW;  // 64 rows per wave and chunk
  constexpr int KS = WK / 32;
  const int h = blockIdx.x, mb = blockIdx.y, col0 = blockIdx.z * MC_COLS;
  const int tid = threadIdx.x, lane = tid & 63, j16 = lane & 15, q4 = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int B = a.B, H = a.H, dl = a.dl;
  // spw = sequences per workgroup, 16 or 8 (then rows 8..15 of the tiles stay zero: half the
  // merge work per workgroup and twice the workgroups, for batches that would not fill the chip)
  const int b = spw * mb + j16;
  const bool b_valid = j16 < spw && b < B;
  const int bc = min(b, B - 1);
  const int L = j16 < spw ? seq_len_clipped(a, bc) : 0;
  const int n_pages = (L + a.page_tokens - 1) / a.page_tokens;
  const int n_v = a.n_shards * B;

  f32x4 acc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kc = 0; kc < d_c; kc += MC_ROWS) {
    if (kc > 0) __syncthreads();       // everybody is done with the previous chunk's slab
    // ---- weight slab, straight into LDS: instruction k fills pieces [64k, 64k + 64)
    {
      const bf16_t* Wh = W + ((size_t)h * d_c + kc) * d_v + col0;
#pragma unroll 8
      for (int k = wave; k < MC_ROWS * PPR / 64; k += MC_NW) {
        const int x = k * 64 + lane, r = x / PPR, p = (x % PPR) ^ wswz(r);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Wh + (size_t)r * d_v + 8 * p),
                                         (__attribute__((address_space(3))) void*)(slab + k * 1024), 16, 0, 0);
      }
    }
    // ---- this lane's (slice, sequence) and its slots ---------------------------
    const int k_base = kc + WK * wave;
    const int sl = k_base / dl, c_lane = k_base - sl * dl + 8 * q4;
    const int vb = sl * B + bc;
    int first, cnt;
    // a balanced plan with fewer pages than workgroups leaves some page ranges empty
    bool sparse = false;
    int T = 1, c0 = 0, w0 = 0;
    if (n_pages == 0) {
      first = 0;
      cnt = 0;
    } else if (!a.balanced) {
      first = vb * a.n_splits;
      cnt = min((n_pages + a.pages_per_split - 1) / a.pages_per_split, a.n_splits);
    } else {
      // the split kernel left the slots of every (slice, sequence) in the plan table
      w0 = a.plan[n_v + 1 + vb];
      cnt = a.plan[2 * n_v + 1 + vb];
      first = w0 + vb;
      sparse = a.plan[3 * n_v + 1] != 0;
      if (sparse) {
        T = a.plan[n_v];
        c0 = a.plan[vb];
      }
    }
    auto live = [&](int s) -> bool {
      if (s >= cnt) return false;
      return !sparse || balanced_range_meets(a.geom, w0 + s, T, c0, c0 + n_pages);
    };

    // ---- merged latent output of this lane: KS pieces of 8 columns -------------
    // (the four lanes of a sequence run these loops together: same cnt, same slots)
    float4 x[KS][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) x[ks][0] = x[ks][1] = float4{0.f, 0.f, 0.f, 0.f};
    float M = -INFINITY, lsum = 0.f;
    for (int base = 0; base < cnt; base += 16) {
      float m4[4], l4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = base + q4 + 4 * i;
        m4[i] = -INFINITY;
        l4[i] = 0.f;
        if (live(s)) {
          const float2 v = *reinterpret_cast<const float2*>(a.part_ml + ((size_t)(first + s) * H + h) * 2);
          m4[i] = v.x;
          l4[i] = v.y;
        }
      }
      float Mr = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
      Mr = fmaxf(Mr, __shfl_xor(Mr, 16));
      Mr = fmaxf(Mr, __shfl_xor(Mr, 32));
      if (Mr == -INFINITY) continue;                 // 16 empty page ranges in a row
      const float M_new = fmaxf(M, Mr);
      const float alpha = exp2f(M - M_new);          // 0 the first time
      float lr = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) lr = fmaf(l4[i], exp2f(m4[i] - M_new), lr);
      lr += __shfl_xor(lr, 16);
      lr += __shfl_xor(lr, 32);
      lsum = fmaf(lsum, alpha, lr);
      M = M_new;
      if (alpha != 1.0f) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            x[ks][e].x *= alpha; x[ks][e].y *= alpha; x[ks][e].z *= alpha; x[ks][e].w *= alpha;
          }
      }
#pragma unroll
      for (int u0 = 0; u0 < 16; u0 += MC_AHEAD) {
        if (base + u0 >= cnt) break;
        float4 p[MC_AHEAD][KS][2];
        float wg[MC_AHEAD];
#pragma unroll
        for (int u = 0; u < MC_AHEAD; ++u) {
          const int s = base + u0 + u;
          // slot u0 + u of the round sits in register (u0 + u) / 4 of lane group (u0 + u) % 4
          const float ms = __shfl(m4[(u0 + u) >> 2], ((u0 + u) & 3) * 16 + j16);
          wg[u] = 0.f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) p[u][ks][0] = p[u][ks][1] = float4{0.f, 0.f, 0.f, 0.f};
          if (live(s)) {
            wg[u] = exp2f(ms - M);
            const float* src = a.part_acc + ((size_t)(first + s) * H + h) * dl + c_lane;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
              p[u][ks][0] = *reinterpret_cast<const float4*>(src + 32 * ks);
              p[u][ks][1] = *reinterpret_cast<const float4*>(src + 32 * ks + 4);
            }
          }
        }
#pragma unroll
        for (int u = 0; u < MC_AHEAD; ++u) {       // slot order
          const float w = wg[u];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              x[ks][e].x = fmaf(p[u][ks][e].x, w, x[ks][e].x);
              x[ks][e].y = fmaf(p[u][ks][e].y, w, x[ks][e].y);
              x[ks][e].z = fmaf(p[u][ks][e].z, w, x[ks][e].z);
              x[ks][e].w = fmaf(p[u][ks][e].w, w, x[ks][e].w);
            }
        }
      }
    }
    if (lsum > 0.f) {
      const float inv = 1.0f / lsum;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          x[ks][e].x *= inv; x[ks][e].y *= inv; x[ks][e].z *= inv; x[ks][e].w *= inv;
        }
    }
    if (b_valid && blockIdx.z == 0) {
      if (a.lse && q4 == 0 && k_base == sl * dl)
        a.lse[(size_t)vb * H + h] = lsum > 0.f ? (M + log2f(lsum)) * 0.6931471805599453f : -INFINITY;
      float* dst = a.o_lat + ((size_t)vb * H + h) * dl + c_lane;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        *reinterpret_cast<float4*>(dst + 32 * ks) = x[ks][0];
        *reinterpret_cast<float4*>(dst + 32 * ks + 4) = x[ks][1];
      }
    }
    // ---- the slab has landed for every wave --------------------------------------
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const float xs[8] = {x[ks][0].x, x[ks][0].y, x[ks][0].z, x[ks][0].w,
                           x[ks][1].x, x[ks][1].y, x[ks][1].z, x[ks][1].w};
      bf16x8 ah, al;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const bf16_t hi16 = (bf16_t)xs[e];
        ah[e] = hi16;
        al[e] = (bf16_t)(xs[e] - (float)hi16);
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const bf16x8 bf = read_b_frag<PPR>(slab, WK * wave + 32 * ks, cb, j16, q4);
        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bf, acc[cb], 0, 0, 0);
        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bf, acc[cb], 0, 0, 0);
      }
    }
  }
  // sum the waves' tiles through LDS; wave w finishes column block w
  static_assert(NCB == MC_NW, "one column block per wave in the final sum");
  __syncthreads();
  f32x4* red = reinterpret_cast<f32x4*>(slab4);    // [wave][cb][lane]
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) red[(wave * NCB + cb) * 64 + lane] = acc[cb];
  __syncthreads();
  f32x4 tsum = red[(0 * NCB + wave) * 64 + lane];
#pragma unroll
  for (int w2 = 1; w2 < MC_NW; ++w2) tsum += red[(w2 * NCB + wave) * 64 + lane];
  // tsum[i]: sequence spw mb + 4 q4 + i, column col0 + 16 wave + j16
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int bb = spw * mb + 4 * q4 + i;
    if (4 * q4 + i < spw && bb < B) store_from_f32(o + ((size_t)bb * H + h) * d_v + col0 + 16 * wave + j16, tsum[i]);
  }
}

bool merge_combine_mfma_supported(const tpla_shape_t& sh) {
  return sh.dtype == TPLA_BF16 && sh.d_v % MC_COLS == 0 && sh.d_c % MC_ROWS == 0 &&
         (sh.d_c / sh.g) % (MC_ROWS / MC_NW) == 0 && sh.d_v / MC_COLS <= 65535 && (sh.B + 7) / 8 <= 65535;
}

int launch_merge_combine_mfma(const DecodeArgs& a, const tpla_shape_t& sh, const void* W_UV_t, void* o, int o_dtype,
                              hipStream_t st) {
  constexpr size_t smem = (size_t)MC_ROWS * MC_COLS * 2;
  // dynamic LDS above the 64 KiB default needs opting in, once
  static const hipError_t attr = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(merge_combine_mfma_kernel<float>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(merge_combine_mfma_kernel<bf16_t>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    return e;
  }();
  if (attr != hipSuccess) {
    (void)hipGetLastError();
    return fail(TPLA_ERR_HIP, "cannot raise the dynamic LDS limit to %zu", smem);
  }
  // 16 sequences per workgroup once that gives every compute unit two workgroups, else 8
  const long long wg16 = (long long)sh.H * ((sh.B + 15) / 16) * (sh.d_v / MC_COLS);
  const int spw = wg16 >= 2LL * device_cu_count() ? 16 : 8;
  const dim3 grid((unsigned)sh.H, (unsigned)((sh.B + spw - 1) / spw), (unsigned)(sh.d_v / MC_COLS));
  if (o_dtype == TPLA_BF16)
    hipLaunchKernelGGL(merge_combine_mfma_kernel<bf16_t>, grid, dim3(MC_NW * 64), smem, st, a,
                       static_cast<const bf16_t*>(W_UV_t), static_cast<bf16_t*>(o), sh.d_c, sh.d_v, spw);
  else
    hipLaunchKernelGGL(merge_combine_mfma_kernel<float>, grid, dim3(MC_NW * 64), smem, st, a,
                       static_cast<const bf16_t*>(W_UV_t), static_cast<float*>(o), sh.d_c, sh.d_v, spw);
  return check_launch("merge_combine_mfma_kernel");
}

// ---------------------------------------------------------------------------
// Output projection  out[b, n] = sum_k x[b, k] W[k, n]  (x = the combined
// per-head outputs flattened to [B, H d_v], W = W_O [H d_v, D]; Sec. 3.3: the
// value up-projection is not merged into W_O, so this runs after the combine).
// A weight-streaming skinny GEMM: grid (D / 128, KSPLIT); a workgroup owns 128
// output columns and one contiguous k-range and walks it in chunks of OP_ROWS
// rows.  A chunk = the weight rows (16 KB) and the matching columns of 32 rows
// of x (8 KB, float), both brought in by direct-to-LDS loads into a ring of
// OP_NST buffers, so that three chunks per workgroup are in flight whatever the
// waves are doing and every vector-memory operation of the loop is one of these
// loads (the wait counts below rely on that).  Wave w owns columns 32w..32w+31
// over all rows of a chunk: no sum across waves.  x is split into bf16 hi + lo
// (two MFMAs) so the product keeps float accuracy.  The float partial tiles of
// the KSPLIT ranges are summed in order by a second kernel.
constexpr int OP_COLS = 128;
constexpr int OP_ROWS = 64;
constexpr int OP_NST = 4;
static_assert(OP_NST >= 3 && OP_NST <= 6, "the wait counts cover one to four younger chunks");
constexpr int OP_W_BYTES = OP_ROWS * OP_COLS * 2;     // 16 rows of 16 pieces per KB: 16 instructions
constexpr int OP_X_BYTES = 32 * OP_ROWS * 4;          // 32 rows of x, 16 pieces each: 8 instructions
constexpr int OP_STAGE = OP_W_BYTES + OP_X_BYTES;
constexpr int OP_LOADS = (OP_W_BYTES + OP_X_BYTES) / 1024 / 4;   // per wave and chunk

template <int OFF>
__device__ __forceinline__ void lds_read_f4(f32x4& dst, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}

__global__ void __launch_bounds__(256) output_projection_mfma_kernel(const float* __restrict__ x,
                                                                        const bf16_t* __restrict__ W,
                                                                        float* __restrict__ part, int B, int K,
                                                                        int N, int k_per_split) {
  extern __shared__ u32x4 ring4[];                 // OP_NST stages of [W chunk | x chunk]
  char* ring = reinterpret_cast<char*>(ring4);
  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)ring4);
  const int c0 = blockIdx.x * OP_COLS, kz = blockIdx.y;
  const int k_begin = kz * k_per_split;
  const int n_chunks = k_per_split / OP_ROWS;
  const int tid = threadIdx.x, lane = tid & 63, j16 = lane & 15, q4 = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_mb = (B + 15) / 16;

  // Direct-to-LDS bookkeeping.  Instruction k of a region fills its pieces [64k, 64k + 64): row
  // 4k + q4, position j16.  This wave issues k = wave + 4j, i.e. rows 4 wave + q4 + 16 j; the
  // piece that belongs at position j16 of such a row is j16 ^ swizzle(row), the same for every j.
  const int wr = 4 * wave + q4;
  const char* w_src = reinterpret_cast<const char*>(W + (size_t)(k_begin + wr) * N + c0 + 8 * (j16 ^ wswz(wr)));
  const size_t w_rows16 = (size_t)16 * N * 2, w_chunk = (size_t)OP_ROWS * N * 2;

  // LDS read offsets.  Weights: rows 32 ks + 8 q4 + (j16 >> 2) (+4), piece pair of column block
  // 2 wave + cb.  x: row 16 m + j16, pieces 8 ks + 2 q4 + {0, 1}, stored at piece ^ (row & 15).
  const int r0 = 8 * q4 + (j16 >> 2);
  unsigned b_off[2], a_off[2][2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
    b_off[cb] = (unsigned)((r0 * 16 + ((2 * (2 * wave + cb) + ((j16 & 3) >> 1)) ^ wswz(r0))) * 16 + (j16 & 1) * 8);
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int h = 0; h < 2; ++h)
      a_off[ks][h] = (unsigned)(OP_W_BYTES + (j16 * 16 + ((8 * ks + 2 * q4 + h) ^ j16)) * 16);

  for (int mb0 = 0; mb0 < n_mb; mb0 += 2) {
    const char* x_src[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int bl = wr + 16 * j;                  // row of the x chunk, 0..31
      const int b = min(16 * mb0 + bl, B - 1);     // rows past the batch repeat the last one, never stored
      x_src[j] = reinterpret_cast<const char*>(x + (size_t)b * K + k_begin + 4 * (j16 ^ (bl & 15)));
    }
    auto issue = [&](int t) {
      char* dst = ring + (t % OP_NST) * OP_STAGE + wave * 1024;
      const char* ws = w_src + (size_t)t * w_chunk;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ws + j * w_rows16),
                                         (__attribute__((address_space(3))) void*)(dst + j * 4096), 16, 0,
                                         2 /* streaming: the weights are read once */);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(x_src[j] + (size_t)t * (OP_ROWS * 4)),
            (__attribute__((address_space(3))) void*)(dst + OP_W_BYTES + j * 4096), 16, 0, 0);
    };
    static_assert(OP_LOADS == 6, "four weight and two x instructions per wave and chunk");

    f32x4 acc[2][2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) acc[m][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // the previous pass is done with LDS and its stores have left (they would share the counter)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
#pragma unroll
    for (int t = 0; t < OP_NST - 1; ++t)
      if (t < n_chunks) issue(t);
    for (int t = 0; t < n_chunks; ++t) {
      // chunk t has landed once only the loads of the chunks requested after it are outstanding
      switch (min(n_chunks - 1 - t, OP_NST - 2)) {
        case 0: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;
        case 1: __builtin_amdgcn_s_waitcnt(vmcnt_imm(OP_LOADS)); break;
        case 2: __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * OP_LOADS)); break;
        case 3: __builtin_amdgcn_s_waitcnt(vmcnt_imm(3 * OP_LOADS)); break;
        default: __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 * OP_LOADS)); break;
      }
      __builtin_amdgcn_s_barrier();          // chunk t visible to all waves, chunk t-1 no longer read
      if (t + OP_NST - 1 < n_chunks) issue(t + OP_NST - 1);
      const unsigned st = lds_base + (unsigned)((t % OP_NST) * OP_STAGE);
      f32x4 xf[2][2][2];                     // [ks][m][half]
      u32x2 wlo[2][2], whi[2][2];            // [ks][cb]
      static_for<2>([&](auto kc) {
        constexpr int ks = decltype(kc)::value;
        lds_read_f4<0>(xf[ks][0][0], st + a_off[ks][0]);
        lds_read_f4<0>(xf[ks][0][1], st + a_off[ks][1]);
        lds_read_f4<4096>(xf[ks][1][0], st + a_off[ks][0]);
        lds_read_f4<4096>(xf[ks][1][1], st + a_off[ks][1]);
        lds_read_tr_b64<ks * 8192>(wlo[ks][0], st + b_off[0]);
        lds_read_tr_b64<ks * 8192 + 1024>(whi[ks][0], st + b_off[0]);
        lds_read_tr_b64<ks * 8192>(wlo[ks][1], st + b_off[1]);
        lds_read_tr_b64<ks * 8192 + 1024>(whi[ks][1], st + b_off[1]);
      });
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(xf[0][0][0]), "+v"(xf[0][0][1]), "+v"(xf[0][1][0]), "+v"(xf[0][1][1]), "+v"(xf[1][0][0]),
                     "+v"(xf[1][0][1]), "+v"(xf[1][1][0]), "+v"(xf[1][1][1]), "+v"(wlo[0][0]), "+v"(whi[0][0]),
                     "+v"(wlo[0][1]), "+v"(whi[0][1]), "+v"(wlo[1][0]), "+v"(whi[1][0]), "+v"(wlo[1][1]),
                     "+v"(whi[1][1])
                   :
                   : "memory");
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 ah[2], al[2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float v = xf[ks][m][e >> 2][e & 3];
            const bf16_t hi16 = (bf16_t)v;
            ah[m][e] = hi16;
            al[m][e] = (bf16_t)(v - (float)hi16);
          }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const u32x4 w4 = {wlo[ks][cb][0], wlo[ks][cb][1], whi[ks][cb][0], whi[ks][cb][1]};
          const bf16x8 bf = __builtin_bit_cast(bf16x8, w4);
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            acc[m][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[m], bf, acc[m][cb], 0, 0, 0);
            acc[m][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[m], bf, acc[m][cb], 0, 0, 0);
          }
        }
      }
    }
    // acc[m][cb][i]: row 16 (mb0 + m) + 4 q4 + i, column c0 + 32 wave + 16 cb + j16
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int bb = 16 * (mb0 + m) + 4 * q4 + i;
          if (bb < B) part[((size_t)kz * B + bb) * N + c0 + 32 * wave + 16 * cb + j16] = acc[m][cb][i];
        }
  }
}

template <typename OT>
__global__ void __launch_bounds__(256) output_projection_reduce_kernel(const float* __restrict__ part,
                                                                       OT* __restrict__ out, size_t n,
                                                                       int ksplit) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float v = part[i];
  for (int z = 1; z < ksplit; ++z) v += part[(size_t)z * n + i];
  store_from_f32(out + i, v);
}

// Any storage type and width: one thread per output element.
template <typename T, typename OT>
__global__ void __launch_bounds__(256) output_projection_simple_kernel(const float* __restrict__ x,
                                                                       const T* __restrict__ W,
                                                                       OT* __restrict__ out, int K, int N) {
  const int n = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
  if (n >= N) return;
  float v = 0.f;
  for (int k = 0; k < K; ++k) v = fmaf(x[(size_t)b * K + k], load_as_f32(W + (size_t)k * N + n), v);
  store_from_f32(out + (size_t)b * N + n, v);
}

// k-range split of the matrix-core path (0 = that path does not apply).
int output_projection_ksplit(const tpla_shape_t& sh, int D) {
  const long long K = (long long)sh.H * sh.d_v;
  if (sh.dtype != TPLA_BF16 || D % OP_COLS != 0 || K % OP_ROWS != 0 || K > 2147483647LL) return 0;
  const int slabs = D / OP_COLS;
  // about one workgroup per compute unit (its ring takes 96 KB of LDS): for D = 7168, K = 8192 at B = 32 that is
  // 224 workgroups of 32 chunks, 27 us for both kernels; 448 of 16 chunks on a ring of 3 took 29.5 us
  int ks = (device_cu_count() + slabs - 1) / slabs;
  const int chunks = (int)(K / OP_ROWS);
  if (ks > chunks) ks = chunks;
  if (ks < 1) ks = 1;
  while (chunks % ks) --ks;                                   // equal k-ranges, whole chunks
  return ks;
}

template <typename OT>
static int launch_output_projection_to(const tpla_shape_t& sh, const float* x, const void* W_O, int D, float* part,
                                       OT* out, hipStream_t st) {
  const int K = sh.H * sh.d_v;
  const int ks = output_projection_ksplit(sh, D);
  constexpr bool direct_ok = sizeof(OT) == sizeof(float);     // the matrix-core kernel writes float tiles
  if (ks == 0) {
    const dim3 grid((unsigned)((D + 255) / 256), (unsigned)sh.B);
    if (sh.dtype == TPLA_F32)
      hipLaunchKernelGGL((output_projection_simple_kernel<float, OT>), grid, dim3(256), 0, st, x,
                         static_cast<const float*>(W_O), out, K, D);
    else
      hipLaunchKernelGGL((output_projection_simple_kernel<bf16_t, OT>), grid, dim3(256), 0, st, x,
                         static_cast<const bf16_t*>(W_O), out, K, D);
    return check_launch("output_projection_simple_kernel");
  }
  constexpr size_t smem = (size_t)OP_NST * OP_STAGE;
  // dynamic LDS above the 64 KiB default needs opting in, once
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(output_projection_mfma_kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr != hipSuccess) {
    (void)hipGetLastError();
    return fail(TPLA_ERR_HIP, "cannot raise the dynamic LDS limit to %zu", smem);
  }
  const bool direct = ks == 1 && direct_ok;
  float* dst = direct ? reinterpret_cast<float*>(out) : part;
  hipLaunchKernelGGL(output_projection_mfma_kernel, dim3((unsigned)(D / OP_COLS), (unsigned)ks), dim3(256), smem,
                     st, x, static_cast<const bf16_t*>(W_O), dst, sh.B, K, D, K / ks);
  int rc = check_launch("output_projection_mfma_kernel");
  if (rc || direct) return rc;
  const size_t n = (size_t)sh.B * D;
  hipLaunchKernelGGL(output_projection_reduce_kernel<OT>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part,
                     out, n, ks);
  return check_launch("output_projection_reduce_kernel");
}

// Scratch floats of the matrix-core path for an output of the given type (a bf16 output always goes
// through the float partial tiles, also with a single k-range).
size_t output_projection_scratch_floats(const tpla_shape_t& sh, int D, int out_dtype) {
  const int ks = output_projection_ksplit(sh, D);
  if (ks == 0 || (ks == 1 && out_dtype == TPLA_F32)) return 0;
  return (size_t)ks * sh.B * D;
}

int launch_output_projection(const tpla_shape_t& sh, const float* x, const void* W_O, int D, float* part, void* out,
                             int out_dtype, hipStream_t st) {
  if (out_dtype == TPLA_BF16)
    return launch_output_projection_to(sh, x, W_O, D, part, static_cast<bf16_t*>(out), st);
  return launch_output_projection_to(sh, x, W_O, D, part, static_cast<float*>(out), st);
}

}  // namespace tpla
