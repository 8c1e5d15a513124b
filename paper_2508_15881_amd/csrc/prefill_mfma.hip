// Prefill with MLA in its un-absorbed form (Sec. 4.5 of the paper: the prefill
// phase keeps MLA with the heads split over devices; Sec. 3.3 for the per-head
// keys and values), bf16 on the matrix cores, for packed variable-length
// sequences with a causal mask.
//
//   prefill_kv_project_kernel     kv[t, h] = [ c_t W_UV[h] | W_UK[h] c_t ]   (values, no-RoPE keys)
//   prefill_attention_mfma_kernel o[t, h]  = sum_{s<=t} softmax_s(scale (q_nope.k + q_pe.k_pe)) v
//
// The attention kernel is the decode kernel's tile machinery turned around: a
// workgroup owns 128 consecutive queries of one (sequence, head), a wave 32 of
// them as two blocks of 16, and 32-key tiles [V 128 | K 128 | k_pe 64] go
// through a ring of 3 LDS buffers with direct-to-LDS loads (the RoPE key comes
// from the array shared by all heads).  Queries are the MFMA N dimension:
//   S^T[key, query] = K[key, :] . Q[query, :]          M = keys, N = queries
//   O^T[dim, query] += V^T[dim, key] . P^T[key, query]  M = value dims, N = queries
// so a lane only ever sees one query per block, the online softmax needs no
// LDS, and P stays in registers between the two products.  Key tiles above the
// diagonal are never loaded; blocks entirely above it skip the tile.
#include "lds_tile.h"

#include <algorithm>
#include <mutex>

namespace tpla {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// Up-projection: Y[t, n] = sum_k c[t, k] B[k, n] per head, B = W_UV[h] (values)
// or W_UK[h]^T (keys).  Same shape of kernel as the dense cache transform: the
// head's weight goes to LDS once in B-operand order, the workgroup (8 waves x
// 4 row tiles) walks over blocks of 512 tokens, A operands straight from
// global memory with 4 k-steps in flight.
constexpr int PJ_WAVES = 8;
constexpr int PJ_ROWS = PJ_WAVES * 64;
constexpr int PJ_AHEAD = 2;

__device__ __forceinline__ int pj_k0(int s, int kg) { return 64 * (s >> 1) + 16 * kg + 8 * (s & 1); }

// grid: (2 H, row workers); blockIdx.x = 2 h + part (0: values, 1: keys)
__global__ void __launch_bounds__(PJ_WAVES * 64) prefill_kv_project_kernel(
    const bf16_t* __restrict__ c, const bf16_t* __restrict__ W_UK, const bf16_t* __restrict__ W_UV,
    bf16_t* __restrict__ kv, int T, int H, int d_c) {
  extern __shared__ u32x4 panel[];                 // [KS][8][64] operands of 8 bf16
  const int KS = d_c >> 5;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 15, hi = lane >> 4;
  const int h = blockIdx.x >> 1, part = blockIdx.x & 1;

  for (int idx = tid; idx < KS * 512; idx += PJ_WAVES * 64) {
    const int ln = idx & 63, nt = (idx >> 6) & 7, s = idx >> 9;
    const int n = 64 * (nt >> 2) + 4 * (ln & 15) + (nt & 3);      // a lane owns 4 adjacent columns per half
    const int k0 = pj_k0(s, ln >> 4);
    u32x4 v;
    if (part) {
      v = *reinterpret_cast<const u32x4*>(W_UK + ((size_t)h * 128 + n) * d_c + k0);      // W_UK[h][n][k], k contiguous
    } else {
      const unsigned short* w = reinterpret_cast<const unsigned short*>(W_UV) + ((size_t)h * d_c + k0) * 128 + n;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) v[jj] = (unsigned)w[(2 * jj) * 128] | ((unsigned)w[(2 * jj + 1) * 128] << 16);
    }
    panel[idx] = v;
  }
  __syncthreads();

  const int last = T - 1;
  const int n_blocks = (T + PJ_ROWS - 1) / PJ_ROWS;
  for (int rb = blockIdx.y; rb < n_blocks; rb += gridDim.y) {
    const int row0 = rb * PJ_ROWS + wave * 64;
    if (row0 > last) continue;                       // whole waves; no barrier below
    const bf16_t* ap[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) ap[mt] = c + (size_t)min(row0 + 16 * mt + lo, last) * d_c;
    f32x4 acc[4][8];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 a[PJ_AHEAD][4];
#pragma unroll
    for (int d = 0; d < PJ_AHEAD; ++d)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) a[d][mt] = *reinterpret_cast<const u32x4*>(ap[mt] + pj_k0(d < KS ? d : KS - 1, hi));
    for (int s0 = 0; s0 < KS; s0 += PJ_AHEAD) {
#pragma unroll
      for (int d = 0; d < PJ_AHEAD; ++d) {
        const int s = s0 + d;                        // KS is a multiple of PJ_AHEAD (d_c % 128 == 0)
        bf16x8 av[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) av[mt] = __builtin_bit_cast(bf16x8, a[d][mt]);
        const int sn = min(s + PJ_AHEAD, KS - 1);    // the last refills repeat a valid address, unused
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) a[d][mt] = *reinterpret_cast<const u32x4*>(ap[mt] + pj_k0(sn, hi));
        __builtin_amdgcn_sched_barrier(0);           // keep the refill ahead of this step's MFMAs
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, panel[(s * 8 + nt) * 64 + lane]);
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], bv, acc[mt][nt], 0, 0, 0);
        }
      }
    }
    // rows 16 mt + 4 hi + i, columns 64 half + 4 lo + (nt & 3)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = row0 + 16 * mt + 4 * hi + i;
        if (r <= last) {
          bf16_t* dst = kv + ((size_t)r * H + h) * 256 + 128 * part + 4 * lo;
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16x2 p0 = __builtin_convertvector(f32x2{acc[mt][4 * half][i], acc[mt][4 * half + 1][i]}, bf16x2);
            const bf16x2 p1 = __builtin_convertvector(f32x2{acc[mt][4 * half + 2][i], acc[mt][4 * half + 3][i]}, bf16x2);
            const u32x2 out = {__builtin_bit_cast(unsigned, p0), __builtin_bit_cast(unsigned, p1)};
            *reinterpret_cast<u32x2*>(dst + 64 * half) = out;
          }
        }
      }
  }
}

// ---------------------------------------------------------------------------
constexpr int PF_TOK = 32;                 // keys per tile
constexpr int PF_NSTAGE = 3;
constexpr int PF_RC = 40;                  // 16-byte pieces per tile row: V 16, K 16, k_pe 8
constexpr int PF_NW = 4;
constexpr int PF_VRING = 4;               // V fragments in flight ahead of the output MFMAs
constexpr int PF_KRING = 8;               // K fragments in flight ahead of the score MFMAs
constexpr int PF_QB = 2;                   // blocks of 16 queries per wave
constexpr int PF_QT = PF_NW * PF_QB * 16;  // queries per workgroup
constexpr int PF_TC = PF_TOK * PF_RC;      // pieces per tile
constexpr int PF_TILE_BYTES = PF_TC * 16;
constexpr int PF_NI = PF_TC / 64;          // direct-to-LDS instructions per tile
constexpr int PF_CPT = PF_NI / PF_NW;      // of which each wave issues this many
static_assert(PF_NI % PF_NW == 0, "every wave issues the same number of tile loads");

struct PrefillArgs {
  const bf16_t* q_nope;   // [T, H, 128]
  const bf16_t* q_pe;     // [T, H, 64]
  const bf16_t* kv;       // [T, H, 256]: values then no-RoPE keys
  const bf16_t* k_pe;     // [T, 64]
  const int32_t* cu;      // [B + 1]
  float* o;               // [T, H, 128]
  int H;
  int T;           // packed tokens in all
  int n_qt;        // query tiles of the longest sequence
  int head_group;  // divides H
  float scale_log2;
};

// grid: (query tiles of the longest sequence x H, sequences).  Order inside a sequence: groups of
// head_group heads; inside a group the query tiles from last (longest key range) to first, the
// heads of the group innermost.  The workgroups in flight then share the keys and values of a
// few heads (they stay in the last-level cache) and the grid ends on short work items.
__global__ void __launch_bounds__(PF_NW * 64, 2) prefill_attention_mfma_kernel(PrefillArgs a) {
  extern __shared__ u32x4 smem[];
  const int seq = blockIdx.y;
  const int per_group = a.n_qt * a.head_group;
  const int hg = blockIdx.x / per_group, rem = blockIdx.x - hg * per_group;
  const int h = hg * a.head_group + rem % a.head_group;
  const int qt = a.n_qt - 1 - rem / a.head_group;          // long key ranges first
  // row ranges are clipped to [0, T): a malformed cu_seqlens gives wrong numbers, never an access outside the buffers
  const int t0 = min(max(a.cu[seq], 0), a.T), L = min(max(a.cu[seq + 1], t0), a.T) - t0;
  if (qt * PF_QT >= L) return;
  const int q0 = qt * PF_QT;
  const int kend = min(L, q0 + PF_QT);                     // keys 0 .. kend-1 are needed
  const int ntiles = (kend + PF_TOK - 1) / PF_TOK;

  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  const int tid = threadIdx.x, lane = tid & 63;
  // scalar on purpose: the per-block skips below must be scalar branches, an MFMA does not honour a lane mask
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j16 = lane & 15, q4 = lane >> 4;

  // ---- direct-to-LDS bookkeeping: instruction k of a tile fills pieces [64k, 64k+64) ----
  // Tiles are issued in order, each exactly once, so every lane keeps a running source pointer per
  // instruction (two VALU adds per load) instead of multiplying the key index out every time.
  int ld_tok[PF_CPT];
  const char* ld_cur[PF_CPT];    // source of this lane's piece in the next tile to be issued
  unsigned ld_step[PF_CPT];      // bytes from one key to the next in that source
  const char* kv_base = reinterpret_cast<const char*>(a.kv) + ((size_t)t0 * a.H + h) * 512;
  const char* kpe_base = reinterpret_cast<const char*>(a.k_pe) + (size_t)t0 * 128;
  const unsigned kv_pitch = (unsigned)a.H * 512u;
#pragma unroll
  for (int j = 0; j < PF_CPT; ++j) {
    const int x = (wave + j * PF_NW) * 64 + lane;          // LDS piece index
    const int tok = x / PF_RC, cs = x % PF_RC;
    const int cg = cs ^ swz(tok);                          // the piece of the row that lives there
    ld_tok[j] = tok;
    const bool from_kv = cg < 32;                          // V and no-RoPE K; else the shared RoPE key
    ld_step[j] = from_kv ? kv_pitch : 128u;
    ld_cur[j] = (from_kv ? kv_base + cg * 16 : kpe_base + (cg - 32) * 16) + (size_t)tok * ld_step[j];
  }
  auto issue = [&](int t) {
    char* dst = reinterpret_cast<char*>(smem) + (t % PF_NSTAGE) * PF_TILE_BYTES;
    if ((t + 1) * PF_TOK <= L) {                           // scalar: every key of the tile exists
#pragma unroll
      for (int j = 0; j < PF_CPT; ++j) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ld_cur[j],
                                         (__attribute__((address_space(3))) void*)(dst + (wave + j * PF_NW) * 1024),
                                         16, 0, 0);
        ld_cur[j] += (size_t)PF_TOK * ld_step[j];
      }
    } else {
      // last tile of the sequence: keys past its end repeat the last key (finite values, masked below)
#pragma unroll
      for (int j = 0; j < PF_CPT; ++j) {
        const int over = max(0, t * PF_TOK + ld_tok[j] - (L - 1));
        const char* src = ld_cur[j] - (size_t)over * ld_step[j];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(dst + (wave + j * PF_NW) * 1024),
                                         16, 0, 0);
      }
    }
  };

  // ---- per-lane LDS byte offsets (as in the decode kernel, row of 40 pieces) ----
  const int xk = swz(j16);
  unsigned k_off[2];
  k_off[0] = (unsigned)((j16 * PF_RC + ((q4) ^ xk)) * 16);
  k_off[1] = (unsigned)((j16 * PF_RC + ((4 | q4) ^ xk)) * 16);
  const int v_tok = 4 * q4 + (j16 >> 2);
  const int xv = swz(v_tok);
  const int cb = (j16 & 3) >> 1;
  unsigned v_off[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
    v_off[d] = (unsigned)((v_tok * PF_RC + (((d << 1) | cb) ^ xv)) * 16 + (j16 & 1) * 8);

  issue(0);
  if (ntiles > 1) issue(1);

  // ---- this wave's queries as B operands: block qb holds queries qbase[qb] + j16 ----
  constexpr int KS = 6;                    // k-steps of the 192-wide score product
  constexpr int DB = 8;                    // 16-wide blocks of the 128 value dims
  bf16x8 qreg[PF_QB][KS];
  int qbase[PF_QB];
#pragma unroll
  for (int qb = 0; qb < PF_QB; ++qb) {
    qbase[qb] = q0 + wave * (16 * PF_QB) + qb * 16;
    const size_t row = (size_t)(t0 + min(qbase[qb] + j16, L - 1)) * a.H + h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 32 + q4 * 8;
      qreg[qb][ks] = (k0 < 128) ? *reinterpret_cast<const bf16x8*>(a.q_nope + row * 128 + k0)
                                : *reinterpret_cast<const bf16x8*>(a.q_pe + row * 64 + (k0 - 128));
    }
  }
#pragma unroll
  for (int qb = 0; qb < PF_QB; ++qb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[qb][ks]));   // complete before the loop

  f32x4 acc[PF_QB][DB];
  // lsum: the softmax denominators, accumulated on the matrix cores as one more output row block
  // whose A operand is all ones (every row of it holds sum_key P[key, query]): the weights that
  // reach the output are the bf16-rounded ones, and these are the ones summed
  float m_run[PF_QB];
  f32x4 lsum[PF_QB];
#pragma unroll
  for (int qb = 0; qb < PF_QB; ++qb) {
    m_run[qb] = -INFINITY;
    lsum[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int d = 0; d < DB; ++d) acc[qb][d] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  for (int t = 0; t < ntiles; ++t) {
    if (t + 1 < ntiles)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(PF_CPT));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();            // tile t visible to all waves, tile t-1 no longer read
    if (t + 2 < ntiles) issue(t + 2);
    const int key0 = t * PF_TOK;
    // Blocks take part while the tile holds a key <= their last query; later blocks have later
    // queries, so the idle ones are the first `idle` blocks (wave-uniform).  The tile body is
    // compiled once per value of `idle`: no branch sits between the MFMAs.
    int idle = 0;
#pragma unroll
    for (int qb = 0; qb < PF_QB; ++qb) idle += (key0 > qbase[qb] + 15) ? 1 : 0;
    if (idle == PF_QB) continue;
    auto tile_body = [&](auto first) {
      constexpr int QB0 = decltype(first)::value;
      const unsigned tile = lds_base + (unsigned)((t % PF_NSTAGE) * PF_TILE_BYTES);

      // ---- scores: pieces 16..39 of the row (k-steps 4..9 of the 40-piece row) ----
      f32x4 sacc[PF_QB][2];
  #pragma unroll
      for (int qb = QB0; qb < PF_QB; ++qb) sacc[qb][0] = sacc[qb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      {
        constexpr int NQ = KS * 2;             // K fragments, in order (ks, tb)
        bf16x8 kf[PF_KRING];
        const unsigned ka[2] = {tile + k_off[0], tile + k_off[1]};
        static_for<PF_KRING>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          constexpr int ks = i / 2 + 4, tb = i % 2;
          lds_read_b128<(ks >> 1) * 128 + tb * (16 * PF_RC * 16)>(kf[i], ka[ks & 1]);
        });
        static_for<NQ>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          constexpr int ks = i / 2, tb = i % 2;
          constexpr int ahead = (NQ - 1 - i) < PF_KRING - 1 ? (NQ - 1 - i) : PF_KRING - 1;
          lds_wait<ahead>(kf[i % PF_KRING]);
  #pragma unroll
          for (int qb = QB0; qb < PF_QB; ++qb)
            sacc[qb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i % PF_KRING], qreg[qb][ks], sacc[qb][tb], 0, 0, 0);
          if constexpr (i + PF_KRING < NQ) {
            constexpr int ks2 = (i + PF_KRING) / 2 + 4, tb2 = (i + PF_KRING) % 2;
            lds_read_b128<(ks2 >> 1) * 128 + tb2 * (16 * PF_RC * 16)>(kf[i % PF_KRING], ka[ks2 & 1]);
          }
        });
      }

      // the first V fragments start now, so that their LDS latency passes under the softmax arithmetic
      u32x2 vlo[PF_VRING], vhi[PF_VRING];
      unsigned va[4];
  #pragma unroll
      for (int d = 0; d < 4; ++d) va[d] = tile + v_off[d];
      static_for<PF_VRING>([&](auto ic) {
        constexpr int d = decltype(ic)::value;
        lds_read_tr_b64<(d >> 2) * 128>(vlo[d], va[d & 3]);
        lds_read_tr_b64<(d >> 2) * 128 + 16 * PF_RC * 16>(vhi[d], va[d & 3]);
      });

      // ---- causal mask + online softmax (lane = one query per block; keys key0 + 16 tb + 4 q4 + i) ----
      bf16x8 pb[PF_QB];
  #pragma unroll
      for (int qb = QB0; qb < PF_QB; ++qb) {
        if (key0 + PF_TOK - 1 > qbase[qb]) {   // the tile reaches past this block's first query
          const int query = qbase[qb] + j16;
  #pragma unroll
          for (int tb = 0; tb < 2; ++tb)
  #pragma unroll
            for (int i = 0; i < 4; ++i)
              if (key0 + 16 * tb + 4 * q4 + i > query) sacc[qb][tb][i] = -INFINITY;
        }
        float mx = sacc[qb][0][0];
  #pragma unroll
        for (int tb = 0; tb < 2; ++tb)
  #pragma unroll
          for (int i = 0; i < 4; ++i) mx = fmaxf(mx, sacc[qb][tb][i]);
        mx *= a.scale_log2;
        if (__any(mx > m_run[qb] + LAZY)) {
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float m_new = fmaxf(m_run[qb], mx);
          const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);   // 0 on the first tile
          lsum[qb] *= alpha;
          m_run[qb] = m_new;
  #pragma unroll
          for (int d = 0; d < DB; ++d) acc[qb][d] *= alpha;
        }
  #pragma unroll
        for (int tb = 0; tb < 2; ++tb)
  #pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[qb][tb][i], a.scale_log2, -m_run[qb]));
            sacc[qb][tb][i] = p;
          }
  #pragma unroll
        for (int i = 0; i < 4; ++i) {
          pb[qb][i] = (bf16_t)sacc[qb][0][i];
          pb[qb][4 + i] = (bf16_t)sacc[qb][1][i];
        }
      }

      // ---- output: O^T += V^T P^T, V = pieces 0..15 of the row ----
      {
        static_for<DB>([&](auto ic) {
          constexpr int d = decltype(ic)::value;
          constexpr int ahead = (DB - 1 - d) < PF_VRING - 1 ? (DB - 1 - d) : PF_VRING - 1;
          lds_wait<2 * ahead>(vlo[d % PF_VRING], vhi[d % PF_VRING]);
          const u32x4 v4 = {vlo[d % PF_VRING][0], vlo[d % PF_VRING][1], vhi[d % PF_VRING][0], vhi[d % PF_VRING][1]};
  #pragma unroll
          for (int qb = QB0; qb < PF_QB; ++qb)
            acc[qb][d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v4), pb[qb], acc[qb][d], 0, 0, 0);
          if constexpr (d + PF_VRING < DB) {
            constexpr int d2 = d + PF_VRING;
            lds_read_tr_b64<(d2 >> 2) * 128>(vlo[d % PF_VRING], va[d2 & 3]);
            lds_read_tr_b64<(d2 >> 2) * 128 + 16 * PF_RC * 16>(vhi[d % PF_VRING], va[d2 & 3]);
          }
        });
        const u32x4 one4 = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  #pragma unroll
        for (int qb = QB0; qb < PF_QB; ++qb)
          lsum[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, one4), pb[qb], lsum[qb], 0, 0, 0);
      }
    };
    static_for<PF_QB>([&](auto ic) {
      if (idle == decltype(ic)::value) tile_body(ic);
    });
  }

  // ---- normalise and store: lane holds query qbase + j16, dims 16 d + 4 q4 .. +4 ----
#pragma unroll
  for (int qb = 0; qb < PF_QB; ++qb) {
    const float l_tot = lsum[qb][0];
    const int query = qbase[qb] + j16;
    if (query < L) {
      const float inv = 1.0f / l_tot;
      float* po = a.o + ((size_t)(t0 + query) * a.H + h) * 128 + 4 * q4;
#pragma unroll
      for (int d = 0; d < DB; ++d) *reinterpret_cast<f32x4*>(po + 16 * d) = acc[qb][d] * inv;
    }
  }
}

// The same kernel with 32 queries per wave as one block on 32x32x16 MFMAs: half as many MFMA issues
// for the same matrix-core cycles, one cross-lane step instead of two in the row maximum, and the tile
// swizzle of the 32-wide fragments (swz32).  Sᵀ[key, query] lands with lane = query (lane & 31) and
// the two half-waves holding keys {0-3, 8-11, 16-19, 24-27} and {4-7, 12-15, 20-23, 28-31}: exactly
// the B operand of Oᵀ += Vᵀ Pᵀ when Vᵀ is fetched with its keys in that order.
__global__ void __launch_bounds__(PF_NW * 64, 2) prefill_attention_mfma32_kernel(PrefillArgs a) {
  extern __shared__ u32x4 smem[];
  constexpr int ROWB = PF_RC * 16;
  static_assert(PF_TILE_BYTES % 4096 == 0, "tile bases must leave address bits 5..11 to the lane offsets");
  static_assert(PF_QT == PF_NW * 32 && PF_TOK == 32, "32 queries per wave, 32 keys per tile");
  const int seq = blockIdx.y;
  const int per_group = a.n_qt * a.head_group;
  const int hg = blockIdx.x / per_group, rem = blockIdx.x - hg * per_group;
  const int h = hg * a.head_group + rem % a.head_group;
  const int qt = a.n_qt - 1 - rem / a.head_group;          // long key ranges first
  const int t0 = min(max(a.cu[seq], 0), a.T), L = min(max(a.cu[seq + 1], t0), a.T) - t0;
  if (qt * PF_QT >= L) return;
  const int q0 = qt * PF_QT;
  const int kend = min(L, q0 + PF_QT);
  const int ntiles = (kend + PF_TOK - 1) / PF_TOK;

  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, hi = lane >> 5;

  // ---- direct-to-LDS bookkeeping (as in the 16-wide kernel, with the other swizzle) ----
  int ld_tok[PF_CPT];
  const char* ld_cur[PF_CPT];
  unsigned ld_step[PF_CPT];
  const char* kv_base = reinterpret_cast<const char*>(a.kv) + ((size_t)t0 * a.H + h) * 512;
  const char* kpe_base = reinterpret_cast<const char*>(a.k_pe) + (size_t)t0 * 128;
  const unsigned kv_pitch = (unsigned)a.H * 512u;
#pragma unroll
  for (int j = 0; j < PF_CPT; ++j) {
    const int x = (wave + j * PF_NW) * 64 + lane;
    const int tok = x / PF_RC, cs = x % PF_RC;
    const int cg = cs ^ swz32(tok);
    ld_tok[j] = tok;
    const bool from_kv = cg < 32;
    ld_step[j] = from_kv ? kv_pitch : 128u;
    ld_cur[j] = (from_kv ? kv_base + cg * 16 : kpe_base + (cg - 32) * 16) + (size_t)tok * ld_step[j];
  }
  auto issue = [&](int t) {
    char* dst = reinterpret_cast<char*>(smem) + (t % PF_NSTAGE) * PF_TILE_BYTES;
    if ((t + 1) * PF_TOK <= L) {
#pragma unroll
      for (int j = 0; j < PF_CPT; ++j) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ld_cur[j],
                                         (__attribute__((address_space(3))) void*)(dst + (wave + j * PF_NW) * 1024),
                                         16, 0, 0);
        ld_cur[j] += (size_t)PF_TOK * ld_step[j];
      }
    } else {
      // last tile of the sequence: keys past its end repeat the last key (finite values, masked below)
#pragma unroll
      for (int j = 0; j < PF_CPT; ++j) {
        const int over = max(0, t * PF_TOK + ld_tok[j] - (L - 1));
        const char* src = ld_cur[j] - (size_t)over * ld_step[j];
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(dst + (wave + j * PF_NW) * 1024),
                                         16, 0, 0);
      }
    }
  };

  // ---- per-lane LDS byte offsets ----
  // score product: key n32, piece 16 + 2 ks + hi = 8 (2 + ks / 4) + (2 (ks % 4) | hi); the swizzle only
  // touches the low three bits of the piece index and (2 j | hi) ^ x = (hi ^ x) ^ 2 j, so the offsets
  // of ks % 4 = 1, 2, 3 are that of 0 with address bits 5 and 6 flipped
  const unsigned k_off = (unsigned)(n32 * ROWB + ((hi ^ swz32(n32)) * 16));
  // output product: 16-lane group (hi, dim half); lane j of it points at key 4 hi + j / 4 of the k-step
  // and dims 32 d + 16 half + 4 (j % 4) .. +3, i.e. piece 4 d + 2 half + (j % 4) / 2
  const int j16 = lane & 15, half = (lane >> 4) & 1;
  const int v_tok = 4 * hi + (j16 >> 2);
  const int pl = 2 * half + ((j16 & 3) >> 1);
  const unsigned v_off = (unsigned)(v_tok * ROWB + ((pl ^ swz32(v_tok)) * 16) + (j16 & 1) * 8);

  issue(0);
  if (ntiles > 1) issue(1);

  // ---- this wave's 32 queries as B operands: lane holds query qbase + n32, k = 16 ks + 8 hi .. +7 ----
  constexpr int KS = 12;                   // 16-wide k-steps of the 192-wide score product
  constexpr int DB = 4;                    // 32-wide blocks of the 128 value dims
  const int qbase = q0 + wave * 32;
  bf16x8 qreg[KS];
  {
    const size_t row = (size_t)(t0 + min(qbase + n32, L - 1)) * a.H + h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 16 + hi * 8;
      qreg[ks] = (k0 < 128) ? *reinterpret_cast<const bf16x8*>(a.q_nope + row * 128 + k0)
                            : *reinterpret_cast<const bf16x8*>(a.q_pe + row * 64 + (k0 - 128));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));   // complete before the loop
  }

  f32x16 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[d][i] = 0.f;
  // lsum: the softmax denominators, accumulated on the matrix cores as one more output block whose A
  // operand is all ones (every row of it holds sum_key P[key, query] of the bf16-rounded weights)
  float m_run = -INFINITY;
  f32x16 lsum;
#pragma unroll
  for (int i = 0; i < 16; ++i) lsum[i] = 0.f;
  const int last_tile = (qbase + 31) / PF_TOK;   // later tiles hold no key <= this wave's last query

  for (int t = 0; t < ntiles; ++t) {
    if (t + 1 < ntiles)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(PF_CPT));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __builtin_amdgcn_s_barrier();            // tile t visible to all waves, tile t-1 no longer read
    if (t + 2 < ntiles) issue(t + 2);
    if (t > last_tile) continue;             // wave-uniform; the barriers above are still reached
    const int key0 = t * PF_TOK;
    const unsigned tile = lds_base + (unsigned)((t % PF_NSTAGE) * PF_TILE_BYTES);

    // ---- scores: one accumulation chain, a ring of 4 K fragments ahead ----
    f32x16 sc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sc[i] = 0.f;
    {
      bf16x8 kf[4];
      const unsigned kb = tile + k_off;
      const unsigned ka[4] = {kb, kb ^ 32u, kb ^ 64u, kb ^ 96u};
      static_for<4>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        lds_read_b128<(2 + (i >> 2)) * 128>(kf[i], ka[i & 3]);
      });
      static_for<KS>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int ahead = (KS - 1 - i) < 3 ? (KS - 1 - i) : 3;
        lds_wait<ahead>(kf[i & 3]);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qreg[i], sc, 0, 0, 0);
        if constexpr (i + 4 < KS) lds_read_b128<(2 + ((i + 4) >> 2)) * 128>(kf[i & 3], ka[i & 3]);
      });
    }

    // the V fragments of the first 16 keys start now: their LDS latency passes under the softmax arithmetic
    u32x2 vlo[DB], vhi[DB];
    const unsigned vb0 = tile + v_off;
    const unsigned va[2] = {vb0, vb0 ^ 64u};
    const unsigned vh[2] = {vb0 ^ 32u, vb0 ^ 96u};
    static_for<DB>([&](auto ic) {
      constexpr int d = decltype(ic)::value;
      lds_read_tr_b64<(d >> 1) * 128>(vlo[d], va[d & 1]);
      lds_read_tr_b64<(d >> 1) * 128 + 8 * ROWB>(vhi[d], vh[d & 1]);
    });

    // ---- causal mask + online softmax: lane = one query, keys key0 + 8 j + 4 hi + i at index 4 j + i ----
    if (key0 + PF_TOK - 1 > qbase) {         // the tile reaches past this wave's first query
      const int query = qbase + n32;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (key0 + 8 * (i >> 2) + 4 * hi + (i & 3) > query) sc[i] = -INFINITY;
    }
    float mx = sc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sc[i]);
    mx *= a.scale_log2;
    if (__any(mx > m_run + LAZY)) {
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile
      lsum *= alpha;
      m_run = m_new;
#pragma unroll
      for (int d = 0; d < DB; ++d) acc[d] *= alpha;
    }
    bf16x8 pb[2];
#pragma unroll
    for (int i = 0; i < 16; ++i)
      pb[i >> 3][i & 7] = (bf16_t)__builtin_amdgcn_exp2f(fmaf(sc[i], a.scale_log2, -m_run));

    // ---- output: O^T += V^T P^T, 16 keys per step; the second step's fragments refill the ring ----
    static_for<DB>([&](auto ic) {
      constexpr int d = decltype(ic)::value;
      lds_wait<6>(vlo[d], vhi[d]);           // fragments d+1.. of this step and 0..d-1 of the next stay in flight
      const u32x4 v4 = {vlo[d][0], vlo[d][1], vhi[d][0], vhi[d][1]};
      acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v4), pb[0], acc[d], 0, 0, 0);
      lds_read_tr_b64<(d >> 1) * 128 + 16 * ROWB>(vlo[d], va[d & 1]);
      lds_read_tr_b64<(d >> 1) * 128 + 24 * ROWB>(vhi[d], vh[d & 1]);
    });
    static_for<DB>([&](auto ic) {
      constexpr int d = decltype(ic)::value;
      lds_wait<2 * (DB - 1 - d)>(vlo[d], vhi[d]);
      const u32x4 v4 = {vlo[d][0], vlo[d][1], vhi[d][0], vhi[d][1]};
      acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v4), pb[1], acc[d], 0, 0, 0);
    });
    const u32x4 one4 = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    lsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, one4), pb[0], lsum, 0, 0, 0);
    lsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, one4), pb[1], lsum, 0, 0, 0);
  }

  // ---- normalise and store: lane holds query qbase + n32, dims 32 d + 8 j + 4 hi .. +3 at index 4 j .. ----
  const float l_tot = lsum[0];
  const int query = qbase + n32;
  if (query < L) {
    const float inv = 1.0f / l_tot;
    float* po = a.o + ((size_t)(t0 + query) * a.H + h) * 128 + 4 * hi;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 v = {acc[d][4 * j] * inv, acc[d][4 * j + 1] * inv, acc[d][4 * j + 2] * inv, acc[d][4 * j + 3] * inv};
        *reinterpret_cast<f32x4*>(po + 32 * d + 8 * j) = v;
      }
  }
}

bool prefill_mfma_supported(const tpla_shape_t& sh) {
  return sh.dtype == TPLA_BF16 && sh.d_n == 128 && sh.d_v == 128 && sh.d_r == 64 && sh.d_c % 128 == 0 &&
         sh.d_c <= 512;
}

int launch_prefill_attention(const tpla_shape_t& sh, const void* q_nope, const void* q_pe, const void* c,
                             const void* k_pe, const void* W_UK, const void* W_UV, const int32_t* cu_seqlens,
                             int T, int max_seq_len, void* kv_workspace, float* o, hipStream_t st) {
  // 1. values and no-RoPE keys of every (token, head)
  const size_t smem = (size_t)(sh.d_c / 32) * 512 * 16;
  static std::mutex mu;
  static bool opted_in[16] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(TPLA_ERR_HIP, "hipGetDevice failed");
  if (smem > 64 * 1024) {
    std::lock_guard<std::mutex> lock(mu);
    if (!opted_in[dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kv_project_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) {
        (void)hipGetLastError();
        return fail(TPLA_ERR_HIP, "cannot reserve 128 KiB of LDS for prefill_kv_project_kernel");
      }
      opted_in[dev] = true;
    }
  }
  const int n_blocks = (T + PJ_ROWS - 1) / PJ_ROWS;
  int workers = (device_cu_count() + 2 * sh.H - 1) / (2 * sh.H);
  workers = std::max(1, std::min(workers, n_blocks));
  hipLaunchKernelGGL(prefill_kv_project_kernel, dim3(2 * sh.H, workers), dim3(PJ_WAVES * 64), smem, st,
                     static_cast<const bf16_t*>(c), static_cast<const bf16_t*>(W_UK),
                     static_cast<const bf16_t*>(W_UV), static_cast<bf16_t*>(kv_workspace), T, sh.H, sh.d_c);
  int rc = check_launch("prefill_kv_project_kernel");
  if (rc) return rc;
  // 2. causal attention
  PrefillArgs a;
  a.q_nope = static_cast<const bf16_t*>(q_nope);
  a.q_pe = static_cast<const bf16_t*>(q_pe);
  a.kv = static_cast<const bf16_t*>(kv_workspace);
  a.k_pe = static_cast<const bf16_t*>(k_pe);
  a.cu = cu_seqlens;
  a.o = o;
  a.H = sh.H;
  a.T = T;
  a.scale_log2 = sh.sm_scale * 1.4426950408889634f;
  a.n_qt = (max_seq_len + PF_QT - 1) / PF_QT;
  a.head_group = sh.H % 8 == 0 ? 8 : (sh.H % 4 == 0 ? 4 : (sh.H % 2 == 0 ? 2 : 1));
  if ((long long)a.n_qt * sh.H > 2147483647LL) return fail(TPLA_ERR_UNSUPPORTED, "grid too large");
  const dim3 grid((unsigned)(a.n_qt * sh.H), sh.B);
  // -DTPLA_PREFILL32 selects the 32-queries-per-wave kernel (same results to rounding order; measured slower)
#ifdef TPLA_PREFILL32
  hipLaunchKernelGGL(prefill_attention_mfma32_kernel, grid, dim3(PF_NW * 64), PF_NSTAGE * PF_TILE_BYTES, st, a);
#else
  hipLaunchKernelGGL(prefill_attention_mfma_kernel, grid, dim3(PF_NW * 64), PF_NSTAGE * PF_TILE_BYTES, st, a);
#endif
  return check_launch("prefill_attention_mfma_kernel");
}

}  // namespace tpla
