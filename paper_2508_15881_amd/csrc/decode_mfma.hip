// bf16 shard decode on the matrix cores (gfx950).
//
// A workgroup processes work items: page ranges of one sequence of one latent
// slice, either a static chunk (decode_mfma_kernel) or whatever falls into
// its equal share of all pages (decode_mfma_balanced_kernel).  It walks an
// item's pages in tiles of TOK tokens.  A tile (TOK rows of d_c/g + d_r bf16, contiguous inside a page)
// goes straight from global memory into a ring of NSTAGE LDS buffers with
// 128-bit direct-to-LDS loads, two tiles ahead of the one being consumed, and
// is shared there by all heads.  Wave w owns heads [16w, 16w+16):
//   S^T[tok, head] = K[tok, :] . Q[head, :]      MFMA 16x16x32, M = tokens, N = heads
//   online softmax per head (a lane only ever sees one head)
//   O^T[dim, head] += V^T[dim, tok] . P^T[tok, head]   M = latent dims, N = heads
// The latent prefix of a row is both key and value, so the same LDS tile is
// read row-wise for the scores and through the transposing LDS read for the
// output.  The S^T accumulator layout is already the B-operand layout of the
// second product once the token order inside a 32-token step is permuted
// identically for V^T, so P never leaves registers.
//
// LDS reads of the tiles are issued from inline assembly with hand-placed
// lgkmcnt waits: the compiler would otherwise make every LDS read wait for
// all outstanding direct-to-LDS loads, which would serialise the prefetch.
// The compiler takes the destination of such a read for valid from the moment
// it is issued: read, wait and first use must stay in straight-line code, or a
// register copy may land between the read and its wait.
//
// Three bodies for a work item: decode_item (16 heads per wave; the default),
// decode_item_shared (576-wide rows: two waves per 16 heads, scores handed
// over through LDS) and decode_item32 (32 heads per wave, build flag TPLA_H32).
#include <hip/hip_ext.h>
#include "lds_tile.h"

namespace tpla {

constexpr int PAGE_TOKENS = 64;
#ifndef TPLA_H32_STAGES
#define TPLA_H32_STAGES 4
#endif

// Measurement build only (-DTPLA_WG_TIMELINE, see bench.py --wg-timeline): every workgroup of the
// balanced kernel leaves four readings of the 100 MHz wall clock (start, first tile landed, tile loop
// done, end) and where it ran (XCC id and hardware id registers).  Nothing of this is compiled otherwise.
#ifdef TPLA_WG_TIMELINE
__device__ unsigned long long g_wg_times[4096 * 4];
__device__ unsigned g_wg_where[4096 * 2];
// per workgroup (wave 0) of the 32-heads-per-wave instances: shader clocks spent in the plain score product of
// an item's first tile, in waiting for / requesting tiles, in the score MFMAs with the previous tile's softmax
// issued between them, in the output MFMAs; and the number of tiles
__device__ unsigned long long g_wg_phase[4096 * 5];
#define TPLA_PH_CLK(x) do { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); x = clock64(); } while (0)
#define TPLA_TL_MARK(k) do { if (threadIdx.x == 0 && blockIdx.x < 4096) g_wg_times[blockIdx.x * 4 + (k)] = wall_clock64(); } while (0)
#define TPLA_TL_MARK_ONCE(k) do { if (threadIdx.x == 0 && blockIdx.x < 4096 && g_wg_times[blockIdx.x * 4 + (k)] == 0) g_wg_times[blockIdx.x * 4 + (k)] = wall_clock64(); } while (0)
#else
#define TPLA_TL_MARK(k) do { } while (0)
#define TPLA_TL_MARK_ONCE(k) do { } while (0)
#define TPLA_PH_CLK(x) do { } while (0)
#endif

// One work item: pages [p0, p1) of sequence b of slice `shard` (L tokens in
// the sequence, p1 <= its page count); the partial result goes to slot
// `slot` of the workspace.  Called by every thread of the workgroup.
template <int DL, int DR, int NW, int TOK, int NSTAGE, int KR>
__device__ __forceinline__ void decode_item(const DecodeArgs& a, u32x4* smem, int shard, int b, int L,
                                            int p0, int p1, size_t slot) {
  constexpr int RC = (DL + DR) / 8;      // 16-byte pieces per row
  constexpr int KS = (DL + DR) / 32;     // k-steps of the score product
  constexpr int DB = DL / 16;            // 16-wide blocks of latent dims
  constexpr int TB = TOK / 16;           // 16-token blocks per tile
  constexpr int S2 = TOK / 32;           // 32-token k-steps of the output product
  constexpr int TC = TOK * RC;           // pieces per tile
  constexpr int NI = TC / 64;            // direct-to-LDS instructions per tile
  constexpr int CPT = (NI + NW - 1) / NW;   // of which each wave issues this many
  constexpr int TPP = PAGE_TOKENS / TOK; // tiles per page
  constexpr int TILE_BYTES = TC * 16;
  static_assert(RC % 8 == 0, "row must be a multiple of 64 elements");
  static_assert(TOK % 32 == 0 && PAGE_TOKENS % TOK == 0 && TC % 64 == 0, "tile size");
  static_assert(NSTAGE >= 2 && NSTAGE <= 4, "the wait counts below cover one to three tiles in flight");
  constexpr int FL = NSTAGE - 1;         // tiles in flight
  static_assert(KR >= 4 && (KR & (KR - 1)) == 0 && KR <= 16, "fragment ring depth");

  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j16 = lane & 15, q4 = lane >> 4;
  const int vb = shard * a.B + b;
  // Page ids of this chunk live in a register, 64 pages at a time (lane i
  // holds page p0 + pg_base + i), and are read back with v_readlane: a memory
  // load per tile would have to wait for every direct-to-LDS load before it.
  int pg_reg = a.block_table[(size_t)b * a.max_pages + min(p0 + lane, p1 - 1)];
  asm volatile("" : "+v"(pg_reg));
  const int t_begin = p0 * PAGE_TOKENS;
  const int t_end = min(p1 * PAGE_TOKENS, L);
  const int ntiles = (t_end - t_begin + TOK - 1) / TOK;
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  const char* pool = static_cast<const char*>(a.pools[shard]);
  // the ring restarts at buffer 0: nobody may still be reading the previous item's tiles
  __syncthreads();

  // ---- direct-to-LDS bookkeeping ---------------------------------------------
  // Instruction k of a tile fills LDS pieces [64k, 64k+64).  This wave issues
  // k = wave + j*NW; when NI is not a multiple of NW the surplus instruction
  // repeats the wave's previous one (same data to the same place).
  int ld_tok[CPT];          // token row of the piece this lane fetches
  unsigned ld_goff[CPT];    // its byte offset inside the tile in global memory
  int ld_k[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    int k = wave + j * NW;
    if (k >= NI) k -= NW;
    const int x = k * 64 + lane;                 // LDS piece index
    const int tok = x / RC, cs = x % RC;         // swizzled position -> source piece
    ld_k[j] = k;
    ld_tok[j] = tok;
    ld_goff[j] = (unsigned)((tok * RC + (cs ^ swz(tok))) * 16);
  }
  int pg_base = 0;
  auto issue = [&](int t) {
    const int T = p0 * TPP + t;
    const int pg = t / TPP;                 // page of this chunk, uniform
    if (pg - pg_base >= 64) {
      pg_base += 64;
      pg_reg = bt[min(p0 + pg_base + lane, p1 - 1)];
      asm volatile("" : "+v"(pg_reg));      // the load's wait stays inside this branch
    }
    const int page = __builtin_amdgcn_readlane(pg_reg, pg - pg_base);
    const char* src = pool + (size_t)page * (PAGE_TOKENS * RC * 16) + (size_t)(T % TPP) * TILE_BYTES;
    const int valid = t_end - (t_begin + t * TOK);   // rows >= valid are not read
    char* dst = reinterpret_cast<char*>(smem) + (t % NSTAGE) * TILE_BYTES;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      // every lane issues (the wait counts rely on it); rows past the end of
      // the sequence fetch row 0 of the tile instead and are zeroed afterwards
      const unsigned off = (ld_tok[j] < valid) ? ld_goff[j] : (ld_goff[j] % (RC * 16));
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                       (__attribute__((address_space(3))) void*)(dst + ld_k[j] * 1024),
                                       16, 0, 2 /* streaming: do not keep in L2 */);
    }
  };

  // ---- per-lane LDS byte offsets -------------------------------------------
  // score product: token 16*tb + j16, piece 4*ks + q4
  const int xk = swz(j16);
  unsigned k_off[2];
  k_off[0] = (unsigned)((j16 * RC + ((q4) ^ xk)) * 16);
  k_off[1] = (unsigned)((j16 * RC + ((4 | q4) ^ xk)) * 16);
  // output product: token 4*q4 + (j16>>2) (+16), dims 16*db + 4*(j16&3) .. +4
  const int v_tok = 4 * q4 + (j16 >> 2);
  const int xv = swz(v_tok);
  const int cb = (j16 & 3) >> 1;
  unsigned v_off[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
    v_off[d] = (unsigned)((v_tok * RC + (((d << 1) | cb) ^ xv)) * 16 + (j16 & 1) * 8);

  f32x4 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  issue(0);
  if (FL >= 2 && ntiles > 1) issue(1);
  if (FL >= 3 && ntiles > 2) issue(2);

  // ---- this wave's 16 heads of the query, as B operands --------------------
  const int head = wave * 16 + j16;
  bf16x8 qreg[KS];
  {
    const bf16_t* ql = static_cast<const bf16_t*>(a.q_lat) + ((size_t)vb * a.H + head) * DL;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q_pe) + ((size_t)b * a.H + head) * DR;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 32 + q4 * 8;
      qreg[ks] = (k0 < DL) ? *reinterpret_cast<const bf16x8*>(ql + k0)
                           : *reinterpret_cast<const bf16x8*>(qp + (k0 - DL));
    }
    // complete these loads here: a wait left for their first use would sit
    // inside the tile loop and drain the prefetched tiles on every iteration
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));
  }


  for (int t = 0; t < ntiles; ++t) {
    // tile t has landed once only the loads of the tiles requested after it are outstanding
    {
      const int later = ntiles - 1 - t;      // tiles after t that exist (FL - 1 of them are in flight at most)
      if (FL >= 3 && later >= 2)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * CPT));
      else if (FL >= 2 && later >= 1)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(CPT));
      else
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    // all waves: tile t visible, tile t-1 no longer read.  A bare barrier:
    // __syncthreads() would add a fence that waits for the loads in flight.
    __builtin_amdgcn_s_barrier();
    if (t == 0) TPLA_TL_MARK_ONCE(1);
    if (t + FL < ntiles) issue(t + FL);
    const unsigned tile = lds_base + (unsigned)((t % NSTAGE) * TILE_BYTES);
    const int valid = t_end - (t_begin + t * TOK);
    if (valid < TOK) {
      // last, partial tile: clear the rows past the end of the sequence so
      // that whatever the pool holds there can never reach the accumulators
      u32x4* tl = smem + (t % NSTAGE) * TC;
      for (int x = tid; x < TC; x += NW * 64)
        if (x / RC >= valid) tl[x] = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }

    // ---- scores: a ring of 4 K fragments ahead of the MFMAs -------------------
    f32x4 sacc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) sacc[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
      constexpr int NQ = KS * TB;          // MFMAs, in order (ks, tb)
      bf16x8 kf[KR];
      const unsigned ka[2] = {tile + k_off[0], tile + k_off[1]};
      static_for<KR>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int ks = i / TB, tb = i % TB;
        lds_read_b128<(ks >> 1) * 128 + tb * (16 * RC * 16)>(kf[i], ka[ks & 1]);
      });
      static_for<NQ>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        constexpr int ks = i / TB, tb = i % TB;
        constexpr int ahead = (NQ - 1 - i) < KR - 1 ? (NQ - 1 - i) : KR - 1;
        lds_wait<ahead>(kf[i & (KR - 1)]);
        sacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i & (KR - 1)], qreg[ks], sacc[tb], 0, 0, 0);
        if constexpr (i + KR < NQ) {
          constexpr int ks2 = (i + KR) / TB, tb2 = (i + KR) % TB;
          lds_read_b128<(ks2 >> 1) * 128 + tb2 * (16 * RC * 16)>(kf[i & (KR - 1)], ka[ks2 & 1]);
        }
      });
    }

    // ---- online softmax (lane = one head; tokens 16*tb + 4*q4 + i) ----------
    // The reference m_run of the exponentials is only moved when some score
    // exceeds it by more than LAZY (weights stay <= 2^LAZY, harmless in
    // float), so the accumulator rescale is off the common path.
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

    // ---- output: O^T += V^T P^T, a ring of 4 V fragments ---------------------
#pragma unroll
    for (int s2 = 0; s2 < S2; ++s2) {
      bf16x8 pb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pb[i] = (bf16_t)sacc[2 * s2][i];
        pb[4 + i] = (bf16_t)sacc[2 * s2 + 1][i];
      }
      constexpr int VR = KR <= 8 ? KR : 8;     // two reads per fragment: the wait counter allows 15 outstanding
      u32x2 vlo[VR], vhi[VR];
      unsigned va[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) va[d] = tile + v_off[d] + (unsigned)(s2 * (32 * RC * 16));
      static_for<VR>([&](auto ic) {
        constexpr int d = decltype(ic)::value;
        lds_read_tr_b64<(d >> 2) * 128>(vlo[d], va[d & 3]);
        lds_read_tr_b64<(d >> 2) * 128 + 16 * RC * 16>(vhi[d], va[d & 3]);
      });
      static_for<DB>([&](auto ic) {
        constexpr int d = decltype(ic)::value;
        constexpr int ahead = (DB - 1 - d) < VR - 1 ? (DB - 1 - d) : VR - 1;
        lds_wait<2 * ahead>(vlo[d & (VR - 1)], vhi[d & (VR - 1)]);
        const u32x4 v4 = {vlo[d & (VR - 1)][0], vlo[d & (VR - 1)][1], vhi[d & (VR - 1)][0], vhi[d & (VR - 1)][1]};
        acc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v4), pb, acc[d], 0, 0, 0);
        if constexpr (d + VR < DB) {
          constexpr int d2 = d + VR;
          lds_read_tr_b64<(d2 >> 2) * 128>(vlo[d & (VR - 1)], va[d2 & 3]);
          lds_read_tr_b64<(d2 >> 2) * 128 + 16 * RC * 16>(vhi[d & (VR - 1)], va[d2 & 3]);
        }
      });
    }
    }

  TPLA_TL_MARK(2);
  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  const size_t item = slot * a.H + head;
  float* pacc = a.part_acc + item * DL + 4 * q4;
#pragma unroll
  for (int d = 0; d < DB; ++d) *reinterpret_cast<f32x4*>(pacc + 16 * d) = acc[d];
  if (q4 == 0) {
    a.part_ml[item * 2 + 0] = m_run;
    a.part_ml[item * 2 + 1] = l_tot;
  }
}

// The same work item for rows too wide for two workgroups per compute unit (576-wide rows: one tile is
// 36 KB), where decode_item would leave every SIMD with a single wave and nothing to run under its MFMAs.
// Two waves share 16 heads.  Of a 32-token tile each computes the scores of 16 tokens (half the score
// MFMAs) and hands them to its partner through LDS; both then run the same softmax on all 32 tokens --
// same inputs, same operations, so their running reference and sum stay equal bit for bit -- and each
// multiplies the weights into its own half of the latent dims (half the output MFMAs, 64 accumulator
// registers instead of 128, which is what lets two waves share a SIMD).  The hand-over would cost a
// second barrier per tile; instead the loop is skewed by one tile: round r computes the scores of tile r
// and the softmax and output product of tile r - 1, and the round's one barrier publishes the tile and
// the partner's scores together.  Ring: tiles r - 1 and r in use, r + 1 and r + 2 in flight.
// LDS: NSTAGE tiles, then two buffers of one f32x4 per lane of every wave for the scores.
template <int DL, int DR, int NW, int TOK, int NSTAGE, int KR>
__device__ __forceinline__ void decode_item_shared(const DecodeArgs& a, u32x4* smem, int shard, int b, int L,
                                                   int p0, int p1, size_t slot) {
  constexpr int RC = (DL + DR) / 8;      // 16-byte pieces per row
  constexpr int KS = (DL + DR) / 32;     // k-steps of the score product
  constexpr int DBH = DL / 32;           // 16-wide blocks of this wave's half of the latent dims
  constexpr int TC = TOK * RC;           // pieces per tile
  constexpr int NI = TC / 64;            // direct-to-LDS instructions per tile
  constexpr int NWT = 2 * NW;            // waves in the workgroup
  constexpr int CPT = (NI + NWT - 1) / NWT;
  constexpr int TPP = PAGE_TOKENS / TOK;
  constexpr int TILE_BYTES = TC * 16;
  constexpr int VR = 4;                  // V fragments in flight
  static_assert(TOK == 32 && NSTAGE == 4, "two tiles in use, two in flight");
  static_assert(RC % 8 == 0 && TC % 64 == 0 && DBH % VR == 0, "tile shape");
  static_assert(KR >= 4 && (KR & (KR - 1)) == 0 && KR <= 16, "fragment ring depth");

  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int half = wv / NW, wave = wv % NW;      // half 0: tokens 0-15 and the first DL/2 dims; wave: heads 16 wave ..
  const int partner = (1 - half) * NW + wave;
  const int j16 = lane & 15, q4 = lane >> 4;
  const int vb = shard * a.B + b;
  int pg_reg = a.block_table[(size_t)b * a.max_pages + min(p0 + lane, p1 - 1)];
  asm volatile("" : "+v"(pg_reg));
  const int t_begin = p0 * PAGE_TOKENS;
  const int t_end = min(p1 * PAGE_TOKENS, L);
  // scalar: the rounds below branch on it, and a branch the compiler takes for divergent would put
  // register copies between an LDS read in assembly and the wait that makes its result valid
  const int ntiles = __builtin_amdgcn_readfirstlane((t_end - t_begin + TOK - 1) / TOK);
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  const char* pool = static_cast<const char*>(a.pools[shard]);
  // the ring and the score buffers restart: nobody may still be reading the previous item's
  __syncthreads();

  // ---- direct-to-LDS bookkeeping (as in decode_item, over all waves of the workgroup) ----
  int ld_tok[CPT];
  unsigned ld_goff[CPT];
  int ld_k[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    int k = wv + j * NWT;
    if (k >= NI) k -= NWT;                       // surplus instruction: repeats the wave's previous one
    const int x = k * 64 + lane;
    const int tok = x / RC, cs = x % RC;
    ld_k[j] = k;
    ld_tok[j] = tok;
    ld_goff[j] = (unsigned)((tok * RC + (cs ^ swz(tok))) * 16);
  }
  int pg_base = 0;
  auto issue = [&](int t) {
    const int T = p0 * TPP + t;
    const int pg = t / TPP;
    if (pg - pg_base >= 64) {
      pg_base += 64;
      pg_reg = bt[min(p0 + pg_base + lane, p1 - 1)];
      asm volatile("" : "+v"(pg_reg));
    }
    const int page = __builtin_amdgcn_readlane(pg_reg, pg - pg_base);
    const char* src = pool + (size_t)page * (PAGE_TOKENS * RC * 16) + (size_t)(T % TPP) * TILE_BYTES;
    const int valid = t_end - (t_begin + t * TOK);
    char* dst = reinterpret_cast<char*>(smem) + (t % NSTAGE) * TILE_BYTES;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const unsigned off = (ld_tok[j] < valid) ? ld_goff[j] : (ld_goff[j] % (RC * 16));
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                       (__attribute__((address_space(3))) void*)(dst + ld_k[j] * 1024),
                                       16, 0, 2 /* streaming: do not keep in L2 */);
    }
  };
  // rows of a tile past the end of the sequence are cleared once it has landed (the last tile only)
  auto clear_tail = [&](int t) {
    const int valid = t_end - (t_begin + t * TOK);
    if (valid < TOK) {
      u32x4* tl = smem + (t % NSTAGE) * TC;
      for (int x = tid; x < TC; x += NWT * 64)
        if (x / RC >= valid) tl[x] = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }
  };

  // ---- per-lane LDS byte offsets ----
  // score product: token 16 half + j16, piece 4 ks + q4
  const int k_tok = 16 * half + j16;
  const int xk = swz(k_tok);
  unsigned k_off[2];
  k_off[0] = (unsigned)((k_tok * RC + ((q4) ^ xk)) * 16);
  k_off[1] = (unsigned)((k_tok * RC + ((4 | q4) ^ xk)) * 16);
  // output product: token 4 q4 + (j16 >> 2) (+16), dims (DL / 2) half + 16 d + 4 (j16 & 3) .. +4
  const int v_tok = 4 * q4 + (j16 >> 2);
  const int xv = swz(v_tok);
  const int cb = (j16 & 3) >> 1;
  unsigned v_off[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
    v_off[d] = (unsigned)((v_tok * RC + (((d << 1) | cb) ^ xv)) * 16 + (j16 & 1) * 8 + half * DL);   // DL bytes = DL / 2 dims

  f32x4 acc[DBH];
#pragma unroll
  for (int d = 0; d < DBH; ++d) acc[d] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  issue(0);
  if (ntiles > 1) issue(1);

  // ---- the 16 heads of this wave pair, as B operands ----
  const int head = wave * 16 + j16;
  bf16x8 qreg[KS];
  {
    const bf16_t* ql = static_cast<const bf16_t*>(a.q_lat) + ((size_t)vb * a.H + head) * DL;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q_pe) + ((size_t)b * a.H + head) * DR;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 32 + q4 * 8;
      qreg[ks] = (k0 < DL) ? *reinterpret_cast<const bf16x8*>(ql + k0)
                           : *reinterpret_cast<const bf16x8*>(qp + (k0 - DL));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));   // complete before the loop
  }

  // scores of this wave's 16 tokens of the tile at LDS address `tile`
  auto scores = [&](unsigned tile) {
    f32x4 sc = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 kf[KR];
    const unsigned ka[2] = {tile + k_off[0], tile + k_off[1]};
    static_for<KR>([&](auto ic) {
      constexpr int ks = decltype(ic)::value;
      lds_read_b128<(ks >> 1) * 128>(kf[ks], ka[ks & 1]);
    });
    static_for<KS>([&](auto ic) {
      constexpr int ks = decltype(ic)::value;
      constexpr int ahead = (KS - 1 - ks) < KR - 1 ? (KS - 1 - ks) : KR - 1;
      lds_wait<ahead>(kf[ks & (KR - 1)]);
      sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks & (KR - 1)], qreg[ks], sc, 0, 0, 0);
      if constexpr (ks + KR < KS) lds_read_b128<((ks + KR) >> 1) * 128>(kf[ks & (KR - 1)], ka[(ks + KR) & 1]);
    });
    return sc;
  };

  // ---- round 0: the scores of tile 0 ----
  if (ntiles > 1)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(CPT));
  else
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __builtin_amdgcn_s_barrier();
  TPLA_TL_MARK_ONCE(1);
  if (ntiles > 2) issue(2);
  clear_tail(0);
  // The hand-over is written with a plain store (the compiler then keeps the wait states an MFMA result
  // needs before an LDS instruction may read it) and read with inline assembly like the tiles (a plain
  // LDS load after a direct-to-LDS load would make the compiler wait for every load in flight).
  f32x4* x_own = reinterpret_cast<f32x4*>(smem + NSTAGE * TC) + wv * 64 + lane;
  const unsigned x_partner = lds_base + (unsigned)(NSTAGE * TILE_BYTES + (partner * 64 + lane) * 16);
  constexpr unsigned XBUF = NWT * 64 * 16;       // bytes per hand-over buffer
  f32x4 s_own = scores(lds_base);
  x_own[0] = s_own;

  // ---- round r: scores of tile r (while there is one), softmax and output product of tile r - 1 ----
  for (int r = 1; r <= ntiles; ++r) {
    const bool more = r < ntiles;
    // tile r has landed once only tile r + 1 (requested in the round before) is outstanding
    if (r + 1 < ntiles)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(CPT));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    // the hand-over written in round r - 1 must have left this wave before the barrier publishes it
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();        // tile r and the partners' scores of tile r - 1 visible; tile r - 2 no longer read
    if (r + 2 < ntiles) issue(r + 2);
    if (more) clear_tail(r);
    const f32x4 s_prev = s_own;
    f32x4 s_partner;
    asm volatile("ds_read_b128 %0, %1" : "=v"(s_partner) : "v"(x_partner + ((r - 1) & 1) * XBUF) : "memory");
    if (more) {
      s_own = scores(lds_base + (unsigned)((r % NSTAGE) * TILE_BYTES));
      x_own[(r & 1) * (XBUF / 16)] = s_own;
    }
    // one wait on one path for both cases, straight after the branch (which does not touch s_partner)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(s_partner) : : "memory");
    const unsigned tile = lds_base + (unsigned)(((r - 1) % NSTAGE) * TILE_BYTES);
    const int valid = t_end - (t_begin + (r - 1) * TOK);

    // the first V fragments start now, under the softmax arithmetic
    u32x2 vlo[VR], vhi[VR];
    unsigned va[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) va[d] = tile + v_off[d];
    static_for<VR>([&](auto ic) {
      constexpr int d = decltype(ic)::value;
      lds_read_tr_b64<(d >> 2) * 128>(vlo[d], va[d & 3]);
      lds_read_tr_b64<(d >> 2) * 128 + 16 * RC * 16>(vhi[d], va[d & 3]);
    });

    // ---- online softmax on all 32 tokens (lane = one head; tokens 16 tb + 4 q4 + i) ----
    f32x4 sacc[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sacc[0][i] = half ? s_partner[i] : s_prev[i];
      sacc[1][i] = half ? s_prev[i] : s_partner[i];
    }
    if (valid < TOK) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (16 * tb + 4 * q4 + i >= valid) sacc[tb][i] = -INFINITY;
    }
    float mx = sacc[0][0];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
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
      for (int d = 0; d < DBH; ++d) acc[d] *= alpha;
    }
    float psum = 0.f;
    bf16x8 pb;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[tb][i], a.scale_log2, -m_run));
        psum += p;
        pb[4 * tb + i] = (bf16_t)p;
      }
    l_run += psum;

    // ---- output: O^T += V^T P^T over this wave's half of the dims ----
    static_for<DBH>([&](auto ic) {
      constexpr int d = decltype(ic)::value;
      constexpr int ahead = (DBH - 1 - d) < VR - 1 ? (DBH - 1 - d) : VR - 1;
      lds_wait<2 * ahead>(vlo[d & (VR - 1)], vhi[d & (VR - 1)]);
      const u32x4 v4 = {vlo[d & (VR - 1)][0], vlo[d & (VR - 1)][1], vhi[d & (VR - 1)][0], vhi[d & (VR - 1)][1]};
      acc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v4), pb, acc[d], 0, 0, 0);
      if constexpr (d + VR < DBH) {
        constexpr int d2 = d + VR;
        lds_read_tr_b64<(d2 >> 2) * 128>(vlo[d & (VR - 1)], va[d2 & 3]);
        lds_read_tr_b64<(d2 >> 2) * 128 + 16 * RC * 16>(vhi[d & (VR - 1)], va[d2 & 3]);
      }
    });
  }

  TPLA_TL_MARK(2);
  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  const size_t item = slot * a.H + head;
  float* pacc = a.part_acc + item * DL + (DL / 2) * half + 4 * q4;
#pragma unroll
  for (int d = 0; d < DBH; ++d) *reinterpret_cast<f32x4*>(pacc + 16 * d) = acc[d];
  if (q4 == 0 && half == 0) {
    a.part_ml[item * 2 + 0] = m_run;
    a.part_ml[item * 2 + 1] = l_tot;
  }
}

// The same work item with 32 heads per wave on 32x32x16 MFMAs.  Every K and V
// fragment read from LDS then serves twice as many heads: half the LDS reads,
// half the MFMA issues and half the operand fetches per cache byte.  The price
// is one wave per SIMD (128 accumulator + 80 query registers for 256-wide
// slices), so nothing else hides a wave's softmax arithmetic: the loop is
// software-pipelined instead.  While tile t+1's score MFMAs run (32 cycles of
// the matrix core each, 8 of the issue port), the wave issues tile t's softmax
// in their shadow, a few instructions after every MFMA:
//   S^T[tok, head] = K[tok, :] . Q[head, :]     M = 32 tokens, N = 32 heads, 16 k per MFMA
//   O^T[dim, head] += V^T[dim, tok] . P^T[tok, head]   M = 32 latent dims, N = 32 heads, 16 tokens per MFMA
// Lane l holds head l % 32; accumulator element i of a 32x32 result is row
// 8 (i / 4) + 4 (l / 32) + i % 4.  For the second product the 16 tokens of a
// k-step are taken in the order in which the score accumulator already holds
// them (k index 8 (l / 32) + e  <->  token 8 (e / 4) + 4 (l / 32) + e % 4 of the
// step), so elements 8 s .. 8 s + 7 of the exponentiated scores are the B
// operand of step s as they stand, and V^T is fetched with two transposing
// reads per fragment (tokens +0..3 and +8..11 of the lane's half).
template <int DL, int DR, int NW, int TOK, int NSTAGE>
__device__ __forceinline__ void decode_item32(const DecodeArgs& a, u32x4* smem, int shard, int b, int L,
                                              int p0, int p1, size_t slot) {
  constexpr int RC = (DL + DR) / 8;      // 16-byte pieces per row
  constexpr int KS = (DL + DR) / 16;     // 16-wide k-steps of the score product
  constexpr int DB = DL / 32;            // 32-wide blocks of latent dims
  constexpr int TC = TOK * RC;           // pieces per tile
  constexpr int NI = TC / 64;            // direct-to-LDS instructions per tile
  constexpr int CPT = (NI + NW - 1) / NW;   // of which each wave issues this many
  constexpr int TPP = PAGE_TOKENS / TOK; // tiles per page
  constexpr int TILE_BYTES = TC * 16;
  constexpr int ROWB = RC * 16;          // bytes per row
  constexpr int FL = NSTAGE - 2;         // tiles in flight: tiles t (values) and t+1 (keys) are both in use
  constexpr int KS1 = 6;                 // score MFMAs issued before the rescale decision
  static_assert(RC % 8 == 0, "row must be a multiple of 64 elements");
  static_assert(TOK == 32 && TC % 64 == 0, "one 32-token score block per tile");
  static_assert(TILE_BYTES % 4096 == 0, "tile bases must leave address bits 5..11 to the lane offsets");
  static_assert(FL == 1 || FL == 2, "one or two tiles in flight");
  static_assert(2 * CPT < 64, "vmcnt");
  static_assert(KS >= KS1 + 4 && KS1 >= 5 && DB >= 4, "pipeline chunking");

  const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n32 = lane & 31, hi = lane >> 5;
  const int vb = shard * a.B + b;
  int pg_reg = a.block_table[(size_t)b * a.max_pages + min(p0 + lane, p1 - 1)];
  asm volatile("" : "+v"(pg_reg));
  const int t_begin = p0 * PAGE_TOKENS;
  const int t_end = min(p1 * PAGE_TOKENS, L);
  const int ntiles = (t_end - t_begin + TOK - 1) / TOK;
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  const char* pool = static_cast<const char*>(a.pools[shard]);
  __syncthreads();      // the ring restarts at buffer 0: nobody may still be reading the previous item's tiles

  // ---- direct-to-LDS bookkeeping (as in decode_item) ------------------------
  int ld_tok[CPT];
  unsigned ld_goff[CPT];
  int ld_k[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    int k = wave + j * NW;
    if (k >= NI) k -= NW;
    const int x = k * 64 + lane;
    const int tok = x / RC, cs = x % RC;
    ld_k[j] = k;
    ld_tok[j] = tok;
    ld_goff[j] = (unsigned)((tok * RC + (cs ^ swz32(tok))) * 16);
  }
  int pg_base = 0;
  auto issue = [&](int t) {
    const int T = p0 * TPP + t;
    const int pg = t / TPP;
    if (pg - pg_base >= 64) {
      pg_base += 64;
      pg_reg = bt[min(p0 + pg_base + lane, p1 - 1)];
      asm volatile("" : "+v"(pg_reg));
    }
    const int page = __builtin_amdgcn_readlane(pg_reg, pg - pg_base);
    const char* src = pool + (size_t)page * (PAGE_TOKENS * ROWB) + (size_t)(T % TPP) * TILE_BYTES;
    const int valid = t_end - (t_begin + t * TOK);
    char* dst = reinterpret_cast<char*>(smem) + (t % NSTAGE) * TILE_BYTES;
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const unsigned off = (ld_tok[j] < valid) ? ld_goff[j] : (ld_goff[j] % ROWB);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                       (__attribute__((address_space(3))) void*)(dst + ld_k[j] * 1024),
                                       16, 0, 2 /* streaming: do not keep in L2 */);
    }
  };
  // rows of the last tile that lie past the end of the sequence are cleared once it has landed
  auto clear_tail = [&](int t) {
    const int valid = t_end - (t_begin + t * TOK);
    if (valid < TOK) {
      u32x4* tl = smem + (t % NSTAGE) * TC;
      for (int x = tid; x < TC; x += NW * 64)
        if (x / RC >= valid) tl[x] = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }
  };

  // ---- per-lane LDS byte offsets --------------------------------------------
  // score product: token n32, piece 2 ks + hi = 8 (ks / 4) + (2 (ks % 4) | hi); the swizzle only
  // touches the low three bits of the piece index, and (2 j | hi) ^ x = (hi ^ x) ^ 2 j, so the
  // offsets of ks % 4 = 1, 2, 3 are that of 0 with address bits 5 and 6 flipped
  const unsigned k_off = (unsigned)(n32 * ROWB + ((hi ^ swz32(n32)) * 16));
  // output product: 16-lane group gq = (hi, dim half); lane j of it points at token 4 hi + j / 4 of the
  // k-step and dims 32 db + 16 half + 4 (j % 4) .. +3, i.e. piece 4 db + 2 half + (j % 4) / 2
  // (db odd: address bit 6 flipped; tokens + 8: swz32 changes by 2, address bit 5 flipped)
  const int j16 = lane & 15, half = (lane >> 4) & 1;
  const int v_tok = 4 * hi + (j16 >> 2);
  const int pl = 2 * half + ((j16 & 3) >> 1);
  const unsigned v_off = (unsigned)(v_tok * ROWB + ((pl ^ swz32(v_tok)) * 16) + (j16 & 1) * 8);

  f32x16 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[d][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  issue(0);
  if (ntiles > 1) issue(1);
  if (FL >= 2 && ntiles > 2) issue(2);

  // ---- this wave's 32 heads of the query, as B operands ----------------------
  const int head = wave * 32 + n32;
  bf16x8 qreg[KS];
  {
    const bf16_t* ql = static_cast<const bf16_t*>(a.q_lat) + ((size_t)vb * a.H + head) * DL;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q_pe) + ((size_t)b * a.H + head) * DR;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k0 = ks * 16 + hi * 8;
      qreg[ks] = (k0 < DL) ? *reinterpret_cast<const bf16x8*>(ql + k0)
                           : *reinterpret_cast<const bf16x8*>(qp + (k0 - DL));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));   // complete before the loop
  }

  // Score MFMAs FIRST .. LAST-1 of the tile at LDS address `tile` into two independent chains (even and
  // odd k-steps), a ring of 4 K fragments ahead; `between(i)` is called after MFMA i has been issued.
  bf16x8 kf[4];
  f32x16 sA, sB;
  auto score_reads_begin = [&](unsigned tile) {
    const unsigned kb = tile + k_off;
    const unsigned ka[4] = {kb, kb ^ 32u, kb ^ 64u, kb ^ 96u};
    static_for<4>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      lds_read_b128<(i >> 2) * 128>(kf[i], ka[i & 3]);
    });
  };
  auto score_mfmas = [&](unsigned tile, auto first_c, auto last_c, auto&& between) {
    constexpr int FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
    const unsigned kb = tile + k_off;
    const unsigned ka[4] = {kb, kb ^ 32u, kb ^ 64u, kb ^ 96u};
    static_for<LAST - FIRST>([&](auto ic) {
      constexpr int i = FIRST + decltype(ic)::value;
      constexpr int ahead = (KS - 1 - i) < 3 ? (KS - 1 - i) : 3;
      lds_wait<ahead>(kf[i & 3]);
      if constexpr (i & 1)
        sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qreg[i], sB, 0, 0, 0);
      else
        sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qreg[i], sA, 0, 0, 0);
      if constexpr (i + 4 < KS) lds_read_b128<((i + 4) >> 2) * 128>(kf[i & 3], ka[i & 3]);
      between(ic);
      __builtin_amdgcn_sched_barrier(0);       // keep the arithmetic of this step in this MFMA's shadow
    });
  };
  auto zero_scores = [&]() {
#pragma unroll
    for (int i = 0; i < 16; ++i) sA[i] = sB[i] = 0.f;
  };
  auto nothing = [](auto) {};
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, KS1>;
  using C2 = std::integral_constant<int, KS>;

  // ---- prologue: tile 0 has landed; its scores -----------------------------------
  if (FL >= 2 && ntiles > 2)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * CPT));
  else if (ntiles > 1)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(CPT));
  else
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __builtin_amdgcn_s_barrier();
  clear_tail(0);
  float s_cur[16];
  [[maybe_unused]] unsigned long long ph[5] = {0, 0, 0, 0, 0}, c0 = 0, c1 = 0, c2 = 0, c3 = 0;
  TPLA_TL_MARK_ONCE(1);
  {
    TPLA_PH_CLK(c0);
    zero_scores();
    score_reads_begin(lds_base);
    score_mfmas(lds_base, C0{}, C2{}, nothing);
#pragma unroll
    for (int i = 0; i < 16; ++i) s_cur[i] = sA[i] + sB[i];
    TPLA_PH_CLK(c1);
    ph[0] += c1 - c0;
  }

  // The accumulators sit in the accumulation registers, which only MFMAs write: rescaling them means
  // copying all 128 out and back.  So the tile loop itself never rescales: when a tile's scores exceed
  // the reference by more than LAZY it stops before using them, the (rare) rescale runs outside, and
  // the loop resumes at the same tile (the score MFMAs of the next tile that were under way start over).
  int t = 0;
  bool resumed = false;      // tile t + 1 has already been waited for
  while (t < ntiles) {
    float m_pending = m_run;
    bool rescale = false;
    for (; t < ntiles; ++t) {
      const bool has_next = t + 1 < ntiles;
      TPLA_PH_CLK(c0);
      if (has_next && !resumed) {
        // tile t + 1 has landed once only the tiles requested after it are outstanding
        if (FL >= 2 && t + 2 < ntiles)
          __builtin_amdgcn_s_waitcnt(vmcnt_imm(CPT));
        else
          __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __builtin_amdgcn_s_barrier();          // tile t + 1 visible to all waves, tile t - 1 no longer read
        if (t + 1 + FL < ntiles) issue(t + 1 + FL);
        clear_tail(t + 1);
      }
      resumed = false;
      TPLA_PH_CLK(c1);
      const unsigned tile = lds_base + (unsigned)((t % NSTAGE) * TILE_BYTES);
      // the last tile has no successor: its own keys are multiplied once more and the result dropped
      const unsigned tile_next = lds_base + (unsigned)(((has_next ? t + 1 : t) % NSTAGE) * TILE_BYTES);
      const int valid = t_end - (t_begin + t * TOK);

      // ---- first score MFMAs of tile t + 1; in their shadow: the maximum of tile t's scores ----
      if (valid < TOK) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (8 * (i >> 2) + 4 * hi + (i & 3) >= valid) s_cur[i] = -INFINITY;
      }
      zero_scores();
      score_reads_begin(tile_next);
      float m4[4], mx = 0.f;
      score_mfmas(tile_next, C0{}, C1{}, [&](auto ic) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i < 4) m4[i] = fmaxf(fmaxf(s_cur[4 * i], s_cur[4 * i + 1]), fmaxf(s_cur[4 * i + 2], s_cur[4 * i + 3]));
        if constexpr (i == 4) mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3])) * a.scale_log2;
      });
      if (__any(mx > m_run + LAZY)) {
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (t == 0) {
          m_run = fmaxf(m_run, mx);      // first tile of the item: nothing accumulated yet, nothing to rescale
        } else {
          m_pending = fmaxf(m_run, mx);
          rescale = true;
          resumed = true;
          break;
        }
      }

      // ---- the other score MFMAs of tile t + 1; in their shadow: tile t's exponentials ----
      float psum = 0.f;
      bf16x8 pb[2];
      score_mfmas(tile_next, C1{}, C2{}, [&](auto ic) {
        constexpr int i = decltype(ic)::value;      // 0 .. KS - KS1 - 1: the 16 scores dealt over these steps
        constexpr int per = (16 + (KS - KS1) - 1) / (KS - KS1);
#pragma unroll
        for (int e = per * i; e < per * (i + 1) && e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s_cur[e], a.scale_log2, -m_run));
          psum += p;
          pb[e >> 3][e & 7] = (bf16_t)p;
        }
      });
      l_run += psum;
      TPLA_PH_CLK(c2);

      // ---- output: O^T += V^T P^T of tile t, a ring of 4 V fragments; in its shadow the new scores
      //      leave the accumulation registers ----
      static_for<2>([&](auto sc) {
        constexpr int s = decltype(sc)::value;
        u32x2 vlo[4], vhi[4];
        const unsigned vb0 = tile + v_off + (unsigned)(s * 16 * ROWB);
        const unsigned va[2] = {vb0, vb0 ^ 64u};
        const unsigned vh[2] = {vb0 ^ 32u, vb0 ^ 96u};
        static_for<4>([&](auto ic) {
          constexpr int d = decltype(ic)::value;
          lds_read_tr_b64<(d >> 1) * 128>(vlo[d], va[d & 1]);
          lds_read_tr_b64<(d >> 1) * 128 + 8 * ROWB>(vhi[d], vh[d & 1]);
        });
        static_for<DB>([&](auto ic) {
          constexpr int d = decltype(ic)::value;
          constexpr int ahead = (DB - 1 - d) < 3 ? (DB - 1 - d) : 3;
          lds_wait<2 * ahead>(vlo[d & 3], vhi[d & 3]);
          const u32x4 v4 = {vlo[d & 3][0], vlo[d & 3][1], vhi[d & 3][0], vhi[d & 3][1]};
          acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v4), pb[s], acc[d], 0, 0, 0);
          if constexpr (d + 4 < DB) {
            constexpr int d2 = d + 4;
            lds_read_tr_b64<(d2 >> 1) * 128>(vlo[d & 3], va[d2 & 1]);
            lds_read_tr_b64<(d2 >> 1) * 128 + 8 * ROWB>(vhi[d & 3], vh[d2 & 1]);
          }
          // 16 sums over the 2 DB output MFMAs of the tile
          constexpr int step = s * DB + d, per = (16 + 2 * DB - 1) / (2 * DB);
#pragma unroll
          for (int e = step * per; e < (step + 1) * per && e < 16; ++e) s_cur[e] = sA[e] + sB[e];
          __builtin_amdgcn_sched_barrier(0);
        });
      });
      TPLA_PH_CLK(c3);
      ph[1] += c1 - c0; ph[2] += c2 - c1; ph[3] += c3 - c2; ph[4] += 1;
    }
    if (rescale) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_pending);
      l_run *= alpha;
      m_run = m_pending;
#pragma unroll
      for (int d = 0; d < DB; ++d) acc[d] *= alpha;
    }
  }

#ifdef TPLA_WG_TIMELINE
  if (tid == 0 && blockIdx.x < 4096)
    for (int k = 0; k < 5; ++k) g_wg_phase[blockIdx.x * 5 + k] += ph[k];
#endif
  TPLA_TL_MARK(2);
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const size_t item = slot * a.H + head;
  float* pacc = a.part_acc + item * DL + 4 * hi;
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<f32x4*>(pacc + 32 * d + 8 * q) = f32x4{acc[d][4 * q], acc[d][4 * q + 1], acc[d][4 * q + 2], acc[d][4 * q + 3]};
  if (hi == 0) {
    a.part_ml[item * 2 + 0] = m_run;
    a.part_ml[item * 2 + 1] = l_tot;
  }
}

// Static chunks: workgroup = (slice, sequence, chunk s), pages [s*pps, (s+1)*pps).
// Waves per SIMD the register allocation must allow: two 4-wave workgroups
// (or one 8-wave workgroup) per compute unit need 2; a 512-wide slice only
// fits one workgroup per compute unit in LDS, so it keeps the full budget.
constexpr int HPW_PAIR = 8;      // value of HPW that selects decode_item_shared: 16 heads per pair of waves
template <int DL, int NW, int HPW = 16>
constexpr int waves_per_simd() {
  if (HPW == HPW_PAIR) return 2 * NW >= 8 ? 2 : 1;
  if (HPW == 32) return DL <= 128 ? 2 : 1;
  return DL >= 512 ? (NW >= 8 ? 2 : 1) : (NW >= 4 ? 2 : 1);
}
// Tiles in the LDS ring (one fewer in flight) and fragment ring depth (LDS reads ahead of the MFMA that
// consumes them).  Measured: a ring of 4 tiles is no faster than 3 for any width (128-wide slices: 1144
// against 1122 us on the ragged batch), and fragment rings of 8 or 16 change nothing even where a wave
// has its SIMD to itself (576-wide rows: 248 / 251 / 261 us for 4 / 8 / 16).
template <int DL>
constexpr int ring_stages() { return 3; }
template <int DL, int NW>
constexpr int frag_ring() { return 4; }

template <int DL, int DR, int NW, int TOK, int NSTAGE, int KR, int HPW>
__global__ void __launch_bounds__(NW * 64 * (HPW == HPW_PAIR ? 2 : 1), (waves_per_simd<DL, NW, HPW>())) decode_mfma_kernel(DecodeArgs a) {
  extern __shared__ u32x4 smem[];        // NSTAGE tiles
  const int vb = blockIdx.x / a.n_splits, s = blockIdx.x % a.n_splits;   // vb = slice * B + sequence
  const int shard = vb / a.B, b = vb % a.B;
  const int L = seq_len_clipped(a, b);
  const int n_pages = (L + PAGE_TOKENS - 1) / PAGE_TOKENS;
  const int p0 = s * a.pages_per_split;
  if (p0 >= n_pages) return;
  const int p1 = min(p0 + a.pages_per_split, n_pages);
  if constexpr (HPW == 32)
    decode_item32<DL, DR, NW, TOK, NSTAGE>(a, smem, shard, b, L, p0, p1, (size_t)vb * a.n_splits + s);
  else if constexpr (HPW == HPW_PAIR)
    decode_item_shared<DL, DR, NW, TOK, NSTAGE, KR>(a, smem, shard, b, L, p0, p1, (size_t)vb * a.n_splits + s);
  else
    decode_item<DL, DR, NW, TOK, NSTAGE, KR>(a, smem, shard, b, L, p0, p1, (size_t)vb * a.n_splits + s);
}

// Balanced ranges: the pages of all (slice, sequence) pairs are laid end to
// end (T pages) and workgroup w of W takes range w of the plan (equal shares,
// or shares weighted by placement round: see BalancedPlan), whatever
// sequences that covers; every (workgroup, sequence) overlap is one work item
// whose partial result goes to slot w + v (v = slice * B + sequence; strictly
// increasing along the items, hence unique).  Workgroup 0 also publishes the
// page offsets of the sequences for the merge.
template <int DL, int DR, int NW, int TOK, int NSTAGE, int KR, int HPW>
__global__ void __launch_bounds__(NW * 64 * (HPW == HPW_PAIR ? 2 : 1), (waves_per_simd<DL, NW, HPW>())) decode_mfma_balanced_kernel(DecodeArgs a) {
  extern __shared__ u32x4 smem[];
#ifdef TPLA_WG_TIMELINE
  if (threadIdx.x == 0 && blockIdx.x < 4096) {
    g_wg_times[blockIdx.x * 4] = wall_clock64();
    g_wg_times[blockIdx.x * 4 + 1] = 0;
    for (int k = 0; k < 5; ++k) g_wg_phase[blockIdx.x * 5 + k] = 0;
    g_wg_where[blockIdx.x * 2] = __builtin_amdgcn_s_getreg((31 << 11) | 20);      // XCC_ID
    g_wg_where[blockIdx.x * 2 + 1] = __builtin_amdgcn_s_getreg((31 << 11) | 4);   // HW_ID
  }
#endif
  const int lane = threadIdx.x & 63;
  const int n_v = a.n_shards * a.B;
  const int w = blockIdx.x;
  // every wave scans the lengths by itself (no LDS, no barrier)
  int total = 0;
  int L_first = 0;               // length of pair `lane`: the later passes do not load the first 64 again
  for (int v0 = 0; v0 < n_v; v0 += 64) {
    const int v = v0 + lane;
    const int L = (v < n_v) ? seq_len_clipped(a, v % a.B) : 0;
    if (v0 == 0) L_first = L;
    int pg = (L + PAGE_TOKENS - 1) / PAGE_TOKENS;
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) pg += __shfl_xor(pg, m);
    total += pg;
  }
  int start, end;
  plan_range(a.geom, total, w, &start, &end);
  int base = 0;
  for (int v0 = 0; v0 < n_v; v0 += 64) {
    const int v = v0 + lane;
    const int L = v0 == 0 ? L_first : ((v < n_v) ? seq_len_clipped(a, v % a.B) : 0);
    const int pg = (L + PAGE_TOKENS - 1) / PAGE_TOKENS;
    int incl = pg;                               // inclusive prefix sum over the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(incl, d);
      if (lane >= d) incl += o;
    }
    const int excl = base + incl - pg;
    if (w == 0 && v < n_v && threadIdx.x < 64) a.plan[v] = excl;
    int p0l, p1l;
    unsigned long long hit = __ballot(balanced_item(start, end, excl, pg, &p0l, &p1l));
    while (hit) {
      const int src = __builtin_ctzll(hit);
      hit &= hit - 1;
      const int Ls = __shfl(L, src), p0 = __shfl(p0l, src), p1 = __shfl(p1l, src);
      const int vs = v0 + src;
      if constexpr (HPW == 32)
        decode_item32<DL, DR, NW, TOK, NSTAGE>(a, smem, vs / a.B, vs % a.B, Ls, p0, p1, (size_t)w + vs);
      else if constexpr (HPW == HPW_PAIR)
        decode_item_shared<DL, DR, NW, TOK, NSTAGE, KR>(a, smem, vs / a.B, vs % a.B, Ls, p0, p1, (size_t)w + vs);
      else
        decode_item<DL, DR, NW, TOK, NSTAGE, KR>(a, smem, vs / a.B, vs % a.B, Ls, p0, p1, (size_t)w + vs);
    }
    base += __shfl(incl, 63);
  }
  if (w == 0 && threadIdx.x == 0) {
    a.plan[n_v] = total;
    a.plan[3 * n_v + 1] = plan_sparse(a.geom, total) ? 1 : 0;
  }
  // What the merge needs of the plan, once per launch instead of once per lane of the merge kernel: for
  // every (slice, sequence) the range that owns its first page and the number of ranges up to the owner
  // of its last.  Dealt over the workgroups (pair v to workgroup v mod W, one lane of its first wave) and
  // done after the workgroup's own range: inside the scan above it cost the ragged batch 7 % (the owner
  // search then lives in the loop that holds the items' registers).
  if (threadIdx.x < 64 && w < n_v) {
    int base2 = 0;
    for (int v0 = 0; v0 < n_v; v0 += 64) {
      const int v = v0 + lane;
      const int L = v0 == 0 ? L_first : ((v < n_v) ? seq_len_clipped(a, v % a.B) : 0);
      const int pg = (L + PAGE_TOKENS - 1) / PAGE_TOKENS;
      int incl = pg;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
      }
      const int excl = base2 + incl - pg;
      if (v < n_v && v % a.n_wg == w) {
        int w0 = 0, cnt = 0;
        if (pg > 0) {
          w0 = balanced_owner(a.geom, excl, total);
          cnt = balanced_owner(a.geom, excl + pg - 1, total) - w0 + 1;
        }
        a.plan[n_v + 1 + v] = w0;
        a.plan[2 * n_v + 1 + v] = cnt;
      }
      base2 += __shfl(incl, 63);
    }
  }
#ifdef TPLA_WG_TIMELINE
  __syncthreads();
  TPLA_TL_MARK(3);
#endif
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
  void (*fn_balanced)(DecodeArgs) = nullptr;
  size_t smem = 0;
  int threads = 0;
  int blocks_per_cu = 0;
  bool ready = false;
};

template <int DL, int NW, int HPW>
static KernelInfo make_kernel_info() {
  constexpr int TOK = 32, KR = frag_ring<DL, NW>();
  constexpr int NSTAGE = HPW == HPW_PAIR ? 4 : HPW == 32 ? (DL <= 128 ? 3 : TPLA_H32_STAGES) : ring_stages<DL>();
  KernelInfo info;
  info.fn = decode_mfma_kernel<DL, 64, NW, TOK, NSTAGE, KR, HPW>;
  info.fn_balanced = decode_mfma_balanced_kernel<DL, 64, NW, TOK, NSTAGE, KR, HPW>;
  info.smem = (size_t)NSTAGE * TOK * ((DL + 64) / 8) * 16;
  info.threads = NW * 64;
  if (HPW == HPW_PAIR) {
    info.smem += (size_t)2 * (2 * NW) * 64 * 16;     // the two hand-over buffers
    info.threads *= 2;
  }
  // dynamic LDS above the 64 KiB default needs opting in
  if (info.smem > 64 * 1024 &&
      (hipFuncSetAttribute(reinterpret_cast<const void*>(info.fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                           (int)info.smem) != hipSuccess ||
       hipFuncSetAttribute(reinterpret_cast<const void*>(info.fn_balanced),
                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)info.smem) != hipSuccess)) {
    (void)hipGetLastError();
    info.ready = false;
    return info;
  }
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(info.fn_balanced), info.threads,
                                                   info.smem) != hipSuccess) {
    (void)hipGetLastError();
    n = 0;
  }
  info.blocks_per_cu = n;
  info.ready = true;
  return info;
}

template <int DL, int NW, int HPW = 16>
static int kernel_info(KernelInfo** out) {
  static KernelInfo info = make_kernel_info<DL, NW, HPW>();   // initialised once, thread-safe
  if (!info.ready) return fail(TPLA_ERR_HIP, "cannot raise the dynamic LDS limit to %zu", info.smem);
  *out = &info;
  return TPLA_OK;
}

template <int DL>
static int kernel_info_dl(int H, KernelInfo** out) {
  switch (H) {
    case 16: return kernel_info<DL, 1>(out);
    case 32:
      if constexpr (DL == 512) {     // as for 64 heads below
        static const bool pair_ok = [] { KernelInfo* k = nullptr; return kernel_info<DL, 2, HPW_PAIR>(&k) == TPLA_OK; }();
        if (pair_ok) return kernel_info<DL, 2, HPW_PAIR>(out);
      }
      return kernel_info<DL, 2>(out);
    // -DTPLA_H32 routes 64 and 128 heads to the 32-heads-per-wave instances.  Measured against the
    // 16-heads-per-wave ones (32 x 32768 tokens, both slices): 266 against 219 us at 64 heads, 432 against
    // 356 us at 128 -- LDS instructions per tile are halved, but a wave's own VALU instructions do not
    // run under its MFMAs (per-phase clocks: the score MFMAs of a tile alone 678 cycles, with the softmax
    // of the previous tile issued between them 1158), so one wave per SIMD loses what two waves overlap;
    // not the default.
#ifdef TPLA_H32
    case 64:
      if constexpr (DL <= 256) return kernel_info<DL, 2, 32>(out);
      return kernel_info<DL, 4>(out);
    case 128:
      if constexpr (DL <= 256) return kernel_info<DL, 4, 32>(out);
      return kernel_info<DL, 8>(out);
#else
    case 64:
      // 576-wide rows: pairs of waves per 16 heads (160 KB of LDS); the plain instance if the device refuses that
      if constexpr (DL == 512) {
        static const bool pair_ok = [] { KernelInfo* k = nullptr; return kernel_info<DL, 4, HPW_PAIR>(&k) == TPLA_OK; }();
        if (pair_ok) return kernel_info<DL, 4, HPW_PAIR>(out);
      }
      return kernel_info<DL, 4>(out);
    case 128: return kernel_info<DL, 8>(out);
#endif
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

// Measured with per-workgroup timestamps on full launches of equal ranges: when two or three workgroups
// share a compute unit and their waves share its SIMDs, the workgroup placed first takes 5 - 9 % less
// time than the average and the one placed last 5 % (two per compute unit) or 10 % (three) more,
// whatever the wave priorities (s_setprio changes nothing).  With two per compute unit the late
// workgroups still keep the memory system full when they are alone at the end, and sizing the ranges by
// round made the launch slower (227 against 222 us at 32 x 32768 tokens); with three (128-wide slices:
// 12 KB tiles, 24 KB in flight per workgroup) the lone last round does not, and weighted ranges take
// the ragged batch from 1122 to 1073 us with 140 : 129 : 115.  With the XCC weights below in place the
// best round weights are further apart (one box, same units: 140:129:115 1047 us, 143:130:112 1035,
// 146:130:109 1026, 149:131:106 1022, 152:131:103 1034, 155:132:100 1040, 160:132:95 1055 us; on
// another box 1072 -> 1051 us for 149:131:106 against 140:129:115).  With one wave per SIMD (32 heads
// and fewer) the rounds run alike.  Weights in units of 1/128 of the average range.
//
// The XCCs differ too, the same way on every box measured: workgroups on the odd-numbered ones take
// 4 % (64 heads, 256-wide slices) to 9 % (32 heads; 128-wide slices) longer over equal ranges than
// those on the even-numbered ones.  Workgroups are dealt to the XCCs in turn, so the odd positions of a
// round get shorter ranges.  Measured on one box with the weight of the odd positions at 128 (equal),
// 123, 118, 113, 108 / 128: 64 heads, 256-wide: 221.9, 219.7, 220.4, 223.6 us; 32 heads: 414.3, 410.8,
// 404.7, 405.5 us (another box: 113 399.2, 108 406.7, 103 414.2); 128-wide ragged batch: 1072, 1061,
// 1051, 1047 us (other box: 113 1043, 108 1057, 103 1069); 576-wide: 232.5, 229.1, 229.6, 229.4 us.
// Whole steps on a third box, equal against weighted: 32 heads 446 -> 431 us, ragged batch 1138 -> 1121 us.
void decode_mfma_round_weights(const tpla_shape_t& sh, int per_cu, int32_t wt[4], int32_t wx[2]) {
  for (int r = 0; r < 4; ++r) wt[r] = 128;
  const int dl = sh.d_c / sh.g;
  wx[0] = wx[1] = 128;
#ifdef TPLA_EQUAL_RANGES      // measurement build: the plan without any weights, for the timeline comparison
  (void)dl;
  (void)per_cu;
  return;
#endif
  // 64 heads over 256-wide slices stay equal: the gain there (1 %) is within the spread between boxes and the
  // layer-step did not follow it (3 us longer with the weights); 128 heads: not measured
  wx[1] = dl == 128 ? 113 : (sh.H <= 32 ? 115 : (sh.H == 64 && dl == 512 ? 123 : 128));
#ifdef TPLA_H32
  const int heads_per_wave = (sh.H >= 64 && dl <= 256) ? 32 : 16;
#else
  const int heads_per_wave = 16;
#endif
  const int waves_per_simd_launched = (sh.H / heads_per_wave) * per_cu / 4;
  if (waves_per_simd_launched < 2) return;
  if (per_cu == 3) {
    wt[0] = 149;
    wt[1] = 131;
    wt[2] = 106;
  }
}

#ifdef TPLA_WG_TIMELINE
// Device addresses of the timeline arrays ([4096][4] uint64 ticks of 10 ns, [4096][2] uint32, [4096][5] uint64).
extern "C" __attribute__((visibility("default"))) int tpla_debug_wg_timeline(void** times, void** where, void** phase) {
  if (hipGetSymbolAddress(times, HIP_SYMBOL(g_wg_times)) != hipSuccess) return TPLA_ERR_HIP;
  if (hipGetSymbolAddress(where, HIP_SYMBOL(g_wg_where)) != hipSuccess) return TPLA_ERR_HIP;
  if (hipGetSymbolAddress(phase, HIP_SYMBOL(g_wg_phase)) != hipSuccess) return TPLA_ERR_HIP;
  return TPLA_OK;
}
#endif

int launch_decode_mfma(const DecodeArgs& a, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  KernelInfo* k = nullptr;
  const int rc = kernel_info_for(a.dl, a.H, &k);
  if (rc) return rc;
  const dim3 grid(a.balanced ? (unsigned)a.n_wg : (unsigned)(a.n_shards * a.B * a.n_splits));
  void (*fn)(DecodeArgs) = a.balanced ? k->fn_balanced : k->fn;
  if (ev_start && ev_stop)
    // the events take the kernel's own begin and end times (no marker packets around it)
    hipExtLaunchKernelGGL(fn, grid, dim3(k->threads), (uint32_t)k->smem, st, ev_start, ev_stop, 0, a);
  else
    hipLaunchKernelGGL(fn, grid, dim3(k->threads), k->smem, st, a);
  return check_launch("decode_mfma_kernel");
}

}  // namespace tpla
