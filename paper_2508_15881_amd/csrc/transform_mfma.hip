// Streaming Hadamard pass over MLA pages on the matrix cores (Sec. 4.3: U =
// diag(s) H / sqrt(d_c), natural order; Sec. 4.1: column slices of c U go to
// the g shard pools, the RoPE key to every one of them).
//
// H_{d_c} = H_NA (x) H_64 with element index e = 64 a + b, NA = d_c / 64:
//   * H_64 over b is a contraction of the row's 64-element sub-rows with a
//     constant +-1 matrix: bf16 inputs are exact operands, the sums are float.
//     A sub-row is 128 contiguous bytes, and the 16 bytes a lane loads straight
//     from global memory are already its share of the MFMA A operand.
//   * H_NA over a runs on the accumulators.  A tile's 16 sub-rows are chosen
//     (4 rows x 4 values of a) so that one lane ends up with all NA values of a
//     for its row and columns: these butterflies stay inside the lane.
//   * The columns of the constant operand are ordered so that a lane owns 4
//     adjacent output columns: 8-byte stores, 128 contiguous bytes per 16 lanes.
// The cross-lane butterflies of the plain-ALU kernel (about 150 instructions
// per row) become 4 MFMAs per row.
#include "lds_tile.h"

#include <mutex>

namespace tpla {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned opaque(unsigned x) {
  asm volatile("" : "+v"(x));
  return x;
}

template <int NA>
struct FwhtGroup {          // one group of 4 rows as loaded: NA/4 tiles x 2 k-steps, and the RoPE keys
  u32x4 a[NA / 4][2];
  u32x4 kpe;
};

// One wave per `rows_per_wave` (a multiple of 4 that divides the page) consecutive
// rows of a page, 4 rows at a time, the next 4 loaded while these are transformed.
template <int NA>
__global__ void __launch_bounds__(256, 4) transform_paged_fwht_mfma_kernel(
    const bf16_t* __restrict__ mla_pool, ShardPools pools, const int32_t* __restrict__ page_ids,
    const float* __restrict__ signs, int n_pages, int page_tokens, int rows_per_wave, int d_r, int g) {
  constexpr int NT = NA / 4, D_C = 64 * NA;
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int waves_per_page = page_tokens / rows_per_wave;
  const int pg = wave / waves_per_page;
  if (pg >= n_pages) return;                       // whole waves leave; the kernel has no barrier
  const int row_first = (wave - pg * waves_per_page) * rows_per_wave;
  const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
  const int dl = D_C / g;
  const int lo = lane & 15, hi = lane >> 4;

  // constant operand: lane (column group lo, k group hi) holds, for k-step s and
  // column tile nt, H_64[k][c] for k = 32 s + 8 hi + j, c = 4 lo + nt.  Bit 5 of
  // k meets bit 3 of lo only, so k-step 1 is k-step 0 with the sign of whole
  // columns flipped: one set of registers and a per-lane sign mask.
  u32x4 hb[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) {
    const unsigned c = 4u * lo + nt;
    const unsigned par_hi = __popc((8u * hi) & c);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const unsigned p0 = (par_hi + __popc((2u * jj) & c)) & 1u;
      const unsigned p1 = (par_hi + __popc((2u * jj + 1u) & c)) & 1u;
      hb[nt][jj] = (0x3F80u | (p0 << 15)) | ((0x3F80u | (p1 << 15)) << 16);
    }
  }
  const unsigned step1_flip = (lo & 8) ? 0x80008000u : 0u;

  // as holder of the data operand: lane (sub-row lo of the tile, k group hi);
  // tile t, sub-row lo = 4 q + i  ->  row q of the group, a = 4 t + i
  const int a_row = lo >> 2, a_sub = lo & 3;
  // sign diagonal, packed: bit 15 - jj of flip[t][s] is set when element 2 jj of the
  // lane's 8 is negated, bit 31 - jj for element 2 jj + 1
  unsigned flip[NT][2];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      unsigned m = 0u;
      if (signs) {
        const float* sp = signs + 64 * (4 * t + a_sub) + 32 * s + 8 * hi;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          m |= ((__float_as_uint(sp[2 * jj]) >> 31) << (15 - jj)) | ((__float_as_uint(sp[2 * jj + 1]) >> 31) << (31 - jj));
      }
      flip[t][s] = m;
    }

  const int in_pitch = D_C + d_r, out_pitch = dl + d_r;
  const size_t tok0 = page * (size_t)page_tokens + row_first;
  const bf16_t* in_lane = mla_pool + (tok0 + a_row) * in_pitch + 64 * a_sub + 8 * hi;
  const int kpe_lanes = d_r >> 3;                   // lanes per row of RoPE key, 4 rows per group
  const bool has_kpe = lane < 4 * kpe_lanes;
  const int kpe_row = has_kpe ? lane / kpe_lanes : 0, kpe_piece = has_kpe ? lane - kpe_row * kpe_lanes : 0;
  const bf16_t* kpe_lane = mla_pool + (tok0 + kpe_row) * in_pitch + D_C + 8 * kpe_piece;

  auto load_group = [&](int gi, FwhtGroup<NA>& grp) {
    const bf16_t* p = in_lane + (size_t)(4 * gi) * in_pitch;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int s = 0; s < 2; ++s)
        grp.a[t][s] = *reinterpret_cast<const u32x4*>(p + 256 * t + 32 * s);
    if (has_kpe)
      grp.kpe = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kpe_lane + (size_t)(4 * gi) * in_pitch));
  };

  const float sc = 1.0f / sqrtf((float)D_C);
  const int n_groups = rows_per_wave >> 2;
  FwhtGroup<NA> cur, nxt;
  load_group(0, cur);
  for (int gi = 0; gi < n_groups; ++gi) {
    if (gi + 1 < n_groups) load_group(gi + 1, nxt);

    f32x4 acc[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc[t][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        // (masks are rebuilt from opaque copies: kept as loop invariants they
        // would cost 28 more registers and a wave per SIMD)
        const unsigned fw = opaque(flip[t][s]);
        u32x4 ax = cur.a[t][s];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) ax[jj] ^= (fw << jj) & 0x80008000u;
        const bf16x8 av = __builtin_bit_cast(bf16x8, ax);
        const unsigned f1 = opaque(step1_flip);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          const u32x4 hv = s ? (hb[nt] ^ f1) : hb[nt];
          acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, hv), acc[t][nt], 0, 0, 0);
        }
      }

    // as holder of the result: row hi of the group, columns 4 lo + nt, a = 4 t + i
    const size_t out_row = (tok0 + 4 * gi + hi) * (size_t)out_pitch;
    float y[4][NA];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) y[nt][4 * t + i] = acc[t][nt][i];
#pragma unroll
      for (int h = 1; h < NA; h <<= 1)
#pragma unroll
        for (int a = 0; a < NA; ++a)
          if (!(a & h)) {
            const float u = y[nt][a], v = y[nt][a | h];
            y[nt][a] = u + v;
            y[nt][a | h] = u - v;
          }
    }
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const bf16x2 p0 = __builtin_convertvector(f32x2{y[0][a] * sc, y[1][a] * sc}, bf16x2);
      const bf16x2 p1 = __builtin_convertvector(f32x2{y[2][a] * sc, y[3][a] * sc}, bf16x2);
      const u32x2 out = {__builtin_bit_cast(unsigned, p0), __builtin_bit_cast(unsigned, p1)};
      const int shard = (64 * a) / dl;
      bf16_t* dst = static_cast<bf16_t*>(pools.p[shard]) + out_row + (64 * a - shard * dl) + 4 * lo;
      __builtin_nontemporal_store(out, reinterpret_cast<u32x2*>(dst));
    }
    if (has_kpe) {
      const size_t kr = (tok0 + 4 * gi + kpe_row) * (size_t)out_pitch + dl + 8 * kpe_piece;
      for (int i = 0; i < g; ++i)
        __builtin_nontemporal_store(cur.kpe, reinterpret_cast<u32x4*>(static_cast<bf16_t*>(pools.p[i]) + kr));
    }
    cur = nxt;
  }
}

// Short runs of rows per wave on purpose: neighbouring waves then read and write
// neighbouring addresses at about the same time, which is what the DRAM wants
// (64 rows per wave: 5.1 TB/s, 8 rows: 5.7 TB/s at a million rows); the constant
// set-up per wave is hidden behind the loads either way.
static int fwht_rows_per_wave(int page_tokens) { return page_tokens % 8 == 0 ? 8 : 4; }

bool transform_paged_mfma_supported(const TransformArgs& t, const tpla_shape_t& sh, int64_t n_pages) {
  if (sh.dtype != TPLA_BF16 || t.mode != TPLA_U_HADAMARD || t.inverse) return false;
  if (sh.d_c != 256 && sh.d_c != 512) return false;
  const int dl = sh.d_c / sh.g;
  if (dl % 64 != 0 || sh.d_r % 8 != 0 || sh.d_r > 128) return false;
  const int pt = sh.page_tokens;
  if (pt % 4 != 0) return false;
  const int64_t waves = n_pages * (pt / fwht_rows_per_wave(pt));
  return waves > 0 && waves < (int64_t)1 << 30;
}

int launch_transform_paged_mfma(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                                const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                                hipStream_t st) {
  const int pt = sh.page_tokens;
  const int rows_per_wave = fwht_rows_per_wave(pt);
  const int64_t waves = n_pages * (pt / rows_per_wave);
  const dim3 grid((unsigned)((waves + 3) / 4));
  const bf16_t* in = static_cast<const bf16_t*>(mla_pool);
  if (sh.d_c == 512)
    hipLaunchKernelGGL(transform_paged_fwht_mfma_kernel<8>, grid, dim3(256), 0, st, in, pools, page_ids,
                       t.signs, (int)n_pages, pt, rows_per_wave, sh.d_r, sh.g);
  else
    hipLaunchKernelGGL(transform_paged_fwht_mfma_kernel<4>, grid, dim3(256), 0, st, in, pools, page_ids,
                       t.signs, (int)n_pages, pt, rows_per_wave, sh.d_r, sh.g);
  return check_launch("transform_paged_fwht_mfma_kernel");
}

// ---------------------------------------------------------------------------
// Dense U (Sec. 4.3.2: the PCA basis) over MLA pages: Y = X U as a GEMM on the
// matrix cores.  X rows are bf16 (exact operands).  U is float: every entry is
// split into bf16 hi + lo and both products are accumulated in float, so the
// result is rounded to bf16 once, from (nearly) the float product.
//
// A workgroup (8 waves) owns 64 output columns: its slab of U (d_c x 64, hi and
// lo) is converted once into LDS in B-operand order, then the workgroup walks
// over blocks of 256 rows.  The rows go through LDS as well, in chunks of 64
// k: the MFMA A layout wants 16 different rows per quarter wave, which read
// straight from global memory costs one cache access per lane; staged, every
// global load is a full 128-byte line per 8 lanes and the operand reads are
// 16-byte LDS reads (pieces XOR-swizzled so that 16 rows hit 16 bank groups).
// A wave stages the 32 rows it multiplies itself, so the loop over the chunks
// has no workgroup barrier.  The next row block is in registers while the
// current one feeds the MFMAs.  Measured and not kept: 64 x 64 outputs per wave
// (4 x 4 MFMA tiles, 32-k chunks, a ring of 4 chunks in registers: 12 instead
// of 20 LDS reads per 32 MFMAs) was 6 % slower, with the fragments read one
// chunk ahead 20 % slower (the registers no longer hold it all); the matrix
// cores are busy 0.38 of the time either way, at 2.25 GHz.
// As in the Hadamard pass the slab's columns are ordered so that a lane owns 4
// adjacent output columns.  The d_c/64 workgroups that read the same rows sit
// on one XCD (block ids congruent mod 8): the rows come from that XCD's L2
// after the first touch.
constexpr int DENSE_WAVES = 8;
constexpr int DENSE_ROWS = DENSE_WAVES * 32;     // rows per workgroup pass: 2 tiles of 16 per wave
constexpr int DENSE_KC = 64;                     // k per staged chunk (two MFMA k-steps)
constexpr int DENSE_STAGE_BYTES = DENSE_ROWS * DENSE_KC * 2;
constexpr int DENSE_LD = DENSE_ROWS * (DENSE_KC / 8) / (DENSE_WAVES * 64);   // 16-byte pieces per thread and chunk

template <int NB>                                 // d_c = 64 NB
__global__ void __launch_bounds__(DENSE_WAVES * 64) transform_paged_dense_mfma_kernel(
    const bf16_t* __restrict__ mla_pool, ShardPools pools, const int32_t* __restrict__ page_ids,
    const float* __restrict__ U, int n_rows, int page_tokens, int page_shift, int d_r, int g,
    int n_row_blocks, int row_workers) {
  extern __shared__ u32x4 lds4[];                  // [2][KS][4][64] operands (hi, lo), then the staged rows
  constexpr int KS = 2 * NB, D_C = 64 * NB, NCH = D_C / DENSE_KC;
  u32x4* const panel = lds4;
  u32x4* const stage = lds4 + 2 * KS * 256;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 15, hi = lane >> 4;
  const int id = blockIdx.x;
  const int nb = (id >> 3) % NB;                   // column block
  const int worker = (id / (8 * NB)) * 8 + (id & 7);
  const int dl = D_C / g;

  // B operand of k-step s, column tile nt: lane (column 4 lo + nt, k group hi) holds k = 32 s + 8 hi + j
  for (int idx = tid; idx < KS * 256; idx += DENSE_WAVES * 64) {
    const int ln = idx & 63, nt = (idx >> 6) & 3, s = idx >> 8;
    const int col = 64 * nb + 4 * (ln & 15) + nt;
    const int k0 = 32 * s + 8 * (ln >> 4);
    u32x4 ph, pl;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const float u0 = U[(k0 + 2 * jj) * D_C + col], u1 = U[(k0 + 2 * jj + 1) * D_C + col];
      const bf16_t h0 = (bf16_t)u0, h1 = (bf16_t)u1;
      const bf16_t l0 = (bf16_t)(u0 - (float)h0), l1 = (bf16_t)(u1 - (float)h1);
      ph[jj] = (unsigned)__builtin_bit_cast(unsigned short, h0) | ((unsigned)__builtin_bit_cast(unsigned short, h1) << 16);
      pl[jj] = (unsigned)__builtin_bit_cast(unsigned short, l0) | ((unsigned)__builtin_bit_cast(unsigned short, l1) << 16);
    }
    panel[idx] = ph;
    panel[KS * 256 + idx] = pl;
  }

  const int in_pitch = D_C + d_r, out_pitch = dl + d_r;
  const int shard = (64 * nb) / dl;
  bf16_t* const out_base = static_cast<bf16_t*>(pools.p[shard]) + (64 * nb - shard * dl) + 4 * lo;
  const int last = n_rows - 1;
  auto token_of = [&](int row) -> size_t {           // physical token index of logical row
    const int pg = page_shift >= 0 ? (row >> page_shift) : (int)((unsigned)row / (unsigned)page_tokens);
    const int slot = row - pg * page_tokens;
    const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
    return page * (size_t)page_tokens + slot;
  };
  // staging: a wave stages the 32 rows it multiplies itself (so no wave ever waits for another): its
  // j-th load takes rows 32 wave + 8 j .. + 8, lane / 8 the row and lane % 8 the 16-byte piece, which
  // lives at piece position (lane % 8) ^ ((row >> 1) & 7) of its row
  static_assert(DENSE_LD * 8 == 32, "a wave stages its own 32 rows");
  int st_row[DENSE_LD];
  unsigned st_dst[DENSE_LD];
#pragma unroll
  for (int j = 0; j < DENSE_LD; ++j) {
    st_row[j] = 32 * wave + 8 * j + (lane >> 3);
    st_dst[j] = (unsigned)(st_row[j] * 8 + ((lane & 7) ^ ((st_row[j] >> 1) & 7)));
  }
  // operand reads: row 32 wave + 16 mt + lo, piece 4 ks + hi of the chunk
  unsigned a_off[2][2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int r = 32 * wave + 16 * mt + lo;
      a_off[mt][ks] = (unsigned)(r * 8 + ((4 * ks + hi) ^ ((r >> 1) & 7)));
    }

  // Physical token index of the 64-row group `grp` of row block rb.  Pages of a multiple of 64
  // tokens hold a whole group, and the page id then comes through a scalar load: a vector load
  // here would have to be waited for with vmcnt(0), which drains the row prefetch below.
  const bool whole_groups = (page_tokens & 63) == 0;
  auto group_token = [&](int rb, int grp) -> size_t {
    int row = rb * DENSE_ROWS + 64 * grp;
    if (row > last) row = rb * DENSE_ROWS;           // group past the end: any valid rows will do, nothing is stored
    const int pg = __builtin_amdgcn_readfirstlane(page_shift >= 0 ? (row >> page_shift)
                                                                   : (int)((unsigned)row / (unsigned)page_tokens));
    const size_t page = page_ids ? (size_t)page_ids[pg] : (size_t)pg;
    return page * (size_t)page_tokens + (row - pg * page_tokens);
  };
  // source of this thread's piece of chunk 0 for its DENSE_LD rows of row block rb
  auto row_sources = [&](int rb, const bf16_t* (&src)[DENSE_LD]) {
#pragma unroll
    for (int j = 0; j < DENSE_LD; ++j) {
      const size_t tok = whole_groups ? group_token(rb, wave >> 1) + (st_row[j] - 64 * (wave >> 1))
                                      : token_of(min(rb * DENSE_ROWS + st_row[j], last));
      src[j] = mla_pool + tok * in_pitch + 8 * (tid & 7);
    }
  };
  // A whole row block (NCH chunks) per thread in registers: chunk ch of the NEXT block is requested
  // as soon as chunk ch of this one has been handed to LDS and is used one block later, so a
  // memory latency has NCH chunks of MFMAs to hide behind.
  u32x4 blk[NCH][DENSE_LD];
  // The RoPE keys of the block are copied to every slice by all NB column-block workgroups, each
  // taking DENSE_ROWS / NB of the rows: 8 lanes per row (a row's first 64 keys are 8 pieces),
  // fetched one block ahead like the rows.
  constexpr int KPE_ROWS = DENSE_ROWS / NB;
  constexpr int KPE_IT = (8 * KPE_ROWS + DENSE_WAVES * 64 - 1) / (DENSE_WAVES * 64);   // rows per thread
  const bool kpe_piece_ok = 8 * (tid & 7) < d_r;
  u32x4 kpe_reg[KPE_IT];
  // row of the block that this thread copies in its it-th turn, or -1
  auto kpe_row = [&](int it) -> int {
    const int r = (tid >> 3) + it * (DENSE_WAVES * 8);
    return r < KPE_ROWS ? nb * KPE_ROWS + r : -1;
  };
  auto kpe_token = [&](int rb, int row) -> size_t {
    return whole_groups ? group_token(rb, row >> 6) + (row & 63) : token_of(min(rb * DENSE_ROWS + row, last));
  };
  auto kpe_request = [&](int rb) {
#pragma unroll
    for (int it = 0; it < KPE_IT; ++it) {
      const int row = kpe_row(it);
      if (row >= 0 && kpe_piece_ok)
        kpe_reg[it] = *reinterpret_cast<const u32x4*>(mla_pool + kpe_token(rb, row) * in_pitch + D_C + 8 * (tid & 7));
    }
  };
  const bf16_t* src[DENSE_LD];
  if (worker < n_row_blocks) {
    row_sources(worker, src);
    static_for<NCH>([&](auto chc) {
      constexpr int ch = decltype(chc)::value;
#pragma unroll
      for (int j = 0; j < DENSE_LD; ++j) blk[ch][j] = *reinterpret_cast<const u32x4*>(src[j] + DENSE_KC * ch);
    });
    kpe_request(worker);
  }

  __syncthreads();                                   // the slab of U is in place
  for (int rb = worker; rb < n_row_blocks; rb += row_workers) {
    const int row0 = rb * DENSE_ROWS;
    const int rb_next = rb + row_workers;
    const bool more = rb_next < n_row_blocks;
    if (more) row_sources(rb_next, src);
    f32x4 acc[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    static_for<NCH>([&](auto chc) {
      constexpr int ch = decltype(chc)::value;
      // The staged rows are private to the wave and a wave's LDS instructions complete in order: the
      // writes below land after the previous chunk's reads and before this chunk's.  The wave barriers
      // only keep the compiler from moving an LDS access across them.
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < DENSE_LD; ++j) stage[st_dst[j]] = blk[ch][j];
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (more) {
#pragma unroll
        for (int j = 0; j < DENSE_LD; ++j) blk[ch][j] = *reinterpret_cast<const u32x4*>(src[j] + DENSE_KC * ch);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 av[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) av[mt] = __builtin_bit_cast(bf16x8, stage[a_off[mt][ks]]);
        constexpr int s0 = 2 * ch;
        const int s = s0 + ks;
        bf16x8 bh[4], bl[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          bh[nt] = __builtin_bit_cast(bf16x8, panel[(s * 4 + nt) * 64 + lane]);
          bl[nt] = __builtin_bit_cast(bf16x8, panel[KS * 256 + (s * 4 + nt) * 64 + lane]);
        }
        // all hi products first, then all lo: two MFMAs on one accumulator are never adjacent
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], bh[nt], acc[mt][nt], 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mt], bl[nt], acc[mt][nt], 0, 0, 0);
      }
    });
    // as holder of the result: rows 32 wave + 16 mt + 4 hi + i, columns 64 nb + 4 lo + nt
    const size_t wave_tok = whole_groups ? group_token(rb, wave >> 1) + 32 * (wave & 1) : 0;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = row0 + 32 * wave + 16 * mt + 4 * hi + i;
        if (r <= last) {
          const bf16x2 p0 = __builtin_convertvector(f32x2{acc[mt][0][i], acc[mt][1][i]}, bf16x2);
          const bf16x2 p1 = __builtin_convertvector(f32x2{acc[mt][2][i], acc[mt][3][i]}, bf16x2);
          const u32x2 out = {__builtin_bit_cast(unsigned, p0), __builtin_bit_cast(unsigned, p1)};
          const size_t tok = whole_groups ? wave_tok + (16 * mt + 4 * hi + i) : token_of(r);
          __builtin_nontemporal_store(out, reinterpret_cast<u32x2*>(out_base + tok * out_pitch));
        }
      }
    // this workgroup's share of the block's RoPE keys, to every slice
#pragma unroll
    for (int it = 0; it < KPE_IT; ++it) {
      const int row = kpe_row(it);
      if (row < 0 || row0 + row > last) continue;
      const size_t tok = kpe_token(rb, row);
      if (kpe_piece_ok) {
        for (int i = 0; i < g; ++i)
          __builtin_nontemporal_store(kpe_reg[it], reinterpret_cast<u32x4*>(static_cast<bf16_t*>(pools.p[i]) +
                                                                           tok * out_pitch + dl + 8 * (tid & 7)));
      }
      // RoPE widths above 64: the remaining pieces, not prefetched
      for (int c = 64 + 8 * (tid & 7); c < d_r; c += 64) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(mla_pool + tok * in_pitch + D_C + c);
        for (int i = 0; i < g; ++i)
          __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(static_cast<bf16_t*>(pools.p[i]) + tok * out_pitch + dl + c));
      }
    }
    if (more) kpe_request(rb_next);
  }
}

bool transform_paged_dense_mfma_supported(const TransformArgs& t, const tpla_shape_t& sh, int64_t n_pages) {
  if (sh.dtype != TPLA_BF16 || t.mode != TPLA_U_DENSE || t.inverse || !t.U) return false;
  if (sh.d_c != 128 && sh.d_c != 256 && sh.d_c != 512) return false;   // the slab of U must fit the LDS
  const int dl = sh.d_c / sh.g;
  if (dl % 64 != 0 || sh.d_r % 8 != 0) return false;
  return n_pages > 0 && n_pages * sh.page_tokens < ((int64_t)1 << 31) - DENSE_ROWS;
}

template <int NB>
static int launch_dense_t(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                          const ShardPools& pools, const int32_t* page_ids, int64_t n_pages, hipStream_t st) {
  const size_t smem = (size_t)(2 * NB) * 256 * 16 * 2 + DENSE_STAGE_BYTES;
  static std::mutex mu;
  static bool opted_in[16] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return fail(TPLA_ERR_HIP, "hipGetDevice failed");
  if (smem > 64 * 1024) {
    std::lock_guard<std::mutex> lock(mu);
    if (!opted_in[dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(transform_paged_dense_mfma_kernel<NB>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) {
        (void)hipGetLastError();
        return fail(TPLA_ERR_HIP, "cannot reserve %zu bytes of LDS for transform_paged_dense_mfma_kernel", smem);
      }
      opted_in[dev] = true;
    }
  }
  const int pt = sh.page_tokens;
  int page_shift = -1;
  if ((pt & (pt - 1)) == 0)
    for (page_shift = 0; (1 << page_shift) < pt; ++page_shift) {}
  const int n_rows = (int)(n_pages * pt);
  const int n_row_blocks = (n_rows + DENSE_ROWS - 1) / DENSE_ROWS;
  // one workgroup per CU where the slab fills the LDS; row workers in multiples of 8 (one per XCD)
  int workers = device_cu_count() * (NB == 8 ? 1 : 2) / NB;
  if (workers > n_row_blocks) workers = n_row_blocks;
  workers = (workers + 7) / 8 * 8;
  const dim3 grid((unsigned)(workers * NB));
  hipLaunchKernelGGL(transform_paged_dense_mfma_kernel<NB>, grid, dim3(DENSE_WAVES * 64), smem, st,
                     static_cast<const bf16_t*>(mla_pool), pools, page_ids, t.U, n_rows, pt, page_shift, sh.d_r,
                     sh.g, n_row_blocks, workers);
  return check_launch("transform_paged_dense_mfma_kernel");
}

int launch_transform_paged_dense_mfma(const TransformArgs& t, const tpla_shape_t& sh, const void* mla_pool,
                                      const ShardPools& pools, const int32_t* page_ids, int64_t n_pages,
                                      hipStream_t st) {
  if (sh.d_c == 512) return launch_dense_t<8>(t, sh, mla_pool, pools, page_ids, n_pages, st);
  if (sh.d_c == 256) return launch_dense_t<4>(t, sh, mla_pool, pools, page_ids, n_pages, st);
  return launch_dense_t<2>(t, sh, mla_pool, pools, page_ids, n_pages, st);
}

}  // namespace tpla
