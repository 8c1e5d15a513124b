// Building blocks shared by the kernels that stream bf16 tiles through LDS with
// direct-to-LDS loads and feed them to 16x16x32 MFMAs (decode_mfma.hip,
// prefill_mfma.hip): compile-time loops, LDS reads in inline assembly with
// hand-placed waits, and the tile swizzle.
#pragma once
#include <utility>
#include "tpla_internal.h"

namespace tpla {


constexpr float LAZY = 8.0f;   // log2 units: the softmax reference lags the running maximum by at most this

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// Compile-time loop: f receives std::integral_constant<int, i>, so i can feed
// instruction immediates.
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// s_waitcnt immediate that only waits on the vector-memory counter.
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

template <int OFF>
__device__ __forceinline__ void lds_read_b128(bf16x8& dst, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
// Transposing read: lane j of each 16-lane group points at 4 bf16 of row j/4,
// columns 4*(j%4)..; lane i receives column i of those 4 rows.
template <int OFF>
__device__ __forceinline__ void lds_read_tr_b64(u32x2& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
// Waits until at most N LDS operations of this wave are outstanding; the
// operands are tied so that their consumers cannot be scheduled before it.
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x2& a, u32x2& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

// 16-byte pieces of a tile are stored at a swizzled position: piece c of
// token `tok` lives at piece index tok * RC + (c ^ swz(tok)), with RC = 8 mod
// 16 (rows alternate between the two halves of the 64 LDS banks) and swz a
// 3-bit value that moves a piece inside its group of 8.  With swz = tok & 7
// both access patterns of these kernels -- row-wise reads (16 lanes = 16
// tokens x 16 B at one column) and transposing reads (16 tokens x 32 B at one
// column pair) -- run without a single bank-conflict cycle (SQ_LDS_BANK_CONFLICT
// reads 0 for the decode kernel; (tok >> 1) & 7, used before, cost two extra
// cycles per transposing read, and a one-bit rotation of that value four per
// row-wise read).  The direct-to-LDS load writes lane l of an instruction at
// base + 16 l, so the swizzle is applied to the global address each lane
// fetches from.
__device__ __forceinline__ int swz(int tok) { return tok & 7; }

// Tile swizzle of the kernels that feed 32x32x16 MFMAs (32 heads or 32 queries per wave): piece c of
// token t sits at c ^ swz32(t) within its group of 8.  Their two read patterns differ from the
// 16-wide kernels': the score operand takes 32 consecutive tokens at one piece (two pieces per
// instruction), the transposing read 4 consecutive tokens x 4 consecutive pieces per 32 lanes.  With
// t & 7 tokens t and t + 8 collide in the first (5.3 against 3.0 cycles per instruction in a read-only
// loop) and tokens t and t + 2 in the second (3.0 against 1.6); of the 3-bit XOR-linear maps of the
// token index, those with output bit 2 = token bit 1 and the other two bits from token bits 2 and 3
// run both at full rate.
__device__ __forceinline__ int swz32(int tok) { return ((tok >> 2) & 3) | ((tok & 2) << 1); }

}  // namespace tpla
