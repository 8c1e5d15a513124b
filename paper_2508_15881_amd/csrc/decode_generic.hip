// Shape-agnostic shard decode (any widths, float or bf16 storage, float
// arithmetic) and the merge of split partials.  This is the float-mode
// implementation and the fallback for bf16 shapes the MFMA kernel does not
// cover; it favours clarity over speed.
#include "tpla_internal.h"

namespace tpla {

constexpr int GEN_THREADS = 128;
constexpr int GEN_MAX_COLS = 8;   // output columns per thread: d_c/g <= 1024

// One workgroup = one (sequence, split, head).  Tokens are processed in
// chunks of GEN_THREADS: thread i scores token i, the chunk's weights go to
// LDS, then thread j accumulates output columns j, j+GEN_THREADS, ...
template <typename T>
__global__ void __launch_bounds__(GEN_THREADS) decode_generic_kernel(DecodeArgs a) {
  extern __shared__ float smem[];
  const int dl = a.dl, dr = a.d_r, w = dl + dr;
  float* q = smem;                  // [w]
  float* p = smem + w;              // [GEN_THREADS]
  float* red = p + GEN_THREADS;     // [GEN_THREADS]
  const int tid = threadIdx.x;
  const int vb = blockIdx.x / a.n_splits, s = blockIdx.x % a.n_splits;   // vb = slice * B + sequence
  const int shard = vb / a.B, b = vb % a.B;
  const int h = blockIdx.y;
  const int L = seq_len_clipped(a, b);
  const int pt = a.page_tokens;
  const int n_pages = (L + pt - 1) / pt;
  const int p0 = s * a.pages_per_split;
  if (p0 >= n_pages) return;
  int p1 = p0 + a.pages_per_split;
  if (p1 > n_pages) p1 = n_pages;
  const int t_begin = p0 * pt;
  const int t_end = min(p1 * pt, L);

  const T* ql = static_cast<const T*>(a.q_lat) + ((size_t)vb * a.H + h) * dl;
  const T* qp = static_cast<const T*>(a.q_pe) + ((size_t)b * a.H + h) * dr;
  for (int i = tid; i < dl; i += GEN_THREADS) q[i] = load_as_f32(ql + i);
  for (int i = tid; i < dr; i += GEN_THREADS) q[dl + i] = load_as_f32(qp + i);
  __syncthreads();

  const T* pool = static_cast<const T*>(a.pools[shard]);
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  float acc[GEN_MAX_COLS];
#pragma unroll
  for (int c = 0; c < GEN_MAX_COLS; ++c) acc[c] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int t0 = t_begin; t0 < t_end; t0 += GEN_THREADS) {
    const int t = t0 + tid;
    float sc = -INFINITY;
    if (t < t_end) {
      const T* row = pool + ((size_t)bt[t / pt] * pt + (t % pt)) * w;
      float d = 0.f;
      for (int i = 0; i < w; ++i) d = fmaf(q[i], load_as_f32(row + i), d);
      sc = d * a.scale_log2;
    }
    // chunk maximum
    red[tid] = sc;
    __syncthreads();
    for (int o = GEN_THREADS / 2; o > 0; o >>= 1) {
      if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
      __syncthreads();
    }
    const float m_new = fmaxf(m_run, red[0]);
    __syncthreads();
    const float pv = (t < t_end) ? exp2f(sc - m_new) : 0.f;
    p[tid] = pv;
    red[tid] = pv;
    __syncthreads();
    for (int o = GEN_THREADS / 2; o > 0; o >>= 1) {
      if (tid < o) red[tid] += red[tid + o];
      __syncthreads();
    }
    const float alpha = exp2f(m_run - m_new);   // 0 on the first chunk
    l_run = l_run * alpha + red[0];
    m_run = m_new;
    const int cnt = min(GEN_THREADS, t_end - t0);
#pragma unroll
    for (int c = 0; c < GEN_MAX_COLS; ++c) {
      const int col = tid + c * GEN_THREADS;
      if (col < dl) {
        float v = acc[c] * alpha;
        for (int i = 0; i < cnt; ++i) {
          const int tt = t0 + i;
          const T* row = pool + ((size_t)bt[tt / pt] * pt + (tt % pt)) * w;
          v = fmaf(p[i], load_as_f32(row + col), v);
        }
        acc[c] = v;
      }
    }
    __syncthreads();
  }
  const size_t item = ((size_t)vb * a.n_splits + s) * a.H + h;
#pragma unroll
  for (int c = 0; c < GEN_MAX_COLS; ++c) {
    const int col = tid + c * GEN_THREADS;
    if (col < dl) a.part_acc[item * dl + col] = acc[c];
  }
  if (tid == 0) {
    a.part_ml[item * 2 + 0] = m_run;
    a.part_ml[item * 2 + 1] = l_run;
  }
}

// One workgroup = one (slice, sequence, head): combines that sequence's
// partial results in ascending order of the work items (fixed order =>
// reproducible bits).  Wave 0 lists the contributing slots and turns their
// (reference, weight-sum) pairs into one normalised factor each; then every
// thread sums its columns over the slots.
constexpr int MERGE_MAX_SPLITS = 1024;
__global__ void __launch_bounds__(128) decode_merge_kernel(DecodeArgs a) {
  __shared__ float wgt[MERGE_MAX_SPLITS];
  __shared__ int slot_of[MERGE_MAX_SPLITS];
  __shared__ int cnt_sh;
  const int vb = blockIdx.x / a.H, h = blockIdx.x % a.H;   // vb = slice * B + sequence
  const int b = vb % a.B;
  const int L = seq_len_clipped(a, b);
  const int n_pages = (L + a.page_tokens - 1) / a.page_tokens;
  const int dl = a.dl;
  float* out = a.o_lat + ((size_t)vb * a.H + h) * dl;
  if (n_pages == 0) {
    for (int c = threadIdx.x; c < dl; c += blockDim.x) out[c] = 0.f;
    if (a.lse && threadIdx.x == 0) a.lse[(size_t)vb * a.H + h] = -INFINITY;
    return;
  }
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int cnt;
    if (!a.balanced) {
      cnt = (n_pages + a.pages_per_split - 1) / a.pages_per_split;
      if (cnt > a.n_splits) cnt = a.n_splits;
      for (int s = lane; s < cnt; s += 64) slot_of[s] = vb * a.n_splits + s;
    } else {
      // workgroups whose page range of the plan meets [c0, c0 + n_pages): those from the
      // owner of the first page to the owner of the last; when there are fewer pages than workgroups
      // some ranges in between are empty and are left out, 64 candidates at a time
      const int n_v = a.n_shards * a.B;
      const int T = a.plan[n_v], c0 = a.plan[vb];
      // first owner and number of ranges: left in the plan table by the split kernel
      const int w0 = a.plan[n_v + 1 + vb], w1 = w0 + a.plan[2 * n_v + 1 + vb] - 1;
      if (a.plan[3 * n_v + 1] == 0) {
        cnt = w1 - w0 + 1;
        for (int s = lane; s < cnt; s += 64) slot_of[s] = w0 + s + vb;
      } else {
        cnt = 0;
        for (int base = w0; base <= w1; base += 64) {
          const int w = base + lane;
          const bool meets = w <= w1 && balanced_range_meets(a.geom, w, T, c0, c0 + n_pages);
          const unsigned long long mask = __ballot(meets);
          if (meets) slot_of[cnt + __popcll(mask & ((1ull << lane) - 1))] = w + vb;
          cnt += __popcll(mask);
        }
      }
    }
    if (lane == 0) cnt_sh = cnt;
    __builtin_amdgcn_wave_barrier();
    float M = -INFINITY;
    for (int s = lane; s < cnt; s += 64) M = fmaxf(M, a.part_ml[((size_t)slot_of[s] * a.H + h) * 2]);
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) M = fmaxf(M, __shfl_xor(M, m));
    float lsum = 0.f;
    for (int s = lane; s < cnt; s += 64) {
      const float* ml = a.part_ml + ((size_t)slot_of[s] * a.H + h) * 2;
      const float e = exp2f(ml[0] - M);
      wgt[s] = e;
      lsum = fmaf(ml[1], e, lsum);
    }
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) lsum += __shfl_xor(lsum, m);
    const float inv = 1.0f / lsum;
    for (int s = lane; s < cnt; s += 64) wgt[s] *= inv;
    if (a.lse && lane == 0) a.lse[(size_t)vb * a.H + h] = (M + log2f(lsum)) * 0.6931471805599453f;
  }
  __syncthreads();
  const int cnt = cnt_sh;
  if ((dl & 3) == 0) {
    for (int c = threadIdx.x * 4; c < dl; c += blockDim.x * 4) {
      float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
      int s = 0;
      for (; s + 4 <= cnt; s += 4) {          // four partial rows in flight; summed in slot order
        float4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          p[u] = *reinterpret_cast<const float4*>(a.part_acc + ((size_t)slot_of[s + u] * a.H + h) * dl + c);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float w = wgt[s + u];
          v0 = fmaf(p[u].x, w, v0); v1 = fmaf(p[u].y, w, v1); v2 = fmaf(p[u].z, w, v2); v3 = fmaf(p[u].w, w, v3);
        }
      }
      for (; s < cnt; ++s) {
        const float4 p = *reinterpret_cast<const float4*>(a.part_acc + ((size_t)slot_of[s] * a.H + h) * dl + c);
        const float w = wgt[s];
        v0 = fmaf(p.x, w, v0); v1 = fmaf(p.y, w, v1); v2 = fmaf(p.z, w, v2); v3 = fmaf(p.w, w, v3);
      }
      *reinterpret_cast<float4*>(out + c) = make_float4(v0, v1, v2, v3);
    }
  } else {
    for (int c = threadIdx.x; c < dl; c += blockDim.x) {
      float v = 0.f;
      for (int s = 0; s < cnt; ++s) v = fmaf(a.part_acc[((size_t)slot_of[s] * a.H + h) * dl + c], wgt[s], v);
      out[c] = v;
    }
  }
}

int launch_decode_generic(const DecodeArgs& a, int dtype, hipStream_t st) {
  if (a.dl > GEN_MAX_COLS * GEN_THREADS)
    return fail(TPLA_ERR_UNSUPPORTED, "d_c/g=%d above %d", a.dl, GEN_MAX_COLS * GEN_THREADS);
  const size_t smem = (size_t)(a.dl + a.d_r + 2 * GEN_THREADS) * sizeof(float);
  if (smem > 64 * 1024) return fail(TPLA_ERR_UNSUPPORTED, "row too wide for the generic kernel");
  if (a.H > 65535) return fail(TPLA_ERR_UNSUPPORTED, "H above 65535");
  dim3 grid((unsigned)(a.n_shards * a.B * a.n_splits), (unsigned)a.H);
  if (dtype == TPLA_F32)
    hipLaunchKernelGGL(decode_generic_kernel<float>, grid, dim3(GEN_THREADS), smem, st, a);
  else
    hipLaunchKernelGGL(decode_generic_kernel<bf16_t>, grid, dim3(GEN_THREADS), smem, st, a);
  return check_launch("decode_generic_kernel");
}

int launch_decode_merge(const DecodeArgs& a, hipStream_t st) {
  const int threads = a.dl >= 512 ? 128 : 64;
  hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)(a.n_shards * a.B * a.H)), dim3(threads), 0, st, a);
  return check_launch("decode_merge_kernel");
}

// ---------------------------------------------------------------------------
// Measurement aid: the plainest possible pass over a buffer -- every lane reads
// 16 bytes per step with the streaming hint, chunks of 20 KB dealt to the
// workgroups round-robin, five loads in flight per lane -- so that the decode
// kernel's rate can be set against what the same box delivers to a reader that
// does nothing else.  The XOR of everything read is stored only if it matches
// a value it cannot have, which keeps the loads alive.
__global__ void __launch_bounds__(256) stream_read_kernel(const u32x4* __restrict__ p, size_t n_chunks,
                                                          unsigned* __restrict__ sink) {
  constexpr int CH = 5;
  unsigned acc = 0;
  for (size_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const u32x4* s = p + c * (CH * 256) + threadIdx.x;
    u32x4 v[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) v[j] = __builtin_nontemporal_load(s + j * 256);
#pragma unroll
    for (int j = 0; j < CH; ++j) acc += v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
  }
  if (acc == 0x9E3779B9u && n_chunks == ~(size_t)0) sink[0] = acc;
}

int launch_stream_read(const void* buf, size_t bytes, void* sink, hipStream_t st) {
  const size_t n_chunks = bytes / (5 * 256 * 16);
  if (n_chunks == 0) return TPLA_OK;
  const int grid = device_cu_count() * 2;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const u32x4*>(buf),
                     n_chunks, static_cast<unsigned*>(sink));
  return check_launch("stream_read_kernel");
}

}  // namespace tpla
