// Embedding gather: H[b,:] = E[tok[b],:], 128-bit copies.  Grid and block depend
// on (B, K) only.
#include "dev_util.h"
#include "kargs.h"

__global__ __launch_bounds__(256) void gather_kernel(const GatherArgs a) {
  const int b = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;  // 8-element chunk within the row
  if (b >= a.B || c * 8 >= a.K) return;
  int t = a.tok[b];
  t = t < 0 ? 0 : (t >= a.V ? a.V - 1 : t);
  st16(a.H + static_cast<size_t>(b) * a.K + c * 8, ld16(a.E + static_cast<size_t>(t) * a.K + c * 8));
}

// Greedy token, second stage: one workgroup per batch row scans the candidates of
// every LM-head workgroup.  (value, index) pairs are totally ordered (larger
// value, then lower index; NaN never wins), so the scan order cannot matter.
__global__ __launch_bounds__(1024) void argmax_finish_kernel(const ArgmaxFinishArgs a) {
  __shared__ float s_v[16];
  __shared__ int s_i[16];
  const int b = blockIdx.x;
  if (b >= a.B) return;
  const uint32_t* cv = a.pairs + static_cast<size_t>(b) * a.nblocks;
  const uint32_t* ci = a.pairs + static_cast<size_t>(a.bt) * a.nblocks + static_cast<size_t>(b) * a.nblocks;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  // eight independent candidates per thread and pass: all loads of a pass are in flight together
  for (int base = 0; base < a.nblocks; base += 8 * 1024) {
    float v[8];
    int idx[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int blk = base + j * 1024 + threadIdx.x;
      const bool in = blk < a.nblocks;
      v[j] = in ? __uint_as_float(cv[blk]) : -INFINITY;
      idx[j] = in ? static_cast<int>(ci[blk]) : 0x7fffffff;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (better(v[j], idx[j], bv, bi)) { bv = v[j]; bi = idx[j]; }
  }
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const float ov = __shfl_xor(bv, d, 64);
    const int oi = __shfl_xor(bi, d, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { s_v[threadIdx.x >> 6] = bv; s_i[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w)
      if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
    a.tok[b] = (bi == 0x7fffffff) ? 0 : bi;
  }
}

// Device-to-device copy and 32-bit fill as launches of their own (the data-movement nodes of a
// virtual-stream graph, Sec. 4.2): 16 bytes per thread and pass, four passes per workgroup, grid from
// the byte count alone.
__global__ __launch_bounds__(256) void copy_kernel(const CopyArgs a) {
  const size_t base = (static_cast<size_t>(blockIdx.x) * 4 * 256 + threadIdx.x) * 16;
  // all four loads before the first store (dst and src may not overlap, but the compiler cannot know:
  // written one by one, every load waits for the store before it)
  u32x4 v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const size_t off = base + static_cast<size_t>(j) * 256 * 16;
    v[j] = off < a.bytes ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a.src + off)) : u32x4{0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const size_t off = base + static_cast<size_t>(j) * 256 * 16;
    if (off < a.bytes) __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4*>(a.dst + off));
  }
}

__global__ __launch_bounds__(256) void fill_kernel(const FillArgs a) {
  const size_t base = (static_cast<size_t>(blockIdx.x) * 4 * 256 + threadIdx.x) * 16;
  const u32x4 v = u32x4{a.value, a.value, a.value, a.value};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const size_t off = base + static_cast<size_t>(j) * 256 * 16;
    if (off < a.bytes) *reinterpret_cast<u32x4*>(a.dst + off) = v;
  }
}

// Softmax probability of the chosen token under the fp32 logits of an LM-head launch (Sec. 7.2:
// the decode replay records it next to the token).  One workgroup of 1024 threads per batch row.
// The maximum is exact whatever the order.  Tree of the sum of exp(l - max), fixed by V: thread t
// adds elements t, t + 1024, ... in ascending order, the 64 lanes of a wave are combined by
// wave_sum(), the 16 wave partials are added in wave order.  p = exp(l[tok] - max) / sum.
__global__ __launch_bounds__(1024) void softmax_prob_kernel(const SoftmaxArgs a) {
  __shared__ float red[16];
  const int b = blockIdx.x;
  if (b >= a.B) return;
  const float* l = a.logits + static_cast<size_t>(b) * a.V;
  float m = -INFINITY;
  for (int v = threadIdx.x; v < a.V; v += 1024) m = fmaxf(m, l[v]);  // fmaxf drops a NaN operand
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) m = fmaxf(m, red[w]);
  __syncthreads();
  float s = 0.f;
  for (int v = threadIdx.x; v < a.V; v += 1024) s += expf(l[v] - m);
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = red[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) tot += red[w];
    const int t = a.tok[b];
    a.prob[b] = (t >= 0 && t < a.V) ? expf(l[t] - m) / tot : 0.f;
  }
}

// Finish launch of the shape-derived K split: output n of batch row b is p[0] + p[1] + ... + p[S-1]
// (fp32, ascending split index) of the partial sums the split launch left behind, then the epilogue
// and one rounding to bf16.  One thread per four consecutive outputs of one batch row.
__global__ __launch_bounds__(256) void split_finish_kernel(const SplitFinishArgs a) {
  const int b = blockIdx.y;
  const int n0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (b >= a.B || n0 >= a.n_out) return;
  float g[4], u[4];
  const size_t stride = static_cast<size_t>(a.bt) * a.N;
  int off[4];  // clamped: a tail thread re-reads the last output
#pragma unroll
  for (int v = 0; v < 4; ++v) off[v] = (n0 + v < a.n_out ? n0 + v : a.n_out - 1) - n0;
  // The parts of an output are added in ascending order; their loads do not depend on one another
  // and are requested eight parts at a time (a loop of load-then-add pays a memory round trip per part).
  auto sum_parts = [&](const float* p0, float(&out)[4]) {
    const bool vec = n0 + 3 < a.n_out && (reinterpret_cast<uintptr_t>(p0) & 15) == 0 && (stride & 3) == 0;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int v = 0; v < 4; ++v) out[v] = 0.f;
    for (int s0 = 0; s0 < a.S; s0 += 8) {
      f32x4 t[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float* q = p0 + static_cast<size_t>(s0 + j) * stride;
        if (s0 + j >= a.S) t[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        else if (vec) t[j] = *reinterpret_cast<const f32x4*>(q);
        else t[j] = f32x4{q[off[0]], q[off[1]], q[off[2]], q[off[3]]};
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (s0 + j >= a.S) break;
#pragma unroll
        for (int v = 0; v < 4; ++v) out[v] = (s0 + j == 0) ? t[j][v] : out[v] + t[j][v];
      }
    }
  };
  const float* p = a.partials + static_cast<size_t>(b) * a.N + n0;
  sum_parts(p, g);
  if (a.silu) sum_parts(p + a.n_out, u);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    if (n0 + v >= a.n_out) break;
    const float r = a.silu ? (g[v] / (1.0f + expf(-g[v]))) * u[v] : g[v];
    a.Y[static_cast<size_t>(b) * a.ldy + n0 + v] = (uint16_t)f32_to_bf16(r);
  }
}

extern "C" const void* vte_split_finish_entry() { return (const void*)split_finish_kernel; }
extern "C" const void* vte_softmax_prob_entry() { return (const void*)softmax_prob_kernel; }
extern "C" const void* vte_copy_entry() { return (const void*)copy_kernel; }
extern "C" const void* vte_fill_entry() { return (const void*)fill_kernel; }
extern "C" const void* vte_argmax_finish_entry() { return (const void*)argmax_finish_kernel; }
extern "C" const void* vte_gather_entry() { return (const void*)gather_kernel; }
