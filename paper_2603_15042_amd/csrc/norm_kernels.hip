// RMSNorm / LayerNorm with a reduction tree fixed by the row length alone
// (operator family: Sec. 1 and Sec. 2.3 of the paper; reshaped variant: the
// negative control of Sec. 7.1).
//
// With a token list the input row is fetched from an embedding table (gather
// fused into the norm); the arithmetic is the same.  The token may also come
// straight from the candidates of the LM-head launch before (greedy-token finish
// fused in as well: Sec. 7.1 / 7.2 decode loop, one launch fewer per step).
// One workgroup of T threads per row.  Thread t owns the 8-element chunks
// t, t+T, t+2T, ... of the row (128-bit loads, coalesced across the wave) and
// keeps them in registers, so the row is read from HBM exactly once.
// Reduction tree of a row sum:
//   1. a thread adds the squares of its elements in ascending index order;
//   2. the 64 lanes of a wave are combined by the fixed butterfly wave_sum();
//   3. wave partials go through LDS and every thread adds them in wave order.
// T is chosen from the row length on the host (never from a CU count), except in
// the *_reshaped descriptor where the caller derives it from a CU count on
// purpose.
#include "dev_util.h"
#include "kargs.h"
#include <limits.h>

constexpr int kMaxChunks = 8;  // per thread: cols <= 8 * 8 * T

template <int T>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  constexpr int NW = T / 64;
  if constexpr (NW == 1) return v;
  const int wave = threadIdx.x >> 6;
  __syncthreads();  // red[] may still be read from a previous reduction
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s += red[w];
  return s;
}

template <int T, bool LAYER>
__global__ __launch_bounds__(T) void norm_kernel(const NormArgs a) {
  __shared__ float red[T / 64];
  __shared__ float s_cv[T / 64];
  __shared__ int s_ci[T / 64];
  const int row = blockIdx.x;
  if (row >= a.rows) return;
  const int nchunks = a.cols >> 3;
  // gamma (and beta) do not depend on anything this launch computes: requested first, so that their
  // latency is covered by the token reduction and the row fetch instead of following the row sum
  u32x4 gv[kMaxChunks], bv4[kMaxChunks];
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c = threadIdx.x + j * T;
    gv[j] = (c < nchunks) ? ld16(a.gamma + c * 8) : u32x4{0u, 0u, 0u, 0u};
    if constexpr (LAYER) bv4[j] = (c < nchunks) ? ld16(a.beta + c * 8) : u32x4{0u, 0u, 0u, 0u};
  }
  size_t src_row = row;
  if (a.cand) {
    // greedy token of this batch row: best (value, lowest index) over the candidates;
    // the comparison is a total order, so the order of the reduction does not matter
    const uint32_t* cv = a.cand + static_cast<size_t>(row) * a.nblocks;
    const uint32_t* ci = a.cand + static_cast<size_t>(a.cand_bt) * a.nblocks + static_cast<size_t>(row) * a.nblocks;
    float bv = -INFINITY;
    int bi = INT_MAX;
    // four candidates per thread are requested before the first is looked at: for up to 4 T
    // workgroups of the LM head (501 at the Llama-8B shape) the reduction costs one memory round trip
    for (int base = 0; base < a.nblocks; base += 4 * T) {
      float v[4];
      int ix[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int blk = base + u * T + static_cast<int>(threadIdx.x);
        const bool ok = blk < a.nblocks;
        v[u] = ok ? __uint_as_float(cv[blk]) : -INFINITY;
        ix[u] = ok ? static_cast<int>(ci[blk]) : INT_MAX;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (better(v[u], ix[u], bv, bi)) { bv = v[u]; bi = ix[u]; }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const float ov = __shfl_xor(bv, d, 64);
      const int oi = __shfl_xor(bi, d, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { s_cv[threadIdx.x >> 6] = bv; s_ci[threadIdx.x >> 6] = bi; }
    __syncthreads();
    bv = s_cv[0];
    bi = s_ci[0];
#pragma unroll
    for (int w = 1; w < T / 64; ++w)
      if (better(s_cv[w], s_ci[w], bv, bi)) { bv = s_cv[w]; bi = s_ci[w]; }
    int t = (bi == INT_MAX) ? 0 : bi;  // all-NaN row
    if (threadIdx.x == 0 && a.tok_out) a.tok_out[row] = t;
    src_row = t < 0 ? 0 : (t >= a.V ? a.V - 1 : t);
  } else if (a.tok) {  // fused embedding gather: the row comes from the table
    int t = a.tok[row];
    src_row = t < 0 ? 0 : (t >= a.V ? a.V - 1 : t);
  }
  const uint16_t* xr = a.x + src_row * a.cols;
  uint16_t* yr = a.y + static_cast<size_t>(row) * a.cols;

  u32x4 xv[kMaxChunks];
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c = threadIdx.x + j * T;
    xv[j] = (c < nchunks) ? ld16(xr + c * 8) : u32x4{0u, 0u, 0u, 0u};
    if (a.h_out && c < nchunks) st16(a.h_out + static_cast<size_t>(row) * a.cols + c * 8, xv[j]);
  }

  float mu = 0.f;
  if constexpr (LAYER) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxChunks; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s += bf16_lo(xv[j][e]);
        s += bf16_hi(xv[j][e]);
      }
    }
    mu = block_sum<T>(s, red) / static_cast<float>(a.cols);  // a true division: exact when the mean is representable
  }

  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const bool live = (threadIdx.x + j * T) < nchunks;  // padding must not add (0-mu)^2
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = bf16_lo(xv[j][e]) - mu, hi = bf16_hi(xv[j][e]) - mu;
      ss = live ? fmaf(lo, lo, ss) : ss;
      ss = live ? fmaf(hi, hi, ss) : ss;
    }
  }
  ss = block_sum<T>(ss, red);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(a.cols) + a.eps);

#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c = threadIdx.x + j * T;
    if (c < nchunks) {
      const u32x4 g = gv[j];
      u32x4 b = u32x4{0u, 0u, 0u, 0u};
      if constexpr (LAYER) b = bv4[j];
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float lo = (bf16_lo(xv[j][e]) - mu) * rstd * bf16_lo(g[e]);
        float hi = (bf16_hi(xv[j][e]) - mu) * rstd * bf16_hi(g[e]);
        if constexpr (LAYER) {
          lo += bf16_lo(b[e]);
          hi += bf16_hi(b[e]);
        }
        o[e] = pack_bf16(lo, hi);
      }
      st16(yr + c * 8, o);
    }
  }
}

// Many short rows (rows >= 512, cols <= 4096, no gather): one wave per row, no LDS
// and no barrier.  A workgroup is four waves, one row each; lane l owns the 8-element
// chunks l, l+64, ... of its row.  Nothing is prefetched in software: the kernel is
// written to need few registers (the row stays packed between the two passes), so five
// waves share a SIMD and the other nineteen waves of a CU cover a wave's wait -- timed
// against a version that walked four rows per wave with the next row requested ahead
// (160 registers, three waves per SIMD): +6 % on 256 CUs, +12 to 19 % on 32 to 192.
// Reduction tree of a row sum: a lane adds its elements in ascending index order, the
// 64 lanes are combined by wave_sum().  Grid and tree follow from (rows, cols) alone.
template <bool LAYER, int NCH>
__global__ __launch_bounds__(256) void norm_rows_kernel(const NormArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunks = a.cols >> 3;
  const int row = blockIdx.x * 4 + wave;
  if (row >= a.rows) return;  // the same for every lane of the wave
  u32x4 g[NCH], bt[NCH], cur[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane + 64 * j;
    g[j] = (c < nchunks) ? ld16(a.gamma + c * 8) : u32x4{0u, 0u, 0u, 0u};
    if constexpr (LAYER) bt[j] = (c < nchunks) ? ld16(a.beta + c * 8) : u32x4{0u, 0u, 0u, 0u};
    cur[j] = (c < nchunks) ? ld16_stream(a.x + static_cast<size_t>(row) * a.cols + c * 8) : u32x4{0u, 0u, 0u, 0u};
  }
  float mu = 0.f;
  if constexpr (LAYER) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s += bf16_lo(cur[j][e]);
        s += bf16_hi(cur[j][e]);
      }
    }
    mu = wave_sum(s) / static_cast<float>(a.cols);
  }
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const bool live = (lane + 64 * j) < nchunks;  // padding must not add (0-mu)^2
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = bf16_lo(cur[j][e]) - mu, hi = bf16_hi(cur[j][e]) - mu;
      ss = live ? fmaf(lo, lo, ss) : ss;
      ss = live ? fmaf(hi, hi, ss) : ss;
    }
  }
  ss = wave_sum(ss);
  const float rstd = 1.0f / sqrtf(ss / static_cast<float>(a.cols) + a.eps);
  uint16_t* yr = a.y + static_cast<size_t>(row) * a.cols;
  // the row stays packed between the two passes: unpacked copies kept across the reduction would
  // cost 64 registers and with them a wave per SIMD
#pragma unroll
  for (int j = 0; j < NCH; ++j) asm volatile("" : "+v"(cur[j]));
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane + 64 * j;
    if (c < nchunks) {
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float lo = (bf16_lo(cur[j][e]) - mu) * rstd * bf16_lo(g[j][e]);
        float hi = (bf16_hi(cur[j][e]) - mu) * rstd * bf16_hi(g[j][e]);
        if constexpr (LAYER) {
          lo += bf16_lo(bt[j][e]);
          hi += bf16_hi(bt[j][e]);
        }
        o[e] = pack_bf16(lo, hi);
      }
      st16(yr + c * 8, o);
    }
  }
}

// Host side: entry of the wave-per-row kernel for `chunks` 8-element chunks per lane (2, 4 or 8).
extern "C" const void* vte_norm_rows_entry(int chunks, int layer) {
  switch (chunks) {
    case 2: return layer ? (const void*)norm_rows_kernel<true, 2> : (const void*)norm_rows_kernel<false, 2>;
    case 4: return layer ? (const void*)norm_rows_kernel<true, 4> : (const void*)norm_rows_kernel<false, 4>;
    case 8: return layer ? (const void*)norm_rows_kernel<true, 8> : (const void*)norm_rows_kernel<false, 8>;
  }
  return nullptr;
}
extern "C" int vte_norm_rows_per_block(void) { return 4; }

// Host side: kernel entry for a thread count (64, 128, 256 or 512).
extern "C" const void* vte_norm_entry(int threads, int layer) {
  switch (threads) {
    case 64:  return layer ? (const void*)norm_kernel<64, true>  : (const void*)norm_kernel<64, false>;
    case 128: return layer ? (const void*)norm_kernel<128, true> : (const void*)norm_kernel<128, false>;
    case 256: return layer ? (const void*)norm_kernel<256, true> : (const void*)norm_kernel<256, false>;
    case 512: return layer ? (const void*)norm_kernel<512, true> : (const void*)norm_kernel<512, false>;
  }
  return nullptr;
}
