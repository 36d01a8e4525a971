// bf16 GEMV family with a K-reduction tree that depends on K alone
// (operator family: Sec. 1 "GEMV", Sec. 2.3 "Split-K GEMMs"; LM-head logits and
// greedy token: Sec. 7.1 / 7.2 of the paper).
//
// Work decomposition (all of it a function of the shape, none of the CU count):
//   * a wave owns RW weight rows at a time ("row group") and walks `groups` of
//     them; a block is WAVES waves; grid.x = ceil(rows / (WAVES*R*groups));
//   * K is cut into tiles of 256 = 32 lanes x 8 contiguous bf16 (one 128-bit
//     load per lane); a wave covers two tiles per load instruction, lane l
//     taking elements [512 i + 8 l, 512 i + 8 l + 8) for i = 0, 1, ...;
//   * X is staged in LDS (kc elements of every batch row at a time) and read
//     back with conflict-free 128-bit reads, once per batch row per group of
//     RW weight loads.
// Reduction tree of one output, fixed by K:
//   1. within a lane: v_dot2 over the 4 bf16 pairs of a load in order, tiles in
//      ascending order, one fp32 accumulator per (row, batch row);
//   2. across the 64 lanes: the butterfly of wave_sum();
//   3. split-K baseline only: S partial sums added in chunk order.
// Epilogues: bf16 store; silu(gate)*up on the fp32 sums; fp32 logits + argmax.
#pragma once
#include "dev_util.h"
#include "kargs.h"
#include <limits.h>

enum { EPI_NONE = 0, EPI_SILU = 1, EPI_ARGMAX = 2 };

__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + expf(-g)); }

// Stage X[b, k0 : k0+klen) for every batch row into LDS rows of `kc` elements;
// positions up to the next multiple of 512 and batch rows >= B are zero-filled.
template <int BT>
__device__ __forceinline__ void stage_x(uint16_t* xs, const GemvArgs& a, int k0, int klen) {
  const int kpad = (klen + 511) & ~511;
  const int chunks_per_row = kpad >> 3;
  const int total = BT * chunks_per_row;
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    const int b = i / chunks_per_row, c = i - b * chunks_per_row;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (b < a.B && c * 8 < klen) v = ld16(a.X + static_cast<size_t>(b) * a.ldx + k0 + c * 8);
    *reinterpret_cast<u32x4*>(xs + b * a.kc + c * 8) = v;
  }
}

// Waves per SIMD the register allocation aims at (more rows in flight -> fewer waves).
constexpr int gemv_occupancy(int bt, int rw) { return rw * bt <= 16 ? 4 : (rw * bt <= 32 ? 3 : 2); }

template <int BT, int RW, int WAVES, int EPI>
__global__ __launch_bounds__(WAVES * 64, gemv_occupancy(BT, RW)) void gemv_kernel(const GemvArgs a) {
  static_assert(RW * BT <= 64, "one lane per (row, batch row) in the epilogue");
  static_assert(EPI != EPI_SILU || (RW % 2 == 0), "gate and up rows come in pairs");
  constexpr int R = (EPI == EPI_SILU) ? RW / 2 : RW;  // outputs per wave per group
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);
  __shared__ float s_bv[WAVES][BT];
  __shared__ int s_bi[WAVES][BT];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: row bases stay scalar
  const int split = blockIdx.y;
  const int k_begin = split * a.k_per_split;
  const int k_end = k_begin + a.k_per_split;
  const bool multi_chunk = a.kc < a.k_per_split;
  // lane i < RW*BT finishes (row r = i / BT, batch row b = i % BT)
  const int my_r = lane / BT, my_b = lane % BT;
  const bool my_live = lane < RW * BT && my_b < a.B;

  float best_v = -INFINITY;
  int best_i = INT_MAX;

  // ---- finish: lane-distributed fp32 totals -> epilogue ------------------------
  auto finish = [&](int out0, float v) {
    if constexpr (EPI == EPI_NONE) {
      const int n = out0 + my_r;
      if (my_live && n < a.n_out) a.Y[static_cast<size_t>(my_b) * a.ldy + n] = (uint16_t)f32_to_bf16(v);
    } else if constexpr (EPI == EPI_SILU) {
      const float u = __shfl(v, lane + R * BT, 64);  // the up row of the same output
      const int n = out0 + my_r;
      if (my_live && my_r < R && n < a.n_out)
        a.Y[static_cast<size_t>(my_b) * a.ldy + n] = (uint16_t)f32_to_bf16(silu_f32(v) * u);
    } else {
      const int n = out0 + my_r;
      if (my_live && n < a.N) {
        if (a.logits) a.logits[static_cast<size_t>(my_b) * a.N + n] = v;
        if (better(v, n, best_v, best_i)) { best_v = v; best_i = n; }
      }
    }
  };
  // weight row behind slot r of the group starting at output out0; -1 past the end
  auto weight_row = [&](int out0, int r) {
    if constexpr (EPI == EPI_SILU) {
      const int n = out0 + (r < R ? r : r - R);
      if (r >= RW || n >= a.n_out) return -1;
      return r < R ? n : a.n_out + n;
    } else {
      const int n = out0 + r;
      return (r >= RW || n >= a.N) ? -1 : n;
    }
  };

  // ---- phase A: accumulate ---------------------------------------------------------
  for (int g = 0; g < a.groups; ++g) {
    const int out0 = ((blockIdx.x * a.groups + g) * WAVES + wave) * R;
    const uint16_t* wp[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      int row = weight_row(out0, r);
      row = row >= 0 ? row : a.N - 1;  // slots past the end re-read the last row; results dropped
      wp[r] = a.W + static_cast<size_t>(row) * a.K;
    }
    float acc[RW][BT];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int b = 0; b < BT; ++b) acc[r][b] = 0.f;

    for (int k0 = k_begin; k0 < k_end; k0 += a.kc) {
      const int klen = (k_end - k0) < a.kc ? (k_end - k0) : a.kc;
      if (g == 0 || multi_chunk) {
        __syncthreads();
        stage_x<BT>(xs, a, k0, klen);
        __syncthreads();
      }
      // full 512-element steps: no lane checks; while one buffer is consumed the
      // other one's loads are in flight
      const int nfull = klen >> 9;
      auto step = [&](const u32x4(&w)[RW], int it) {
        const uint16_t* xrow = xs + it * 512 + lane * 8;
#pragma unroll
        for (int b = 0; b < BT; ++b) {
          const u32x4 xv = *reinterpret_cast<const u32x4*>(xrow + b * a.kc);
#pragma unroll
          for (int r = 0; r < RW; ++r) acc[r][b] = dot8_bf16(w[r], xv, acc[r][b]);
        }
      };
      auto load = [&](u32x4(&w)[RW], int it) {
#pragma unroll
        for (int r = 0; r < RW; ++r) w[r] = ld16_stream(wp[r] + k0 + it * 512 + lane * 8);
      };
      u32x4 w0[RW], w1[RW];
      if (nfull > 0) load(w0, 0);
      int it = 0;
      for (; it + 2 <= nfull; it += 2) {
        load(w1, it + 1);
        step(w0, it);
        if (it + 2 < nfull) load(w0, it + 2);
        step(w1, it + 1);
      }
      if (it < nfull) {
        step(w0, it);
        ++it;
      }
      if (klen & 511) {  // ragged tail: lanes past the end contribute +0
        const int kk = it * 512 + lane * 8;
#pragma unroll
        for (int r = 0; r < RW; ++r)
          w0[r] = (kk < klen) ? ld16_stream(wp[r] + k0 + kk) : u32x4{0u, 0u, 0u, 0u};
        step(w0, it);
      }
    }

    // butterfly over lanes, then hand (r, b) to lane r*BT + b
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        const float t = wave_sum(acc[r][b]);
        if (lane == r * BT + b) mine = t;
      }

    if (a.S == 1) {
      finish(out0, mine);
    } else {
      const int row = weight_row(out0, my_r);
      if (my_live && row >= 0)
        a.partials[(static_cast<size_t>(split) * BT + my_b) * a.N + row] = mine;
    }
  }

  // ---- phase B (split-K baseline): the last chunk-block of this row block sums ----
  if (a.S > 1) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t t = atomicAdd(&a.ws[1 + blockIdx.x], 1u);
      s_last = (t == static_cast<uint32_t>(a.S) - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int g = 0; g < a.groups; ++g) {
      const int out0 = ((blockIdx.x * a.groups + g) * WAVES + wave) * R;
      const int row = weight_row(out0, my_r);
      float v = 0.f;
      if (my_live && row >= 0) {
        for (int s = 0; s < a.S; ++s)  // chunk order
          v += __builtin_nontemporal_load(&a.partials[(static_cast<size_t>(s) * BT + my_b) * a.N + row]);
      }
      finish(out0, v);
    }
    if (threadIdx.x == 0) a.ws[1 + blockIdx.x] = 0u;  // ready for the next launch
  }

  // ---- phase C (LM head): block argmax -> workspace -> last block picks the token --
  if constexpr (EPI == EPI_ARGMAX) {
    // lanes with the same batch row sit BT apart
#pragma unroll
    for (int d = BT; d < 64; d <<= 1) {
      const float ov = __shfl_xor(best_v, d, 64);
      const int oi = __shfl_xor(best_i, d, 64);
      if (better(ov, oi, best_v, best_i)) { best_v = ov; best_i = oi; }
    }
    if (lane < BT) { s_bv[wave][lane] = best_v; s_bi[wave][lane] = best_i; }
    __syncthreads();
    uint32_t* part = a.ws + 1 + gridDim.x;  // [gridDim.x][BT][2]
    if (threadIdx.x < BT) {
      float bv = s_bv[0][threadIdx.x];
      int bi = s_bi[0][threadIdx.x];
#pragma unroll
      for (int w = 1; w < WAVES; ++w)
        if (better(s_bv[w][threadIdx.x], s_bi[w][threadIdx.x], bv, bi)) { bv = s_bv[w][threadIdx.x]; bi = s_bi[w][threadIdx.x]; }
      part[(blockIdx.x * BT + threadIdx.x) * 2 + 0] = __float_as_uint(bv);
      part[(blockIdx.x * BT + threadIdx.x) * 2 + 1] = static_cast<uint32_t>(bi);
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t t = atomicAdd(&a.ws[0], 1u);
      s_last = (t == gridDim.x - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    // every block has published its (value, index) pairs: reduce them per batch row
    for (int b = wave; b < a.B; b += WAVES) {
      float bv = -INFINITY;
      int bi = INT_MAX;
      for (unsigned blk = lane; blk < gridDim.x; blk += 64) {
        const float v = __uint_as_float(__builtin_nontemporal_load(&part[(blk * BT + b) * 2 + 0]));
        const int i = static_cast<int>(__builtin_nontemporal_load(&part[(blk * BT + b) * 2 + 1]));
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
      }
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const float ov = __shfl_xor(bv, d, 64);
        const int oi = __shfl_xor(bi, d, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (lane == 0) a.tok[b] = (bi == INT_MAX) ? 0 : bi;
    }
    if (threadIdx.x == 0) a.ws[0] = 0u;
  }
}

#define VTE_GEMV_CASE(BT, RW, WV, EPI) \
  if (bt == BT && rw == RW && waves == WV && epi == EPI) return (const void*)gemv_kernel<BT, RW, WV, EPI>;

// One translation unit per BT instantiates these.
#define VTE_GEMV_ENTRY_FOR_BT(BT)                                                   \
  extern "C" const void* vte_gemv_entry_b##BT(int bt, int rw, int waves, int epi) { \
    VTE_GEMV_CASES(BT)                                                              \
    return nullptr;                                                                 \
  }
