// bf16 GEMV family with a K-reduction tree that depends on K alone
// (operator family: Sec. 1 "GEMV", Sec. 2.3 "Split-K GEMMs"; LM-head logits and
// greedy token: Sec. 7.1 / 7.2 of the paper).
//
// Work decomposition (all of it a function of the shape, none of the CU count):
//   * K is cut into tiles of 256 = 32 lanes x 8 contiguous bf16 (one 128-bit
//     load per lane); a wave covers two tiles (512 elements) per load
//     instruction ("k-step"), lane l taking elements [512 i + 8 l, +8);
//   * a workgroup is one wave per K-slice of KS consecutive k-steps: wave w owns
//     k-steps [w KS, (w+1) KS) and keeps its slice of X in registers for the
//     whole launch, so X costs no LDS or cache traffic in the hot loop;
//   * the workgroup walks `groups` row groups of R weight rows; the waves of a
//     workgroup together read each row contiguously, once, with R*KS 128-bit
//     loads per lane in flight (and the next group's loads behind them).
// Reduction tree of one output, fixed by K:
//   1. within a lane: v_dot2 over the 4 bf16 pairs of a load in order, the KS
//      k-steps of the slice in ascending order, one fp32 accumulator (what one
//      v_dot2c_f32_bf16 does to it was measured; tests/tree_emulator.py reproduces it);
//   2. across the 64 lanes of the wave: partner distances 32, 16 (lane-half and
//      row swaps), then 8, 4, 2, 1 (row rotations); the R*BT sums of a group
//      are reduced together so that the swaps halve the live values each time,
//      but every sum goes through exactly this butterfly;
//   3. across the waves (K-slices) of the workgroup in ascending slice order,
//      through LDS;
//   4. split-K baseline only: S chunk sums added in chunk order.
// Epilogues: bf16 store; silu(gate)*up on the fp32 sums; fp32 logits + per-workgroup
// argmax candidates (value, lowest index), one pair per batch row.
#pragma once
#include "dev_util.h"
#include "kargs.h"
#include <limits.h>

enum { EPI_NONE = 0, EPI_SILU = 1, EPI_ARGMAX = 2 };
constexpr int kMaxWaves = 16;

__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + expf(-g)); }

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Sum over the 16 lanes of a row by rotations 8, 4, 2, 1: every lane of the row
// ends with the same bits.
__device__ __forceinline__ float row_allsum(float v) {
  v += dpp_mov<0x128>(v);
  v += dpp_mov<0x124>(v);
  v += dpp_mov<0x122>(v);
  v += dpp_mov<0x121>(v);
  return v;
}
// a <- {a.lanes[0:32), b.lanes[0:32)}, b <- {a.lanes[32:64), b.lanes[32:64)}; returns a + b:
// lanes < 32 hold a[l] + a[l+32], lanes >= 32 hold b[l-32] + b[l].
// (Written as an instruction because the two-result builtin of this compiler
// returns its first result twice; the s_nop covers the VALU-write -> swap hazard.)
__device__ __forceinline__ float swap_add32(float a, float b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return a + b;
}
// Same with rows of 16 lanes: odd rows of a swap with even rows of b.
__device__ __forceinline__ float swap_add16(float a, float b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return a + b;
}
// Butterfly-sums NV per-lane values over the wave; lane l ends with the total of
// value value_of_lane<NV>(l) (or nothing if that is -1).
template <int NV>
__device__ __forceinline__ float reduce_values(float (&v)[NV], int lane) {
  static_assert(NV == 16 || NV == 32 || NV == 64, "");
  float a[NV / 2];
#pragma unroll
  for (int j = 0; j < NV / 2; ++j) a[j] = swap_add32(v[j], v[j + NV / 2]);
  float b[NV / 4];
#pragma unroll
  for (int j = 0; j < NV / 4; ++j) b[j] = swap_add16(a[j], a[j + NV / 4]);
  float mine = 0.f;
#pragma unroll
  for (int j = 0; j < NV / 4; ++j) {
    const float t = row_allsum(b[j]);
    if ((lane & 15) == j) mine = t;
  }
  return mine;
}
template <int NV>
__device__ __forceinline__ int value_of_lane(int l) {
  return ((l & 15) < NV / 4) ? (l & 15) + (NV / 4) * ((l >> 4) & 1) + (NV / 2) * (l >> 5) : -1;
}

template <int BT, int R, int KS, bool PF, int MAXW, int EPI>
__global__ __launch_bounds__(MAXW * 64) void gemv_kernel(const GemvArgs a) {
  constexpr int NV = R * BT;  // sums per wave per group
  static_assert(NV == 16 || NV == 32 || NV == 64, "R * BT must be 16, 32 or 64");
  static_assert(EPI != EPI_SILU || (R % 2 == 0), "gate and up rows come in pairs");
  constexpr int ROUT = (EPI == EPI_SILU) ? R / 2 : R;  // outputs per group
  __shared__ float part[2][MAXW][NV];
  __shared__ float s_bv[MAXW][BT];
  __shared__ int s_bi[MAXW][BT];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: row bases stay scalar
  const int nw = blockDim.x >> 6;
  const int split = blockIdx.y;
  const int k_begin = split * a.k_per_split;
  const int k_end = k_begin + a.k_per_split;
  // batch rows [b0, b0 + nb) of this workgroup (a second batch chunk re-reads the weights)
  const int b0 = blockIdx.z * BT;
  const int nb = (a.B - b0) < BT ? (a.B - b0) : BT;

  // this wave's slice of X, for every batch row, in registers
  u32x4 xs[KS][BT];
  int koff[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    koff[s] = k_begin + (wave * KS + s) * 512 + lane * 8;
#pragma unroll
    for (int b = 0; b < BT; ++b)
      xs[s][b] = (koff[s] < k_end && b < nb) ? ld16(a.X + static_cast<size_t>(b0 + b) * a.ldx + koff[s])
                                              : u32x4{0u, 0u, 0u, 0u};
  }

  // weight row behind slot r of group g; -1 past the end
  auto weight_row = [&](int g, int r) {
    const int out0 = (blockIdx.x * a.groups + g) * ROUT;
    if constexpr (EPI == EPI_SILU) {
      const int n = out0 + (r < ROUT ? r : r - ROUT);
      if (n >= a.n_out) return -1;
      return r < ROUT ? n : a.n_out + n;
    } else {
      const int n = out0 + r;
      return n >= a.N ? -1 : n;
    }
  };
  auto load = [&](u32x4(&dst)[R][KS], int g) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      int row = weight_row(g, r);
      row = row >= 0 ? row : a.N - 1;  // slots past the end re-read the last row; results dropped
      const uint16_t* wp = a.W + static_cast<size_t>(row) * a.K;
#pragma unroll
      for (int s = 0; s < KS; ++s)
        dst[r][s] = (koff[s] < k_end) ? ld16_stream(wp + koff[s]) : u32x4{0u, 0u, 0u, 0u};
    }
  };

  // lane j < NV of the finishing wave owns (slot r = j / BT, batch row b = j % BT)
  const int fin_r = lane / BT, fin_b = b0 + lane % BT;  // fin_b: global batch row
  const bool fin_live = lane < NV && (lane % BT) < nb;
  float best_v = -INFINITY;
  int best_i = INT_MAX;
  auto finish = [&](int g, float v) {  // called by all lanes of one wave
    const int row = fin_live ? weight_row(g, fin_r) : -1;
    if constexpr (EPI == EPI_NONE) {
      if (row >= 0) a.Y[static_cast<size_t>(fin_b) * a.ldy + row] = (uint16_t)f32_to_bf16(v);
    } else if constexpr (EPI == EPI_SILU) {
      const float u = __shfl(v, lane + ROUT * BT, 64);  // the up row of the same output
      if (row >= 0 && fin_r < ROUT)
        a.Y[static_cast<size_t>(fin_b) * a.ldy + row] = (uint16_t)f32_to_bf16(silu_f32(v) * u);
    } else {
      if (row >= 0) {
        if (a.logits) a.logits[static_cast<size_t>(fin_b) * a.N + row] = v;
        if (better(v, row, best_v, best_i)) { best_v = v; best_i = row; }
      }
    }
  };

  // ---- phase A: stream the rows ------------------------------------------------------
  const int my_value = value_of_lane<NV>(lane);
  u32x4 w[R][KS], wn[R][KS];
  load(w, 0);
  for (int g = 0; g < a.groups; ++g) {
    if constexpr (PF) {
      if (g + 1 < a.groups) load(wn, g + 1);
    }
    float v[NV];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int b = 0; b < BT; ++b) {
        float acc = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = dot8_bf16(w[r][s], xs[s][b], acc);
        v[r * BT + b] = acc;
      }
    if constexpr (!PF) {
      if (g + 1 < a.groups) load(w, g + 1);
    }
    const float mine = reduce_values<NV>(v, lane);
    float* slot = part[g & 1][wave];
    if (my_value >= 0) slot[my_value] = mine;
    __syncthreads();
    // slices are added in ascending order by one wave; the others move on (the
    // other half of part[] is not rewritten before the next barrier)
    if (wave == g % nw) {
      float s = 0.f;
      if (lane < NV) {
        // all MAXW slots exist in LDS: read them at once (one LDS latency, not one per wave), then
        // add those of the waves there are, in ascending order
        float pw[MAXW];
#pragma unroll
        for (int ww = 0; ww < MAXW; ++ww) pw[ww] = part[g & 1][ww][lane];
        s = pw[0];
#pragma unroll
        for (int ww = 1; ww < MAXW; ++ww) s = ww < nw ? s + pw[ww] : s;
      }
      if (a.S == 1) {
        finish(g, s);
      } else {
        const int row = fin_live ? weight_row(g, fin_r) : -1;
        if (row >= 0) a.partials[(static_cast<size_t>(split) * a.bt + fin_b) * a.N + row] = s;
      }
    }
    if constexpr (PF) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int s = 0; s < KS; ++s) w[r][s] = wn[r][s];
    }
  }

  // ---- phase B (split-K baseline): the last chunk-block of this row block sums ----
  if (a.S > 1) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t t = atomicAdd(&a.ws[1 + blockIdx.z * gridDim.x + blockIdx.x], 1u);
      s_last = (t == static_cast<uint32_t>(a.S) - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int g = wave; g < a.groups; g += nw) {
      const int row = fin_live ? weight_row(g, fin_r) : -1;
      float v = 0.f;
      if (row >= 0) {
        for (int s = 0; s < a.S; ++s)  // chunk order
          v += __builtin_nontemporal_load(&a.partials[(static_cast<size_t>(s) * a.bt + fin_b) * a.N + row]);
      }
      finish(g, v);
    }
    if (threadIdx.x == 0) a.ws[1 + blockIdx.z * gridDim.x + blockIdx.x] = 0u;  // ready for the next launch
  }

  // ---- phase C (LM head): block argmax -> (value, index) pair per batch row in the workspace;
  // the pairs of all workgroups are reduced by the argmax-finish launch that follows ----
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
    // candidates: values [a.bt][gridDim.x] then indices [a.bt][gridDim.x], so the finish reads rows
    uint32_t* cand_v = a.ws + 1 + gridDim.x * gridDim.z;
    uint32_t* cand_i = cand_v + static_cast<size_t>(a.bt) * gridDim.x;
    if (threadIdx.x < BT) {
      float wv[MAXW];
      int wi[MAXW];
#pragma unroll
      for (int ww = 0; ww < MAXW; ++ww) { wv[ww] = s_bv[ww][threadIdx.x]; wi[ww] = s_bi[ww][threadIdx.x]; }
      float bv = wv[0];
      int bi = wi[0];
#pragma unroll
      for (int ww = 1; ww < MAXW; ++ww)
        if (ww < nw && better(wv[ww], wi[ww], bv, bi)) { bv = wv[ww]; bi = wi[ww]; }
      cand_v[static_cast<size_t>(b0 + threadIdx.x) * gridDim.x + blockIdx.x] = __float_as_uint(bv);
      cand_i[static_cast<size_t>(b0 + threadIdx.x) * gridDim.x + blockIdx.x] = static_cast<uint32_t>(bi);
    }
  }
}

#define VTE_GEMV_CASE(BT, R, KS, PF, MAXW)                                                            \
  if (bt == BT && r == R && ks == KS && pf == PF && maxw == MAXW) {                                    \
    if (epi == 0) return (const void*)gemv_kernel<BT, R, KS, (PF != 0), MAXW, EPI_NONE>;               \
    if (epi == 2) return (const void*)gemv_kernel<BT, R, KS, (PF != 0), MAXW, EPI_ARGMAX>;             \
    if constexpr (R % 2 == 0) { if (epi == 1) return (const void*)gemv_kernel<BT, R, KS, (PF != 0), MAXW, EPI_SILU>; } \
  }

// One translation unit per BT instantiates these.
#define VTE_GEMV_ENTRY_FOR_BT(BT)                                                                 \
  extern "C" const void* vte_gemv_entry_b##BT(int bt, int r, int ks, int pf, int maxw, int epi) { \
    VTE_GEMV_CASES(BT)                                                                            \
    return nullptr;                                                                               \
  }
