// Skinny-batch GEMV on the matrix cores for up to 64 batch rows in one pass over the
// weights: Y[b, n] = sum_k W[n, k] X[b, k], four column tiles of 16 batch rows per
// weight tile of 16 rows (v_mfma_f32_16x16x32_bf16); two for wide outputs at batch 17 to 32.  Operator family: Sec. 1 "GEMV",
// Sec. 2.3; LM-head logits and greedy token: Sec. 7.1 / 7.2 of the paper.
//
// At this batch X no longer fits a wave's registers (64 rows x a 512-element chunk
// would take 256 of them), so the waves of a workgroup do not split K: each wave owns
// G row tiles for the whole of K, and the workgroup shares one copy of X through LDS.
//
// Work decomposition (a function of the shape and the plan, never of the CU count):
//   * a workgroup has WR waves and walks `groups` rounds; in a round wave w owns the
//     G row tiles ((blockIdx.x groups + round) WR + w) G + g;
//   * K advances in steps of 128 elements, the same step for every wave.  Per step the
//     workgroup stages X[16 CT x 128] in LDS (16 KB at four column tiles, double buffered: the waves fetch the
//     next step's part while they compute, store it after their MFMAs, and one
//     workgroup barrier per step publishes it); a wave reads its 16 B operands of the
//     step from there once and uses them for all its G tiles;
//   * a wave streams its tiles as blocks of 16 rows x 128 K (4 KB): four coalesced
//     wave loads (4 rows x 256 B each), transposed through a 4 KB wave-private LDS
//     area (16-byte pieces XOR-swizzled by row) into the MFMA A layout; the loads run
//     KA K-steps ahead of the MFMAs, across round boundaries.
//   * the K steps of a workgroup's round are walked from a start that depends on where its outputs
//     lie: outputs [512 j, 512 j + 512) start at step floor((j mod 32) * steps / 32) and wrap around.  Every
//     workgroup streams its rows at the same pace, and a row is 2^13 bytes long at K = 4096: walked
//     from step 0 everywhere, all requests in flight on the device at one moment share their address bits
//     8 to 12, and how well they spread over the memory channels is left to the upper bits, i.e. to
//     where the tensor happens to lie -- the same LM head took 160 to 228 us depending on the
//     allocation.  With up to 32 starts it takes 160 to 175 us wherever the tensor lies.
// Reduction tree of one output, fixed by K and the output's index alone (not by the plan: a round of
// a workgroup covers 32 to 512 consecutive outputs and starts at a multiple of its length, so it
// never straddles a block of 512):
//   1. inside one MFMA: four groups of 8 consecutive K (a lane's operand), in ascending K, each
//      added to the accumulator with one rounding (measured; tests/tree_emulator.py reproduces it);
//   2. along K through the accumulator operand: the 4 MFMAs of a step, then step after step in
//      the rotated order above (ascending from the start, then from step 0 up to the start).  No
//      sum crosses a wave.
// The batch columns of an MFMA are independent and every column tile runs the same
// chain, so a row's result does not depend on its position or on the rows beside it.
#include "gemv_kernels.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int CT, int G, int KA, int WR, int EPI>
__global__ __launch_bounds__(WR * 64) void gemv_rows_kernel(const GemvArgs a) {
  // CT column tiles: batch rows 16 ct + c (4 for batch 33 to 64, 2 for 17 to 32)
  constexpr int ROUT = (EPI == EPI_SILU) ? 8 : 16;  // outputs per tile: gate rows 0-7 pair with up rows 8-15
  constexpr int XU = 4 * CT / WR;                   // (column tile, 4-row group) units of X a wave stages per step
  static_assert((CT == 2 || CT == 4) && (WR == 4 || WR == 8), "X is staged as 4 CT units spread over the waves; 64 KB of LDS at most");
  __shared__ u32x4 xstage[2][CT * 256];   // per column tile: 16 rows x 16 pieces of 16 B, piece p of row r at r * 16 + (p ^ r)
  __shared__ u32x4 wstage_all[WR * 256];  // one 4 KB transposition area per wave (at the end: its argmax candidates)

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, q = lane >> 4;    // MFMA operand coordinates
  const int lr = lane >> 4, lp = lane & 15;  // load coordinates: row within a 4-row group, 16-byte piece of 256 B
  const int nk = (a.K + 127) >> 7;           // K steps
  const int nsteps = a.groups * nk;          // steps of the launch, round-major
  // position p of round rd's walk along K -> K step (see the header: the start is chosen by the outputs' block of 512)
  auto kstep = [&](int rd, int p) {
    const int out0 = ((blockIdx.x * a.groups + rd) * WR) * G * ROUT;  // first output of the workgroup's round
    const int k = p + (((out0 >> 9) & 31) * nk >> 5);
    return k >= nk ? k - nk : k;
  };
  u32x4* wstage = wstage_all + wave * 256;

  // Tile t of (round, g): first output row, and where its loads start.  A tile that would run
  // past the end is moved up to end at the last row; the rows it then shares with its
  // predecessor are computed twice and stored once (by the predecessor).
  const int n_rows = (EPI == EPI_SILU) ? a.n_out : a.N;
  auto tile_first = [&](int rd, int g) { return (((blockIdx.x * a.groups + rd) * WR + wave) * G + g) * ROUT; };
  auto tile_start = [&](int rd, int g) {
    const int out0 = tile_first(rd, g);
    const int last = n_rows - ROUT;
    return out0 < last ? out0 : last;
  };
  // Loads go through buffer resources: a scalar base, a scalar offset per block, one per-lane
  // offset for the whole launch.  The scalar part is relative to the wave's first tile.  The
  // range check of a buffer load looks at the per-lane offset only; a lane that must not fetch
  // (K tail, batch rows past B) gets an offset beyond the resource and reads zeros.
  constexpr int kRsrcFlags = 0x00020000;  // raw 32-bit data format
  constexpr uint32_t kNoFetch = 0x80000000u;
  const int base_row = tile_start(0, 0);
  const uint16_t* wbase = a.W + static_cast<size_t>(base_row) * a.K;
  __amdgpu_buffer_rsrc_t rs_w[4];  // one per 4-row group of a tile (with the SiLU epilogue groups 2, 3 are the up rows)
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const size_t row = (EPI == EPI_SILU) ? (u < 2 ? 4 * u : static_cast<size_t>(a.n_out) + 4 * (u - 2)) : 4 * u;
    rs_w[u] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(wbase + row * a.K), 0, 0x7fffffff, kRsrcFlags);
  }
  const uint32_t voff_w = (static_cast<uint32_t>(lr) * a.K + lp * 8) * 2u;  // bytes
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(a.X), 0, static_cast<int>((static_cast<uint32_t>(a.B - 1) * a.ldx + a.K) * 2u), kRsrcFlags);
  uint32_t voff_x[XU];  // unit j = wave XU + i: column tile j / 4, rows 4 (j % 4) + lr of it
  int xdst[XU];         // where the unit's piece goes in a stage buffer
  bool x_live[XU];      // wave-uniform: some of the unit's four batch rows exist (else its load is not issued at all)
#pragma unroll
  for (int i = 0; i < XU; ++i) {
    const int j = wave * XU + i, ct = j >> 2, r = 4 * (j & 3) + lr, row = 16 * ct + r;
    voff_x[i] = row < a.B ? (static_cast<uint32_t>(row) * a.ldx + lp * 8) * 2u : kNoFetch;
    xdst[i] = ct * 256 + r * 16 + (lp ^ r);
    x_live[i] = 16 * ct + 4 * (j & 3) < a.B;
  }
  const bool k_ragged = (a.K & 127) != 0;  // only then can a piece lie past K

  auto load_w = [&](u32x4(&dst)[4], int rd, int p, int g) {
    const int k = kstep(rd, p);
    const int soff = ((tile_start(rd, g) - base_row) * a.K + k * 128) * 2;
    const uint32_t vo = (!k_ragged || k * 128 + lp * 8 < a.K) ? voff_w : kNoFetch;
#pragma unroll
    for (int u = 0; u < 4; ++u) dst[u] = __builtin_amdgcn_raw_buffer_load_b128(rs_w[u], vo, soff, 2);  // streaming
  };
  auto load_x = [&](u32x4(&dst)[XU], int rd, int p) {
    const int k = kstep(rd, p);
    const bool in = !k_ragged || k * 128 + lp * 8 < a.K;
#pragma unroll
    for (int i = 0; i < XU; ++i) {
      if (x_live[i]) dst[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, in ? voff_x[i] : kNoFetch, k * 256, 0);
      else dst[i] = u32x4{0u, 0u, 0u, 0u};
    }
  };
  auto store_x = [&](const u32x4(&src)[XU], int buf) {
#pragma unroll
    for (int i = 0; i < XU; ++i) xstage[buf][xdst[i]] = src[i];
  };
  // Publishes LDS stores to the other waves.  (No fence builtin here: a release fence also
  // waits for the weight loads in flight, which must stay in flight across the barrier.)
  auto lds_barrier = [&]() {
    asm volatile("" ::: "memory");       // the compiler keeps LDS accesses on their side of the barrier
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS traffic is done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  f32x4_t acc[G][CT];
  float best_v[CT];
  int best_i[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) { best_v[ct] = -INFINITY; best_i[ct] = INT_MAX; }

  // what a round leaves: lane (c, q), register v holds tile row 4 q + v of batch row 16 ct + c
  auto epilogue = [&](int rd) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int first = tile_first(rd, g);  // rows below belong to the previous tile
      const int n0 = tile_start(rd, g) + 4 * q;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const int col = 16 * ct + c;
        float up[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (EPI == EPI_SILU) {
#pragma unroll
          for (int v = 0; v < 4; ++v) up[v] = __shfl_xor(acc[g][ct][v], 32, 64);  // quarters 2, 3 hold the up rows
        }
        if (col >= a.B) continue;
        if (EPI == EPI_SILU && q >= 2) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int n = n0 + v;
          if (n < first || n >= n_rows) continue;
          const float s = acc[g][ct][v];
          if constexpr (EPI == EPI_NONE) {
            a.Y[static_cast<size_t>(col) * a.ldy + n] = (uint16_t)f32_to_bf16(s);
          } else if constexpr (EPI == EPI_SILU) {
            a.Y[static_cast<size_t>(col) * a.ldy + n] = (uint16_t)f32_to_bf16(silu_f32(s) * up[v]);
          } else {
            if (a.logits) a.logits[static_cast<size_t>(col) * a.N + n] = s;
            if (better(s, n, best_v[ct], best_i[ct])) { best_v[ct] = s; best_i[ct] = n; }
          }
        }
      }
    }
  };

  // ---- prologue: the first KA steps' weight blocks, X of step 0 ----
  u32x4 wbuf[KA][G][4];
  u32x4 xr[XU];
  int ld_rd = 0, ld_k = 0;  // the step the next weight loads belong to
  auto advance_load = [&]() {
    if (++ld_k == nk) { ld_k = 0; ++ld_rd; }
  };
  load_x(xr, 0, 0);
#pragma unroll
  for (int ka = 0; ka < KA; ++ka) {
    if (ld_rd < a.groups) {
#pragma unroll
      for (int g = 0; g < G; ++g) load_w(wbuf[ka][g], ld_rd, ld_k, g);
    }
    advance_load();
  }
  store_x(xr, 0);
  lds_barrier();

  int rd = 0, k = 0;
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[g][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  for (int i = 0; i < nsteps; i += KA) {
#pragma unroll
    for (int ka = 0; ka < KA; ++ka) {
      const int step = i + ka;
      if (step < nsteps) {  // uniform over the workgroup
        const int buf = step & 1;
        const bool more = step + 1 < nsteps;
        const int kn = (k + 1 == nk) ? 0 : k + 1;
        if (more) load_x(xr, kn == 0 ? rd + 1 : rd, kn);
        // this step's X operands: lane (c, q) takes piece 4 s + q of batch row 16 ct + c
        u32x4 xf[CT][4];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int s = 0; s < 4; ++s) xf[ct][s] = xstage[buf][ct * 256 + c * 16 + ((4 * s + q) ^ c)];
#pragma unroll
        for (int g = 0; g < G; ++g) {
          // keep the written order (the scheduler would otherwise sink the loads next to their uses)
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int r = 4 * u + lr;
            wstage[r * 16 + (lp ^ r)] = wbuf[ka][g][u];
          }
          // the slot is free again: request the block KA steps ahead
          if (ld_rd < a.groups) load_w(wbuf[ka][g], ld_rd, ld_k, g);
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          u32x4 av[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) av[s] = wstage[c * 16 + ((4 * s + q) ^ c)];
#pragma unroll
          for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
              acc[g][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[s]),
                                                                   __builtin_bit_cast(bf16x8_t, xf[ct][s]), acc[g][ct], 0, 0, 0);
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
        }
        __builtin_amdgcn_sched_barrier(0);
        advance_load();
        if (more) store_x(xr, buf ^ 1);
        lds_barrier();
        if (++k == nk) {  // the round is complete
          epilogue(rd);
          k = 0;
          ++rd;
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[g][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
      }
    }
  }

  // ---- LM head: workgroup argmax -> one (value, index) candidate per batch row ----
  if constexpr (EPI == EPI_ARGMAX) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
      for (int d = 16; d < 64; d <<= 1) {
        const float ov = __shfl_xor(best_v[ct], d, 64);
        const int oi = __shfl_xor(best_i[ct], d, 64);
        if (better(ov, oi, best_v[ct], best_i[ct])) { best_v[ct] = ov; best_i[ct] = oi; }
      }
      if (lane < 16) {  // the wave's own area: its transpositions are over
        reinterpret_cast<float*>(wstage)[16 * ct + lane] = best_v[ct];
        reinterpret_cast<int*>(wstage)[64 + 16 * ct + lane] = best_i[ct];
      }
    }
    __syncthreads();
    uint32_t* cand_v = a.ws + 1 + gridDim.x;
    uint32_t* cand_i = cand_v + static_cast<size_t>(a.bt) * gridDim.x;
    if (threadIdx.x < 16 * CT && static_cast<int>(threadIdx.x) < a.B) {
      float wv[WR];  // every wave's candidate, read at once
      int wi[WR];
#pragma unroll
      for (int w = 0; w < WR; ++w) {
        wv[w] = reinterpret_cast<const float*>(wstage_all + w * 256)[threadIdx.x];
        wi[w] = reinterpret_cast<const int*>(wstage_all + w * 256)[64 + threadIdx.x];
      }
      float bv = wv[0];
      int bi = wi[0];
#pragma unroll
      for (int w = 1; w < WR; ++w)
        if (better(wv[w], wi[w], bv, bi)) { bv = wv[w]; bi = wi[w]; }
      cand_v[static_cast<size_t>(threadIdx.x) * gridDim.x + blockIdx.x] = __float_as_uint(bv);
      cand_i[static_cast<size_t>(threadIdx.x) * gridDim.x + blockIdx.x] = static_cast<uint32_t>(bi);
    }
  }
}

#define VTE_ROWS_CASE(CT, G, KA, WR)                                                      \
  if (ct == CT && g == G && ka == KA && wr == WR) {                                       \
    if (epi == 0) return (const void*)gemv_rows_kernel<CT, G, KA, WR, EPI_NONE>;          \
    if (epi == 1) return (const void*)gemv_rows_kernel<CT, G, KA, WR, EPI_SILU>;          \
    if (epi == 2) return (const void*)gemv_rows_kernel<CT, G, KA, WR, EPI_ARGMAX>;        \
  }

// ct = column tiles (2 or 4), g = row tiles per wave, ka = K steps the weight loads run ahead,
// wr = waves per workgroup; nullptr when the combination is not built.
extern "C" const void* vte_gemv_entry_rows(int ct, int g, int ka, int wr, int epi) {
  VTE_ROWS_CASE(4, 1, 2, 4)
  VTE_ROWS_CASE(4, 1, 2, 8)
  VTE_ROWS_CASE(4, 2, 2, 4)
  VTE_ROWS_CASE(4, 2, 2, 8)
  VTE_ROWS_CASE(4, 2, 1, 8)
  VTE_ROWS_CASE(4, 4, 1, 4)
  VTE_ROWS_CASE(4, 4, 1, 8)
  VTE_ROWS_CASE(2, 2, 2, 4)
  VTE_ROWS_CASE(2, 2, 2, 8)
  VTE_ROWS_CASE(2, 4, 1, 4)
  VTE_ROWS_CASE(2, 4, 1, 8)
  VTE_ROWS_CASE(2, 4, 2, 4)
  VTE_ROWS_CASE(2, 4, 2, 8)
  return nullptr;
}
