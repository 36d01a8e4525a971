// Skinny-batch GEMV on the matrix cores: Y[b, n] = sum_k W[n, k] X[b, k] for up to
// 16 CT batch rows per workgroup (CT = 1 or 2 column tiles; a larger batch runs as chunks of
// 16 CT rows in grid z, each reading the weights), 16 weight rows per v_mfma_f32_16x16x32_bf16 tile
// (operator family: Sec. 1 "GEMV", Sec. 2.3; LM-head logits and greedy token:
// Sec. 7.1 / 7.2 of the paper).
//
// From batch 8 up the dot-product kernels are bound by vector-ALU issue, not by
// HBM; one MFMA consumes a full 1 KB wave load of weights in a few cycles, so the
// same stream becomes memory-bound again.
//
// Work decomposition (a function of the shape and the plan, never of the CU count):
//   * K is cut into chunks of KC = 128 NBK elements; wave w of a workgroup owns
//     chunks w, w + nw, ... and keeps the chunk of X in registers (as MFMA B
//     operand: lane (c = l % 16, q = l / 16) holds 8 consecutive K elements of
//     batch row c per MFMA step, the quarters q taking 8 of the step's 32 each);
//   * the workgroup walks `groups` rounds of G row tiles of 16 weight rows; a wave
//     streams its K range of every tile in blocks of 16 rows x 128 K (4 KB).  With
//     one chunk per wave X is loaded once per workgroup, so rounds are what keeps
//     the X re-reads (L2 -> CU traffic that competes with the weight stream) small;
//     with several chunks per wave a chunk's X is requested block by block while the
//     last row tile of the chunk before it is being multiplied.  With one chunk per wave
//     and one column tile the first NB weight blocks are requested in front of X (theirs is the longer round
//     trip, and a CU's address unit needs about 0.6 us for a workgroup's X requests), and
//     X is turned into operand order block by block, right before a block's first use:
//     turned all at once in front of the stream it held the stream's window still;
//   * a block is fetched with four coalesced wave loads (4 rows x 256 B each; the
//     MFMA operand layout itself would make every load touch 16 cache lines,
//     which the texture addresser cannot sustain), transposed through a 4 KB
//     wave-private LDS area (16-byte pieces XOR-swizzled by row, conflict-free
//     both ways) and consumed by four MFMAs;
//   * loads run NB blocks ahead of the MFMAs, across tile and chunk boundaries.
// Reduction tree of one output, fixed by K and the plan:
//   1. inside one MFMA: four groups of 8 consecutive K (a lane's operand), in ascending K, each
//      added to the accumulator with one rounding (measured; tests/tree_emulator.py reproduces it);
//   2. along a wave's chunk, then along its chunks: the accumulator operand, in
//      ascending K;
//   3. across the waves of the workgroup in ascending wave order, through LDS
//      (after each round: every wave leaves its partial tiles in its own LDS
//      area, all threads of the workgroup add and store, then the next round);
//   4. split-K baseline only: S chunk sums added in chunk order.
// The batch columns of an MFMA are independent of each other and every column tile runs the
// same chain, so a row's result does not depend on its position or on the rows beside it.
//
// PRO = true (one column tile, one 1024-element chunk per wave, K = 4096, 256 threads): the decode
// loop's step boundary runs in the kernel's own prologue instead of in a launch of its own.  Every
// workgroup finishes the greedy tokens from the LM head's candidates (a total order: no tree), fetches
// the embedding rows, computes each row's sum of squares in exactly the tree of the stand-alone
// RMSNorm launch for this row length (256 threads: thread t adds chunks t and t + 256 in ascending
// order, fixed 64-lane butterfly, four wave sums added in wave order -- which is why the rows are
// fetched a second time in that layout) and scales its own K range of every row with the same
// expression, rounding to bf16 once: the B operand is then, bit for bit, what the RMSNorm launch
// would have stored, and the GEMV proceeds as usual.  The first weights are requested right behind
// the prologue's first loads and nothing in the prologue waits for them, so its latencies (candidates,
// then rows: two dependent fetches) run beside the weight stream's first-byte latency.  Workgroup 0
// stores the tokens and, if asked, the gathered and the normalised rows.
#pragma once
#include "gemv_kernels.h"
#include "trace_stamps.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <bool PRO> struct gemv_mfma_args { typedef GemvArgs type; };
template <> struct gemv_mfma_args<true> { typedef GemvNormArgs type; };
__device__ __forceinline__ const GemvArgs& gemv_part(const GemvArgs& a) { return a; }
__device__ __forceinline__ const GemvArgs& gemv_part(const GemvNormArgs& a) { return a.g; }

template <int NBK, int G, int NB, int MAXW, bool ALLFULL, bool ONECHUNK, int EPI, int CT, bool PRO = false>
__global__ __launch_bounds__(MAXW * 64) void gemv_mfma_kernel(const typename gemv_mfma_args<PRO>::type aa) {
  static_assert(!PRO || (CT == 1 && ONECHUNK && ALLFULL && NBK == 8 && MAXW == 4 && EPI == EPI_NONE),
                "the fused prologue is built for one column tile and one 1024-element chunk per wave");
  const GemvArgs& a = gemv_part(aa);
  constexpr int KC = 128 * NBK;
  constexpr int T = G * NBK;  // blocks of one chunk, tile-major
  static_assert(NB <= T && T % NB == 0, "the load window must divide a chunk's blocks");
  constexpr int ROUT = (EPI == EPI_SILU) ? 8 : 16;  // outputs per tile: gate rows 0-7 pair with up rows 8-15
  constexpr int WAVE_LDS = (G * CT > 4 ? G * CT : 4) * 64;  // 16-byte units per wave: transpose area, later G x CT partial tiles
  __shared__ u32x4 stage_all[MAXW * WAVE_LDS];
  __shared__ float s_bv[MAXW][16 * CT];
  __shared__ int s_bi[MAXW][16 * CT];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int c = lane & 15, q = lane >> 4;    // MFMA operand coordinates
  VTE_STAMP(0);  // entry
  const int lr = lane >> 4, lp = lane & 15;  // load coordinates: row within a 4-row group, 16-byte piece of 256 B
  const int split = blockIdx.y;
  const int row0 = blockIdx.z * 16 * CT;  // first batch row of this workgroup (a batch above 16 CT runs as chunks in z)
  const int k_begin = split * a.k_per_split;
  const int k_end = k_begin + a.k_per_split;
  const int nchunks = (a.k_per_split + KC - 1) / KC;
  u32x4* stage = stage_all + wave * WAVE_LDS;

  // First weight row of the 4-row group u of tile g (wave-uniform, so the loads
  // take a scalar base and one per-lane offset).  A tile that would run past the
  // end is moved up to end at the last row; the rows it then shares with its
  // predecessor are computed twice and stored once (by the predecessor).
  auto tile_first = [&](int rd, int g) { return ((blockIdx.x * a.groups + rd) * G + g) * ROUT; };
  auto tile_start = [&](int rd, int g) {
    const int out0 = tile_first(rd, g);
    const int last = ((EPI == EPI_SILU) ? a.n_out : a.N) - ROUT;
    return out0 < last ? out0 : last;
  };
  // Loads go through buffer resources: a scalar base, a scalar offset per 4-row
  // group and block, one per-lane offset for the whole launch.  The scalar part
  // stays below 32 bits because it is relative to the workgroup's first tile.
  constexpr int kRsrcFlags = 0x00020000;  // raw 32-bit data format
  // one resource per 4-row group of a tile (with the SiLU epilogue groups 2, 3 are the up rows)
  const uint16_t* wbase = a.W + static_cast<size_t>(tile_start(0, 0)) * a.K;
  __amdgpu_buffer_rsrc_t rs_w[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const size_t row = (EPI == EPI_SILU) ? (u < 2 ? 4 * u : static_cast<size_t>(a.n_out) + 4 * (u - 2)) : 4 * u;
    rs_w[u] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(wbase + row * a.K), 0, 0x7fffffff, kRsrcFlags);
  }
  const uint32_t voff = (static_cast<uint32_t>(lr) * a.K + lp * 8) * 2u;  // bytes
  // X: rows past B lie outside the resource and read as zero
  __amdgpu_buffer_rsrc_t rs_x;
  if constexpr (PRO)  // the rows come from the embedding table (the host checked that it stays below 2 GiB)
    rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(aa.E), 0,
                                             static_cast<int>(static_cast<uint32_t>(aa.V) * static_cast<uint32_t>(a.K) * 2u), kRsrcFlags);
  else
    rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.X), 0,
                                             static_cast<int>((static_cast<uint32_t>(a.B - 1) * a.ldx + a.K) * 2u), kRsrcFlags);
  // X is fetched like the weights, coalesced (an instruction takes 4 batch rows x 256 B) and turned
  // into operand order through the wave's LDS area: fetched in operand order (lane = row + 16 x
  // K group) every lane of an instruction sits on its own cache line and the address unit, not the
  // cache, sets the pace -- a quarter of the coalesced rate.
  uint32_t voff_x[CT][4];  // instruction u of column tile ct: batch row row0 + 16 ct + 4 u + lr, piece lp
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int br = row0 + 16 * ct + 4 * u + lr;
      voff_x[ct][u] = br < a.B ? (static_cast<uint32_t>(br) * a.ldx + lp * 8) * 2u : 0x80000000u;
    }

  f32x4_t acc[G][CT];
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};

  u32x4 wbuf[NB][4];
  u32x4 xs[CT][NBK][4];
  auto load_block = [&](u32x4(&dst)[4], int rd, int ch, int g, int bi) {
    const int kb = k_begin + ch * KC + bi * 128;
    const int soff = ((tile_start(rd, g) - tile_start(0, 0)) * a.K + k_begin + ch * KC) * 2;
    // K tail: a piece past k_end is not fetched at all (behind the last row of W it would lie
    // outside the allocation).  The range check of a buffer load looks at the per-lane offset
    // only, so such a lane gets an offset beyond the resource and reads zeros.
    const uint32_t vo = (ALLFULL || kb + lp * 8 < k_end) ? voff : 0x80000000u;
#pragma unroll
    for (int t = 0; t < 4; ++t)
      dst[t] = __builtin_amdgcn_raw_buffer_load_b128(rs_w[t], vo, soff + bi * 256, 2);  // streaming
  };
  auto load_x_block = [&](int ch, int bi) {  // block bi (128 K) of chunk ch, still in load order
    const int soff = (k_begin + ch * KC) * 2;
    const bool in_k = ALLFULL || k_begin + ch * KC + bi * 128 + lp * 8 < k_end;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        // an instruction whose four batch rows all lie past B is not issued at all (uniform over the
        // workgroup): it would fetch nothing, but still take the CU's address unit for as long as a
        // full one, in front of the first weights
        if (row0 + 16 * ct + 4 * u < a.B)
          xs[ct][bi][u] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, in_k ? voff_x[ct][u] : 0x80000000u, soff + bi * 256, 0);
        else
          xs[ct][bi][u] = zero;
      }
  };
  // load order -> operand order, in place, through the wave's transposition area (free between blocks)
  auto transpose_x_block = [&](int bi) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int r = 4 * u + lr;
        stage[r * 16 + (lp ^ r)] = xs[ct][bi][u];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int s = 0; s < 4; ++s) xs[ct][bi][s] = stage[c * 16 + ((4 * s + q) ^ c)];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  };
  auto transpose_x = [&]() {
#pragma unroll
    for (int bi = 0; bi < NBK; ++bi) transpose_x_block(bi);
  };
  // One chunk per wave, no fused prologue: the first weights are requested in front of X (their HBM
  // round trip is the longer one), and X is turned block by block right before its first use
  // instead of all at once in front of the stream (which holds the stream's window still).  Timed
  // in an interleaved A/B of two builds: 0.6 % of a batch-8 step; with several chunks per wave, or
  // with two or four column tiles (more X than weights in a wave's first requests), it loses
  // (0.5 to 1.7 % of a batch-64 step) and is not used.
  constexpr bool WFIRST = ONECHUNK && !PRO && CT == 1;
  auto load_x = [&](int ch) {
#pragma unroll
    for (int bi = 0; bi < NBK; ++bi) load_x_block(ch, bi);
  };

  // the finishing part of a round: a thread owns four consecutive tile rows of one
  // batch row of one tile
  float best_v[CT];
  int best_i[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) { best_v[ct] = -INFINITY; best_i[ct] = INT_MAX; }
  auto epilogue = [&](int rd, int g, int lcol, int qq, const float(&s)[4], const float(&u)[4]) {
    const int col = row0 + lcol;
    if (col >= a.B) return;
    const int first = tile_first(rd, g);  // rows below belong to the previous tile
    const int out0 = tile_start(rd, g) + 4 * qq;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = out0 + v;
      if (n < first) continue;
      if constexpr (EPI == EPI_NONE) {
        if (n < a.N) a.Y[static_cast<size_t>(col) * a.ldy + n] = (uint16_t)f32_to_bf16(s[v]);
      } else if constexpr (EPI == EPI_SILU) {
        if (n < a.n_out) a.Y[static_cast<size_t>(col) * a.ldy + n] = (uint16_t)f32_to_bf16(silu_f32(s[v]) * u[v]);
      } else {
        if (n < a.N) {
          if (a.logits) a.logits[static_cast<size_t>(col) * a.N + n] = s[v];
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)  // col / 16 selects the candidate; written so that the arrays stay in registers
            if (ct == (lcol >> 4) && better(s[v], n, best_v[ct], best_i[ct])) { best_v[ct] = s[v]; best_i[ct] = n; }
        }
      }
    }
  };
  constexpr int QOUT = (EPI == EPI_SILU) ? 2 : 4;  // quarters that own outputs
  float* part_all = reinterpret_cast<float*>(stage_all);
  constexpr int WAVE_F = WAVE_LDS * 4;  // floats per wave area

  const bool active = wave < nchunks;
  if constexpr (PRO) {
    __shared__ int s_tok[16];
    __shared__ float s_part[4][16];
    __shared__ float s_rstd[16];
    // Publishes LDS stores to the other waves without a fence: a fence would also wait for the
    // weight loads, which are meant to stay in flight through the whole prologue.
    auto lds_barrier = [&]() {
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };
    // The first weights are requested right behind the first loads of the prologue (loads return in
    // order: in front of them they would hold the tokens back by an HBM round trip), and nothing
    // below waits for them.
    bool w_requested = false;
    auto request_weights = [&]() {
      if (w_requested) return;
      w_requested = true;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < NB; ++t) load_block(wbuf[t], 0, wave, t / NBK, t % NBK);
      __builtin_amdgcn_sched_barrier(0);
    };
    // 1. the tokens: from the LM head's candidates (best value, lowest index; a total order), or given
    if (aa.cand) {
      // wave w takes batch rows w, w + 4, ...; the candidates of all its rows are requested before the
      // first is looked at (512 per row and pass), so the reduction costs one memory round trip
      float bv[4];
      int bi[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) { bv[j] = -INFINITY; bi[j] = INT_MAX; }
      for (int base = 0; base < aa.nblocks; base += 512) {
        float v[4][8];
        int ix[4][8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int r = wave + 4 * j;
          const uint32_t* cv = aa.cand + static_cast<size_t>(r) * aa.nblocks;
          const uint32_t* ci = aa.cand + static_cast<size_t>(aa.cand_bt) * aa.nblocks + static_cast<size_t>(r) * aa.nblocks;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int blk = base + 64 * i + lane;
            const bool ok = r < a.B && blk < aa.nblocks;
            v[j][i] = ok ? __uint_as_float(cv[blk]) : -INFINITY;
            ix[j][i] = ok ? static_cast<int>(ci[blk]) : INT_MAX;
          }
        }
        request_weights();
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            if (better(v[j][i], ix[j][i], bv[j], bi[j])) { bv[j] = v[j][i]; bi[j] = ix[j][i]; }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = wave + 4 * j;
        if (r >= a.B) break;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const float ov = __shfl_xor(bv[j], d, 64);
          const int oi = __shfl_xor(bi[j], d, 64);
          if (better(ov, oi, bv[j], bi[j])) { bv[j] = ov; bi[j] = oi; }
        }
        const int t = (bi[j] == INT_MAX) ? 0 : bi[j];  // all-NaN row
        if (lane == 0) {
          s_tok[r] = t < 0 ? 0 : (t >= aa.V ? aa.V - 1 : t);
          if (blockIdx.x == 0 && aa.tok_out) aa.tok_out[r] = t;
        }
      }
    } else {
      int t = 0;
      if (static_cast<int>(threadIdx.x) < a.B) t = aa.tok[threadIdx.x];
      request_weights();
      if (static_cast<int>(threadIdx.x) < a.B) s_tok[threadIdx.x] = t < 0 ? 0 : (t >= aa.V ? aa.V - 1 : t);
    }
    request_weights();
    lds_barrier();
    // 2. this wave's K range of the raw rows, in the load layout of the B operand
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int br = 4 * u + lr;
      voff_x[0][u] = br < a.B ? (static_cast<uint32_t>(s_tok[br]) * a.K + lp * 8) * 2u : 0x80000000u;
    }
    load_x(wave);
    u32x4 gam[NBK];
#pragma unroll
    for (int bi = 0; bi < NBK; ++bi) gam[bi] = ld16(aa.gamma + wave * KC + bi * 128 + lp * 8);
    // 3. every row's sum of squares in the tree of the stand-alone RMSNorm launch for this row length
    const int nch = a.K >> 3;
    const bool two = static_cast<int>(threadIdx.x) + 256 < nch;
    for (int half = 0; half < 2; ++half) {
      if (half * 8 >= a.B) break;
      u32x4 v0[8], v1[8];
#pragma unroll
      for (int r8 = 0; r8 < 8; ++r8) {
        const int r = half * 8 + r8;
        const bool live = r < a.B;
        const uint16_t* xr = aa.E + static_cast<size_t>(s_tok[live ? r : 0]) * a.K;
        v0[r8] = live ? ld16(xr + threadIdx.x * 8) : zero;
        v1[r8] = (live && two) ? ld16(xr + (threadIdx.x + 256) * 8) : zero;
      }
#pragma unroll
      for (int r8 = 0; r8 < 8; ++r8) {
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = bf16_lo(v0[r8][e]), hi = bf16_hi(v0[r8][e]);
          ss = fmaf(lo, lo, ss);
          ss = fmaf(hi, hi, ss);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = bf16_lo(v1[r8][e]), hi = bf16_hi(v1[r8][e]);
          ss = two ? fmaf(lo, lo, ss) : ss;
          ss = two ? fmaf(hi, hi, ss) : ss;
        }
        ss = wave_sum(ss);
        if (lane == 0) s_part[wave][half * 8 + r8] = ss;
      }
    }
    lds_barrier();
    if (static_cast<int>(threadIdx.x) < a.B) {
      float s = s_part[0][threadIdx.x];
#pragma unroll
      for (int w = 1; w < 4; ++w) s += s_part[w][threadIdx.x];
      s_rstd[threadIdx.x] = 1.0f / sqrtf(s / static_cast<float>(a.K) + aa.eps);
    }
    lds_barrier();
    // 4. scale this wave's K range of every row, one rounding: the B operand, still in load order
    const bool keep = blockIdx.x == 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (4 * u >= a.B) break;  // nothing but padding from here on: those registers already hold zeros
      const int br = 4 * u + lr;
      const float rstd = br < a.B ? s_rstd[br] : 0.f;
#pragma unroll
      for (int bi = 0; bi < NBK; ++bi) {
        const u32x4 raw = xs[0][bi][u];
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = bf16_lo(raw[e]) * rstd * bf16_lo(gam[bi][e]);
          const float hi = bf16_hi(raw[e]) * rstd * bf16_hi(gam[bi][e]);
          o[e] = pack_bf16(lo, hi);
        }
        if (br >= a.B) o = zero;
        xs[0][bi][u] = o;
        if (keep && br < a.B) {
          const size_t at = static_cast<size_t>(br) * a.K + wave * KC + bi * 128 + lp * 8;
          if (aa.h_out) st16(aa.h_out + at, raw);
          if (aa.n_out) st16(aa.n_out + at, o);
        }
      }
    }
  } else if (active) {
    if constexpr (WFIRST) {
#pragma unroll
      for (int t = 0; t < NB; ++t) load_block(wbuf[t], 0, wave, t / NBK, t % NBK);
      __builtin_amdgcn_sched_barrier(0);
      VTE_STAMP(7);  // first weights requested
      load_x(wave);
    } else {
      load_x(wave);  // the first chunk; with several chunks per wave the next one's X follows block by block below
#pragma unroll
      for (int t = 0; t < NB; ++t) load_block(wbuf[t], 0, wave, t / NBK, t % NBK);
    }
  }
  VTE_STAMP(1);  // launch arguments in, first loads issued
  for (int rd = 0; rd < a.groups; ++rd) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) acc[g][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (active) {
      int ch = wave;
      while (true) {
        // X of this chunk arrived in load order: once per launch when a wave has a single chunk, else per chunk pass
        if (!WFIRST && (!ONECHUNK || rd == 0)) transpose_x();
        if (!WFIRST && rd == 0 && ch == wave) VTE_STAMP(2);  // X arrived and turned
        const int chn = ch + nw;
        const bool more = !ONECHUNK && chn < nchunks;  // ONECHUNK: the launch has no more chunks than waves
        const bool next_round = rd + 1 < a.groups;
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const int g = t / NBK, bi = t % NBK, slot = t % NB;
          // keep the written order (the scheduler would otherwise sink the loads
          // next to their uses and leave two or three in flight)
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (WFIRST) {
            if (rd == 0 && g == 0) {  // the first use of this block of X
              transpose_x_block(bi);
              if (bi == 0) VTE_STAMP(2);  // the first block of X arrived and turned
            }
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int r = 4 * u + lr;
            stage[r * 16 + (lp ^ r)] = wbuf[slot][u];
          }
          // the slot is free again: request the block NB positions ahead (next
          // tile, next chunk of this round, or the first chunk of the next round)
          if (t + NB < T) load_block(wbuf[slot], rd, ch, (t + NB) / NBK, (t + NB) % NBK);
          else if (more) load_block(wbuf[slot], rd, chn, (t + NB - T) / NBK, (t + NB - T) % NBK);
          else if (next_round) load_block(wbuf[slot], rd + 1, wave, (t + NB - T) / NBK, (t + NB - T) % NBK);
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          u32x4 av[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) av[s] = stage[c * 16 + ((4 * s + q) ^ c)];
#pragma unroll
          for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
              acc[g][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[s]),
                                                                   __builtin_bit_cast(bf16x8_t, xs[ct][bi][s]), acc[g][ct], 0, 0, 0);
          // the chunk's last row tile is done with this block of X: fetch the block of the chunk the
          // wave turns to next (its next chunk, or its first one again in the next round), so that
          // X is on its way a chunk pass ahead of its use
          if constexpr (!ONECHUNK) {
            if (g == G - 1) {
              if (more) load_x_block(chn, bi);
              else if (next_round) load_x_block(wave, bi);
            }
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          if (t == 0 && rd == 0 && ch == wave) VTE_STAMP(3);  // first block of weights multiplied
        }
        __builtin_amdgcn_sched_barrier(0);
        if (ONECHUNK || !more) break;
        ch = chn;
      }
    }

    if (rd == a.groups - 1) VTE_STAMP(4);  // the wave's share of the stream is through
    // wave partial tiles -> the wave's own LDS area (its transposes of this round are
    // done): lane (c, q), register v holds tile row 4 q + v of batch row c
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int v = 0; v < 4; ++v) part_all[wave * WAVE_F + ((g * CT + ct) * 4 + v) * 64 + lane] = acc[g][ct][v];
    __syncthreads();
    if (rd == a.groups - 1) VTE_STAMP(5);  // every wave of the workgroup is through
    for (int f = threadIdx.x; f < G * CT * 64; f += blockDim.x) {
      const int gc = f >> 6, g = gc / CT, ln = f & 63, col = 16 * (gc % CT) + (ln & 15), qq = ln >> 4;
      if (qq >= QOUT) continue;
      float s[4], u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        // every wave area exists in LDS whether or not its wave does, so all MAXW partial sums are
        // read at once (one LDS latency instead of one per wave) and those of absent waves left out
        const float* pp = part_all + (gc * 4 + v) * 64 + ln;
        float pw[MAXW];
#pragma unroll
        for (int w = 0; w < MAXW; ++w) pw[w] = pp[w * WAVE_F];
        float t = pw[0];
#pragma unroll
        for (int w = 1; w < MAXW; ++w) t = w < nw ? t + pw[w] : t;  // ascending wave (K) order
        s[v] = t;
        if constexpr (EPI == EPI_SILU) {
#pragma unroll
          for (int w = 0; w < MAXW; ++w) pw[w] = pp[w * WAVE_F + 32];
          float t2 = pw[0];
#pragma unroll
          for (int w = 1; w < MAXW; ++w) t2 = w < nw ? t2 + pw[w] : t2;
          u[v] = t2;
        }
      }
      if (a.S == 1) {
        epilogue(rd, g, col, qq, s, u);
      } else if (row0 + col < a.B) {
        const int first = tile_first(rd, g);
        const int out0 = tile_start(rd, g) + 4 * qq;
        float* pp = a.partials + (static_cast<size_t>(split) * a.bt + row0 + col) * a.N;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int n = out0 + v;
          if (n < first) continue;
          if constexpr (EPI == EPI_SILU) {
            if (n < a.n_out) { pp[n] = s[v]; pp[a.n_out + n] = u[v]; }
          } else {
            if (n < a.N) pp[n] = s[v];
          }
        }
      }
    }
    if (rd + 1 < a.groups) __syncthreads();  // the LDS areas are transposition space again
    else VTE_STAMP(6);  // cross-wave sums added, outputs stored
  }

  // ---- split-K baseline: the last chunk-block of this row block adds the chunk sums.  Without a
  // ticket array (the shape-derived split) the partial sums are all this launch leaves: a finish
  // launch adds them in split order. ----
  if (a.S > 1 && a.ws) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t t = atomicAdd(&a.ws[1 + blockIdx.z * gridDim.x + blockIdx.x], 1u);
      s_last = (t == static_cast<uint32_t>(a.S) - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int f = threadIdx.x; f < a.groups * G * CT * 64; f += blockDim.x) {
      const int rd = f / (G * CT * 64), gc = (f >> 6) % (G * CT), g = gc / CT, ln = f & 63, col = 16 * (gc % CT) + (ln & 15), qq = ln >> 4;
      if (qq >= QOUT || row0 + col >= a.B) continue;
      const int first = tile_first(rd, g);
      const int out0 = tile_start(rd, g) + 4 * qq;
      float s[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int n = out0 + v;
        const bool live = n >= first && ((EPI == EPI_SILU) ? n < a.n_out : n < a.N);
        if (!live) continue;
        for (int sp = 0; sp < a.S; ++sp) {  // chunk order
          const float* pp = a.partials + (static_cast<size_t>(sp) * a.bt + row0 + col) * a.N;
          s[v] += __builtin_nontemporal_load(pp + n);
          if constexpr (EPI == EPI_SILU) u[v] += __builtin_nontemporal_load(pp + a.n_out + n);
        }
      }
      epilogue(rd, g, col, qq, s, u);
    }
    if (threadIdx.x == 0) a.ws[1 + blockIdx.z * gridDim.x + blockIdx.x] = 0u;  // ready for the next launch
  }

  // ---- LM head: workgroup argmax -> one (value, index) candidate per batch row ----
  if constexpr (EPI == EPI_ARGMAX) {
    // a thread's batch row within a column tile is lane % 16 in every pass of the finishing loop
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
      for (int d = 16; d < 64; d <<= 1) {
        const float ov = __shfl_xor(best_v[ct], d, 64);
        const int oi = __shfl_xor(best_i[ct], d, 64);
        if (better(ov, oi, best_v[ct], best_i[ct])) { best_v[ct] = ov; best_i[ct] = oi; }
      }
      if (lane < 16) { s_bv[wave][16 * ct + lane] = best_v[ct]; s_bi[wave][16 * ct + lane] = best_i[ct]; }
    }
    __syncthreads();
    uint32_t* cand_v = a.ws + 1 + gridDim.x * gridDim.z;
    uint32_t* cand_i = cand_v + static_cast<size_t>(a.bt) * gridDim.x;
    if (threadIdx.x < 16 * CT && row0 + static_cast<int>(threadIdx.x) < a.B) {
      float wv[MAXW];
      int wi[MAXW];
#pragma unroll
      for (int w = 0; w < MAXW; ++w) { wv[w] = s_bv[w][threadIdx.x]; wi[w] = s_bi[w][threadIdx.x]; }
      float bv = wv[0];
      int bi = wi[0];
#pragma unroll
      for (int w = 1; w < MAXW; ++w)
        if (w < nw && better(wv[w], wi[w], bv, bi)) { bv = wv[w]; bi = wi[w]; }
      cand_v[static_cast<size_t>(row0 + threadIdx.x) * gridDim.x + blockIdx.x] = __float_as_uint(bv);
      cand_i[static_cast<size_t>(row0 + threadIdx.x) * gridDim.x + blockIdx.x] = static_cast<uint32_t>(bi);
    }
  }
}

