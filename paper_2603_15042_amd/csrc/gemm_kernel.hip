// bf16 GEMM C = A * Bm^T on the matrix cores, fp32 accumulation, bf16 output:
// the training-shaped co-tenant.  The structure is fixed by (M, N, K): a 2-D grid
// of 256x256 output tiles, each reduced over K in steps of 64 in ascending order
// by one workgroup; no split-K, no stream-K, no dependence on the CU count.
//
// Workgroup = 4 waves as 2 (M) x 2 (N); a wave owns 128 x 128 of the tile as
// 4 x 4 MFMA blocks of 32x32 (v_mfma_f32_32x32x16_bf16): 16 MFMAs per 8 operand
// reads from LDS, which keeps the LDS port at half the MFMA pipe's time (with
// 4 x 2 blocks per wave and padded rows the kernel was LDS-bound at 36 % of the
// MFMA peak).  The 256 accumulator registers leave one wave per SIMD, so operand
// fragments for the next 16 K are read while the MFMAs of the current 16 run.
// A and Bm tiles (256 rows x 64 K, 128 B per row) are staged in LDS unpadded;
// the 16-byte pieces of a row are XOR-swizzled with row % 8, so any 8 consecutive
// rows of an MFMA operand read, and the 8 pieces a row is written with, fall on
// distinct banks.  Two LDS stages; the tiles of step i+1 are loaded straight into
// the other stage (global_load_lds, no register stop, no LDS write instructions)
// while step i computes.  LDS moves 64 B per cycle and CU with 128-bit accesses
// (measured), which is exactly what 4 x 4 blocks need at the full MFMA rate, so every
// LDS cycle saved counts.
// Tile order: consecutive workgroup ids are dealt round-robin to the 8 XCDs, so
// id % 8 selects a band of tile rows and each XCD's L2 sees a compact set of
// A rows and Bm columns.
#include "dev_util.h"
#include "kargs.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int ROW_BYTES = TK * 2;                    // 128
constexpr int OPERAND_BYTES = TM * ROW_BYTES;        // 32 KB per operand per stage
constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;
constexpr int GEMM_THREADS = 256;

__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(const GemmArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];     // [stage][A | B][256 rows][8 swizzled pieces of 16 B]

  // ---- tile selection (fixed function of blockIdx) ----
  const int ntiles = a.tiles_m * a.tiles_n;
  int tile = blockIdx.x;
  int tm, tn;
  if ((a.tiles_m & 31) == 0 && (a.tiles_n & 7) == 0) {
    // XCD x = id % 8 works through bands of 4 tile rows, each band in blocks of 4 x 8 tiles:
    // the ~32 tiles an XCD has in flight then share 4 A bands and 8 Bm bands in its L2
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;          // j: position in this XCD's sequence
    const int per_band = 4 * a.tiles_n;                          // tiles in a band of 4 rows
    const int band = j / per_band, jb = j % per_band;           // band index within this XCD's share
    const int blk = jb >> 5, in = jb & 31;
    tm = (band * 8 + x) * 4 + (in & 3);
    tn = blk * 8 + (in >> 2);
  } else {
    if ((ntiles & 7) == 0) tile = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
    tm = tile / a.tiles_n;
    tn = tile % a.tiles_n;
  }
  const uint16_t* Ag = a.A + static_cast<size_t>(tm) * TM * a.K;
  const uint16_t* Bg = a.Bm + static_cast<size_t>(tn) * TN * a.K;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;            // 2 x 2 waves

  // global -> LDS copy without a register stop (global_load_lds_dwordx4: lane L of a wave
  // instruction lands at the instruction's LDS base + 16 L).  One instruction fills 8 rows;
  // lane L fetches, for row L / 8, the piece that belongs in slot L % 8 of the swizzled row.
  // Wave w fills rows [64 w, 64 w + 64) of both operands: 16 instructions per K step.
  const int grow = lane >> 3;                                   // row within the 8-row group
  const int gpiece = (lane & 7) ^ grow;                         // (row & 7) == grow: groups start at multiples of 8
  const uint16_t* Ap = Ag + static_cast<size_t>(wave * 64 + grow) * a.K + gpiece * 8;
  const uint16_t* Bp = Bg + static_cast<size_t>(wave * 64 + grow) * a.K + gpiece * 8;
  const size_t group_step = static_cast<size_t>(8) * a.K;
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto fill_stage = [&](int stage, int k0) {
    uint8_t* base = smem + stage * STAGE_BYTES + wave * 64 * ROW_BYTES;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_global_load_lds((gptr_t)(Ap + i * group_step + k0), (lptr_t)(base + i * 8 * ROW_BYTES), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr_t)(Bp + i * group_step + k0), (lptr_t)(base + OPERAND_BYTES + i * 8 * ROW_BYTES), 16, 0, 0);
    }
  };

  // operand fragments: lane l supplies row l % 32 of a 32-row block and K pieces 2 kk + l / 32
  const int frow = lane & 31, fhalf = lane >> 5, fsw = frow & 7;
  const int a_row0 = (wm * 128 + frow) * ROW_BYTES;
  const int b_row0 = OPERAND_BYTES + (wn * 128 + frow) * ROW_BYTES;
  auto read_frags = [&](bf16x8_t(&af)[4], bf16x8_t(&bfr)[4], const uint8_t* st, int kk) {
    const int piece = 16 * ((2 * kk + fhalf) ^ fsw);
    // Bm fragments first: the MFMAs run i-major, so af[3] is needed last
#pragma unroll
    for (int j = 0; j < 4; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(st + b_row0 + j * 32 * ROW_BYTES + piece);
#pragma unroll
    for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(st + a_row0 + i * 32 * ROW_BYTES + piece);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // One K step of 64: 64 MFMAs per wave.  The instruction stream is laid out by hand
  // (sched_group_barrier): the LDS fills of the next step first, then two MFMAs for
  // every fragment read of the following 16 K -- with one wave per SIMD nothing else
  // would cover the LDS latency.  The last 16 MFMAs of a step need registers only, so
  // the compiler may run them behind the barrier, over the first reads of the next stage.
  const int nk = a.K / TK;
  bf16x8_t af[2][4], bfr[2][4];
  auto mfma16 = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[buf][i], bfr[buf][j], acc[i][j], 0, 0, 0);
  };
  fill_stage(0, 0);
  __builtin_amdgcn_s_waitcnt(0);  // everything outstanding, the LDS fills included
  __syncthreads();
  read_frags(af[0], bfr[0], smem, 0);
  for (int ks = 0; ks + 1 < nk; ++ks) {
    const int stage = ks & 1;
    const uint8_t* st = smem + stage * STAGE_BYTES;
    fill_stage(stage ^ 1, (ks + 1) * TK);  // the other stage was last read before the previous barrier
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
      read_frags(af[(kk + 1) & 1], bfr[(kk + 1) & 1], st, kk + 1);
      mfma16(kk & 1);
    }
    mfma16(1);
    __builtin_amdgcn_sched_group_barrier(0x020, 16, 0);  // the LDS fills (VMEM)
#pragma unroll
    for (int n = 0; n < 24; ++n) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    read_frags(af[0], bfr[0], smem + (stage ^ 1) * STAGE_BYTES, 0);
  }
  {  // last step: nothing left to fetch
    const uint8_t* st = smem + ((nk - 1) & 1) * STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
      read_frags(af[(kk + 1) & 1], bfr[(kk + 1) & 1], st, kk + 1);
      mfma16(kk & 1);
    }
    mfma16(1);
  }

  // ---- epilogue: fp32 -> bf16, row-major C ----
  // 32x32 block layout: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
  uint16_t* Cg = a.C + (static_cast<size_t>(tm) * TM + wm * 128) * a.N + static_cast<size_t>(tn) * TN + wn * 128;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int col = j * 32 + (lane & 31);
        Cg[static_cast<size_t>(row) * a.N + col] = (uint16_t)f32_to_bf16(acc[i][j][v]);
      }
}

extern "C" const void* vte_gemm_entry() { return (const void*)gemm_kernel; }
extern "C" unsigned vte_gemm_lds_bytes() { return 2u * STAGE_BYTES; }
extern "C" unsigned vte_gemm_threads() { return GEMM_THREADS; }
