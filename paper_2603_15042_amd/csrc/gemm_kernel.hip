// bf16 GEMM C = A * Bm^T on the matrix cores, fp32 accumulation, bf16 output:
// the training-shaped co-tenant.  The structure is fixed by (M, N, K): a 2-D grid
// of 256x256 output tiles, each reduced over K in steps of 64 in ascending order
// by one workgroup; no split-K, no stream-K, no dependence on the CU count.
//
// Workgroup = 8 waves as 2 (M) x 4 (N); a wave owns 128 x 64 of the tile as
// 4 x 2 MFMA blocks of 32x32 (v_mfma_f32_32x32x16_bf16, 16 fp32 per lane each).
// A and Bm tiles (256 x 64 bf16 each) are staged in LDS with rows padded to
// 72 elements so that the 32 rows read by one MFMA operand fall on distinct
// banks; two LDS stages, global loads for step i+1 in flight during step i.
// Tile order: consecutive workgroup ids are dealt round-robin to the 8 XCDs, so
// id % 8 selects a band of tile rows and each XCD's L2 sees a compact set of
// A rows and Bm columns.
#include "dev_util.h"
#include "kargs.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int LDS_ROW = TK + 8;                      // padded row, in elements
constexpr int TILE_ELEMS = TM * LDS_ROW;             // per operand per stage
constexpr int GEMM_THREADS = 512;

__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_kernel(const GemmArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  uint16_t* lds = reinterpret_cast<uint16_t*>(smem);  // [stage][A|B][256][72]

  // ---- tile selection (fixed function of blockIdx) ----
  const int ntiles = a.tiles_m * a.tiles_n;
  int tile = blockIdx.x;
  if ((ntiles & 7) == 0) tile = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
  const int tm = tile / a.tiles_n, tn = tile % a.tiles_n;
  const uint16_t* Ag = a.A + static_cast<size_t>(tm) * TM * a.K;
  const uint16_t* Bg = a.Bm + static_cast<size_t>(tn) * TN * a.K;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;           // 2 x 4 waves
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

  // global -> LDS copy assignment: 2048 16-byte chunks per operand tile
  // chunk c: row = c / 8, kchunk = c % 8
  u32x4 ga[4], gb[4];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * GEMM_THREADS;
      const int row = c >> 3, kc = (c & 7) * 8;
      ga[i] = ld16(Ag + static_cast<size_t>(row) * a.K + k0 + kc);
      gb[i] = ld16(Bg + static_cast<size_t>(row) * a.K + k0 + kc);
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t* As = lds + stage * 2 * TILE_ELEMS;
    uint16_t* Bs = As + TILE_ELEMS;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * GEMM_THREADS;
      const int row = c >> 3, kc = (c & 7) * 8;
      *reinterpret_cast<u32x4*>(As + row * LDS_ROW + kc) = ga[i];
      *reinterpret_cast<u32x4*>(Bs + row * LDS_ROW + kc) = gb[i];
    }
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = a.K / TK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int ks = 0; ks < nk; ++ks) {
    const int stage = ks & 1;
    if (ks + 1 < nk) load_global((ks + 1) * TK);
    const uint16_t* As = lds + stage * 2 * TILE_ELEMS + (wm * 128 + frag_row) * LDS_ROW + frag_k;
    const uint16_t* Bs = lds + stage * 2 * TILE_ELEMS + TILE_ELEMS + (wn * 64 + frag_row) * LDS_ROW + frag_k;
#pragma unroll
    for (int kk = 0; kk < TK; kk += 16) {
      bf16x8_t af[4], bfr[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(As + i * 32 * LDS_ROW + kk);
#pragma unroll
      for (int j = 0; j < 2; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(Bs + j * 32 * LDS_ROW + kk);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (ks + 1 < nk) store_lds(stage ^ 1);  // the other stage was last read before the previous barrier
    __syncthreads();
  }

  // ---- epilogue: fp32 -> bf16, row-major C ----
  // 32x32 block layout: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, column l%32
  uint16_t* Cg = a.C + (static_cast<size_t>(tm) * TM + wm * 128) * a.N + static_cast<size_t>(tn) * TN + wn * 64;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int col = j * 32 + (lane & 31);
        Cg[static_cast<size_t>(row) * a.N + col] = (uint16_t)f32_to_bf16(acc[i][j][v]);
      }
}

extern "C" const void* vte_gemm_entry() { return (const void*)gemm_kernel; }
extern "C" unsigned vte_gemm_lds_bytes() { return 2u * 2u * TILE_ELEMS * 2u; }
extern "C" unsigned vte_gemm_threads() { return GEMM_THREADS; }
