// Descriptor constructors: turn a problem shape into an immutable launch
// descriptor D_k (Sec. 4.2).  Every grid, block, LDS size and work split below is
// a function of the shape arguments only.  Nothing here looks at the device, at
// the pool or at a CU count, except the *_reshaped / *_splitk baselines, whose
// caller passes a CU-derived parameter on purpose (Sec. 2.3).
#include <cstring>
#include <new>

#include "kargs.h"
#include "runtime.h"

extern "C" {
const void* vte_norm_entry(int threads, int layer);
const void* vte_norm_rows_entry(int chunks, int layer);
const void* vte_copy_entry();
const void* vte_softmax_prob_entry();
const void* vte_fill_entry();
int vte_norm_rows_per_block(void);
const void* vte_gemv_entry_b1(int, int, int, int, int, int);
const void* vte_gemv_entry_b2(int, int, int, int, int, int);
const void* vte_gemv_entry_b4(int, int, int, int, int, int);
const void* vte_gemv_entry_b8(int, int, int, int, int, int);
const void* vte_gemv_entry_b16(int, int, int, int, int, int);
const void* vte_gemv_entry_mfma(int, int, int, int, int, int, int);
const void* vte_gemv_entry_mfma32(int, int, int, int, int, int, int);
const void* vte_gemv_entry_rows(int, int, int, int, int);
const void* vte_gemv_entry_mfma64(int, int, int, int, int, int, int);
const void* vte_gemv_entry_mfma_norm(int);
const void* vte_gather_entry();
const void* vte_argmax_finish_entry();
const void* vte_split_finish_entry();
const void* vte_gemm_entry();
unsigned vte_gemm_lds_bytes();
unsigned vte_gemm_threads();
}

namespace vte {

uint64_t fnv1a(const void* data, size_t n, uint64_t h) {
  const unsigned char* p = static_cast<const unsigned char*>(data);
  for (size_t i = 0; i < n; ++i) { h ^= p[i]; h *= 1099511628211ull; }
  return h;
}

uint64_t desc_hash(const vte_desc* d) {
  uint64_t h = fnv1a(&d->kernel, sizeof d->kernel);
  h = fnv1a(&d->entry, sizeof d->entry, h);
  h = fnv1a(d->grid, sizeof d->grid, h);
  h = fnv1a(d->block, sizeof d->block, h);
  h = fnv1a(&d->lds_bytes, sizeof d->lds_bytes, h);
  h = fnv1a(&d->arg_bytes, sizeof d->arg_bytes, h);
  return fnv1a(d->args, d->arg_bytes, h);
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Fills *d (caller's storage: heap or stack) from the shape-derived launch parameters.
// Allocates nothing and touches no context state.
template <class Args>
int fill_desc(vte_desc* d, vte_ctx* ctx, int kernel, const void* entry, const Args& a, uint32_t gx, uint32_t gy,
              uint32_t threads, uint32_t lds, uint64_t shape_key, uint64_t bytes, uint64_t flops, uint32_t gz = 1) {
  static_assert(sizeof(Args) <= sizeof(vte_desc::args), "argument block too large");
  if (!entry) { set_error("no kernel instance for this configuration"); return VTE_EINVAL; }
  if (gx == 0 || gy == 0 || gz == 0 || gx > 0x7fffffffu || gy > 65535u || gz > 65535u) { set_error("grid out of range"); return VTE_EINVAL; }
  std::memset(d, 0, sizeof *d);
  d->ctx = ctx;
  d->kernel = kernel;
  d->entry = entry;
  d->grid[0] = gx; d->grid[1] = gy; d->grid[2] = gz;
  d->block[0] = threads; d->block[1] = 1; d->block[2] = 1;
  d->lds_bytes = lds;
  d->arg_bytes = sizeof(Args);
  std::memcpy(d->args, &a, sizeof(Args));
  d->bytes = bytes;
  d->flops = flops;
  uint64_t k = fnv1a(&kernel, sizeof kernel);
  k = fnv1a(d->grid, sizeof d->grid, k);
  k = fnv1a(d->block, sizeof d->block, k);
  d->profile_key = fnv1a(&shape_key, sizeof shape_key, k);
  d->hash = desc_hash(d);
  return VTE_OK;
}

// Copies a filled descriptor to the heap, applies its one-time kernel attributes and hands
// ownership of the copy to the caller through *out (the context keeps it listed).
int register_desc(vte_ctx* ctx, const vte_desc& filled, vte_desc** out) {
  vte_desc* d = new (std::nothrow) vte_desc(filled);
  if (!d) { set_error("out of host memory"); return VTE_ENOMEM; }
  int rc = ctx->backend->prepare_kernel(d);
  if (rc != VTE_OK) { delete d; return rc; }
  {
    std::lock_guard<std::mutex> lk(ctx->mu);
    ctx->descs.push_back(d);
  }
  *out = d;
  return VTE_OK;
}

template <class Args>
int finish_desc(vte_ctx* ctx, int kernel, const void* entry, const Args& a, uint32_t gx, uint32_t gy,
                uint32_t threads, uint32_t lds, uint64_t shape_key, uint64_t bytes, uint64_t flops,
                vte_desc** out, uint32_t gz = 1) {
  vte_desc tmp;
  int rc = fill_desc(&tmp, ctx, kernel, entry, a, gx, gy, threads, lds, shape_key, bytes, flops, gz);
  if (rc != VTE_OK) return rc;
  return register_desc(ctx, tmp, out);
}

int norm_threads(int cols) {
  const int chunks = cols / 8;
  int t = 64;
  while (t < 256 && t < chunks) t *= 2;  // 64, 128, 256: one chunk per thread up to 2048 columns
  return t;
}

int build_norm(vte_ctx* ctx, int kernel, bool layer, const void* x, const void* gamma, const void* beta,
               void* y, int rows, int cols, float eps, int threads, vte_desc** out,
               const int32_t* tok = nullptr, void* h_out = nullptr, int V = 0, const uint32_t* cand = nullptr,
               int nblocks = 0, int cand_bt = 0, int32_t* tok_out = nullptr) {
  if (!ctx || !out || !x || !gamma || !y || (layer && !beta)) { set_error("norm: null argument"); return VTE_EINVAL; }
  if (rows <= 0 || cols <= 0 || cols % 8 != 0 || cols > 16384) { set_error("norm: need rows > 0, cols % 8 == 0, cols <= 16384"); return VTE_EINVAL; }
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(y) || (layer && !aligned16(beta))) { set_error("norm: pointers must be 16-byte aligned"); return VTE_EINVAL; }
  while (cols > 64 * threads && threads < 512) threads *= 2;  // at most 8 chunks of 8 per thread
  if (cols > 64 * threads) { set_error("norm: row too long for this thread count"); return VTE_EINVAL; }
  NormArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.gamma = static_cast<const uint16_t*>(gamma);
  a.beta = static_cast<const uint16_t*>(beta);
  a.y = static_cast<uint16_t*>(y);
  a.rows = rows; a.cols = cols; a.eps = eps; a.inv_cols = 1.0f / static_cast<float>(cols);
  a.tok = tok; a.h_out = static_cast<uint16_t*>(h_out); a.V = V;
  a.cand = cand; a.nblocks = nblocks; a.cand_bt = cand_bt; a.tok_out = tok_out;
  if (h_out && !aligned16(h_out)) { set_error("norm: pointers must be 16-byte aligned"); return VTE_EINVAL; }
  // many short rows and nothing fused in: one wave per row (structure from rows and cols alone)
  const bool by_wave = kernel != VTE_K_RMSNORM_RESHAPED && !tok && !cand && !h_out && rows >= 512 && cols <= 4096;
  const int shape_v[3] = {rows, cols, nblocks};
  const uint64_t shape = nblocks ? fnv1a(shape_v, sizeof shape_v) : ((static_cast<uint64_t>(rows) << 32) | static_cast<uint32_t>(cols));
  const uint64_t bytes = static_cast<uint64_t>(rows) * cols * 4 + static_cast<uint64_t>(cols) * (layer ? 4 : 2) +
                         (cand ? 8ull * nblocks * rows + 4ull * rows : 0);
  if (by_wave) {
    const int chunks = cols <= 1024 ? 2 : (cols <= 2048 ? 4 : 8);
    const int per_block = vte_norm_rows_per_block();
    return finish_desc(ctx, kernel, vte_norm_rows_entry(chunks, layer ? 1 : 0), a,
                       static_cast<uint32_t>((rows + per_block - 1) / per_block), 1, 256, 0, shape, bytes,
                       static_cast<uint64_t>(rows) * cols * 4, out);
  }
  return finish_desc(ctx, kernel, vte_norm_entry(threads, layer ? 1 : 0), a, static_cast<uint32_t>(rows), 1,
                     static_cast<uint32_t>(threads), 0, shape, bytes, static_cast<uint64_t>(rows) * cols * 4, out);
}

const void* gemv_entry(const vte_gemv_plan& p, int epi, int k_per_split) {
  if (p.kind == VTE_GEMV_MFMA_ROWS) {
    if ((p.batch_tile != 64 && p.batch_tile != 32) || p.rows < 16 || p.rows % 16 != 0) return nullptr;
    return vte_gemv_entry_rows(p.batch_tile / 16, p.rows / 16, p.prefetch, p.max_waves, epi);
  }
  if (p.kind == VTE_GEMV_MFMA) {
    if (p.ksteps < 1) return nullptr;
    const int kc = 128 * p.ksteps;
    return (p.batch_tile == 64 ? vte_gemv_entry_mfma64 : p.batch_tile == 32 ? vte_gemv_entry_mfma32 : vte_gemv_entry_mfma)(
        p.ksteps, p.rows / 16, p.prefetch, p.max_waves, k_per_split % kc == 0 ? 1 : 0,
        (k_per_split + kc - 1) / kc <= p.max_waves ? 1 : 0, epi);
  }
  switch (p.batch_tile) {
    case 1: return vte_gemv_entry_b1(1, p.rows, p.ksteps, p.prefetch, p.max_waves, epi);
    case 2: return vte_gemv_entry_b2(2, p.rows, p.ksteps, p.prefetch, p.max_waves, epi);
    case 4: return vte_gemv_entry_b4(4, p.rows, p.ksteps, p.prefetch, p.max_waves, epi);
    case 8: return vte_gemv_entry_b8(8, p.rows, p.ksteps, p.prefetch, p.max_waves, epi);
    case 16: return vte_gemv_entry_b16(16, p.rows, p.ksteps, p.prefetch, p.max_waves, epi);
  }
  return nullptr;
}

int batch_tile(int B) { int bt = 1; while (bt < B) bt *= 2; return bt; }

int plan_waves(const vte_gemv_plan& p, int k_per_split) {
  if (p.kind == VTE_GEMV_MFMA_ROWS) return p.max_waves;  // every wave walks all of K for its own row tiles
  if (p.kind == VTE_GEMV_MFMA) {  // waves share the K chunks round-robin
    if (p.ksteps < 1) return 0;
    const int nchunks = (k_per_split + 128 * p.ksteps - 1) / (128 * p.ksteps);
    return nchunks < p.max_waves ? nchunks : p.max_waves;
  }
  const int nsteps = (k_per_split + 511) / 512;
  return (nsteps + p.ksteps - 1) / p.ksteps;
}

// Default decomposition, from the shape alone (a table found by timing every
// built combination on the Llama-8B shapes; it never looks at the device).
// outputs = logical outputs per batch row (N, or N/2 with the SiLU epilogue);
// kps = K / S.
int plan_gemv(int B, int outputs, int kps, int epi, vte_gemv_plan* p) {
  if (B < 1 || B > 64 || outputs < 1 || kps < 8) return VTE_EINVAL;
  const bool silu = epi == VTE_EPI_SILU_MUL;
  const int tile_out = silu ? 8 : 16;
  const int tiles = (outputs + tile_out - 1) / tile_out;
  if (B > 32) {
    // Batch 33 to 64: four column tiles per weight tile; the waves of a workgroup split the row
    // tiles, not K, and share X through LDS.  More row tiles per workgroup mean fewer fetches of
    // X; narrow outputs keep the workgroups small so that there are enough of them.
    if (outputs < tile_out) return VTE_EINVAL;
    if (tiles >= 1024) {
      // timed on the Llama-8B shapes: the LM head takes four tiles per wave and eight waves (X is
      // fetched once per 32 tiles); the gate/up projection has too few tiles for that and runs
      // one tile per wave, eight waves
      const bool wide = tiles >= 4096;
      p->batch_tile = 64; p->rows = 16 * (wide ? 4 : 1); p->ksteps = 1; p->prefetch = wide ? 1 : 2;
      p->max_waves = 8; p->groups = 1;
      p->kind = VTE_GEMV_MFMA_ROWS;
      return VTE_OK;
    }
    // Narrow outputs have too few row tiles to fill the device without splitting K: the K-split
    // kernel with four column tiles and 256-element chunks (X for 64 rows and a wider chunk would
    // not fit a wave's registers).  Timed against two chunks of 32 rows in one launch (grid z of
    // the two-column-tile kernel, which a plan with batch_tile 32 still selects): 20 % faster.
    p->batch_tile = 64; p->rows = tiles > 256 ? 32 : 16; p->ksteps = 2; p->prefetch = 2; p->max_waves = 4; p->groups = 1;
    p->kind = VTE_GEMV_MFMA;
    return VTE_OK;
  }
  if (B > 16) {
    // Batch 17 to 32: two column tiles per weight tile, four waves (a wave holds X for 32 rows).
    // Fewer than one full tile of outputs is not offered at this batch.
    if (outputs < tile_out) return VTE_EINVAL;
    // Found by timing the built combinations on the Llama-8B shapes at batch 24 and 32: eight waves
    // (X of a 4096-wide row loaded once per workgroup) and rounds for the wide outputs.
    if (tiles >= 4096) {
      // the LM head: the row-split kind with two column tiles (four tiles per wave, eight waves)
      // streams it 9 % faster than the K-split kind, whose X registers leave little room
      p->batch_tile = 32; p->rows = 16 * 4; p->ksteps = 1; p->prefetch = 1; p->max_waves = 8; p->groups = 1;
      p->kind = VTE_GEMV_MFMA_ROWS;
      return VTE_OK;
    }
    int g = 1, nb = 2, rounds = 1, mw = 8;
    if (tiles >= 1024) { g = 2; rounds = 4; }
    else if (tiles > 256) { g = 2; mw = 4; }
    p->batch_tile = 32; p->rows = 16 * g; p->ksteps = 4; p->prefetch = nb; p->max_waves = mw; p->groups = rounds;
    p->kind = VTE_GEMV_MFMA;
    return VTE_OK;
  }
  if (outputs >= tile_out && B >= 3) {
    // Batch 3 and up: matrix-core tiles.  From batch 8 the dot-product kernels are ALU-bound; at
    // batch 3 and 4 their four-row batch tile already loses to the matrix cores on every Llama-8B
    // shape and width (O 9.6 -> 8.8 us, QKV 13.4 -> 11.4, LM head 153 -> 151 us at 256 CUs, 231 -> 190 at
    // 128); at batch 1 and 2 the two-row dot-product tile is as fast at full width and faster on a
    // narrow pCtx for the small projections, and stays.  Found by timing every built combination on
    // the Llama-8B shapes.  Large outputs walk several rounds so that X is fetched once per many rows.
    int g = 1, nb = 2, mw = 8, rounds = 1, nbk = 4;
    if (tiles >= 4096 && kps <= 4096) {
      // the LM head: 1024-element chunks, so that four waves hold all of X (fetched once per
      // workgroup) and a workgroup of eight rounds of two tiles re-reads none of it.  As fast as
      // the best 512-element plan at full width and 15-18 % faster on pCtxs of 32 to 128 CUs,
      // where a CU's fill path is the bound and re-read X competes with the weights for it.
      nbk = 8; g = 2; mw = 4; rounds = 8;
    }
    else if (tiles >= 4096) { mw = 4; if (B <= 8) { g = 2; rounds = 4; } else { g = 4; rounds = 2; } }
    else if (tiles >= 1024) { g = 8; }
    else if (tiles > 256 && kps <= 4096) { nbk = 8; g = 2; mw = 4; }  // X once per workgroup, as above
    else if (tiles > 256 && kps <= 8192) { g = 2; mw = 4; }
    else if (kps > 2048 && kps <= 4096) { nbk = 8; mw = 4; }  // one 1024-element chunk per wave: X is fetched and turned once,
                                                              // ahead of the weights; 6-8 % faster than 512-element chunks at every width
    else if (kps <= 4096) { nb = 4; mw = 4; }  // four-wave workgroups share a CU three at a time: as fast at full
                                               // width, up to 30 % faster on 32 to 128 CUs than eight waves
    p->batch_tile = 16; p->rows = 16 * g; p->ksteps = nbk; p->prefetch = nb; p->max_waves = mw; p->groups = rounds;
    p->kind = VTE_GEMV_MFMA;
    return VTE_OK;
  }
  const int nsteps = (kps + 511) / 512;
  if (nsteps > 32) return VTE_EINVAL;
  int bt = batch_tile(B);
  if (bt == 1) bt = 2;                    // one row rides in the two-row tile
  if (nsteps > 16 && bt < 4) bt = 4;      // long rows: the wider tile keeps a wave's slice in registers
  if (nsteps > 16 && bt == 16) bt = 8;    // long rows at batch 16: two batch chunks of 8
  int r, ks, pf = 1, mw = 8, gmax = 8;
  if (bt == 2) {
    if (nsteps <= 1) { r = 16; ks = 1; } else { r = 8; ks = 2; }
    if ((nsteps + ks - 1) / ks > 8) { bt = 4; }
    gmax = 4;
  }
  if (bt == 4) {
    if (nsteps <= 1) { r = 16; ks = 1; }
    else if (nsteps <= 16 && outputs < 16384) { r = 8; ks = 2; }
    else { r = 4; ks = 4; pf = 0; }
    gmax = 4;
  } else if (bt == 8) {
    if (nsteps <= 1) { r = 8; ks = 1; }
    else if (nsteps <= 3) { r = 8; ks = 2; }
    else if (silu && nsteps <= 16) { r = 4; ks = 2; gmax = 2; }
    else { r = 2; ks = 4; pf = 0; }
  } else if (bt == 16) {
    if (nsteps <= 1) { r = 4; ks = 1; } else { r = 4; ks = 2; }
    if (silu) gmax = 2;
  }
  if ((nsteps + ks - 1) / ks > mw) return VTE_EINVAL;
  const int rout = silu ? r / 2 : r;
  int groups = outputs / (rout * 256);
  groups = groups < 1 ? 1 : (groups > gmax ? gmax : groups);
  p->batch_tile = bt; p->rows = r; p->ksteps = ks; p->prefetch = pf; p->max_waves = mw; p->groups = groups;
  p->kind = VTE_GEMV_DOT2;
  return VTE_OK;
}

struct GemvBuild {
  int kernel, epi_kernel;  // VTE_K_*, EPI_* of the kernel template
  const void *W, *X; void* Y; float* logits; int32_t* tok; void* ws; void* partials;
  int B, N, K, epilogue, S;
  const vte_gemv_plan* plan;
  int ldx = 0, ldy = 0;  // 0 = dense
  bool fixed_split = false;  // S is derived from the shape: partial sums only, no ticket array, a finish launch follows
};

// Validates the shape and the plan and fills *d; allocates nothing.
int build_gemv_into(vte_ctx* ctx, const GemvBuild& g, vte_desc* d) {
  if (!d || !g.W || !g.X) { set_error("gemv: null argument"); return VTE_EINVAL; }
  const bool lm = (g.epi_kernel == 2);
  if (!lm && !g.Y && !g.fixed_split) { set_error("gemv: null output"); return VTE_EINVAL; }
  if (lm && (!g.tok || !g.ws)) { set_error("lmhead: tok and workspace are required"); return VTE_EINVAL; }
  if (g.B < 1 || g.B > 64 || g.N < 1 || g.K < 8 || g.K % 8 != 0) { set_error("gemv: need 1 <= B <= 64, N >= 1, K % 8 == 0"); return VTE_EINVAL; }
  if (g.S < 1 || g.S > 64 || g.K % (g.S * 8) != 0) { set_error("gemv: K must split into S chunks of a multiple of 8"); return VTE_EINVAL; }
  if (g.S > 1 && (!g.partials || (!g.ws && !g.fixed_split))) { set_error("split-K: partials and workspace are required"); return VTE_EINVAL; }
  if (g.epilogue == VTE_EPI_SILU_MUL && (g.N % 2 != 0)) { set_error("gemv: SiLU-mul needs an even N"); return VTE_EINVAL; }
  if (g.epilogue != VTE_EPI_NONE && g.epilogue != VTE_EPI_SILU_MUL) { set_error("gemv: unknown epilogue"); return VTE_EINVAL; }
  if (!aligned16(g.W) || !aligned16(g.X)) { set_error("gemv: W and X must be 16-byte aligned"); return VTE_EINVAL; }
  const int n_out = (g.epilogue == VTE_EPI_SILU_MUL) ? g.N / 2 : g.N;
  vte_gemv_plan p;
  if (g.plan) p = *g.plan;
  else if (plan_gemv(g.B, n_out, g.K / g.S, g.epilogue, &p) != VTE_OK) { set_error("gemv: no plan for this shape (K / S at most 16384; a batch above 16 needs a full tile of outputs)"); return VTE_EINVAL; }
  const int kps = g.K / g.S;
  const int waves = plan_waves(p, kps);
  const bool by_rows = p.kind == VTE_GEMV_MFMA_ROWS;
  if (by_rows) {
    if (g.S != 1) { set_error("gemv plan: the row-split MFMA kind has no split-K variant"); return VTE_EINVAL; }
    if ((p.batch_tile != 64 && p.batch_tile != 32) || g.B > p.batch_tile) { set_error("gemv plan: the row-split MFMA kind has batch_tile 32 or 64 and takes the whole batch in one tile"); return VTE_EINVAL; }
    if (n_out < (g.epi_kernel == 1 ? 8 : 16)) { set_error("gemv plan: the MFMA kinds need at least one full tile of outputs (16, or 8 with SiLU-mul)"); return VTE_EINVAL; }
  }
  const bool mfma = p.kind == VTE_GEMV_MFMA;
  if (p.kind != VTE_GEMV_DOT2 && !mfma && !by_rows) { set_error("gemv plan: unknown kind"); return VTE_EINVAL; }
  if (g.fixed_split && !mfma) { set_error("gemv plan: the shape-derived K split runs on the MFMA kind"); return VTE_EINVAL; }
  if (g.B > 32 && !by_rows && !(mfma && p.batch_tile >= 32 && (g.S == 1 || g.fixed_split))) {
    set_error("gemv plan: batch 33 to 64 needs the row-split MFMA kind (batch_tile 64) or the MFMA kind with batch_tile 32 (two chunks), S = 1");
    return VTE_EINVAL;
  }
  if (mfma && n_out < (g.epi_kernel == 1 ? 8 : 16)) { set_error("gemv plan: the MFMA kind needs at least one full tile of outputs (16, or 8 with SiLU-mul)"); return VTE_EINVAL; }
  if (mfma && ((p.batch_tile != 16 && p.batch_tile != 32 && p.batch_tile != 64) || p.rows < 16 || p.rows % 16 != 0)) { set_error("gemv plan: the MFMA kind has batch_tile 16, 32 or 64 and rows a multiple of 16"); return VTE_EINVAL; }
  if (mfma && g.B > p.batch_tile && p.batch_tile != 32) { set_error("gemv plan: the MFMA kind with batch_tile 16 takes the whole batch in one tile"); return VTE_EINVAL; }
  if (!mfma && !by_rows && g.B > 16) { set_error("gemv plan: batch 17 to 32 needs the MFMA kind with batch_tile 32"); return VTE_EINVAL; }
  const int zchunks = (g.B + p.batch_tile - 1) / (p.batch_tile > 0 ? p.batch_tile : 1);
  if (p.batch_tile < 1 || p.groups < 1 || p.rows < 1 || p.ksteps < 1 || waves < 1 || waves > p.max_waves) {
    set_error("gemv plan: groups >= 1 and ceil(K/S/512/ksteps) <= max_waves are required"); return VTE_EINVAL;
  }
  if (!gemv_entry(p, g.epi_kernel, kps)) { set_error("gemv plan: this combination is not built"); return VTE_EINVAL; }
  const int rout = (g.epi_kernel == 1) ? p.rows / 2 : p.rows;
  if (rout < 1) { set_error("gemv plan: the SiLU epilogue needs an even number of rows"); return VTE_EINVAL; }
  const int per_block = rout * p.groups * (by_rows ? p.max_waves : 1);
  const uint32_t gx = static_cast<uint32_t>((n_out + per_block - 1) / per_block);
  // the MFMA kernels address a workgroup's weight rows with 32-bit byte offsets from its first row
  if ((mfma || by_rows) && (static_cast<uint64_t>(per_block) + 4) * g.K * 2 >= (1ull << 31)) {
    set_error("gemv plan: the weight rows of one workgroup span 2 GiB or more (fewer groups or rows)"); return VTE_EINVAL;
  }
  GemvArgs a{};
  a.W = static_cast<const uint16_t*>(g.W);
  a.X = static_cast<const uint16_t*>(g.X);
  a.Y = static_cast<uint16_t*>(g.Y);
  a.logits = g.logits; a.tok = g.tok;
  a.ws = static_cast<uint32_t*>(g.ws);
  a.partials = static_cast<float*>(g.partials);
  a.B = g.B; a.N = g.N; a.K = g.K; a.n_out = n_out;
  a.ldx = g.ldx > 0 ? g.ldx : g.K;
  a.ldy = g.ldy > 0 ? g.ldy : n_out;
  if (static_cast<uint64_t>(g.B - 1) * a.ldx + g.K >= (1ull << 30)) { set_error("gemv: X spans 2 GiB or more"); return VTE_EINVAL; }
  if (a.ldx < g.K || a.ldx % 8 != 0 || a.ldy < n_out) { set_error("gemv: need ldx >= K, ldx % 8 == 0, ldy >= outputs per row"); return VTE_EINVAL; }
  a.groups = p.groups; a.S = g.S; a.k_per_split = kps; a.bt = p.batch_tile * zchunks;
  const uint64_t shape = fnv1a(&a.B, sizeof(int) * 9);
  uint64_t bytes = 2ull * g.N * g.K + 2ull * g.B * g.K + (lm ? 4ull * g.B : 2ull * g.B * n_out);
  if (lm && g.logits) bytes += 4ull * g.B * g.N;
  if (g.fixed_split) bytes = 2ull * g.N * g.K + 2ull * g.B * g.K + 4ull * g.S * g.B * g.N;
  const uint64_t flops = 2ull * g.B * g.N * g.K;
  return fill_desc(d, ctx, g.kernel, gemv_entry(p, g.epi_kernel, kps), a, gx, static_cast<uint32_t>(g.S),
                   static_cast<uint32_t>(waves * 64), 0, shape, bytes, flops, static_cast<uint32_t>(zchunks));
}

int build_gemv(vte_ctx* ctx, const GemvBuild& g, vte_desc** out) {
  if (!ctx || !out) { set_error("gemv: null argument"); return VTE_EINVAL; }
  vte_desc tmp;
  int rc = build_gemv_into(ctx, g, &tmp);
  if (rc != VTE_OK) return rc;
  return register_desc(ctx, tmp, out);
}

// The argmax-finish launch that reads the candidates the LM-head launch *lm leaves behind.
int fill_argmax_finish(vte_ctx* ctx, const vte_desc* lm, vte_desc* d) {
  GemvArgs g;
  std::memcpy(&g, lm->args, sizeof g);
  // candidates sit behind the ticket words: [1 + grid.x * grid.z] uint32, then values and indices [batch slots][grid.x]
  ArgmaxFinishArgs a{};
  a.pairs = g.ws + 1 + lm->grid[0] * lm->grid[2];
  a.tok = g.tok;
  a.nblocks = static_cast<int>(lm->grid[0]);
  a.bt = g.bt;
  a.B = g.B;
  const uint64_t shape = (static_cast<uint64_t>(a.nblocks) << 32) | static_cast<uint32_t>(a.B * 64 + a.bt);
  return fill_desc(d, ctx, VTE_K_ARGMAX_FINISH, vte_argmax_finish_entry(), a, static_cast<uint32_t>(a.B), 1, 1024, 0,
                   shape, 8ull * a.nblocks * a.B + 4ull * a.B, 0);
}

}  // namespace

// The LM head with its default plan and the finish launch behind it, filled into the caller's
// storage with `ws` as the workspace; *ws_words = 32-bit words of `ws` the two launches touch
// (ticket words first: *ticket_words of them).  Nothing is allocated or registered.
int fill_lmhead_pair(const void* W, const void* H, int32_t* tok, float* logits_or_null, void* ws, int B, int V, int K,
                     vte_desc* lm, vte_desc* fin, size_t* ticket_words, size_t* ws_words) {
  if (!tok) { set_error("lmhead: tok is required"); return VTE_EINVAL; }
  GemvBuild g{VTE_K_LMHEAD, 2, W, H, nullptr, logits_or_null, tok, ws, nullptr, B, V, K, VTE_EPI_NONE, 1, nullptr};
  int rc = build_gemv_into(nullptr, g, lm);
  if (rc != VTE_OK) return rc;
  rc = fill_argmax_finish(nullptr, lm, fin);
  if (rc != VTE_OK) return rc;
  GemvArgs a;
  std::memcpy(&a, lm->args, sizeof a);
  *ticket_words = 1 + static_cast<size_t>(lm->grid[0]) * lm->grid[2];
  *ws_words = *ticket_words + 2 * static_cast<size_t>(a.bt) * lm->grid[0];
  return VTE_OK;
}

}  // namespace vte

using namespace vte;

extern "C" {

int vte_desc_rmsnorm(vte_ctx* ctx, const void* x, const void* gamma, void* y, int rows, int cols, float eps,
                     vte_desc** out) {
  return build_norm(ctx, VTE_K_RMSNORM, false, x, gamma, nullptr, y, rows, cols, eps, norm_threads(cols), out);
}

int vte_desc_rmsnorm_gather(vte_ctx* ctx, const void* E, const int32_t* tok, const void* gamma, void* y,
                            void* h_or_null, int B, int V, int cols, float eps, vte_desc** out) {
  if (!tok || V < 1) { set_error("rmsnorm_gather: tok and V >= 1 are required"); return VTE_EINVAL; }
  return build_norm(ctx, VTE_K_RMSNORM_GATHER, false, E, gamma, nullptr, y, B, cols, eps, norm_threads(cols), out,
                    tok, h_or_null, V);
}

int vte_desc_rmsnorm_gather_argmax(vte_ctx* ctx, const void* E, const vte_desc* lmhead, int32_t* tok_out_or_null,
                                   const void* gamma, void* y, void* h_or_null, int V, int cols, float eps,
                                   vte_desc** out) {
  if (!ctx || !lmhead || V < 1) { set_error("rmsnorm_gather_argmax: lmhead and V >= 1 are required"); return VTE_EINVAL; }
  if (lmhead->ctx != ctx || (lmhead->kernel != VTE_K_LMHEAD && lmhead->kernel != VTE_K_LMHEAD_SPLITK)) {
    set_error("rmsnorm_gather_argmax: needs an LM-head descriptor of this context"); return VTE_EINVAL;
  }
  GemvArgs g;
  std::memcpy(&g, lmhead->args, sizeof g);
  const uint32_t* cand = g.ws + 1 + lmhead->grid[0] * lmhead->grid[2];
  return build_norm(ctx, VTE_K_RMSNORM_GATHER_ARGMAX, false, E, gamma, nullptr, y, g.B, cols, eps, norm_threads(cols),
                    out, nullptr, h_or_null, V, cand, static_cast<int>(lmhead->grid[0]), g.bt, tok_out_or_null);
}

// The first projection of a decode step with the step boundary in its prologue (kargs.h: GemvNormArgs).
static int build_gemv_norm(vte_ctx* ctx, const void* W, const void* E, const int32_t* tok, const uint32_t* cand, int nblocks,
                           int cand_bt, int32_t* tok_out, const void* gamma, void* Y, void* h_out, void* n_out, int B,
                           int V, int N, int K, float eps, vte_desc** out) {
  if (!ctx || !out || !W || !E || !gamma || !Y || (!tok && !cand)) { set_error("gemv_rmsnorm: null argument"); return VTE_EINVAL; }
  if (B < 1 || B > 16 || N < 16 || V < 1) { set_error("gemv_rmsnorm: need 1 <= B <= 16, N >= 16, V >= 1"); return VTE_EINVAL; }
  if (K != 4096) { set_error("gemv_rmsnorm: the fused form is built for K = 4096 (one 1024-element chunk for each of four waves)"); return VTE_EINVAL; }
  if (static_cast<uint64_t>(V) * K * 2 >= (1ull << 31)) { set_error("gemv_rmsnorm: the embedding table spans 2 GiB or more"); return VTE_EINVAL; }
  if (!aligned16(W) || !aligned16(E) || !aligned16(gamma) || (h_out && !aligned16(h_out)) || (n_out && !aligned16(n_out))) {
    set_error("gemv_rmsnorm: pointers must be 16-byte aligned"); return VTE_EINVAL;
  }
  const int tiles = (N + 15) / 16;
  const int g = tiles > 256 ? 2 : 1;  // the row tiles per workgroup of the default plan for these shapes
  GemvNormArgs a{};
  a.g.W = static_cast<const uint16_t*>(W);
  a.g.Y = static_cast<uint16_t*>(Y);
  a.g.B = B; a.g.N = N; a.g.K = K; a.g.n_out = N;
  a.g.ldx = K; a.g.ldy = N;
  a.g.groups = 1; a.g.S = 1; a.g.k_per_split = K; a.g.bt = 16;
  a.E = static_cast<const uint16_t*>(E);
  a.gamma = static_cast<const uint16_t*>(gamma);
  a.tok = cand ? nullptr : tok;
  a.cand = cand;
  a.tok_out = tok_out;
  a.h_out = static_cast<uint16_t*>(h_out);
  a.n_out = static_cast<uint16_t*>(n_out);
  a.V = V; a.nblocks = nblocks; a.cand_bt = cand_bt; a.eps = eps;
  const int shape_v[5] = {B, N, K, V, nblocks};
  const uint64_t bytes = 2ull * N * K + 2ull * B * N + 2ull * B * K + 2ull * K + (cand ? 8ull * nblocks * B : 0) + 4ull * B;
  return finish_desc(ctx, VTE_K_GEMV_NORM, vte_gemv_entry_mfma_norm(g), a, static_cast<uint32_t>((N + 16 * g - 1) / (16 * g)),
                     1, 256, 0, fnv1a(shape_v, sizeof shape_v), bytes, 2ull * B * N * K, out);
}

int vte_desc_gemv_rmsnorm_gather(vte_ctx* ctx, const void* W, const void* E, const int32_t* tok, const void* gamma,
                                 void* Y, void* h_or_null, void* n_or_null, int B, int V, int N, int K, float eps,
                                 vte_desc** out) {
  if (!tok) { set_error("gemv_rmsnorm_gather: tok is required"); return VTE_EINVAL; }
  return build_gemv_norm(ctx, W, E, tok, nullptr, 0, 0, nullptr, gamma, Y, h_or_null, n_or_null, B, V, N, K, eps, out);
}

int vte_desc_gemv_rmsnorm_gather_argmax(vte_ctx* ctx, const void* W, const void* E, const vte_desc* lmhead,
                                        int32_t* tok_out_or_null, const void* gamma, void* Y, void* h_or_null,
                                        void* n_or_null, int V, int N, int K, float eps, vte_desc** out) {
  if (!ctx || !lmhead) { set_error("gemv_rmsnorm_gather_argmax: lmhead is required"); return VTE_EINVAL; }
  if (lmhead->ctx != ctx || (lmhead->kernel != VTE_K_LMHEAD && lmhead->kernel != VTE_K_LMHEAD_SPLITK)) {
    set_error("gemv_rmsnorm_gather_argmax: needs an LM-head descriptor of this context"); return VTE_EINVAL;
  }
  GemvArgs g;
  std::memcpy(&g, lmhead->args, sizeof g);
  const uint32_t* cand = g.ws + 1 + lmhead->grid[0] * lmhead->grid[2];
  return build_gemv_norm(ctx, W, E, nullptr, cand, static_cast<int>(lmhead->grid[0]), g.bt, tok_out_or_null, gamma, Y,
                         h_or_null, n_or_null, g.B, V, N, K, eps, out);
}

int vte_desc_layernorm(vte_ctx* ctx, const void* x, const void* gamma, const void* beta, void* y, int rows,
                       int cols, float eps, vte_desc** out) {
  return build_norm(ctx, VTE_K_LAYERNORM, true, x, gamma, beta, y, rows, cols, eps, norm_threads(cols), out);
}

int vte_desc_rmsnorm_reshaped(vte_ctx* ctx, const void* x, const void* gamma, void* y, int rows, int cols,
                              float eps, int active_cus, vte_desc** out) {
  if (active_cus < 1) { set_error("rmsnorm_reshaped: active_cus must be positive"); return VTE_EINVAL; }
  int t = 64 * (active_cus / 32);
  t = t < 64 ? 64 : (t > 512 ? 512 : t);
  int p2 = 64;
  while (p2 * 2 <= t) p2 *= 2;
  return build_norm(ctx, VTE_K_RMSNORM_RESHAPED, false, x, gamma, nullptr, y, rows, cols, eps, p2, out);
}

int vte_gemv_default_plan(int B, int N, int K, int epilogue, int S, vte_gemv_plan* plan) {
  if (!plan) { set_error("null plan"); return VTE_EINVAL; }
  const int n_out = (epilogue == VTE_EPI_SILU_MUL) ? N / 2 : N;
  if (S < 1 || K % S != 0) { set_error("gemv plan: S must divide K"); return VTE_EINVAL; }
  int rc = plan_gemv(B, n_out, K / S, epilogue, plan);
  if (rc != VTE_OK) set_error("gemv plan: need 1 <= B <= 64 (from 17: at least one full tile of outputs), N >= 1, 8 <= K / S <= 16384");
  return rc;
}

int vte_desc_gemv(vte_ctx* ctx, const void* W, const void* X, void* Y, int B, int N, int K, int epilogue,
                  vte_desc** out) {
  GemvBuild g{VTE_K_GEMV, epilogue == VTE_EPI_SILU_MUL ? 1 : 0, W, X, Y, nullptr, nullptr, nullptr, nullptr,
              B, N, K, epilogue, 1, nullptr};
  return build_gemv(ctx, g, out);
}

int vte_desc_gemv_strided(vte_ctx* ctx, const void* W, const void* X, int ldx, void* Y, int ldy, int B, int N,
                          int K, int epilogue, vte_desc** out) {
  GemvBuild g{VTE_K_GEMV, epilogue == VTE_EPI_SILU_MUL ? 1 : 0, W, X, Y, nullptr, nullptr, nullptr, nullptr,
              B, N, K, epilogue, 1, nullptr};
  g.ldx = ldx;
  g.ldy = ldy;
  return build_gemv(ctx, g, out);
}

int vte_desc_gemv_planned(vte_ctx* ctx, const void* W, const void* X, void* Y, int B, int N, int K,
                          int epilogue, const vte_gemv_plan* plan, vte_desc** out) {
  GemvBuild g{VTE_K_GEMV, epilogue == VTE_EPI_SILU_MUL ? 1 : 0, W, X, Y, nullptr, nullptr, nullptr, nullptr,
              B, N, K, epilogue, 1, plan};
  return build_gemv(ctx, g, out);
}

// split-K workspace: [tickets: one uint32 per possible row block, rounded up][fp32 partials [S][BT][N]]
static size_t splitk_ticket_bytes(int N) { return ((static_cast<size_t>(N) + 2) * 4 + 255) & ~static_cast<size_t>(255); }

int vte_splitk_workspace_bytes(int B, int N, int S, size_t* bytes) {
  if (!bytes || B < 1 || B > 64 || N < 1 || S < 1) { set_error("splitk workspace: bad argument"); return VTE_EINVAL; }
  *bytes = splitk_ticket_bytes(N) + static_cast<size_t>(S) * (B > 32 ? 64 : (B > 16 ? 32 : 16)) * N * 4;  // partials [S][batch tile][N]
  return VTE_OK;
}

int vte_desc_gemv_splitk(vte_ctx* ctx, const void* W, const void* X, void* Y, void* workspace, int B, int N,
                         int K, int epilogue, int S, vte_desc** out) {
  if (!workspace || N < 1) { set_error("split-K: workspace is required"); return VTE_EINVAL; }
  void* partials = static_cast<unsigned char*>(workspace) + splitk_ticket_bytes(N);
  GemvBuild g{VTE_K_GEMV_SPLITK, epilogue == VTE_EPI_SILU_MUL ? 1 : 0, W, X, Y, nullptr, nullptr, workspace,
              partials, B, N, K, epilogue, S, nullptr};
  return build_gemv(ctx, g, out);
}

// Shape-derived K split for outputs too narrow to fill the device at a large batch: every
// workgroup then needs only its K part of X.  1 = do not split.
int vte_gemv_fixed_split(int B, int N, int K, int epilogue, int* S) {
  if (!S || B < 1 || B > 64 || N < 1 || K < 8) { set_error("gemv_fixed_split: bad argument"); return VTE_EINVAL; }
  const int n_out = (epilogue == VTE_EPI_SILU_MUL) ? N / 2 : N;
  const int tiles = (n_out + (epilogue == VTE_EPI_SILU_MUL ? 8 : 16) - 1) / (epilogue == VTE_EPI_SILU_MUL ? 8 : 16);
  *S = 1;
  // Batch 33 to 64, fewer than 1024 row tiles and a long K (the down projection): parts of 2048 K
  // elements, eight waves of one 256-element chunk each, X of a part fetched once per workgroup.
  // Timed on cold weights at batch 64 against the single launch: 4096 x 14336 41 us against 45;
  // with K = 4096 (QKV, O) the single launch wins (16 and 20 us against 19 and 24).
  if (B > 32 && tiles < 1024 && K >= 8192 && K % 2048 == 0 && K / 2048 <= 64) *S = K / 2048;
  return VTE_OK;
}

int vte_desc_gemv_split(vte_ctx* ctx, const void* W, const void* X, int ldx, void* workspace, int B, int N, int K,
                        int epilogue, int S, const vte_gemv_plan* plan_or_null, vte_desc** out) {
  if (!workspace || N < 1 || S < 2) { set_error("gemv_split: a workspace and S >= 2 are required"); return VTE_EINVAL; }
  if (!aligned16(workspace)) { set_error("gemv_split: the workspace must be 16-byte aligned"); return VTE_EINVAL; }
  if (S < 1 || K % S != 0) { set_error("gemv_split: S must divide K"); return VTE_EINVAL; }
  void* partials = static_cast<unsigned char*>(workspace) + splitk_ticket_bytes(N);
  vte_gemv_plan p;
  if (plan_or_null) p = *plan_or_null;
  else {
    // parts of K / S elements in 256-element chunks (512 below batch 33), one per wave where that fits
    const int n_out = (epilogue == VTE_EPI_SILU_MUL) ? N / 2 : N;
    const int tiles = (n_out + (epilogue == VTE_EPI_SILU_MUL ? 8 : 16) - 1) / (epilogue == VTE_EPI_SILU_MUL ? 8 : 16);
    p.kind = VTE_GEMV_MFMA; p.batch_tile = B > 32 ? 64 : (B > 16 ? 32 : 16);
    p.ksteps = p.batch_tile == 64 ? 2 : 4; p.prefetch = p.batch_tile == 64 ? 2 : 4;
    const int chunks = (K / S + 128 * p.ksteps - 1) / (128 * p.ksteps);
    if (p.batch_tile == 64 && chunks > 4) { p.max_waves = 8; p.rows = 16; p.groups = tiles >= 256 ? 8 : 1; }  // timed best for 4096 x 14336
    else { p.max_waves = 4; p.rows = 16 * (p.batch_tile == 64 ? 2 : 1); p.groups = tiles >= 512 ? 2 : 1; }
  }
  GemvBuild g{VTE_K_GEMV_SPLIT, epilogue == VTE_EPI_SILU_MUL ? 1 : 0, W, X, nullptr, nullptr, nullptr, nullptr,
              partials, B, N, K, epilogue, S, &p};
  g.ldx = ldx;
  g.fixed_split = true;
  return build_gemv(ctx, g, out);
}

int vte_desc_gemv_split_finish(vte_ctx* ctx, const vte_desc* split, void* Y, int ldy, vte_desc** out) {
  if (!ctx || !split || !Y || !out) { set_error("gemv_split_finish: null argument"); return VTE_EINVAL; }
  if (split->ctx != ctx || split->kernel != VTE_K_GEMV_SPLIT) { set_error("gemv_split_finish: needs a vte_desc_gemv_split descriptor of this context"); return VTE_EINVAL; }
  GemvArgs g;
  std::memcpy(&g, split->args, sizeof g);
  if (ldy == 0) ldy = g.n_out;
  if (ldy < g.n_out) { set_error("gemv_split_finish: ldy must hold a row of outputs"); return VTE_EINVAL; }
  SplitFinishArgs a{};
  a.partials = g.partials; a.Y = static_cast<uint16_t*>(Y);
  a.B = g.B; a.N = g.N; a.n_out = g.n_out; a.ldy = ldy; a.S = g.S; a.bt = g.bt; a.silu = g.n_out != g.N ? 1 : 0;
  const int v[4] = {a.B, a.N, a.n_out, a.S};
  const uint32_t gx = static_cast<uint32_t>((a.n_out + 1023) / 1024);
  return finish_desc(ctx, VTE_K_GEMV_SPLIT_FINISH, vte_split_finish_entry(), a, gx, static_cast<uint32_t>(a.B), 256, 0,
                     fnv1a(v, sizeof v), 4ull * a.S * a.B * a.N + 2ull * a.B * a.n_out, 0, out);
}

int vte_lmhead_workspace_bytes(int B, int V, int K, size_t* bytes) {
  if (!bytes) { set_error("null bytes"); return VTE_EINVAL; }
  // sized for the finest decomposition there is: one workgroup per output row, batch tile 16
  (void)K;
  if (B < 1 || B > 64 || V < 1) { set_error("lmhead workspace: bad argument"); return VTE_EINVAL; }
  const size_t blocks = static_cast<size_t>(V) + 1;
  *bytes = 4 * (1 + blocks + blocks * (B > 32 ? 64 : (B > 16 ? 32 : 16)) * 2) + 256;
  return VTE_OK;
}

int vte_desc_lmhead_argmax(vte_ctx* ctx, const void* W, const void* H, int32_t* tok, float* logits_or_null,
                           void* workspace, int B, int V, int K, vte_desc** out) {
  GemvBuild g{VTE_K_LMHEAD, 2, W, H, nullptr, logits_or_null, tok, workspace, nullptr, B, V, K, VTE_EPI_NONE, 1, nullptr};
  return build_gemv(ctx, g, out);
}

int vte_desc_lmhead_argmax_planned(vte_ctx* ctx, const void* W, const void* H, int32_t* tok,
                                   float* logits_or_null, void* workspace, int B, int V, int K,
                                   const vte_gemv_plan* plan, vte_desc** out) {
  GemvBuild g{VTE_K_LMHEAD, 2, W, H, nullptr, logits_or_null, tok, workspace, nullptr, B, V, K, VTE_EPI_NONE, 1, plan};
  return build_gemv(ctx, g, out);
}

int vte_desc_lmhead_argmax_splitk(vte_ctx* ctx, const void* W, const void* H, int32_t* tok,
                                  float* logits_or_null, void* workspace, void* partials, int B, int V, int K,
                                  int S, vte_desc** out) {
  GemvBuild g{VTE_K_LMHEAD_SPLITK, 2, W, H, nullptr, logits_or_null, tok, workspace, partials, B, V, K,
              VTE_EPI_NONE, S, nullptr};
  return build_gemv(ctx, g, out);
}

int vte_desc_argmax_finish(vte_ctx* ctx, const vte_desc* lmhead, vte_desc** out) {
  if (!ctx || !lmhead || !out) { set_error("argmax_finish: null argument"); return VTE_EINVAL; }
  if (lmhead->ctx != ctx || (lmhead->kernel != VTE_K_LMHEAD && lmhead->kernel != VTE_K_LMHEAD_SPLITK)) {
    set_error("argmax_finish: needs an LM-head descriptor of this context"); return VTE_EINVAL;
  }
  vte_desc tmp;
  int rc = fill_argmax_finish(ctx, lmhead, &tmp);
  if (rc != VTE_OK) return rc;
  return register_desc(ctx, tmp, out);
}

int vte_desc_gather(vte_ctx* ctx, const void* E, const int32_t* tok, void* H, int B, int V, int K, vte_desc** out) {
  if (!ctx || !out || !E || !tok || !H) { set_error("gather: null argument"); return VTE_EINVAL; }
  if (B < 1 || B > 65535 || V < 1 || K < 8 || K % 8 != 0) { set_error("gather: need 1 <= B <= 65535, V >= 1, K % 8 == 0"); return VTE_EINVAL; }
  if (!aligned16(E) || !aligned16(H)) { set_error("gather: E and H must be 16-byte aligned"); return VTE_EINVAL; }
  GatherArgs a{static_cast<const uint16_t*>(E), tok, static_cast<uint16_t*>(H), B, V, K};
  const uint32_t gx = static_cast<uint32_t>((K / 8 + 255) / 256);
  const uint64_t shape = (static_cast<uint64_t>(B) << 32) | static_cast<uint32_t>(K);
  return finish_desc(ctx, VTE_K_GATHER, vte_gather_entry(), a, gx, static_cast<uint32_t>(B), 256, 0, shape,
                     4ull * B * K + 4ull * B, 0, out);
}

int vte_desc_softmax_prob(vte_ctx* ctx, const float* logits, const int32_t* tok, float* prob, int B, int V,
                          vte_desc** out) {
  if (!ctx || !out || !logits || !tok || !prob) { set_error("softmax_prob: null argument"); return VTE_EINVAL; }
  if (B < 1 || B > 65535 || V < 1) { set_error("softmax_prob: need 1 <= B <= 65535, V >= 1"); return VTE_EINVAL; }
  SoftmaxArgs a{logits, tok, prob, B, V};
  const uint64_t shape = (static_cast<uint64_t>(B) << 32) | static_cast<uint32_t>(V);
  return finish_desc(ctx, VTE_K_SOFTMAX_PROB, vte_softmax_prob_entry(), a, static_cast<uint32_t>(B), 1, 1024, 0, shape,
                     8ull * B * V + 8ull * B, 4ull * B * V, out);
}

int vte_desc_memcpy(vte_ctx* ctx, void* dst, const void* src, size_t bytes, vte_desc** out) {
  if (!ctx || !out || !dst || !src) { set_error("memcpy: null argument"); return VTE_EINVAL; }
  if (bytes == 0 || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) { set_error("memcpy: need bytes > 0, bytes % 16 == 0, 16-byte aligned pointers"); return VTE_EINVAL; }
  const size_t blocks = (bytes + 16383) / 16384;
  if (blocks > 0x7fffffffull) { set_error("memcpy: too large for one launch"); return VTE_EINVAL; }
  CopyArgs a{static_cast<const unsigned char*>(src), static_cast<unsigned char*>(dst), bytes};
  return finish_desc(ctx, VTE_K_MEMCPY, vte_copy_entry(), a, static_cast<uint32_t>(blocks), 1, 256, 0,
                     static_cast<uint64_t>(bytes), 2ull * bytes, 0, out);
}

int vte_desc_memset32(vte_ctx* ctx, void* dst, uint32_t value, size_t bytes, vte_desc** out) {
  if (!ctx || !out || !dst) { set_error("memset: null argument"); return VTE_EINVAL; }
  if (bytes == 0 || bytes % 16 != 0 || !aligned16(dst)) { set_error("memset: need bytes > 0, bytes % 16 == 0, a 16-byte aligned pointer"); return VTE_EINVAL; }
  const size_t blocks = (bytes + 16383) / 16384;
  if (blocks > 0x7fffffffull) { set_error("memset: too large for one launch"); return VTE_EINVAL; }
  FillArgs a{static_cast<unsigned char*>(dst), bytes, value};
  return finish_desc(ctx, VTE_K_MEMSET, vte_fill_entry(), a, static_cast<uint32_t>(blocks), 1, 256, 0,
                     static_cast<uint64_t>(bytes), 1ull * bytes, 0, out);
}

int vte_desc_gemm(vte_ctx* ctx, const void* A, const void* Bm, void* C, int M, int N, int K, vte_desc** out) {
  if (!ctx || !out || !A || !Bm || !C) { set_error("gemm: null argument"); return VTE_EINVAL; }
  if (M < 256 || N < 256 || K < 64 || M % 256 != 0 || N % 256 != 0 || K % 64 != 0) { set_error("gemm: need M,N % 256 == 0 and K % 64 == 0"); return VTE_EINVAL; }
  if (!aligned16(A) || !aligned16(Bm) || !aligned16(C)) { set_error("gemm: pointers must be 16-byte aligned"); return VTE_EINVAL; }
  GemmArgs a{static_cast<const uint16_t*>(A), static_cast<const uint16_t*>(Bm), static_cast<uint16_t*>(C), M, N, K, M / 256, N / 256};
  const uint64_t tiles = static_cast<uint64_t>(a.tiles_m) * a.tiles_n;
  if (tiles > 0x7fffffffull) { set_error("gemm: too many tiles"); return VTE_EINVAL; }
  const uint64_t shape = fnv1a(&a.M, sizeof(int) * 3);
  return finish_desc(ctx, VTE_K_GEMM, vte_gemm_entry(), a, static_cast<uint32_t>(tiles), 1, vte_gemm_threads(),
                     vte_gemm_lds_bytes(), shape,
                     2ull * (static_cast<uint64_t>(M) * K + static_cast<uint64_t>(N) * K + static_cast<uint64_t>(M) * N),
                     2ull * M * N * K, out);
}

int vte_desc_info(const vte_desc* d, vte_desc_view* v) {
  if (!d || !v) { set_error("desc_info: null argument"); return VTE_EINVAL; }
  v->kernel = d->kernel;
  for (int i = 0; i < 3; ++i) { v->grid[i] = d->grid[i]; v->block[i] = d->block[i]; }
  v->lds_bytes = d->lds_bytes;
  v->arg_bytes = d->arg_bytes;
  v->hash = desc_hash(d);  // recomputed from the bytes as they are now
  v->profile_key = d->profile_key;
  v->bytes = d->bytes;
  v->flops = d->flops;
  return VTE_OK;
}

int vte_desc_args(const vte_desc* d, void* dst, size_t cap) {
  if (!d || !dst) { set_error("desc_args: null argument"); return VTE_EINVAL; }
  std::memcpy(dst, d->args, cap < d->arg_bytes ? cap : d->arg_bytes);
  return VTE_OK;
}

}  // extern "C"
