// Argument blocks of the fixed-structure kernels.  A descriptor stores one of
// these by value (pointer values included) and the kernel receives exactly those
// bytes, so "submitting the descriptor unchanged" is a memcpy-level statement
// (Sec. 4.2, "Immutable Operation Descriptors").
#pragma once
#include <stddef.h>
#include <stdint.h>

struct NormArgs {
  const uint16_t* x;
  const uint16_t* gamma;
  const uint16_t* beta;   // LayerNorm only
  uint16_t* y;
  const int32_t* tok;     // fused gather: row r is x[tok[r], :] (x = embedding table of V rows); else null
  uint16_t* h_out;        // fused gather: optional copy of the gathered rows
  int rows, cols, V;
  float eps;
  float inv_cols;
  // fused greedy-token finish: the token of row r is first reduced from the
  // (value, index) candidates an LM-head launch left behind (else null)
  const uint32_t* cand;   // values [cand_bt][nblocks] (fp32 bits), then indices [cand_bt][nblocks]
  int32_t* tok_out;       // optional: where the finished tokens are also stored
  int nblocks, cand_bt;
};

// GEMV family: plain, SiLU-mul, LM head (+argmax), and the split-K baselines.
struct GemvArgs {
  const uint16_t* W;      // [N,K] bf16, K contiguous
  const uint16_t* X;      // [B,K] bf16
  uint16_t* Y;            // [B,N_out] bf16 (null for LM head)
  float* logits;          // LM head: [B,N] fp32 or null
  int32_t* tok;           // LM head: [B]
  uint32_t* ws;           // LM head: block partials + ticket; split-K: tickets
  float* partials;        // split-K: [S][B][N] fp32
  int B, N, K;
  int ldx, ldy;           // row strides of X and Y in elements (K and n_out when dense)
  int n_out;              // outputs per batch row (N, or N/2 with SiLU-mul)
  int groups;             // row groups each workgroup walks through
  int bt;                 // batch slots of the launch: kernel batch tile x gridDim.z
  int S;                  // K split (1 = fixed structure)
  int k_per_split;        // K / S
};

// A GEMV whose input rows are produced in its own prologue: the decode loop's step boundary
// (greedy-token finish, embedding gather, RMSNorm) fused in front of the first projection.
struct GemvNormArgs {
  GemvArgs g;             // g.X is unused: the rows come from E
  const uint16_t* E;      // embedding table [V,K] bf16
  const uint16_t* gamma;  // [K] bf16
  const int32_t* tok;     // tokens [B], or null when they come from the candidates
  const uint32_t* cand;   // LM-head candidates: values [cand_bt][nblocks] (fp32 bits), then indices; or null
  int32_t* tok_out;       // optional: where the finished tokens are also stored
  uint16_t* h_out;        // optional [B,K]: the gathered rows
  uint16_t* n_out;        // optional [B,K]: the normalised rows
  int V, nblocks, cand_bt;
  float eps;
};

struct GatherArgs {
  const uint16_t* E;
  const int32_t* tok;
  uint16_t* H;
  int B, V, K;
};

struct CopyArgs {
  const unsigned char* src;
  unsigned char* dst;
  size_t bytes;           // multiple of 16
};

struct FillArgs {
  unsigned char* dst;
  size_t bytes;           // multiple of 16
  uint32_t value;
};

struct SoftmaxArgs {
  const float* logits;    // [B,V] fp32
  const int32_t* tok;     // [B]
  float* prob;            // [B]
  int B, V;
};

struct GemmArgs {
  const uint16_t* A;      // [M,K]
  const uint16_t* Bm;     // [N,K]
  uint16_t* C;            // [M,N]
  int M, N, K;
  int tiles_m, tiles_n;
};

// Finish of a GEMV whose K range was split by a shape-derived factor S: adds the S partial sums
// of every output in split order and applies the epilogue.
struct SplitFinishArgs {
  const float* partials;  // [S][bt][N] fp32 (SiLU: gate sums at [0,n_out), up sums at [n_out, 2 n_out) of a row)
  uint16_t* Y;            // [B, ldy] bf16
  int B, N, n_out, ldy, S, bt, silu;
};

// Second stage of the greedy token: reduce the per-workgroup (value, index)
// candidates the LM head left in its workspace.
struct ArgmaxFinishArgs {
  const uint32_t* pairs;  // values [bt][nblocks] (fp32 bits), then indices [bt][nblocks]
  int32_t* tok;           // [B]
  int nblocks, bt, B;
};
