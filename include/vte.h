/*
 * vte.h — C ABI of the late-binding runtime and its fixed-structure kernels
 * for one MI355X (gfx950, 256 CUs in 8 XCDs).
 *
 * What the library does, in the paper's terms:
 *   - an *immutable operation descriptor* D_k holds a kernel entry, the values
 *     of its launch arguments (pointers by value), grid and block dimensions,
 *     dynamic LDS bytes and attributes (Sec. 4.2, "Immutable Operation
 *     Descriptors").  Nothing in scheduling ever modifies one;
 *   - a *physical context* (pCtx) is one replaceable allocation of compute
 *     units: here a HIP stream created with a CU mask (Sec. 3.4 names
 *     CU-masked queues as the AMD primitive; Sec. 4.3 defines the pCtx, its
 *     four states and the bounded, pre-created hierarchical pool);
 *   - a *virtual stream* keeps the logical order of the launches submitted to
 *     it as a chain of completion tokens (Sec. 4.2, "Token-Based Logical
 *     Dependencies");
 *   - the *dispatcher* binds each logically ready launch to an eligible,
 *     non-conflicting pCtx proposed by a policy, re-validates the proposal,
 *     submits the descriptor unchanged and propagates completion (Sec. 4.4);
 *   - the policy is three callbacks Pick / Select / Prepare (Sec. 4.5).
 * Because the grid, block shape and floating-point reduction tree of every
 * kernel below are functions of the problem shape only, the output bits of a
 * descriptor are the same on every pCtx (the parallel-structure invariant,
 * Sec. 3.1).  The *_splitk / *_reshaped descriptors are the negative control:
 * their structure is derived from a CU count (Sec. 2.3, C~_k = g(C_k, R_k)).
 *
 * Conventions
 *   - every function returns int: VTE_OK (0) or a negative VTE_E* code; no
 *     exception crosses the boundary.  vte_last_error() returns a thread-local
 *     message for the last failure on the calling thread, vte_last_hip_error()
 *     the HIP error code behind a VTE_EHIP.
 *   - "device pointer" = address in the HBM of the device given to vte_init,
 *     owned by the caller, who keeps the buffer alive and free of races until
 *     the launch's token is done (Sec. 4.2: contents of referenced memory and
 *     their synchronisation stay under application control).  "host pointer"
 *     = ordinary process memory.  The library never allocates or frees device
 *     memory on the launch path; descriptors, streams, events and tokens are
 *     owned by the library.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE binary32),
 *     row-major, innermost dimension contiguous.
 *   - thread safety: every call may be made from any thread; one internal
 *     dispatcher thread per vte_ctx does policy-driven binding and completion
 *     polling (Sec. 6: client-side submission thread, batched event polling).
 */
#ifndef VTE_H_
#define VTE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes ---------------------------------------------------------- */
enum {
  VTE_OK = 0,
  VTE_EINVAL = -1,    /* bad argument (null pointer, shape not supported, bad id) */
  VTE_ENOMEM = -2,    /* host allocation failed */
  VTE_EHIP = -3,      /* a HIP call failed; see vte_last_hip_error() */
  VTE_EBUSY = -4,     /* lease conflict, closed gate or reservation held by another owner */
  VTE_ENOTREADY = -5, /* a predecessor token is not yet satisfied */
  VTE_EINCOMPAT = -6, /* the pCtx cannot run the descriptor unchanged */
  VTE_ESTATE = -7,    /* call not valid in the current state (e.g. fake-only hook on HIP backend) */
  VTE_ETIMEOUT = -8   /* a bounded wait expired */
};

/* Every call returns VTE_OK or one of the codes above; nothing is thrown across the ABI.
 * The message and, after VTE_EHIP, the failing HIP error code of the calling thread's last
 * failed call (thread-local; the string stays valid until that thread's next failure). */
const char* vte_last_error(void);
int vte_last_hip_error(void);

/* ---- opaque handles ------------------------------------------------------- */
typedef struct vte_ctx vte_ctx;         /* one device + pool + dispatcher */
typedef struct vte_desc vte_desc;       /* immutable launch descriptor D_k */
typedef struct vte_vstream vte_vstream; /* logical stream of a virtual context */
typedef uint64_t vte_token;             /* completion token; 0 = "already satisfied" */

/* ---- pool configuration (Sec. 4.3, "Hierarchical pCtx Pool") --------------- */
enum { VTE_BACKEND_HIP = 0, VTE_BACKEND_FAKE = 1 };
/* STRICT: an op is bound only after the host has observed every predecessor's
 * completion (Sec. 4.4, "Readiness Before Binding").  PIPELINED: up to
 * `lookahead` successors of in-flight ops are bound early and the edge is kept
 * on the device (stream order on the same pCtx, an event wait across pCtxs);
 * descriptors, H and therefore output bits are the same in both modes. */
enum { VTE_MODE_STRICT = 0, VTE_MODE_PIPELINED = 1 };
/* STRIPED: mask bit i is handed to hipExtStreamCreateWithCUMask unchanged; on
 * MI355X consecutive bits fall on consecutive XCDs, so a run of w bits is w/8
 * CUs on each of the 8 XCDs.  It is the only layout offered. */
enum { VTE_LAYOUT_STRIPED = 0 };

/* Every pCtx is a hardware queue.  An MI355X process that keeps more than about
 * 22 compute queues alive is time-sliced by the queue scheduler (measured: 11 ms
 * stalls of the running queue every ~50 ms from 24 queues on), so the default
 * pool is the full tree (15 nodes for 256 CUs / 32) plus one remainder per tree
 * level: 17 queues.  ALL gives every non-root node its remainder (27 queues). */
enum { VTE_REMAINDERS_NONE = 0, VTE_REMAINDERS_ALL = 1, VTE_REMAINDERS_PER_LEVEL = 2 };

typedef struct vte_pool_cfg {
  int backend;         /* VTE_BACKEND_* */
  int total_cus;       /* 0 = ask the device (HIP) / 256 (FAKE) */
  int leaf_cus;        /* minimum allocation unit; 0 = 32 */
  int layout;          /* VTE_LAYOUT_STRIPED */
  int with_remainders; /* VTE_REMAINDERS_*: which nodes get a pre-created remainder pCtx */
  int mode;            /* VTE_MODE_* */
  int lookahead;       /* PIPELINED: max unfinished ops bound ahead per vstream; 0 = 16 */
  int stats_capacity;  /* ring size of per-op records kept for vte_stats_read; 0 = 65536 */
  unsigned device_timing_mask; /* bit k set: launches of kernel VTE_K_k carry a pair of timing events on
                                  their own stream (the kernel's begin and end on the device) and
                                  vte_op_record.gpu_seconds is filled */
  int dispatch_pipes;  /* compute pipes the device deals its queues to, round-robin in creation order
                          (measured: 4 on MI355X); 0 = 4.  Queues are created in an order that puts
                          disjoint pCtxs on different pipes where it can (Sec. 4.3, bounded pool). */
  int device_timing_stride; /* of the launches device_timing_mask selects, every stride-th per kernel id
                               is timed (the first one included); 0 or 1 = all.  A timed launch keeps
                               the stream idle for a few microseconds around it, so a sampled average
                               disturbs a throughput measurement less. */
} vte_pool_cfg;

/* Fills *cfg with the defaults (HIP, device CU count, leaf 32, one remainder per level, STRICT). */
int vte_pool_cfg_default(vte_pool_cfg* cfg);

/* Creates the context on `device`: builds the pool tree, pre-creates one
 * CU-masked stream per pCtx and starts the dispatcher thread.  Nothing is
 * created on the dispatch path afterwards.  FAKE backend: no HIP call at all;
 * launches are logged and complete when vte_fake_complete() says so. */
int vte_init(vte_ctx** out, int device, const vte_pool_cfg* cfg);
/* Waits for all submitted work, stops the dispatcher, destroys streams/events.
 * Descriptors and vstreams still alive are destroyed too. */
int vte_shutdown(vte_ctx* ctx);

/* ---- pCtx pool introspection ------------------------------------------------ */
enum { VTE_PCTX_NODE = 0, VTE_PCTX_REMAINDER = 1 };
enum { VTE_PCTX_IDLE = 0, VTE_PCTX_LEASED = 1, VTE_PCTX_DRAINING = 2, VTE_PCTX_RESERVED = 3 };

typedef struct vte_pctx_info {
  int id;
  int kind;          /* VTE_PCTX_NODE | VTE_PCTX_REMAINDER */
  int width;         /* number of CUs */
  int level;         /* NODE: depth in the tree (0 = root); REMAINDER: level of its node */
  int parent;        /* NODE: parent node id or -1; REMAINDER: the node it complements */
  int child[2];      /* NODE: children or -1,-1 (leaf); REMAINDER: -1,-1 */
  int remainder;     /* NODE: id of the pCtx spanning every other CU, -1 for the root */
  int state;         /* VTE_PCTX_* */
  int gate_open;     /* 1 = admits new operations */
  int outstanding;   /* submitted, not yet observed complete */
  int reserved_for;  /* vstream id holding (or waiting for) a reservation, else -1 */
  uint32_t mask[8];  /* CU mask, bit i of word i/32 */
  int pipe;          /* dispatch pipe of its queue; pCtxs on one pipe dispatch one kernel at a time */
} vte_pctx_info;

/* The pool of Sec. 4.3: *count pCtxs with ids 0 .. *count - 1, fixed from vte_init to
 * vte_shutdown.  vte_pool_info copies a snapshot of one pCtx (host struct owned by the
 * caller); VTE_EINVAL for an id out of range. */
int vte_pool_count(vte_ctx* ctx, int* count);
int vte_pool_info(vte_ctx* ctx, int pctx_id, vte_pctx_info* info);
/* The order in which the backend queues were created: ids[k] is the pCtx whose queue
 * was the k-th, or -1 for a placeholder queue; the k-th queue sits on pipe
 * k % dispatch_pipes.  Copies min(cap, *n_out) entries. */
int vte_pool_creation_order(vte_ctx* ctx, int* ids, int cap, int* n_out);
/* First pCtx of kind NODE with this width (lowest id), or the n-th with `index`. */
int vte_pool_find(vte_ctx* ctx, int kind, int width, int index, int* pctx_id);
/* 1 if the two pCtxs share a CU.  Decided by walking the hierarchy, not by
 * comparing masks (tests compare it with the mask intersection). */
int vte_pool_conflict(vte_ctx* ctx, int pctx_a, int pctx_b, int* conflict);
/* The hipStream_t behind a pCtx (HIP backend), so device allocations and copies
 * made elsewhere can be ordered against it.  Owned by the library. */
int vte_pctx_native_stream(vte_ctx* ctx, int pctx_id, void** hip_stream);

/* ---- descriptors: one typed constructor per fixed-structure kernel ---------- */
/* All constructors copy the argument VALUES now (pointer values included) and
 * derive grid/block/LDS from the shape alone — never from a CU count.  The only
 * HIP call they make is a one-time attribute on kernels that need more than
 * 48 KiB of LDS.  *out is owned by the caller (vte_desc_destroy) and must outlive
 * every launch made from it.  A descriptor may be launched any number of times. */

/* y[r,i] = bf16( x[r,i] * rsqrt(mean_j x[r,j]^2 + eps) * gamma[i] ), fp32 sum of
 * squares in a fixed tree, one rounding at the end.  x,y: device [rows,cols]
 * bf16; gamma: device [cols] bf16.  cols % 8 == 0, cols <= 16384.
 * (Operator family: Sec. 1 / Sec. 2.3 "reductions".) */
int vte_desc_rmsnorm(vte_ctx* ctx, const void* x, const void* gamma, void* y, int rows,
                     int cols, float eps, vte_desc** out);
/* The same RMSNorm with the embedding gather fused in front: row b of the input
 * is E[tok[b], :] (E: device [V,cols] bf16; tok: device [B] int32, clamped to
 * [0,V)); h_or_null: optional device [B,cols] copy of the gathered rows.  One
 * launch instead of gather + norm; the arithmetic and its tree are unchanged. */
int vte_desc_rmsnorm_gather(vte_ctx* ctx, const void* E, const int32_t* tok, const void* gamma, void* y,
                            void* h_or_null, int B, int V, int cols, float eps, vte_desc** out);
/* The decode loop's step boundary in one launch: finishes the greedy token of
 * the LM-head launch before it (tok[b] = lowest index attaining the maximum over
 * the candidates `lmhead` leaves in its workspace; NaN never wins, all-NaN -> 0),
 * gathers E[tok[b], :] and applies the RMSNorm above.  tok_out_or_null: optional
 * device [B] int32 that also receives the tokens.  B is the LM head's batch.
 * Replaces vte_desc_argmax_finish + vte_desc_rmsnorm_gather between two steps;
 * the token and the norm bits are the same. (Sec. 7.1 / 7.2) */
int vte_desc_rmsnorm_gather_argmax(vte_ctx* ctx, const void* E, const vte_desc* lmhead,
                                   int32_t* tok_out_or_null, const void* gamma, void* y, void* h_or_null,
                                   int V, int cols, float eps, vte_desc** out);
/* The step boundary folded into the launch that consumes it: Y[b,:] = W * rmsnorm(E[tok[b],:]) with
 * the RMSNorm above (same tree, same single rounding to bf16) computed in the prologue of the GEMV,
 * by every workgroup for itself, while the first weights are on their way; one launch fewer per
 * decode step (Sec. 7.1 / 7.2 decode loop; Sec. 3.1: the structure depends on the shape alone).
 * W: device [N,K] bf16; E: device [V,K] bf16, below 2 GiB; gamma: device [K] bf16; Y: device [B,N]
 * bf16; h_or_null, n_or_null: optional device [B,K] bf16 copies of the gathered and of the
 * normalised rows (for inspection; what vte_desc_rmsnorm_gather stores).  Built for K = 4096,
 * 1 <= B <= 16, N >= 16; anything else returns VTE_EINVAL.  The GEMV is the matrix-core kind with
 * one 1024-element chunk per wave: its output bits equal vte_desc_gemv_planned with that plan
 * (batch_tile 16, ksteps 8, prefetch 2, max_waves 4, groups 1, rows 32 above 256 row tiles, else 16)
 * on the output of vte_desc_rmsnorm_gather.
 * _gather takes the tokens (device [B] int32, clamped to [0,V)); _gather_argmax finishes them from
 * the candidates of `lmhead` first (as vte_desc_rmsnorm_gather_argmax; B is the LM head's batch) and
 * stores them to tok_out_or_null. */
int vte_desc_gemv_rmsnorm_gather(vte_ctx* ctx, const void* W, const void* E, const int32_t* tok, const void* gamma,
                                 void* Y, void* h_or_null, void* n_or_null, int B, int V, int N, int K, float eps,
                                 vte_desc** out);
int vte_desc_gemv_rmsnorm_gather_argmax(vte_ctx* ctx, const void* W, const void* E, const vte_desc* lmhead,
                                        int32_t* tok_out_or_null, const void* gamma, void* Y, void* h_or_null,
                                        void* n_or_null, int V, int N, int K, float eps, vte_desc** out);
/* y = (x - mu) * rsqrt(var + eps) * gamma + beta, biased variance, two fixed-tree
 * fp32 reductions (mean, then centred squares).  Same layout and limits. (Sec. 1) */
int vte_desc_layernorm(vte_ctx* ctx, const void* x, const void* gamma, const void* beta,
                       void* y, int rows, int cols, float eps, vte_desc** out);

enum { VTE_EPI_NONE = 0, VTE_EPI_SILU_MUL = 1 };
/* Y[b,n] = bf16( sum_k W[n,k] X[b,k] ).  W: device [N,K] bf16 (each output's K
 * contiguous); X: device [B,K] bf16; Y: device [B,N] bf16.  1 <= B <= 64
 * (from 17 up N must hold at least one tile of 16 outputs, 8 with SILU_MUL),
 * K % 8 == 0, K <= 16384.  fp32 accumulation in a tree that depends on K and the
 * plan only (vte_gemv_plan; by default chosen from B, N, K): for the small batches
 * a K-tile of 256 is 32 lanes x 8 contiguous elements; a lane adds the products
 * of its slice in ascending order, a fixed butterfly adds the 64 lanes of a
 * wave, and the per-slice sums are added in ascending K order; the matrix-core
 * kinds accumulate 32 K positions per instruction and chain them in ascending K.
 * The weights are read once whatever the batch.
 * epilogue SILU_MUL: N must be even; rows [0,N/2) are gate, [N/2,N) up;
 * Y is [B,N/2] = bf16( silu(g_fp32) * u_fp32 ).  (Sec. 1 "GEMV"; Sec. 2.3.) */
int vte_desc_gemv(vte_ctx* ctx, const void* W, const void* X, void* Y, int B, int N, int K,
                  int epilogue, vte_desc** out);

/* The same GEMV reading X rows ldx elements apart and writing Y rows ldy
 * elements apart (ldx >= K, ldx % 8 == 0, ldy >= outputs per row): lets a launch
 * consume a column slice of a wider activation tensor in place.  The reduction
 * tree is that of vte_desc_gemv. */
int vte_desc_gemv_strided(vte_ctx* ctx, const void* W, const void* X, int ldx, void* Y, int ldy,
                          int B, int N, int K, int epilogue, vte_desc** out);

/* The greedy token takes two launches: the LM head, then vte_desc_argmax_finish
 * built from it and submitted right behind it.
 * LM head: logits[b,v] = sum_k W[v,k] H[b,k] in fp32 (never rounded to bf16),
 * and per workgroup the best (value, lowest index) candidate of each batch row,
 * left in the workspace.  Finish: tok[b] = lowest v attaining the maximum over
 * all candidates (NaN never wins; all-NaN -> 0).
 * W: device [V,K] bf16; H: device [B,K] bf16; tok: device [B] int32;
 * logits_or_null: device [B,V] fp32 or NULL; workspace: device buffer of
 * vte_lmhead_workspace_bytes() bytes, zero-filled by the caller before the
 * first launch and private to launches of this descriptor that do not overlap
 * in time.  (Sec. 7.1 / 7.2: LM-head logits and the greedy token.) */
int vte_lmhead_workspace_bytes(int B, int V, int K, size_t* bytes);
int vte_desc_lmhead_argmax(vte_ctx* ctx, const void* W, const void* H, int32_t* tok,
                           float* logits_or_null, void* workspace, int B, int V, int K,
                           vte_desc** out);
/* Second stage: reads the candidates `lmhead` (an LM-head descriptor, fixed or
 * split-K) leaves in its workspace and writes its tok[].  Comparison of
 * (value, index) pairs is a total order, so no reduction order is involved. */
int vte_desc_argmax_finish(vte_ctx* ctx, const vte_desc* lmhead, vte_desc** out);

/* The work decomposition of a GEMV-family descriptor, spelled out.  It is part
 * of the submitted structure C_k: chosen from the shape by vte_gemv_default_plan,
 * or given by the caller, and frozen in the descriptor.
 *   batch_tile  batch rows the kernel is built for (1,2,4,8,16; 32 and 64: MFMA kinds); a batch
 *               larger than the tile runs as ceil(B / batch_tile) chunks that each re-read the
 *               weights
 *   rows        weight rows a wave streams at once (rows * batch_tile in {16,32,64})
 *   ksteps      512-element K steps per wave: a workgroup has
 *               ceil(ceil(K/S/512) / ksteps) waves, one per K-slice
 *   prefetch    1: the next row group's loads are issued before the current one is reduced
 *   max_waves   8 or 16: the register budget the kernel was compiled for
 *   groups      row groups a workgroup walks through
 *   kind        VTE_GEMV_DOT2: the fields above (batch <= 16).  VTE_GEMV_MFMA (matrix-core
 *               tiles of 16 weight rows x 16 batch columns): batch_tile = 16 (B <= 16), or 32
 *               for two column tiles per weight tile (batch 17 to 32 in one tile; batch 33 to
 *               64 as two chunks of 32 rows in one launch, each reading the weights), or 64 for
 *               four column tiles (batch 33 to 64; ksteps <= 2: the default for outputs too
 *               narrow to fill the device without splitting K); rows = 16 x the tiles
 *               accumulated at once; ksteps = number of 128-element blocks per K chunk (4; 8 in
 *               the default plan of wide LM heads with K <= 4096, where four waves then hold all
 *               of X; 2 with batch_tile 64);
 *               the workgroup has min(max_waves, chunks) waves that take the chunks
 *               round-robin; prefetch = blocks the loads run ahead; groups as above.
 *               VTE_GEMV_MFMA_ROWS (batch 17 to 64, one pass over the weights): batch_tile
 *               = 64 (four column tiles per weight tile) or 32 (two; B <= batch_tile); the
 *               workgroup has max_waves (4 or 8) waves that split the row tiles, not K, and
 *               share X through LDS; rows =
 *               16 x the tiles a wave accumulates at once; prefetch = 128-element K steps
 *               the weight loads run ahead; ksteps = 1; groups = rounds of a workgroup.
 *               An output is one accumulator chain along K, nothing crosses a wave.
 * Only combinations the library was built with are accepted.  The reduction tree
 * of an output depends on K and the plan alone — never on the device. */
enum { VTE_GEMV_DOT2 = 0, VTE_GEMV_MFMA = 1, VTE_GEMV_MFMA_ROWS = 2 };
typedef struct vte_gemv_plan {
  int batch_tile, rows, ksteps, prefetch, max_waves, groups;
  int kind;
} vte_gemv_plan;
int vte_gemv_default_plan(int B, int N, int K, int epilogue, int S, vte_gemv_plan* plan);
int vte_desc_gemv_planned(vte_ctx* ctx, const void* W, const void* X, void* Y, int B, int N, int K,
                          int epilogue, const vte_gemv_plan* plan, vte_desc** out);
int vte_desc_lmhead_argmax_planned(vte_ctx* ctx, const void* W, const void* H, int32_t* tok,
                                   float* logits_or_null, void* workspace, int B, int V, int K,
                                   const vte_gemv_plan* plan, vte_desc** out);

/* A GEMV as two launches, for outputs too narrow to fill the device at a large batch (Sec. 1
 * "GEMV"; the structure stays a function of the shape, Sec. 3.1).  The K range is cut into S
 * contiguous parts, S derived from the SHAPE (vte_gemv_fixed_split; never from a CU count): the
 * split launch has N-tiles x S workgroups, each needing only its part of X, and leaves the fp32
 * partial sums of every output in the workspace; the finish launch adds the S partial sums of an
 * output in ascending part order, applies the epilogue and rounds to bf16 once.  No tickets, no
 * atomics, no fences: the order between the two is the virtual stream's.
 * Tree of an output: inside a part the K-split matrix-core tree of vte_desc_gemv (chunks of 256 or
 * 512 elements chained per wave, waves added in order), then p[0] + p[1] + ... + p[S-1].
 * workspace: device, vte_splitk_workspace_bytes(B, N, S) bytes, 16-byte aligned, private to launches
 * of this pair that do not overlap in time; need not be zeroed.  X rows are ldx elements apart
 * (0 = K), Y rows ldy (0 = outputs per row).  1 <= B <= 64, K % S == 0, (K / S) % 8 == 0. */
int vte_gemv_fixed_split(int B, int N, int K, int epilogue, int* S); /* *S = 1: one launch (vte_desc_gemv) is the default */
int vte_desc_gemv_split(vte_ctx* ctx, const void* W, const void* X, int ldx, void* workspace, int B, int N,
                        int K, int epilogue, int S, const vte_gemv_plan* plan_or_null, vte_desc** out);
int vte_desc_gemv_split_finish(vte_ctx* ctx, const vte_desc* split, void* Y, int ldy, vte_desc** out);

/* H[b,:] = E[tok[b],:].  E: device [V,K] bf16; tok: device [B] int32 (values in
 * [0,V), clamped otherwise); H: device [B,K] bf16.  K % 8 == 0. */
int vte_desc_gather(vte_ctx* ctx, const void* E, const int32_t* tok, void* H, int B, int V,
                    int K, vte_desc** out);

/* prob[b] = softmax(logits[b,:])[tok[b]] = exp(l[tok] - max) / sum_v exp(l[v] - max), fp32, for
 * the fp32 logits an LM-head launch stored (Sec. 7.2: the decode replay records the softmax
 * probability next to the token).  logits: device [B,V] fp32; tok: device [B] int32; prob:
 * device [B] fp32; a token outside [0,V) gives 0.  One workgroup per row; the sum's tree
 * depends on V alone (thread t adds elements t, t+1024, ... in order, fixed butterfly over a
 * wave, wave partials in wave order). */
int vte_desc_softmax_prob(vte_ctx* ctx, const float* logits, const int32_t* tok, float* prob, int B, int V,
                          vte_desc** out);

/* Data movement as operations of a virtual stream (Sec. 4.2: memory operations are
 * nodes of the same dependency graph as kernels).  dst, src: device pointers, 16-byte
 * aligned; bytes a positive multiple of 16; the ranges must not overlap.  The launch
 * geometry follows from `bytes` alone.  memset32 stores the 32-bit `value` repeatedly. */
int vte_desc_memcpy(vte_ctx* ctx, void* dst, const void* src, size_t bytes, vte_desc** out);
int vte_desc_memset32(vte_ctx* ctx, void* dst, uint32_t value, size_t bytes, vte_desc** out);

/* C = A * Bm^T, bf16 in, fp32 MFMA accumulation, bf16 out.  A: device [M,K];
 * Bm: device [N,K]; C: device [M,N].  M,N % 256 == 0, K % 64 == 0.  Fixed 2-D
 * tile grid, no split-K.  (The background training-shaped co-tenant; Sec. 7.5
 * uses a BF16 GEMM as its probe.) */
int vte_desc_gemm(vte_ctx* ctx, const void* A, const void* Bm, void* C, int M, int N, int K,
                  vte_desc** out);

/* ---- reshaping baselines (the negative control, Sec. 2.3 / Sec. 7.1) -------- */
/* GEMV whose K range is cut into S contiguous chunks (S = active CUs / 32 in the
 * experiments); the S fp32 partial sums of an output are written to the
 * workspace and added in chunk order by whichever chunk-block finishes last.
 * Same lanes, same instructions — only the grouping changes with S.
 * workspace: device, vte_splitk_workspace_bytes(), zero-filled by the caller
 * before the first launch, private to non-overlapping launches. */
int vte_splitk_workspace_bytes(int B, int N, int S, size_t* bytes);
int vte_desc_gemv_splitk(vte_ctx* ctx, const void* W, const void* X, void* Y, void* workspace,
                         int B, int N, int K, int epilogue, int S, vte_desc** out);
/* LM head with the same split: `workspace` as for vte_desc_lmhead_argmax,
 * `partials` a second device buffer of vte_splitk_workspace_bytes(B,V,S). */
int vte_desc_lmhead_argmax_splitk(vte_ctx* ctx, const void* W, const void* H, int32_t* tok,
                                  float* logits_or_null, void* workspace, void* partials,
                                  int B, int V, int K, int S, vte_desc** out);
/* RMSNorm whose threads-per-row is derived from a CU count (64 threads per 32
 * active CUs, clamped to [64,512]), which regroups the sum of squares. */
int vte_desc_rmsnorm_reshaped(vte_ctx* ctx, const void* x, const void* gamma, void* y,
                              int rows, int cols, float eps, int active_cus, vte_desc** out);

/* ---- descriptor inspection --------------------------------------------------- */
enum {
  VTE_K_RMSNORM = 1, VTE_K_LAYERNORM = 2, VTE_K_GEMV = 3, VTE_K_LMHEAD = 4, VTE_K_GATHER = 5,
  VTE_K_GEMM = 6, VTE_K_GEMV_SPLITK = 7, VTE_K_LMHEAD_SPLITK = 8, VTE_K_RMSNORM_RESHAPED = 9,
  VTE_K_ARGMAX_FINISH = 10, VTE_K_RMSNORM_GATHER = 11, VTE_K_RMSNORM_GATHER_ARGMAX = 12,
  VTE_K_MEMCPY = 13, VTE_K_MEMSET = 14, VTE_K_SOFTMAX_PROB = 15, VTE_K_GEMV_SPLIT = 16, VTE_K_GEMV_SPLIT_FINISH = 17,
  VTE_K_GEMV_NORM = 18
};
typedef struct vte_desc_view {
  int kernel;           /* VTE_K_* */
  uint32_t grid[3];
  uint32_t block[3];
  uint32_t lds_bytes;   /* dynamic LDS */
  uint32_t arg_bytes;   /* size of the copied argument block */
  uint64_t hash;        /* FNV-1a over kernel, grid, block, lds and the argument bytes */
  uint64_t profile_key; /* equal for descriptors of the same kernel and shape */
  uint64_t bytes;       /* algorithmic HBM bytes of one launch */
  uint64_t flops;       /* algorithmic flops of one launch */
} vte_desc_view;
/* Read-only view of a descriptor (Sec. 4.2): the hash is recomputed from the bytes as they
 * are now, so equal views before and after a launch show that it was submitted unchanged. */
int vte_desc_info(const vte_desc* desc, vte_desc_view* view);
/* Copies min(cap, arg_bytes) bytes of the argument block to `dst` (host). */
int vte_desc_args(const vte_desc* desc, void* dst, size_t cap);
/* The caller owns its descriptors.  VTE_EBUSY while a launch of this descriptor is queued or
 * in flight; descriptors still alive at vte_shutdown are freed there. */
int vte_desc_destroy(vte_desc* desc);

/* ---- explicit binding (tests, width sweeps, profiling) ------------------------ */
/* Submits `desc` unchanged on pCtx `pctx_id` from the calling thread.  Bypasses
 * the policy but not validation: VTE_EINCOMPAT if the pCtx cannot run it,
 * VTE_EBUSY if the pCtx conflicts with another active lease, its gate is closed
 * or it is reserved for a vstream.  Has no logical predecessor.  *token_out
 * (may be NULL) is satisfied when the launch has completed. */
int vte_bind_and_launch(vte_ctx* ctx, const vte_desc* desc, int pctx_id, vte_token* token_out);

/* ---- virtual streams and policy-driven dispatch ------------------------------ */
enum { VTE_CLASS_LATENCY = 0, VTE_CLASS_BEST_EFFORT = 1 };
int vte_vstream_create(vte_ctx* ctx, int klass, vte_vstream** out);
int vte_vstream_destroy(vte_vstream* vs); /* waits for its tail first */
int vte_vstream_id(const vte_vstream* vs, int* id);
/* Restricts the vstream's launches to one pCtx (the fixed-binding baseline);
 * pctx_id = -1 removes the restriction. */
int vte_vstream_pin(vte_vstream* vs, int pctx_id);
/* The new op depends on the stream's tail token and becomes the new tail; an
 * empty stream's tail is already satisfied (Sec. 4.2). */
int vte_submit(vte_vstream* vs, const vte_desc* desc, vte_token* token_out);
/* As vte_submit, with extra predecessor tokens from other vstreams (the edges an
 * event wait would add; each token is an immutable completion point). */
int vte_submit_after(vte_vstream* vs, const vte_desc* desc, const vte_token* deps, int n_deps,
                     vte_token* token_out);
/* vte_submit for descs[0..n) in order, validated as a whole before the first is
 * submitted; *last_out (may be NULL) = token of the last op submitted. */
int vte_submit_batch(vte_vstream* vs, const vte_desc* const* descs, int n, vte_token* last_out);
/* Events (Sec. 4.2, "Token-Based Logical Dependencies"): recording captures the stream's
 * current tail as an immutable completion point (0, already satisfied, for an empty
 * stream); work submitted to the recorded stream later does not move it.  Waiting makes
 * every op submitted to `vs` from now on depend on that point, whichever stream it came
 * from (a token of this context that was issued; VTE_EINVAL otherwise). */
int vte_event_record(vte_vstream* vs, vte_token* event_out);
int vte_vstream_wait_event(vte_vstream* vs, vte_token event);
/* A token is satisfied when its launch has been observed complete (Sec. 4.2, 4.4); token 0
 * and tokens of finished launches are satisfied.  query never blocks; wait blocks the caller
 * (not the dispatcher) until the token is satisfied and makes the dispatcher record a
 * completion behind the launch if none covers it yet.  Callable from any thread.
 * Failures.  A launch whose completion reports a device error, an operation whose backend
 * submission failed 8 times in a row (Sec. 4.4: until then it stays ready), and every operation
 * that depends on a failed one are retired as FAILED: their tokens count as done (nothing
 * waits for ever), and vte_token_wait / vte_token_query (*done = 1) / vte_vstream_sync return
 * the failure's code (VTE_EHIP) with its message and HIP code in vte_last_error() /
 * vte_last_hip_error() of the calling thread.  vte_vstream_sync, having reported a failed
 * tail, empties the tail: later submissions do not inherit the failure.  vte_device_sync
 * returns the first failure that no earlier vte_device_sync has returned.  After a device
 * fault HIP itself stays in error: expect every later launch of the process to fail.
 * A waiting call sleeps while what it waits for is still queued; once all of it has been handed to
 * the device the calling thread polls instead (for 20 ms at most per call, then it sleeps again):
 * the completion of a short launch is then seen a wake-up sooner, at the price of a busy core. */
int vte_token_query(vte_ctx* ctx, vte_token token, int* done);
int vte_token_wait(vte_ctx* ctx, vte_token token);
int vte_vstream_sync(vte_vstream* vs); /* waits on the stream tail */
int vte_device_sync(vte_ctx* ctx);     /* waits on every vstream tail and explicit launch */

/* ---- lease control used by policies (Sec. 4.3) -------------------------------- */
/* LEASED -> DRAINING: outstanding work continues, nothing new is admitted; at
 * zero outstanding the pCtx becomes IDLE (or RESERVED if a reservation waits). */
int vte_pctx_close_gate(vte_ctx* ctx, int pctx_id);
/* Holds the pCtx for `vs`: excluded, with every overlapping pCtx, from all other
 * leases.  If overlapping work is still running the reservation is pending and
 * takes effect when it has drained (VTE_OK either way; VTE_EBUSY if another
 * vstream already holds or awaits a reservation that overlaps). */
int vte_pctx_reserve(vte_ctx* ctx, int pctx_id, vte_vstream* vs);
int vte_pctx_unreserve(vte_ctx* ctx, int pctx_id);

/* ---- policy interface (Sec. 4.5) ------------------------------------------------ */
typedef struct vte_ready_op {
  vte_token token;
  int vstream;          /* id, -1 for explicit launches */
  int klass;            /* VTE_CLASS_* */
  int pinned_pctx;      /* -1 if the vstream is not pinned */
  uint64_t age;         /* submission sequence number (smaller = older) */
  int pred_pctx;        /* PIPELINED: pCtx of an unfinished predecessor, else -1 */
  vte_desc_view desc;
} vte_ready_op;

typedef struct vte_pool_view {     /* S: states, leases, reservations, gates */
  int count;
  const vte_pctx_info* pctx;       /* valid during the callback only */
  int ready_by_class[2];           /* ready ops per class */
  int inflight_by_class[2];        /* submitted, unfinished ops per class */
} vte_pool_view;

typedef struct vte_hint {          /* lookahead hint h */
  int vstream;                     /* who will need the resources */
  int want_width;                  /* CUs wanted */
  double ready_in_s;               /* expected time until the op is ready */
  double deadline_in_s;            /* <= 0: none */
} vte_hint;

typedef struct vte_prepare_plan {  /* R */
  int target_pctx;                 /* -1: nothing to do */
  int reserve;                     /* 1: reserve target for the hint's vstream */
  int n_close;                     /* gates to close (only pCtxs overlapping target are accepted) */
  int close[32];
} vte_prepare_plan;

typedef struct vte_policy_vtbl {
  /* Pick(Q,S): index into ready[0..n) or -1 to defer. */
  int (*pick)(void* user, const vte_ready_op* ready, int n, const vte_pool_view* S);
  /* Select(o,E,S): one id out of eligible[0..n) or -1 to leave o ready. */
  int (*select)(void* user, const vte_ready_op* op, const int* eligible, int n,
                const vte_pool_view* S);
  /* Prepare(h,S): fills *plan; may be NULL. */
  int (*prepare)(void* user, const vte_hint* hint, const vte_pool_view* S, vte_prepare_plan* plan);
} vte_policy_vtbl;

/* Installs callbacks (called on the dispatcher thread with the runtime lock
 * held: they must not call back into the library).  NULL restores the default. */
int vte_set_policy(vte_ctx* ctx, const vte_policy_vtbl* vtbl, void* user);

/* Built-in policies.
 *  WIDEST      oldest ready op first; the widest eligible pCtx (pinned pCtx if pinned).
 *  QUEUE_STATE launch-granular sharing from the instantaneous queue state and the
 *              width profiles.  A LATENCY op is placed by the profiled time of its
 *              recurring chain (the sum over the distinct descriptors its vstream
 *              submitted lately): it stays on its predecessor's pCtx while that is
 *              within `slack` of the best candidate, else takes the fastest pCtx
 *              when no BEST_EFFORT work is ready or in flight and the narrowest
 *              within `slack` when there is.  A BEST_EFFORT op takes the widest
 *              pCtx that leaves `keep_free_cus` CUs unclaimed while LATENCY ops are
 *              ready or in flight, and the widest of all otherwise.  In both
 *              classes an op stays ready, rather than settling for less, when the
 *              pCtx it should get is blocked only by leases of its own vstream. */
enum { VTE_POLICY_WIDEST = 0, VTE_POLICY_QUEUE_STATE = 1, VTE_POLICY_TPUT_PLAN = 2, VTE_POLICY_TPOT_FIRST = 3 };
/*  TPUT_PLAN   the Throughput-Oriented policy (Sec. 5, Algorithm 1): every round plans
 *              all ready ops together.  MinBind gives as many of them as possible, in
 *              age order (one head per vstream), a minimum-size pCtx that overlaps no
 *              other assignment; then the feasible expansion with the largest marginal
 *              gain G_o(p,p') = (P_o(m(p')) - P_o(m(p))) / (m(p') - m(p)),
 *              P_o(m) = T^_o(m_min) / T^_o(m), is applied until none is positive.  An op
 *              without a profile counts as scaling perfectly.  Pick returns the next
 *              planned op, Select returns A[o]; an op planned onto a pCtx that only
 *              leases of its own vstream block stays ready until they drain.  `slack`
 *              and `keep_free_cus` are unused.
 *  TPOT_FIRST  TPUT_PLAN for everything except vstreams with a TPOT target
 *              (vte_vstream_set_tpot).  Each of those gets an exclusive standing pCtx
 *              once the ops of one token have been submitted (they define its chain):
 *              the narrowest node whose profiled token time times (1 + slack) meets the
 *              target (the whole device if none does), lowest pool ids first; a stream
 *              idle for two target periods gives it back until its next submission.  The next-token deadline is the
 *              previous token's completion plus the target; completion is predicted
 *              from the profiles of the ops in flight and queued, scaled by a running
 *              average of how much slower than its solo profile the stream's last tokens
 *              ran (sharing HBM and caches with co-tenants).  When the token is
 *              at risk on the standing pCtx, Prepare closes the gates of overlapping
 *              leases of other vstreams and reserves the smallest wider pCtx predicted
 *              to meet the deadline (the widest if none is); Pick takes at-risk decodes
 *              by earliest deadline and Select binds them to the prepared pCtx, or to
 *              the standing one while preparation is incomplete.  The wider pCtx is
 *              given back at a token boundary once the standing one suffices. */
int vte_set_builtin_policy(vte_ctx* ctx, int which, double slack, int keep_free_cus);

/* Declares `vs` a decode stream with a time-per-output-token target: every
 * `ops_per_token` completed ops are one token.  tpot_seconds = 0 removes the target
 * and releases its reservations.  VTE_EBUSY while the vstream has work. */
int vte_vstream_set_tpot(vte_vstream* vs, double tpot_seconds, int ops_per_token);
typedef struct vte_tpot_info {
  double tpot_seconds;
  int ops_per_token;
  int standing_pctx;    /* -1 until profiles exist to size it from */
  int escalated_pctx;   /* wider pCtx currently prepared, or -1 */
  int at_risk;
  uint64_t tokens_done, deadline_misses, escalations;
} vte_tpot_info;
int vte_vstream_tpot_info(vte_vstream* vs, vte_tpot_info* out);

/* Gives the policy a lookahead hint; the plan it returns is validated and
 * applied (gates closed, reservation placed or left pending). */
int vte_hint_submit(vte_ctx* ctx, const vte_hint* hint);

/* ---- width profiles T^_o(m) (Sec. 5, "Performance Profiles") ----------------- */
/* Times `desc` alone on one pCtx of every width the pool exposes (warmup + reps
 * launches each, device events) and stores seconds per launch under the
 * descriptor's profile_key.  Must be called while nothing else is in flight. */
int vte_profile_measure(vte_ctx* ctx, const vte_desc* desc, int warmup, int reps);
/* Times `desc` on one pCtx only; *seconds = device time per launch.  Same conditions. */
int vte_profile_measure_on(vte_ctx* ctx, const vte_desc* desc, int pctx_id, int warmup, int reps,
                           double* seconds);
/* Stores a profile entry by hand (seconds > 0, width > 0: CUs; VTE_EINVAL otherwise). */
int vte_profile_set(vte_ctx* ctx, uint64_t profile_key, int width, double seconds);
/* VTE_EINVAL if no profile exists for (key,width). */
int vte_profile_get(vte_ctx* ctx, uint64_t profile_key, int width, double* seconds);

/* ---- statistics ------------------------------------------------------------------ */
typedef struct vte_op_record {
  vte_token token;
  int vstream, klass, kernel, pctx, width;
  double t_submit;   /* host seconds since vte_init: op handed to the library */
  double t_ready;    /* predecessors satisfied (STRICT) or bindable (PIPELINED) */
  double t_bound;    /* descriptor submitted to the backend stream */
  double t_done;     /* completion observed by the dispatcher */
  double gpu_seconds; /* device time of the launch (event pair on its stream), or -1 */
  double gpu_begin;   /* timed launches: begin and end of the kernel on the device clock, seconds since
                         vte_init (float32 milliseconds inside: about 1 us of resolution per 8 s); else -1 */
  double gpu_end;
} vte_op_record;
typedef struct vte_stats_t {
  uint64_t submitted, completed, leases_opened, leases_reused, lease_conflicts,
      stale_proposals, submit_failures, gates_closed, reservations,
      completion_records, /* stream markers made to observe completions (PIPELINED: far fewer than launches) */
      failed;             /* operations retired as failed (device error behind their completion, a submission
                             that kept failing, a predecessor that failed) */
} vte_stats_t;
/* Copies the counters since vte_init or the last vte_stats_reset. */
int vte_stats(vte_ctx* ctx, vte_stats_t* out);
/* Copies up to `cap` most recent completed-op records, oldest first; *n_out = count. */
int vte_stats_read(vte_ctx* ctx, vte_op_record* dst, int cap, int* n_out);
/* Zeroes the counters and empties the record ring; launches in flight are still recorded. */
int vte_stats_reset(vte_ctx* ctx);
/* Changes which launches carry device timing events from now on (vte_pool_cfg.device_timing_mask and
 * device_timing_stride; same meaning, same limits; the per-kernel sampling counters restart).
 * Launches already submitted keep what they have.  VTE_EINVAL for a negative stride. */
int vte_set_device_timing(vte_ctx* ctx, unsigned mask, int stride);

/* ---- fake backend hooks (VTE_BACKEND_FAKE only; VTE_ESTATE otherwise) ---------- */
/* With the fake backend a submitted op stays in flight until completed here. */
int vte_fake_complete(vte_ctx* ctx, vte_token token);
/* Completes the op as vte_fake_complete does, with its completion reporting a device error. */
int vte_fake_complete_error(vte_ctx* ctx, vte_token token);
int vte_fake_set_autocomplete(vte_ctx* ctx, int on); /* 1: ops complete as soon as submitted */
int vte_fake_fail_next_submits(vte_ctx* ctx, int n); /* next n backend submissions fail */
typedef struct vte_fake_log_entry {
  vte_token token;
  int pctx;
  uint64_t desc_hash;  /* hash of the descriptor bytes as seen by the backend */
  int waited_on_pctx;  /* device-side wait inserted on this pCtx's stream, or -1 */
} vte_fake_log_entry;
/* Copies up to `cap` entries of what the fake backend was handed, in submission order. */
int vte_fake_log(vte_ctx* ctx, vte_fake_log_entry* dst, int cap, int* n_out);

/* Blocks until the dispatcher has nothing left to do without outside input
 * (no ready op it could bind, no unobserved completion).  For tests. */
int vte_dispatcher_quiesce(vte_ctx* ctx);

/* ---- for callers that cannot allocate ---------------------------------------------------- */
/* For code that may not call hipMalloc where it stands: a stream under HIP graph capture, a
 * tight serving loop, a harness that forbids allocation.  vte_lmhead_argmax_static is
 * vte_desc_lmhead_argmax (default plan) + vte_desc_argmax_finish as one call that enqueues three
 * launches on `hip_stream` (a hipStream_t of the calling thread's current device; NULL = the
 * null stream) and returns without waiting: tok[b] and, if given, logits[b,:] are valid once
 * the stream has passed them, and hold the same bits as the descriptor pair's.  It needs no
 * vte_ctx, builds no descriptor and calls no allocating routine: the per-workgroup candidates
 * live in an array of vte_static_scratch_bytes() (1 MiB) inside the library's device image,
 * one copy per GPU, held until the process ends, its address looked up once per device (at
 * vte_init on that device, else on the first call there).
 * W: device [V,K] bf16; H: device [B,K] bf16; tok: device [B] int32; logits_or_null: device
 * [B,V] fp32 or NULL — all owned by the caller.  Same limits as vte_desc_lmhead_argmax.
 * VTE_EINVAL if the shape's candidates do not fit the array (the message gives both sizes;
 * every vocabulary up to 262144 rows fits at every batch), VTE_EHIP if a launch fails.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents
 * (what must start at zero is cleared by a fill launch in front, on the same stream): calls
 * that overlap in time on one GPU — different streams without an edge between them — race. */
int vte_static_scratch_bytes(size_t* bytes);
int vte_lmhead_argmax_static(void* hip_stream, const void* W, const void* H, int32_t* tok,
                             float* logits_or_null, int B, int V, int K);

/* ---- device utilities -------------------------------------------------------------- */
/* Host seconds since vte_init on the library's clock (the one the records use). */
int vte_now(vte_ctx* ctx, double* seconds);

#ifdef __cplusplus
}
#endif
#endif /* VTE_H_ */
