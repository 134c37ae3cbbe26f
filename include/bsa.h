/*
 * bsa.h -- C ABI of the Bidirectional Sparse Attention (BSA) hot path for AMD MI355X (gfx950).
 *
 * One attention layer of a video diffusion transformer, sparsified in two directions
 * (paper Sec. 3.2): queries that are redundant inside their 3D block are pruned
 * (Sec. 3.2.2, Eq. 2) and every query block attends only to the minimal set of KV blocks
 * whose pooled softmax mass reaches a threshold (Sec. 3.2.3, Eq. 4); exact softmax
 * attention then runs over the survivors (Sec. 3.2.4, Eq. 5) and pruned positions are
 * filled with the output of their window's critical token (Sec. 3.2.2, "Token Filling").
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device unless stated,
 *     16-byte aligned (tensors, workspaces) or 4-byte aligned (index arrays).
 *   - Q, K, V, O, dO, dQ, dK, dV are contiguous [B, H, L, d], L = T*Hs*Ws, in RASTER token
 *     order n = t*Hs*Ws + h*Ws + w (Sec. 3.1) unless shape.layout says block-major;
 *     element type per shape.dtype.
 *   - Blocks: (Ct, Ch, Cw) must divide (T, Hs, Ws) (Sec. 3.2.1).  Bk = Ct*Ch*Cw tokens
 *     per block, N = L / Bk blocks, block id = (bt*Nh + bh)*Nw + bw, intra-block id
 *     = (ct*Ch + ch)*Cw + cw.  "rows" = B*H*N (one row per head and query block).
 *   - Ownership: the caller allocates and frees every buffer, including workspaces.
 *     The library never allocates device memory and keeps no state between calls (the one
 *     built-in scratch buffer, used by bsa_select_kv_static only, carries nothing over).
 *   - Asynchrony: a call only enqueues work on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and returns; it never synchronises, so a sequence
 *     of calls can be recorded into a HIP graph once every kernel has run once eagerly.
 *   - Errors: 0 on success, a negative bsa_status otherwise.  All argument checks are
 *     done on the host before anything is launched; a failed call launches nothing.
 *   - Determinism: equal inputs give bit-identical outputs (no floating-point atomics).
 */
#ifndef BSA_H_
#define BSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum bsa_dtype { BSA_F32 = 0, BSA_BF16 = 1 };

/* Token order of the [B,H,L,d] tensors.  RASTER: n = t*Hs*Ws + h*Ws + w (Sec. 3.1).
 * BLOCK_MAJOR: the one-time reorder of Sec. 3.2.1, tokens of a block adjacent: row
 * i*Bk + c holds intra-block token c of block i.  Both layouts give the same results for
 * the same video, token for token. */
enum bsa_layout { BSA_LAYOUT_RASTER = 0, BSA_LAYOUT_BLOCK_MAJOR = 1 };

enum bsa_status {
  BSA_OK = 0,
  BSA_ERR_NULL = -1,        /* a required pointer is NULL */
  BSA_ERR_SHAPE = -2,       /* non-positive extent, block does not divide grid, unsupported d / Bk / N */
  BSA_ERR_RANGE = -3,       /* threshold or keep ratio outside (0, 1], n_keep outside [1, Bk], sm_scale <= 0 */
  BSA_ERR_CAPACITY = -4,    /* index buffer smaller than the worst case rows*N */
  BSA_ERR_DTYPE = -5,       /* shape.dtype is neither BSA_F32 nor BSA_BF16 */
  BSA_ERR_LAUNCH = -6,      /* the HIP runtime reported a launch error */
  BSA_ERR_WORKSPACE = -7,   /* workspace NULL or smaller than the *_workspace_bytes() figure */
  BSA_ERR_STATIC_LIMIT = -8 /* bsa_select_kv_static: the shape needs more than BSA_STATIC_SELECT_BYTES */
};

typedef struct bsa_shape {
  int32_t B, H;          /* batch, heads */
  int32_t T, Hs, Ws;     /* latent grid (Sec. 3.1) */
  int32_t Ct, Ch, Cw;    /* 3D block shape (Sec. 3.2.1) */
  int32_t d;             /* head dimension, multiple of 8, <= 256 */
  int32_t dtype;         /* enum bsa_dtype of Q/K/V/O and the gradients */
  int32_t Wt, Wh, Ww;    /* window of the critical-token mechanism (Sec. 3.2.2, "Critical Token"):
                            must divide (Ct, Ch, Cw) evenly; 0,0,0 = the whole block, one critical
                            token per block.  Windows are numbered raster-wise over the block's
                            window grid; a window's critical token is its local (Wt/2, Wh/2, Ww/2). */
  int32_t layout;        /* enum bsa_layout of every [B,H,L,d] tensor */
} bsa_shape_t;

/* Limits: Bk <= 256, N <= 8192, d % 8 == 0 and d <= 256. */

const char* bsa_strerror(int status);

/* Number of retained queries per block (Eq. 2): every window keeps ceil(keep_ratio * Wk) of
 * its Wk tokens, so nwin * ceil(keep_ratio * Wk); ceil(keep_ratio * Bk) with one window.
 * <0 on bad arguments. */
int bsa_n_keep(const bsa_shape_t* shape, double keep_ratio);

/*
 * Block-level representations (Sec. 3.2.3): Xbar[b,h,i,:] = arithmetic mean of the Bk
 * token vectors of block i, accumulated in fp64 in ascending intra-block order.
 *   X    in   [B,H,L,d]  shape.dtype
 *   Xbar out  [B,H,N,d]  double
 */
int bsa_pool_blocks(const bsa_shape_t* shape, const void* X, double* Xbar, void* stream);

/*
 * Sparse KV selection (Sec. 3.2.3, Eq. 4).  Block logits s_ij = score_scale * <Qbar_i, Kbar_j>
 * (fp64, channel-ascending, multiply and add rounded separately).  For every row the
 * blocks are ordered by (s descending, j ascending) and the shortest prefix whose
 * softmax mass is >= threshold is kept (threshold >= 1 keeps all N).  Output is CSR:
 *   q2k_ptr  out [rows+1] int32   q2k_ptr[r+1]-q2k_ptr[r] = number of KV blocks of row r
 *                                 (the paper's q2k_num), q2k_ptr[rows] = nnz
 *   q2k_idx  out [nnz]    int32   KV block ids of each row, ascending (the paper's q2k_index)
 *   k2q_ptr / k2q_idx             the exact transpose per head: for row (b,h,j) the query
 *                                 blocks i that list j, ascending.  Both NULL to skip.
 *   nnz_dev  out int64 device scalar (may be NULL)
 *   idx_capacity  number of int32 slots behind q2k_idx (and k2q_idx); must be >= rows*N,
 *                 the data-independent worst case, else BSA_ERR_CAPACITY.
 *   workspace     bsa_select_workspace_bytes(shape) bytes of device scratch.
 * score_scale is normally 1/sqrt(d).
 */
size_t bsa_select_workspace_bytes(const bsa_shape_t* shape);
int bsa_select_kv(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                  double threshold, double score_scale,
                  int32_t* q2k_ptr, int32_t* q2k_idx, int64_t idx_capacity,
                  int32_t* k2q_ptr, int32_t* k2q_idx, int64_t* nnz_dev,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * bsa_select_kv for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * bsa_select_kv, bit for bit, without the workspace: the scratch (block logits, selection bit
 * masks, counts) lives in a buffer of BSA_STATIC_SELECT_BYTES that is part of the library's
 * device image, so every GPU the library runs on holds one copy from load until the process
 * ends.  The call allocates and frees nothing.
 *   - A shape with bsa_select_workspace_bytes(shape) > BSA_STATIC_SELECT_BYTES is refused with
 *     BSA_ERR_STATIC_LIMIT before anything is launched (the 33,280-token, 12-head layer needs
 *     26.4 MB and fits; larger layers use bsa_select_kv with a caller-owned workspace).
 *   - All calls on one GPU share that GPU's buffer.  Nothing in it has to start at zero (every
 *     part is written before it is read within a call), but calls that overlap on one GPU, on
 *     different streams, race on it: keep them on one stream or order them with events.
 */
#define BSA_STATIC_SELECT_BYTES (32u << 20)
int bsa_select_kv_static(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                         double threshold, double score_scale,
                         int32_t* q2k_ptr, int32_t* q2k_idx, int64_t idx_capacity,
                         int32_t* k2q_ptr, int32_t* k2q_idx, int64_t* nnz_dev, void* stream);

/*
 * The same selection behind the statistical dynamic threshold of Sec. 3.2.3, Eq. 3: per row,
 * only the blocks whose logit reaches tau = mean(s_i.) + std(s_i.) * stat_z (std with the
 * n-1 divisor) are candidates, and the minimal prefix of Eq. 4 is cut to them; a row with no
 * candidate keeps its best block.  stat_z is the standard-normal quantile U(1 - k/n) for k
 * desired blocks of n, computed by the caller; -inf disables the filter, NaN is
 * BSA_ERR_RANGE.  The softmax mass of Eq. 4 stays normalised over all N blocks.
 * (The paper's equation leaves U, the divisor and the composition with Eq. 4 open: this is
 * one documented reading.)  All other arguments as bsa_select_kv.
 */
int bsa_select_kv_stat(const bsa_shape_t* shape, const double* Qbar, const double* Kbar,
                       double threshold, double stat_z, double score_scale,
                       int32_t* q2k_ptr, int32_t* q2k_idx, int64_t idx_capacity,
                       int32_t* k2q_ptr, int32_t* k2q_idx, int64_t* nnz_dev,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Sparse Query (Sec. 3.2.2, Eq. 2, and "Critical Token").  Per window of every block (the
 * whole block when shape.Wt/Wh/Ww are 0): cosine similarity (fp64) of every token of the
 * window to the window's critical token, local coordinate (Wt/2, Wh/2, Ww/2); the critical
 * token plus the other ceil(keep_ratio * Wk) - 1 tokens of the window with the smallest
 * cosine are retained (ties: lower intra-block id first; a zero vector has cosine 0).
 * n_keep = nwin * ceil(keep_ratio * Wk): the windows' selections concatenated.
 *   keep_idx out [B,H,N,n_keep] int32  intra-block ids, ascending
 */
int bsa_prune_q(const bsa_shape_t* shape, const void* Q, double keep_ratio,
                int32_t* keep_idx, void* stream);

/*
 * Sparse attention forward with token filling (Eq. 5; Sec. 3.2.2 "Token Filling").
 * Retained queries of block i attend, with exact softmax at scale sm_scale, to all Bk
 * tokens of every KV block listed for row i; a pruned position receives the row of its
 * window's critical token.
 *   O   out [B,H,L,d] shape.dtype,  LSE out [B,H,L] float (natural-log sum-exp, filled too)
 * Every row must list at least one KV block (Eq. 4 always selects one).
 * keep_idx rows must be ascending, distinct, in [0,Bk) and contain every window's critical
 * token (a window whose critical token is missing is left unfilled).
 *   workspace   bsa_fwd_workspace_bytes(shape, n_keep) bytes of device scratch (may be NULL
 *               when that is 0), else BSA_ERR_WORKSPACE.  It holds the partial results of
 *               the query blocks whose KV walk is split over several workgroups to balance a
 *               short launch; contents are undefined afterwards.
 */
size_t bsa_fwd_workspace_bytes(const bsa_shape_t* shape, int n_keep);
int bsa_attn_fwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                 const int32_t* q2k_ptr, const int32_t* q2k_idx,
                 const int32_t* keep_idx, int n_keep, float sm_scale,
                 void* O, float* LSE, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of bsa_attn_fwd with the index sets held constant (Sec. 3.3: the backward
 * kernel reuses the forward's masks and mappings).  The fill copy back-propagates into
 * the center row.  dQ rows of pruned queries and dK/dV of never-listed blocks are zero.
 * dK/dV of a KV block are accumulated by one owner over its k2q list: no atomics.
 *   O, LSE: the forward's outputs;  dO in [B,H,L,d];  dQ, dK, dV out [B,H,L,d]
 *   workspace: bsa_bwd_workspace_bytes(shape, n_keep) bytes of device scratch.
 */
size_t bsa_bwd_workspace_bytes(const bsa_shape_t* shape, int n_keep);
int bsa_attn_bwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                 const void* O, const float* LSE, const void* dO,
                 const int32_t* q2k_ptr, const int32_t* q2k_idx,
                 const int32_t* k2q_ptr, const int32_t* k2q_idx,
                 const int32_t* keep_idx, int n_keep, float sm_scale,
                 void* dQ, void* dK, void* dV,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same backward, restricted to a subset of its three kernels, so that a profiler or
 * benchmark can time each one between its own pair of events: BSA_BWD_PRE gathers the
 * retained rows and forms delta, BSA_BWD_DQ and BSA_BWD_DKV read what PRE left in the
 * workspace.  bsa_attn_bwd() is stages = BSA_BWD_PRE | BSA_BWD_DQ | BSA_BWD_DKV, in that order.
 */
enum bsa_bwd_stage { BSA_BWD_PRE = 1, BSA_BWD_DQ = 2, BSA_BWD_DKV = 4 };
int bsa_attn_bwd_stages(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                        const void* O, const float* LSE, const void* dO,
                        const int32_t* q2k_ptr, const int32_t* q2k_idx,
                        const int32_t* k2q_ptr, const int32_t* k2q_idx,
                        const int32_t* keep_idx, int n_keep, float sm_scale,
                        void* dQ, void* dK, void* dV,
                        void* workspace, size_t workspace_bytes, unsigned stages, void* stream);

/*
 * Full (dense) softmax attention of Eq. 1 at the same shape, forward and backward: the
 * baseline the sparse path is timed against.  Same layouts; the block fields of `shape`
 * only fix the tile granularity (Bk) and must still divide the grid.
 */
size_t bsa_dense_bwd_workspace_bytes(const bsa_shape_t* shape);
int bsa_dense_attn_fwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                       float sm_scale, void* O, float* LSE, void* stream);
int bsa_dense_attn_bwd(const bsa_shape_t* shape, const void* Q, const void* K, const void* V,
                       const void* O, const float* LSE, const void* dO, float sm_scale,
                       void* dQ, void* dK, void* dV,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid, not a step of the method: launches `workgroups` workgroups of four
 * wavefronts that each run `iters` rounds of four independent 32 x 32 x 16 bf16 matrix-core
 * products with operands and accumulators held in registers, and returns the number of
 * floating-point operations the launch performs (negative: an error code).  Timed by the
 * caller, it gives the matrix-core rate this GPU sustains with no memory traffic at all: the
 * second denominator (beside the published peak) for the attention kernels' achieved rates.
 * `sink` is a device array of workgroups * 256 floats that receives one value per thread.
 */
int64_t bsa_mfma_probe(int workgroups, int iters, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BSA_H_ */
