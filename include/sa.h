/*
 * sa.h - C ABI of the MI355X (gfx950) dynamic sparse prefill attention library.
 *
 * One attention layer, batch 1, causal.  Per query head the library
 *   1. scores a window of the last queries against all keys
 *      (sa_estimate_patterns),
 *   2. decides which sparsity pattern the head follows and selects its
 *      columns, diagonals and blocks (sa_build_index),
 *   3. runs causal softmax attention over the selected entries only
 *      (sa_sparse_prefill).
 * Beside this path: steps 1 and 2 as one call (sa_estimate_and_index), one
 * decode step over the same index (sa_sparse_decode) and the offline per-head
 * pattern search (sa_search_patterns).
 *
 * Conventions
 *   - C99 types only.  Q, K, V, O are DEVICE pointers to raw bf16 (16-bit)
 *     elements; O is written with round-to-nearest-even.
 *   - The caller owns every device buffer (Q, K, V, O, scores, index,
 *     workspace).  Sizes come from the *_bytes queries.  The library never
 *     allocates or frees device memory and the compute calls never synchronise
 *     the host: they enqueue kernels on the given HIP stream and return.  The
 *     offline search is the exception on the host side: the host steers it, so
 *     it waits for the stream after every probe and creates and frees small
 *     host-memory contexts on the way (still no device memory), see there.
 *     sa_estimate_patterns (and sa_estimate_and_index) runs part of its kernels on a side stream that the
 *     context owns (created by sa_create, default priority); that stream waits
 *     for the given stream at entry and the given stream waits for it at exit,
 *     so work enqueued on the given stream before and after the call is
 *     ordered with all of it.
 *   - Errors are return codes.  Argument checks are synchronous;
 *     SA_ERR_HIP wraps a failed launch; sa_last_error gives a text.
 *     Unsupported shapes are rejected, nothing is silently padded.
 *   - Index arrays are plain int32 and canonical (ascending, -1 padded): two
 *     index sets are equal iff their bytes are equal.  Same inputs give the
 *     same bytes, run to run.
 *   - A context serialises nothing: do not run two calls on one context
 *     concurrently (they share its workspace).
 */
#ifndef SA_H_
#define SA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sa_ctx sa_ctx; /* opaque, host memory */

typedef enum {
  SA_OK = 0,
  SA_ERR_INVALID_ARG = 1,
  SA_ERR_UNSUPPORTED = 2,
  SA_ERR_BUFFER_TOO_SMALL = 3,
  SA_ERR_HIP = 4
} sa_status;

/* The three patterns named in the paper's contributions list. */
typedef enum {
  SA_PATTERN_AUTO = -1,
  SA_TRIANGULAR = 0,     /* sink key blocks + local band (static) */
  SA_INTERVAL_SLASH = 1, /* top vertical columns + top diagonals (Alg. 2) */
  SA_BLOCK_CLUSTER = 2   /* top blocks of the block-mean map (Alg. 3) */
} sa_pattern;

/* How a Block-Cluster head spends k_blocks (Alg. 3 TopKBlocks names one k_b and
 * does not say whether it is per sequence or per query block):
 *   SA_BLOCKS_GLOBAL   one top-k over all causal blocks of the head (the literal reading);
 *   SA_BLOCKS_PER_ROW  row block R keeps min(R+1, ceil(k_blocks (R+1) / (nb (nb+1)/2))) blocks:
 *                      its diagonal block and its best lower blocks, ties to the lower block id,
 *                      i.e. the same fraction of every row (at most nb blocks above k_blocks);
 *   SA_BLOCKS_GLOBAL_ROW_NORMALISED  one top-k like SA_BLOCKS_GLOBAL, on the key blk[R][C] * (R+1)
 *                      (one fp32 multiplication): an entry is measured against the uniform value
 *                      1/(R+1) of its own softmax row, so short early rows no longer win by construction. */
typedef enum { SA_BLOCKS_GLOBAL = 0, SA_BLOCKS_PER_ROW = 1, SA_BLOCKS_GLOBAL_ROW_NORMALISED = 2 } sa_block_select;

/* Granularity of the selected diagonals of an Interval-Slash head (Alg. 2 combines vertical and
 * slash indices but does not say at which granularity the kernel applies them):
 *   SA_DIAGONALS_EXACT   query i attends key i - o for every selected offset o (element-exact);
 *   SA_DIAGONALS_BLOCKS  every block pair (i / block, (i - o) / block) is kept whole: the offsets
 *                        become part of the block CSR (at most two key blocks per offset and row
 *                        block) and the offs list of the index comes back empty (n_offs = 0). */
typedef enum { SA_DIAGONALS_EXACT = 0, SA_DIAGONALS_BLOCKS = 1 } sa_diagonal_select;

typedef struct {
  int32_t n_q_heads, n_kv_heads, head_dim; /* n_q_heads % n_kv_heads == 0, <= 128 heads; head_dim must be 128 */
  int32_t seq_len, block, last_q;          /* seq_len % block == 0; block in {64,128}; 1 <= last_q <= 64 */
  float softmax_scale;                     /* 0 => 1/sqrt(head_dim) */
  int32_t sink_blocks, local_blocks;       /* Triangular: key blocks [0,sink) and the band R-C < local */
  int32_t k_vertical, k_slash, k_blocks;   /* Alg. 2 k_v, k_s; Alg. 3 k_b (includes the forced diagonal blocks) */
  int32_t probe_v, probe_s, lift_num, lift_den; /* pattern rule; 0 => defaults 4,4,4,1 */
  int64_t q_head_stride, q_row_stride;     /* in elements; 0 => contiguous [H][N][d]; O uses Q's strides */
  int64_t kv_head_stride, kv_row_stride;   /* K and V; row strides must be multiples of 8 elements */
  int32_t block_select;                    /* sa_block_select; 0 => SA_BLOCKS_GLOBAL */
  int32_t diagonal_select;                 /* sa_diagonal_select; 0 => SA_DIAGONALS_EXACT */
  int32_t lazy_block_map;                  /* 0 or 1; 1: sa_estimate_and_index computes the block map (Alg. 3) only
                                            * for the heads that turn out Block-Cluster; see that call */
} sa_config;

/* Device score buffers written by sa_estimate_patterns (Alg. 2 SumRows /
 * SumDiagonals on the last-query window; Alg. 3 blocked attention map):
 *   v   [n_q_heads][seq_len]   fp32  vertical score of key column j
 *   s   [n_q_heads][seq_len]   fp32  slash score of diagonal offset o = i - j
 *   blk [n_q_heads][nb][nb]    fp32  block map, nb = seq_len/block, entries C > R are 0 */
typedef struct { float *v, *s, *blk; } sa_scores;

/* Device index buffers written by sa_build_index, read by sa_sparse_prefill:
 *   pattern [H]            chosen sa_pattern
 *   n_cols  [H]            number of selected key columns
 *   cols    [H][k_vertical] strictly ascending (no repeats), -1 padded
 *   n_offs  [H]            number of selected diagonal offsets
 *   offs    [H][k_slash]   strictly ascending (no repeats), -1 padded
 *   rowptr  [H][nb+1]      block CSR row pointers
 *   blkcols [H][cap]       key-block ids, ascending within a row, -1 padded;
 *                          cap = sizes[6]/(4*H) from sa_index_bytes
 * A query i attends key j <= i iff (i/block, j/block) is in the CSR, or j is
 * in cols, or i-j is in offs (a union: each key counted once). */
typedef struct { int32_t *pattern, *n_cols, *cols, *n_offs, *offs, *rowptr, *blkcols; } sa_index;

/* Fill sink_blocks, local_blocks, k_vertical, k_slash, k_blocks from a keep
 * fraction of the causal blocks (0 < keep <= 1).  seq_len and block must be
 * set.  The paper leaves these budgets as inputs of Alg. 2 / Alg. 3. */
sa_status sa_default_budgets(sa_config *cfg, double keep_fraction);

/* Validate cfg and create a context (host memory only). */
sa_status sa_create(const sa_config *cfg, sa_ctx **out);
void sa_destroy(sa_ctx *ctx);

/* Byte sizes of the three score buffers {v, s, blk}. */
sa_status sa_scores_bytes(const sa_ctx *ctx, size_t v_s_blk[3]);
/* Byte sizes of the seven index buffers, in sa_index member order. */
sa_status sa_index_bytes(const sa_ctx *ctx, size_t sizes[7]);
/* Device workspace the compute calls need; attach it before the first call.
 * The pointer must be 256-byte aligned and stays owned by the caller. */
sa_status sa_workspace_bytes(const sa_ctx *ctx, size_t *bytes);
sa_status sa_set_workspace(sa_ctx *ctx, void *dev, size_t bytes);

/* Alg. 2 "Compute Dense Attention Scores" + SumRows / SumDiagonals restricted
 * to the last last_q query rows, and Alg. 3 "Compute Blocked Representation".
 * Q [Hq][N][d], K [Hkv][N][d] bf16 device.  Writes all of out.v, out.s, out.blk. */
sa_status sa_estimate_patterns(sa_ctx *ctx, const void *Q, const void *K, sa_scores out,
                               void *hip_stream);

/* Per-head pattern choice (Main Idea, "Categorization of Attention Heads") and
 * Alg. 2 TopK / CombineIndices, Alg. 3 TopKBlocks.  Integer-exact: scores are
 * compared by their fp32 bit patterns, ties go to the lower index.
 * pattern_override_host: HOST array of n_q_heads sa_pattern values
 * (SA_PATTERN_AUTO = decide), or NULL for all-auto.  Writes all of `out`.
 * The scores must be what sa_estimate_patterns writes: finite and >= +0 (sign
 * bit clear).  Other values are selected among in an unspecified order; no
 * access leaves the buffers. */
sa_status sa_build_index(sa_ctx *ctx, sa_scores in, const int32_t *pattern_override_host,
                         sa_index out, void *hip_stream);

/* sa_estimate_patterns followed by sa_build_index as one call: same score
 * buffers, same index, byte for byte (Alg. 2 l.1-7 on the last-query window,
 * Alg. 3 l.1-6, and the categorisation of the heads).  The two are interleaved
 * on the caller's stream and the context's side stream: the selections on v
 * and s run while the block map is still being computed, and the block
 * selection runs beside them.  Towards the caller it behaves like a sequence
 * of kernels on `stream`.  Arguments as in the two calls; errors likewise.
 * With cfg.lazy_block_map = 1 the call follows the order of the categorisation
 * instead (the blocked representation of Alg. 3 belongs to the Block-Cluster
 * branch only): window passes, selections on v and s, pattern decision, and
 * then block means, block map and block selection for the Block-Cluster heads
 * alone, all on `stream`.  The index is the same, byte for byte; scores.blk of
 * the other heads is not written (it keeps what it held), and Q is read for
 * the Block-Cluster heads only. */
sa_status sa_estimate_and_index(sa_ctx *ctx, const void *Q, const void *K, sa_scores scores,
                                const int32_t *pattern_override_host, sa_index index, void *hip_stream);

/* Alg. 2 / Alg. 3 "Compute Sparse Attention": O[h][i] = sum over the kept
 * keys j of softmax_j(scale * Q_h[i].K[j]) V[j].  Q, O [Hq][N][d]; K, V
 * [Hkv][N][d] bf16 device.  Any index in the documented layout is accepted,
 * not only one produced by sa_build_index; a query that keeps no key (its row
 * block lists no block that reaches it, and no column or offset applies) gets
 * a row of zeros. */
sa_status sa_sparse_prefill(sa_ctx *ctx, const void *Q, const void *K, const void *V,
                            sa_index idx, void *O, void *hip_stream);

/* Same computation and output as sa_sparse_prefill, plus work accounting for
 * the FLOP figures of a benchmark: adds to counters_dev[0] the number of
 * 32-query x 32-key sub-tiles the kernel multiplied (a 64-key tile of one wave
 * counts 2, a selected diagonal of one wave counts 1; 4*head_dim*32*32 FLOP
 * each) and to counters_dev[1] the number of kept (query, key) pairs, |M| of the sparse
 * softmax of Alg. 2 / Alg. 3.  counters_dev: DEVICE uint64[2], zeroed by the
 * caller.  A benchmark times sa_sparse_prefill, not this variant. */
sa_status sa_sparse_prefill_counted(sa_ctx *ctx, const void *Q, const void *K, const void *V,
                                    sa_index idx, void *O, uint64_t *counters_dev,
                                    void *hip_stream);

/* One decode step over the prefill index (Abstract / Introduction: gains "in the decoding phase";
 * Proposed Method: decode queries are [B, 1, H]; the paper gives no method, this is a reading).
 * The prompt of seq_len = N tokens was prefilled with idx.  The query at position pos >= N attends,
 * per query head, the union of: the generated keys N..pos (itself included), the selected columns,
 * the keys pos - o of the selected diagonal offsets o, and the keys of the key blocks idx keeps for
 * the last row block of the prompt - each key once - with the prefill's scaled softmax.
 * q, o [Hq][128] bf16 device, contiguous; K, V as in the prefill (same strides) but holding rows
 * 0..pos, so kv_head_stride must leave room for them; pos < N + 2^20.  Uses ctx's workspace. */
sa_status sa_sparse_decode(sa_ctx *ctx, const void *q, const void *K, const void *V, sa_index idx,
                           int64_t pos, void *o, void *hip_stream);

/* sa_sparse_decode for callers that cannot allocate device memory or attach a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same
 * kernels, same output bytes, but the partial results of the step live in a static device array
 * inside the library (270336 bytes per GPU, held until the process ends) instead of ctx's
 * workspace, which need not be attached.  The call allocates and frees nothing.  Limit: n_q_heads
 * times the split count the library picks must not exceed 512 partial results (every context
 * sa_create accepts today fits; a larger one gets SA_ERR_UNSUPPORTED).  All calls on one GPU - from
 * any context or thread - share that array: calls that overlap in time on one GPU race, so keep
 * them on one stream or order them with events.  Nothing in the array needs clearing between calls
 * (every slot a call reads it has written first). */
sa_status sa_sparse_decode_static(sa_ctx *ctx, const void *q, const void *K, const void *V, sa_index idx,
                                  int64_t pos, void *o, void *hip_stream);

/* Offline pattern search, "Kernel-Aware Sparse Pattern Search Algorithm" (Alg. 1), one head at a
 * time.  Candidates: the three patterns, each with one integer size (its search space):
 *   SA_TRIANGULAR      local_blocks = x,                       1 <= x <= nb
 *   SA_INTERVAL_SLASH  k_slash = x, k_vertical = min(N, 32 x), 1 <= x <= max(1, N/32)
 *   SA_BLOCK_CLUSTER   k_blocks = x,                           nb <= x <= nb (nb+1)/2
 * (sink_blocks, block, last_q, scale and strides come from ctx's config).  FLOPs of a candidate =
 * 4 * head_dim * kept (query, key) pairs of the index built from it, so the target and the
 * tolerance are given in pairs.  RefineSearchSpace: bisection on x; it stops at the first probe
 * within eps_pairs of target_pairs, else takes of the two adjacent sizes around the target the
 * closer one (the smaller on a tie).  Evaluate Patterns: Frobenius norm of (sparse output - dense
 * causal output) of the head for every refined candidate; `pattern` is the smallest (ties: lowest
 * id), ready for sa_build_index's pattern_override.
 * Q, K, V, scores: device, as for the other calls (scores from sa_estimate_patterns).  scratch:
 * DEVICE, 256-byte aligned, sa_search_scratch_bytes bytes, owned by the caller.  out_host: HOST
 * array of n_q_heads results, candidates in pattern-id order.  The call runs the index builder and
 * the attention kernel of this library on one-head contexts it creates and destroys, waits for the
 * stream after every probe (do not capture it in a graph) and returns when all results are in
 * out_host.  ctx's own workspace is not used. */
typedef struct {
  int32_t pattern;   /* argmin of err */
  int32_t param[3];  /* refined size x of each candidate */
  int64_t pairs[3];  /* kept (query, key) pairs at that size */
  double err[3];     /* || O_sparse - O_dense ||_F at that size */
} sa_search_head;
sa_status sa_search_scratch_bytes(const sa_ctx *ctx, size_t *bytes);
sa_status sa_search_patterns(sa_ctx *ctx, const void *Q, const void *K, const void *V, sa_scores scores,
                             int64_t target_pairs, int64_t eps_pairs, void *scratch_dev,
                             size_t scratch_bytes, sa_search_head *out_host, void *hip_stream);

const char *sa_last_error(const sa_ctx *ctx);

/* Library version string. */
const char *sa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SA_H_ */
