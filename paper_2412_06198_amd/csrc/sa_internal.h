// Internal declarations shared by the host API and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sa.h"

namespace sa {

constexpr int kHeadDim = 128;
constexpr int kMaxHeads = 128;
constexpr int kWin = 64;          // rows of the last-query window the estimator tiles for
constexpr int kMaxSeq = 262144;   // key-tile bitmaps of the attention kernel cover this many keys

struct Override { int8_t pat[kMaxHeads]; };

// Everything the kernels need, resolved from sa_config at sa_create time.
struct Shape {
  int Hq, Hkv, g, N, b, nb, w;
  int k_v, k_s, k_b, cap_b, sink, local;
  int probe_v, probe_s, lift_num, lift_den;
  int row_select;                 // Block-Cluster heads: 1 = every row keeps its own share of k_b
  int row_norm;                   // Block-Cluster heads: 1 = global top-k on blk[R][C] * (R + 1)
  int diag_blocks;                // Interval-Slash heads: 1 = selected diagonals kept as whole blocks
  int lazy_blk;                   // one-call form: 1 = block map only for the heads decided Block-Cluster
  int chunk, nchunks;             // keys per estimator workgroup (window passes), ceil(N / chunk)
  int n_cu;                       // compute units of the device the context was created on
  int64_t q_hs, q_rs, kv_hs, kv_rs;
  float scale;
};

struct Workspace {
  float *qblk, *kblk;             // [Hq][ceil(nb/16)] and [Hkv][ceil(nb/16)] tiles (8 KB) of block means
  float2 *part;                   // [Hq][nchunks][64] partial (max, sum) of the window rows
  float2 *stats;                  // [Hq][64] (max * scale*log2e, 1/sum)
  uint32_t *colbits;              // [Hq][N/32] membership bitmap of the selected columns
  int32_t *colprefix;             // [Hq][N/32] number of selected columns before each word of colbits
  float *dec_part;                // [Hq][splits][132] partial (max, sum, output) of the decode step
  unsigned int *queue;            // [8] work-queue heads of the attention kernel
  void *idx;                      // per-head scratch of the index builder
  uint16_t *kg, *vg;              // [Hq][roundup64(k_v)][kv_rs] gathered K / V rows of the selected columns
  int32_t *hperm;                 // [Hkv][g + 1] order of a KV head's query heads in the attention kernel's queues
};

size_t index_scratch_bytes(int n_heads);

// Side stream of a context with the events that fork it from and join it back into the caller's
// stream inside one call (the estimator runs its Q chain beside its K chain).  aux == nullptr:
// everything is enqueued on the caller's stream.
struct Fork { hipStream_t aux; hipEvent_t fork, mid, join; };

// Parts of the index builder when it runs interleaved with the estimator.
enum class IndexStage { Zero, ColumnsDiagonals, Decide, Blocks, Emit };

// Which of the estimator's two chains a call enqueues.
enum class EstimatePart { Both, KChain, QChain };

}  // namespace sa

// The context behind the opaque handle of the C ABI (host memory).
struct sa_ctx {
  sa_config cfg;
  sa::Shape sh;
  sa::Workspace ws;
  sa::Fork fork;
  bool have_ws;
  size_t ws_bytes;
  size_t off[12];
  char err[256];
};

namespace sa {

// sa_create, optionally without the estimator's side stream and its events
sa_status create_context(const sa_config *cfg, sa_ctx **out, bool side_stream);

hipError_t launch_estimate(const Shape &sh, const Workspace &ws, const uint16_t *Q,
                           const uint16_t *K, sa_scores out, hipStream_t st, const Fork &fk,
                           bool join_back = true);
// One chain alone on st.  QChain needs the K block means that KChain leaves in the workspace;
// only_block_cluster (device, [Hq] patterns, or nullptr = every head) restricts it to the heads
// whose entry is SA_BLOCK_CLUSTER.
hipError_t launch_estimate_part(const Shape &sh, const Workspace &ws, const uint16_t *Q, const uint16_t *K,
                                sa_scores out, EstimatePart part, const int32_t *only_block_cluster,
                                hipStream_t st);
hipError_t launch_build_index(const Shape &sh, const Workspace &ws, sa_scores in,
                              const Override &ov, sa_index out, hipStream_t st);
// lazy: the block-map part of the work is done only for the heads whose out.pattern (written by
// the Decide stage) is SA_BLOCK_CLUSTER.
hipError_t launch_index_stage(const Shape &sh, const Workspace &ws, sa_scores in, const Override &ov,
                              sa_index out, IndexStage stage, hipStream_t st, bool lazy = false);
size_t decode_partial_bytes(const Shape &sh);
// partials: decode_partial_bytes(sh) bytes of device memory (the context's workspace, or the static array)
hipError_t launch_sparse_decode(const Shape &sh, float *partials, const uint16_t *q, const uint16_t *K,
                                const uint16_t *V, sa_index idx, int pos, uint16_t *o, hipStream_t st);
size_t decode_static_bytes();                       // size of the library's static decode scratch
hipError_t decode_static_scratch(float **out);      // its address on the current device
hipError_t launch_sparse_prefill(const Shape &sh, const Workspace &ws, const uint16_t *Q,
                                 const uint16_t *K, const uint16_t *V, sa_index idx, uint16_t *O,
                                 unsigned long long *counters, hipStream_t st);

}  // namespace sa
