// Offline pattern search (Kernel-Aware Sparse Pattern Search Algorithm, Alg. 1), head by head:
//   Initialize Search Space - each candidate pattern has one integer size (Triangular: band
//     blocks; Interval-Slash: diagonals, with 32 columns per diagonal; Block-Cluster: blocks);
//     RefineSearchSpace is a bisection on it until the kept (query, key) pairs - FLOPs / (4 d) -
//     meet the target within the tolerance, or the two sizes around the target are adjacent;
//   Evaluate Patterns - the head's dense causal output against the sparse output of every
//     refined candidate, Frobenius norm of the difference, smallest wins (ties: lowest id).
// Every evaluation runs the library's own index builder and attention kernel on a one-head
// context, so the cost that is matched is the cost of these kernels' masks; the host only steers.
#include <cmath>
#include <cstdio>
#include <cstring>

#include "sa_internal.h"

namespace {

constexpr int kNormBlocks = 1024;

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// partial[blockIdx.x] = sum over the block's rows of (A - B)^2, A and B [N][128] bf16 with row
// stride rs (elements); fp64 accumulation, fixed order: bit-reproducible.
__global__ __launch_bounds__(256) void sq_diff_kernel(const uint16_t *__restrict__ A,
                                                      const uint16_t *__restrict__ B, int N, int64_t rs,
                                                      double *__restrict__ partial) {
  __shared__ double red[256];
  const int cc = threadIdx.x & 15, rg = threadIdx.x >> 4;
  double acc = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * 16 + rg; i < N; i += (int64_t)gridDim.x * 16) {
    const uint4 a = *(const uint4 *)(A + i * rs + cc * 8), b = *(const uint4 *)(B + i * rs + cc * 8);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float d0 = __uint_as_float(aw[e] << 16) - __uint_as_float(bw[e] << 16);
      const float d1 = __uint_as_float(aw[e] & 0xFFFF0000u) - __uint_as_float(bw[e] & 0xFFFF0000u);
      acc += (double)d0 * (double)d0 + (double)d1 * (double)d1;
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int d = 128; d >= 1; d >>= 1) {
    if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

struct Sizes {
  int64_t x_lo[3], x_hi[3];
  int kv_max, ks_max;
  int64_t cap_max;
  size_t ws_child, o_bytes, off[12], total;
};

void candidate_config(const sa_config &parent, int pattern, int64_t x, sa_config *c) {
  *c = parent;
  c->n_q_heads = c->n_kv_heads = 1;
  const int nb = parent.seq_len / parent.block;
  c->local_blocks = 1; c->k_vertical = 1; c->k_slash = 1; c->k_blocks = nb;
  c->block_select = SA_BLOCKS_GLOBAL;  // the search's Block-Cluster candidate is the one-top-k rule,
  c->diagonal_select = SA_DIAGONALS_EXACT;  // its Interval-Slash candidate the element-exact one
  c->lazy_block_map = 0;
  if (pattern == SA_TRIANGULAR) {
    c->local_blocks = (int32_t)x;
  } else if (pattern == SA_INTERVAL_SLASH) {
    c->k_slash = (int32_t)x;
    const int64_t kv = 32 * x;
    c->k_vertical = (int32_t)(kv < parent.seq_len ? kv : parent.seq_len);
  } else {
    c->k_blocks = (int32_t)x;
  }
}

sa_status plan(const sa_ctx *ctx, Sizes *z) {
  const sa_config &p = ctx->cfg;
  const int N = p.seq_len, nb = N / p.block;
  z->x_lo[0] = 1; z->x_hi[0] = nb;
  z->x_lo[1] = 1; z->x_hi[1] = N / 32 > 1 ? N / 32 : 1;
  z->x_lo[2] = nb; z->x_hi[2] = (int64_t)nb * (nb + 1) / 2;
  if (z->x_hi[2] > 0x7FFFFFFFll) return SA_ERR_UNSUPPORTED;
  z->ks_max = (int)z->x_hi[1];
  z->kv_max = 32 * (int64_t)z->ks_max < N ? 32 * z->ks_max : N;
  z->cap_max = z->x_hi[2];
  // the largest child workspace is the one with the most gathered columns
  sa_config c;
  candidate_config(p, SA_INTERVAL_SLASH, z->x_hi[1], &c);
  sa_ctx *child = nullptr;
  sa_status st = sa::create_context(&c, &child, false);
  if (st != SA_OK) return st;
  st = sa_workspace_bytes(child, &z->ws_child);
  sa_destroy(child);
  if (st != SA_OK) return st;
  z->o_bytes = (size_t)N * (size_t)ctx->sh.q_rs * 2;
  const size_t parts[12] = {z->ws_child, z->o_bytes, z->o_bytes, (size_t)nb * nb * 4, 256, 256,
                            (size_t)z->kv_max * 4, 256, (size_t)z->ks_max * 4, (size_t)(nb + 1) * 4,
                            (size_t)z->cap_max * 4, 256 + (size_t)kNormBlocks * 8};
  size_t o = 0;
  for (int i = 0; i < 12; ++i) { z->off[i] = o; o += align256(parts[i]); }
  z->total = o;
  return SA_OK;
}

sa_status failp(sa_ctx *c, sa_status st, const char *msg) {
  snprintf(c->err, sizeof(c->err), "%s", msg);
  return st;
}

}  // namespace

extern "C" {

sa_status sa_search_scratch_bytes(const sa_ctx *ctx, size_t *bytes) {
  if (!ctx || !bytes) return SA_ERR_INVALID_ARG;
  Sizes z;
  const sa_status st = plan(ctx, &z);
  if (st == SA_OK) *bytes = z.total;
  return st;
}

sa_status sa_search_patterns(sa_ctx *ctx, const void *Q, const void *K, const void *V, sa_scores scores,
                             int64_t target_pairs, int64_t eps_pairs, void *scratch, size_t scratch_bytes,
                             sa_search_head *out_host, void *hip_stream) {
  if (!ctx) return SA_ERR_INVALID_ARG;
  if (!Q || !K || !V || !scores.v || !scores.s || !scores.blk || !scratch || !out_host)
    return failp(ctx, SA_ERR_INVALID_ARG, "null pointer");
  if (target_pairs < 0 || eps_pairs < 0) return failp(ctx, SA_ERR_INVALID_ARG, "negative target or tolerance");
  if ((uintptr_t)scratch & 255) return failp(ctx, SA_ERR_INVALID_ARG, "scratch must be 256-byte aligned");
  Sizes z;
  sa_status st = plan(ctx, &z);
  if (st != SA_OK) return failp(ctx, st, "search: sizes not supported");
  if (scratch_bytes < z.total) return failp(ctx, SA_ERR_BUFFER_TOO_SMALL, "scratch smaller than sa_search_scratch_bytes");
  hipStream_t stream = (hipStream_t)hip_stream;
  const sa::Shape &sh = ctx->sh;
  const int N = sh.N, nb = sh.nb;
  char *base = (char *)scratch;
  void *ws = base + z.off[0];
  uint16_t *o_dense = (uint16_t *)(base + z.off[1]), *o_sparse = (uint16_t *)(base + z.off[2]);
  float *blk1 = (float *)(base + z.off[3]);
  sa_index ix;
  ix.pattern = (int32_t *)(base + z.off[4]); ix.n_cols = (int32_t *)(base + z.off[5]);
  ix.cols = (int32_t *)(base + z.off[6]); ix.n_offs = (int32_t *)(base + z.off[7]);
  ix.offs = (int32_t *)(base + z.off[8]); ix.rowptr = (int32_t *)(base + z.off[9]);
  ix.blkcols = (int32_t *)(base + z.off[10]);
  uint64_t *counters = (uint64_t *)(base + z.off[11]);
  double *partial = (double *)(base + z.off[11] + 256);

  hipError_t he = hipSuccess;
  auto hip_fail = [&](hipError_t e) {
    snprintf(ctx->err, sizeof(ctx->err), "HIP: %s", hipGetErrorString(e));
    return SA_ERR_HIP;
  };

  for (int h = 0; h < sh.Hq; ++h) {
    const uint16_t *Qh = (const uint16_t *)Q + (size_t)h * sh.q_hs;
    const uint16_t *Kh = (const uint16_t *)K + (size_t)(h / sh.g) * sh.kv_hs;
    const uint16_t *Vh = (const uint16_t *)V + (size_t)(h / sh.g) * sh.kv_hs;
    // the head's block map goes to an aligned copy (its slice need not be 16-byte aligned)
    if ((he = hipMemcpyAsync(blk1, scores.blk + (size_t)h * nb * nb, (size_t)nb * nb * 4,
                             hipMemcpyDeviceToDevice, stream)) != hipSuccess)
      return hip_fail(he);
    const sa_scores sc{scores.v + (size_t)h * N, scores.s + (size_t)h * N, blk1};

    // one evaluation: index of candidate (pattern, x), sparse output into O, kept pairs
    auto evaluate = [&](int pattern, int64_t x, uint16_t *O, bool count, int64_t *pairs) -> sa_status {
      sa_config c;
      candidate_config(ctx->cfg, pattern, x, &c);
      sa_ctx *child = nullptr;
      sa_status s_ = sa::create_context(&c, &child, false);  // host memory only: no stream, no events
      if (s_ != SA_OK) return failp(ctx, s_, "search: candidate rejected by sa_create");
      const int32_t ov = pattern;
      s_ = sa_set_workspace(child, ws, z.ws_child);
      if (s_ == SA_OK) s_ = sa_build_index(child, sc, &ov, ix, stream);
      if (s_ == SA_OK && count) {
        if ((he = hipMemsetAsync(counters, 0, 16, stream)) != hipSuccess) s_ = hip_fail(he);
        if (s_ == SA_OK) s_ = sa_sparse_prefill_counted(child, Qh, Kh, Vh, ix, O, counters, stream);
      } else if (s_ == SA_OK) {
        s_ = sa_sparse_prefill(child, Qh, Kh, Vh, ix, O, stream);
      }
      if (s_ != SA_OK && s_ != SA_ERR_HIP) snprintf(ctx->err, sizeof(ctx->err), "search: %s", sa_last_error(child));
      if (s_ == SA_OK && count) {
        uint64_t hc[2];
        if ((he = hipMemcpyAsync(hc, counters, 16, hipMemcpyDeviceToHost, stream)) != hipSuccess ||
            (he = hipStreamSynchronize(stream)) != hipSuccess)
          s_ = hip_fail(he);
        else
          *pairs = (int64_t)hc[1];
      } else if (s_ == SA_OK) {
        if ((he = hipStreamSynchronize(stream)) != hipSuccess) s_ = hip_fail(he);
      }
      sa_destroy(child);  // the stream is idle: nothing of the child is in flight
      return s_;
    };

    // dense reference: the band as wide as the sequence
    if ((st = evaluate(SA_TRIANGULAR, nb, o_dense, false, nullptr)) != SA_OK) return st;

    sa_search_head &r = out_host[h];
    for (int p = 0; p < 3; ++p) {
      int64_t lo = z.x_lo[p], hi = z.x_hi[p], p_lo = 0, p_hi = 0, x = lo, px = 0;
      // RefineSearchSpace: bisection, the pair count does not decrease with the size
      if ((st = evaluate(p, lo, o_sparse, true, &p_lo)) != SA_OK) return st;
      x = lo; px = p_lo;
      bool done = p_lo >= target_pairs || llabs(p_lo - target_pairs) <= eps_pairs || lo == hi;
      if (!done) {
        if ((st = evaluate(p, hi, o_sparse, true, &p_hi)) != SA_OK) return st;
        if (p_hi <= target_pairs || llabs(p_hi - target_pairs) <= eps_pairs) { x = hi; px = p_hi; done = true; }
      }
      while (!done && hi - lo > 1) {
        const int64_t mid = (lo + hi) / 2;
        int64_t pm = 0;
        if ((st = evaluate(p, mid, o_sparse, true, &pm)) != SA_OK) return st;
        if (llabs(pm - target_pairs) <= eps_pairs) { x = mid; px = pm; done = true; break; }
        if (pm < target_pairs) { lo = mid; p_lo = pm; } else { hi = mid; p_hi = pm; }
      }
      if (!done) {
        if (target_pairs - p_lo <= p_hi - target_pairs) { x = lo; px = p_lo; } else { x = hi; px = p_hi; }
      }
      // Evaluate Patterns: sparse output of the refined candidate against the dense one
      if ((st = evaluate(p, x, o_sparse, false, nullptr)) != SA_OK) return st;
      sq_diff_kernel<<<kNormBlocks, 256, 0, stream>>>(o_sparse, o_dense, N, sh.q_rs, partial);
      if ((he = hipGetLastError()) != hipSuccess) return hip_fail(he);
      double hp[kNormBlocks];
      if ((he = hipMemcpyAsync(hp, partial, sizeof(hp), hipMemcpyDeviceToHost, stream)) != hipSuccess ||
          (he = hipStreamSynchronize(stream)) != hipSuccess)
        return hip_fail(he);
      double sum = 0.0;
      for (int i = 0; i < kNormBlocks; ++i) sum += hp[i];
      r.param[p] = (int32_t)x;
      r.pairs[p] = px;
      r.err[p] = std::sqrt(sum);
    }
    r.pattern = 0;
    for (int p = 1; p < 3; ++p)
      if (r.err[p] < r.err[r.pattern]) r.pattern = p;
  }
  return SA_OK;
}

}  // extern "C"
