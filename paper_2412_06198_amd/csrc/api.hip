// Host side of the C ABI declared in include/sa.h: argument checks, shape
// resolution, workspace carving, and the three launch sequences.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "sa_internal.h"

namespace {

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

long long triangular_count(int nb, int sink, int local) {
  long long n = 0;
  for (int R = 0; R < nb; ++R) {
    const int bs = R - local + 1 > 0 ? R - local + 1 : 0;
    n += (sink < bs ? sink : bs) + (R - bs + 1);
  }
  return n;
}

sa_status fail(sa_ctx *c, sa_status st, const char *msg) {
  if (c) snprintf(c->err, sizeof(c->err), "%s", msg);
  return st;
}

void carve(sa_ctx *c) {
  const sa::Shape &s = c->sh;
  size_t o = 0;
  const size_t nb16 = (size_t)(s.nb + 15) / 16 * 16;  // block means are stored in tiles of 16 rows
  c->off[0] = o; o += align256((size_t)s.Hq * nb16 * sa::kHeadDim * 4);
  c->off[1] = o; o += align256((size_t)s.Hkv * nb16 * sa::kHeadDim * 4);
  c->off[2] = o; o += align256((size_t)s.Hq * s.nchunks * sa::kWin * 8);
  c->off[3] = o; o += align256((size_t)s.Hq * sa::kWin * 8);
  c->off[4] = o; o += align256((size_t)s.Hq * (s.N / 32) * 4);
  const size_t kvg = (size_t)s.Hq * ((s.k_v + 63) / 64 * 64) * (size_t)s.kv_rs * 2;
  c->off[5] = o; o += align256(kvg);
  c->off[6] = o; o += align256(kvg);
  c->off[7] = o; o += 256;
  c->off[8] = o; o += align256(sa::index_scratch_bytes(s.Hq));
  c->off[9] = o; o += align256((size_t)s.Hq * (s.N / 32) * 4);
  c->off[10] = o; o += align256(sa::decode_partial_bytes(s));
  c->off[11] = o; o += align256((size_t)(s.Hq + s.Hkv) * 4);
  c->ws_bytes = o;
}

}  // namespace

extern "C" {

const char *sa_version(void) { return "sa-prefill-gfx950 0.1"; }

sa_status sa_default_budgets(sa_config *cfg, double keep) {
  if (!cfg || !(keep > 0.0) || keep > 1.0) return SA_ERR_INVALID_ARG;
  if (cfg->block <= 0 || cfg->seq_len <= 0 || cfg->seq_len % cfg->block) return SA_ERR_INVALID_ARG;
  const long long N = cfg->seq_len, nb = N / cfg->block;
  const long long causal = nb * (nb + 1) / 2;
  long long T = (long long)std::floor(keep * (double)causal + 0.5);
  if (T < nb) T = nb;
  const int sink = 1;
  int L = 1;
  for (long long cand = 1; cand <= nb; ++cand)
    if (cand * nb - cand * (cand - 1) / 2 + (nb - cand) * sink <= T) L = (int)cand;
  long long ks = (long long)std::floor(keep * (double)N / 128.0 + 0.5);
  long long kv = (long long)std::floor(keep * (double)N / 256.0 + 0.5);
  if (ks < 1) ks = 1;
  if (kv < 1) kv = 1;
  kv *= 64;
  if (kv > N) kv = N;
  if (ks > N) ks = N;
  cfg->sink_blocks = sink;
  cfg->local_blocks = L;
  cfg->k_vertical = (int32_t)kv;
  cfg->k_slash = (int32_t)ks;
  cfg->k_blocks = (int32_t)T;
  return SA_OK;
}

sa_status sa_create(const sa_config *cfg, sa_ctx **out) { return sa::create_context(cfg, out, true); }

}  // extern "C"

// side_stream == false: a context for callers inside the library that never run the estimator (the
// probes of the offline search): no stream and no events are created.
sa_status sa::create_context(const sa_config *cfg, sa_ctx **out, bool side_stream) {
  if (!cfg || !out) return SA_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->head_dim != sa::kHeadDim) return SA_ERR_UNSUPPORTED;
  if (cfg->block != 64 && cfg->block != 128) return SA_ERR_UNSUPPORTED;
  if (cfg->seq_len <= 0 || cfg->seq_len % cfg->block) return SA_ERR_UNSUPPORTED;
  if (cfg->seq_len > sa::kMaxSeq) return SA_ERR_UNSUPPORTED;
  if (cfg->last_q < 1 || cfg->last_q > sa::kWin || cfg->last_q > cfg->seq_len) return SA_ERR_UNSUPPORTED;
  if (cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->n_q_heads % cfg->n_kv_heads ||
      cfg->n_q_heads > sa::kMaxHeads)
    return SA_ERR_INVALID_ARG;
  const int nb = cfg->seq_len / cfg->block;
  if (cfg->sink_blocks < 0 || cfg->local_blocks < 1 || cfg->local_blocks > nb) return SA_ERR_INVALID_ARG;
  if (cfg->k_vertical < 1 || cfg->k_slash < 1 || cfg->k_blocks < nb) return SA_ERR_INVALID_ARG;
  if (cfg->probe_v < 0 || cfg->probe_s < 0 || cfg->lift_num < 0 || cfg->lift_den < 0) return SA_ERR_INVALID_ARG;
  if (cfg->softmax_scale < 0.f) return SA_ERR_INVALID_ARG;
  if (cfg->block_select < SA_BLOCKS_GLOBAL || cfg->block_select > SA_BLOCKS_GLOBAL_ROW_NORMALISED) return SA_ERR_INVALID_ARG;
  if (cfg->diagonal_select != SA_DIAGONALS_EXACT && cfg->diagonal_select != SA_DIAGONALS_BLOCKS) return SA_ERR_INVALID_ARG;
  if (cfg->lazy_block_map != 0 && cfg->lazy_block_map != 1) return SA_ERR_INVALID_ARG;

  sa_ctx *c = new (std::nothrow) sa_ctx();
  if (!c) return SA_ERR_INVALID_ARG;
  c->cfg = *cfg;
  sa::Shape &s = c->sh;
  s.Hq = cfg->n_q_heads; s.Hkv = cfg->n_kv_heads; s.g = s.Hq / s.Hkv;
  s.N = cfg->seq_len; s.b = cfg->block; s.nb = nb; s.w = cfg->last_q;
  s.k_v = cfg->k_vertical; s.k_s = cfg->k_slash; s.k_b = cfg->k_blocks;
  s.sink = cfg->sink_blocks; s.local = cfg->local_blocks;
  s.probe_v = cfg->probe_v ? cfg->probe_v : 4;
  s.probe_s = cfg->probe_s ? cfg->probe_s : 4;
  s.lift_num = cfg->lift_num ? cfg->lift_num : 4;
  s.lift_den = cfg->lift_den ? cfg->lift_den : 1;
  const long long tri = triangular_count(nb, s.sink, s.local);
  s.row_select = cfg->block_select == SA_BLOCKS_PER_ROW;
  s.row_norm = cfg->block_select == SA_BLOCKS_GLOBAL_ROW_NORMALISED;
  // the per-row rule rounds every row's share up: at most one block per row above k_b
  const long long kcap = (long long)s.k_b + (s.row_select ? nb : 0);
  long long cap = tri > kcap ? tri : kcap;
  s.diag_blocks = cfg->diagonal_select == SA_DIAGONALS_BLOCKS;
  s.lazy_blk = cfg->lazy_block_map;
  if (s.diag_blocks) {
    // a diagonal touches at most two key blocks per row block: row R holds min(R + 1, 2 k_s + 1)
    const long long ks = s.k_s < s.N ? s.k_s : s.N, m = 2 * ks + 1;
    const long long dcap = m >= nb ? (long long)nb * (nb + 1) / 2 : m * (m + 1) / 2 + (nb - m) * m;
    if (dcap > cap) cap = dcap;
  }
  if (cap > 0x7FFFFFFFll) { delete c; return SA_ERR_UNSUPPORTED; }
  s.cap_b = (int)cap;
  // keys per workgroup of the window passes: 1024 measured 3 % faster than 512 at 128K, equal at
  // 32K-64K; short sequences keep 512 for the sake of parallelism
  s.chunk = s.N >= 32768 ? 1024 : 512;
  s.nchunks = (s.N + s.chunk - 1) / s.chunk;
  s.q_rs = cfg->q_row_stride ? cfg->q_row_stride : sa::kHeadDim;
  s.q_hs = cfg->q_head_stride ? cfg->q_head_stride : (int64_t)s.N * s.q_rs;
  s.kv_rs = cfg->kv_row_stride ? cfg->kv_row_stride : sa::kHeadDim;
  s.kv_hs = cfg->kv_head_stride ? cfg->kv_head_stride : (int64_t)s.N * s.kv_rs;
  if (s.q_rs % 8 || s.kv_rs % 8 || s.q_hs % 8 || s.kv_hs % 8 || s.q_rs < sa::kHeadDim ||
      s.kv_rs < sa::kHeadDim) {
    delete c;
    return SA_ERR_UNSUPPORTED;
  }
  {
    // the attention kernel is persistent: it launches two workgroups per compute unit.
    // Without a usable device (a CPU-only build check) fall back to the MI355X count.
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0) {
      (void)hipGetLastError();
      ncu = 256;
    }
    s.n_cu = ncu;
  }
  s.scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)sa::kHeadDim);
  // Side stream of the estimator (default priority).  Without a usable device the creation
  // fails and the context simply enqueues everything on the caller's stream.
  c->fork = sa::Fork{nullptr, nullptr, nullptr, nullptr};
  if (!side_stream) {
    // everything is enqueued on the caller's stream
  } else if (hipStreamCreateWithFlags(&c->fork.aux, hipStreamNonBlocking) == hipSuccess) {
    if (hipEventCreateWithFlags(&c->fork.fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->fork.mid, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->fork.join, hipEventDisableTiming) != hipSuccess) {
      if (c->fork.fork) (void)hipEventDestroy(c->fork.fork);
      if (c->fork.mid) (void)hipEventDestroy(c->fork.mid);
      if (c->fork.join) (void)hipEventDestroy(c->fork.join);
      (void)hipStreamDestroy(c->fork.aux);
      c->fork = sa::Fork{nullptr, nullptr, nullptr, nullptr};
    }
  } else {
    c->fork.aux = nullptr;
  }
  (void)hipGetLastError();
  c->have_ws = false;
  c->err[0] = 0;
  carve(c);
  *out = c;
  return SA_OK;
}

extern "C" {

void sa_destroy(sa_ctx *ctx) {
  if (!ctx) return;
  if (ctx->fork.aux) {
    (void)hipEventDestroy(ctx->fork.fork);
    (void)hipEventDestroy(ctx->fork.mid);
    (void)hipEventDestroy(ctx->fork.join);
    (void)hipStreamDestroy(ctx->fork.aux);
  }
  delete ctx;
}

sa_status sa_scores_bytes(const sa_ctx *c, size_t out[3]) {
  if (!c || !out) return SA_ERR_INVALID_ARG;
  out[0] = out[1] = (size_t)c->sh.Hq * c->sh.N * 4;
  out[2] = (size_t)c->sh.Hq * c->sh.nb * c->sh.nb * 4;
  return SA_OK;
}

sa_status sa_index_bytes(const sa_ctx *c, size_t out[7]) {
  if (!c || !out) return SA_ERR_INVALID_ARG;
  const sa::Shape &s = c->sh;
  out[0] = (size_t)s.Hq * 4;
  out[1] = (size_t)s.Hq * 4;
  out[2] = (size_t)s.Hq * s.k_v * 4;
  out[3] = (size_t)s.Hq * 4;
  out[4] = (size_t)s.Hq * s.k_s * 4;
  out[5] = (size_t)s.Hq * (s.nb + 1) * 4;
  out[6] = (size_t)s.Hq * s.cap_b * 4;
  return SA_OK;
}

sa_status sa_workspace_bytes(const sa_ctx *c, size_t *bytes) {
  if (!c || !bytes) return SA_ERR_INVALID_ARG;
  *bytes = c->ws_bytes;
  return SA_OK;
}

sa_status sa_set_workspace(sa_ctx *c, void *dev, size_t bytes) {
  if (!c) return SA_ERR_INVALID_ARG;
  if (!dev || ((uintptr_t)dev & 255)) return fail(c, SA_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
  if (bytes < c->ws_bytes) return fail(c, SA_ERR_BUFFER_TOO_SMALL, "workspace smaller than sa_workspace_bytes");
  char *p = (char *)dev;
  c->ws.qblk = (float *)(p + c->off[0]);
  c->ws.kblk = (float *)(p + c->off[1]);
  c->ws.part = (float2 *)(p + c->off[2]);
  c->ws.stats = (float2 *)(p + c->off[3]);
  c->ws.colbits = (uint32_t *)(p + c->off[4]);
  c->ws.kg = (uint16_t *)(p + c->off[5]);
  c->ws.vg = (uint16_t *)(p + c->off[6]);
  c->ws.queue = (unsigned int *)(p + c->off[7]);
  c->ws.idx = (void *)(p + c->off[8]);
  c->ws.colprefix = (int32_t *)(p + c->off[9]);
  c->ws.dec_part = (float *)(p + c->off[10]);
  c->ws.hperm = (int32_t *)(p + c->off[11]);
  c->have_ws = true;
  return SA_OK;
}

static sa_status hip_result(sa_ctx *c, hipError_t e) {
  if (e == hipSuccess) return SA_OK;
  snprintf(c->err, sizeof(c->err), "HIP: %s", hipGetErrorString(e));
  return SA_ERR_HIP;
}

sa_status sa_estimate_patterns(sa_ctx *c, const void *Q, const void *K, sa_scores out, void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  if (!Q || !K || !out.v || !out.s || !out.blk) return fail(c, SA_ERR_INVALID_ARG, "null pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)out.blk) & 15) return fail(c, SA_ERR_INVALID_ARG, "Q, K, blk must be 16-byte aligned");
  if (!c->have_ws) return fail(c, SA_ERR_INVALID_ARG, "no workspace attached");
  return hip_result(c, sa::launch_estimate(c->sh, c->ws, (const uint16_t *)Q, (const uint16_t *)K, out,
                                           (hipStream_t)stream, c->fork));
}

static sa_status check_index_args(sa_ctx *c, sa_scores in, const int32_t *override_host, sa_index out,
                                  sa::Override *ov) {
  if (!in.v || !in.s || !in.blk || !out.pattern || !out.n_cols || !out.cols || !out.n_offs ||
      !out.offs || !out.rowptr || !out.blkcols)
    return fail(c, SA_ERR_INVALID_ARG, "null pointer");
  if (((uintptr_t)in.v | (uintptr_t)in.s | (uintptr_t)in.blk) & 15)
    return fail(c, SA_ERR_INVALID_ARG, "v, s, blk must be 16-byte aligned");
  for (int h = 0; h < sa::kMaxHeads; ++h) ov->pat[h] = -1;
  if (override_host)
    for (int h = 0; h < c->sh.Hq; ++h) {
      const int32_t p = override_host[h];
      if (p < -1 || p > 2) return fail(c, SA_ERR_INVALID_ARG, "pattern override out of range");
      ov->pat[h] = (int8_t)p;
    }
  return SA_OK;
}

sa_status sa_build_index(sa_ctx *c, sa_scores in, const int32_t *override_host, sa_index out,
                         void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  sa::Override ov;
  const sa_status s = check_index_args(c, in, override_host, out, &ov);
  if (s != SA_OK) return s;
  if (!c->have_ws) return fail(c, SA_ERR_INVALID_ARG, "no workspace attached");
  return hip_result(c, sa::launch_build_index(c->sh, c->ws, in, ov, out, (hipStream_t)stream));
}

sa_status sa_estimate_and_index(sa_ctx *c, const void *Q, const void *K, sa_scores scores,
                                const int32_t *override_host, sa_index out, void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  if (!Q || !K) return fail(c, SA_ERR_INVALID_ARG, "null pointer");
  if (((uintptr_t)Q | (uintptr_t)K) & 15) return fail(c, SA_ERR_INVALID_ARG, "Q, K must be 16-byte aligned");
  if (!c->have_ws) return fail(c, SA_ERR_INVALID_ARG, "no workspace attached");
  sa::Override ov;
  const sa_status s = check_index_args(c, scores, override_host, out, &ov);
  if (s != SA_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  const sa::Fork &fk = c->fork;
  if (c->sh.lazy_blk) {
    // In the order of the categorisation, on one stream: what the Block-Cluster branch needs is
    // computed once the heads that take it are known.
    const uint16_t *q = (const uint16_t *)Q, *k = (const uint16_t *)K;
    using sa::IndexStage;
    using sa::EstimatePart;
    hipError_t e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, IndexStage::Zero, st);
    if (e == hipSuccess) e = sa::launch_estimate_part(c->sh, c->ws, q, k, scores, EstimatePart::KChain, nullptr, st);
    if (e == hipSuccess) e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, IndexStage::ColumnsDiagonals, st);
    if (e == hipSuccess) e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, IndexStage::Decide, st);
    if (e == hipSuccess)
      e = sa::launch_estimate_part(c->sh, c->ws, q, k, scores, EstimatePart::QChain, out.pattern, st);
    if (e == hipSuccess) e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, IndexStage::Blocks, st, true);
    if (e == hipSuccess) e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, IndexStage::Emit, st, true);
    return hip_result(c, e);
  }
  // Caller's stream: window passes -> selections on v and s; side stream: block means and block
  // map -> block selection; joined before the pattern decision and the emission.
  hipError_t e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, sa::IndexStage::Zero, st);
  if (e == hipSuccess)
    e = sa::launch_estimate(c->sh, c->ws, (const uint16_t *)Q, (const uint16_t *)K, scores, st, fk, false);
  if (e == hipSuccess)
    e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, sa::IndexStage::ColumnsDiagonals, st);
  if (e == hipSuccess)
    e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, sa::IndexStage::Blocks, fk.aux ? fk.aux : st);
  if (fk.aux) {
    // join even after an error above, so that the side stream never outlives the call unjoined
    hipError_t j = hipEventRecord(fk.join, fk.aux);
    if (j == hipSuccess) j = hipStreamWaitEvent(st, fk.join, 0);
    if (e == hipSuccess) e = j;
  }
  if (e == hipSuccess) e = sa::launch_index_stage(c->sh, c->ws, scores, ov, out, sa::IndexStage::Emit, st);
  return hip_result(c, e);
}

static sa_status prefill_common(sa_ctx *c, const void *Q, const void *K, const void *V, sa_index idx,
                                void *O, uint64_t *counters, void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  if (!Q || !K || !V || !O || !idx.n_cols || !idx.cols || !idx.n_offs || !idx.offs || !idx.rowptr ||
      !idx.blkcols)
    return fail(c, SA_ERR_INVALID_ARG, "null pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15)
    return fail(c, SA_ERR_INVALID_ARG, "Q, K, V, O must be 16-byte aligned");
  if (!c->have_ws) return fail(c, SA_ERR_INVALID_ARG, "no workspace attached");
  return hip_result(c, sa::launch_sparse_prefill(c->sh, c->ws, (const uint16_t *)Q, (const uint16_t *)K,
                                                 (const uint16_t *)V, idx, (uint16_t *)O,
                                                 (unsigned long long *)counters, (hipStream_t)stream));
}

sa_status sa_sparse_prefill(sa_ctx *c, const void *Q, const void *K, const void *V, sa_index idx,
                            void *O, void *stream) {
  return prefill_common(c, Q, K, V, idx, O, nullptr, stream);
}

sa_status sa_sparse_prefill_counted(sa_ctx *c, const void *Q, const void *K, const void *V,
                                    sa_index idx, void *O, uint64_t *counters_dev, void *stream) {
  if (c && (!counters_dev || ((uintptr_t)counters_dev & 7)))
    return fail(c, SA_ERR_INVALID_ARG, "counters must be an 8-byte aligned device pointer");
  return prefill_common(c, Q, K, V, idx, O, counters_dev, stream);
}

static sa_status check_decode_args(sa_ctx *c, const void *q, const void *K, const void *V, sa_index idx,
                                   int64_t pos, void *o) {
  if (!q || !K || !V || !o || !idx.n_cols || !idx.cols || !idx.n_offs || !idx.offs || !idx.rowptr ||
      !idx.blkcols)
    return fail(c, SA_ERR_INVALID_ARG, "null pointer");
  if (((uintptr_t)q | (uintptr_t)K | (uintptr_t)V) & 15)
    return fail(c, SA_ERR_INVALID_ARG, "q, K, V must be 16-byte aligned");
  if (pos < c->sh.N || pos - c->sh.N >= (1 << 20))
    return fail(c, SA_ERR_INVALID_ARG, "pos must lie in [seq_len, seq_len + 2^20)");
  // rows 0..pos of a KV head must fit inside its own stride, or they would alias the next head's
  // rows (and leave the buffer behind the last head)
  if ((pos + 1) * c->sh.kv_rs > c->sh.kv_hs)
    return fail(c, SA_ERR_INVALID_ARG, "kv_head_stride leaves no room for key rows up to pos");
  return SA_OK;
}

sa_status sa_sparse_decode(sa_ctx *c, const void *q, const void *K, const void *V, sa_index idx,
                           int64_t pos, void *o, void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  const sa_status s = check_decode_args(c, q, K, V, idx, pos, o);
  if (s != SA_OK) return s;
  if (!c->have_ws) return fail(c, SA_ERR_INVALID_ARG, "no workspace attached");
  return hip_result(c, sa::launch_sparse_decode(c->sh, c->ws.dec_part, (const uint16_t *)q, (const uint16_t *)K,
                                                (const uint16_t *)V, idx, (int)pos, (uint16_t *)o,
                                                (hipStream_t)stream));
}

sa_status sa_sparse_decode_static(sa_ctx *c, const void *q, const void *K, const void *V, sa_index idx,
                                  int64_t pos, void *o, void *stream) {
  if (!c) return SA_ERR_INVALID_ARG;
  const sa_status s = check_decode_args(c, q, K, V, idx, pos, o);
  if (s != SA_OK) return s;
  if (sa::decode_partial_bytes(c->sh) > sa::decode_static_bytes())
    return fail(c, SA_ERR_UNSUPPORTED, "n_q_heads x decode splits exceeds the static scratch (512 partials)");
  float *partials = nullptr;
  const hipError_t e = sa::decode_static_scratch(&partials);
  if (e != hipSuccess) return hip_result(c, e);
  return hip_result(c, sa::launch_sparse_decode(c->sh, partials, (const uint16_t *)q, (const uint16_t *)K,
                                                (const uint16_t *)V, idx, (int)pos, (uint16_t *)o,
                                                (hipStream_t)stream));
}

const char *sa_last_error(const sa_ctx *c) { return c ? c->err : "null context"; }

}  // extern "C"
