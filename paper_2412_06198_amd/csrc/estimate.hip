// Pattern estimator for gfx950.
//
//  * window scores (Alg. 2 "Compute Dense Attention Scores" on the last w query
//    rows only, then SumRows -> v and SumDiagonals -> s).  The softmax of a
//    window row needs its maximum and normaliser over ALL keys before any
//    column can be summed, so K is streamed twice:
//      pass 1  S^T = K Qwin^T  (lane = query)  -> per-chunk (max, sum) partials,
//                                                 and the block sums of K on the way
//      pass 2  S   = Qwin K^T  (lane = key)    -> normalised weights, column sums in
//                                                 the lane, diagonal sums by lane shifts
//    The 4 query heads of a GQA group ride on one K stream: wave w = head w.
//    K tiles go global -> LDS directly (global_load_lds_dwordx4), double-buffered.
//  * block map (Alg. 3 "Compute Blocked Representation"): fp32 block means of Q
//    and K, then one kernel that forms a 16-row strip of block logits with fp32
//    MFMA, keeps it in registers, and writes its causal row softmax once.
#include "sa_internal.h"

namespace sa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Block means are kept as two bf16 numbers, head + remainder (x = hi + lo to about 2^-17 |x|), so
// that the block map can form their products on the bf16 matrix pipe: hi.hi + hi.lo + lo.hi with
// fp32 accumulation differs from the fp32 product by about 2^-16 of it.
// A means array is laid out in the order in which the block map's matrix instruction wants its
// operands: per head ceil(nb/16) tiles of 16 rows, 8 KB each = [part: heads, remainders][k-step
// st = d/32][g = d%32/8][row n = R%16][8 elements], so that lane n + 16 g of a wave reads 16
// contiguous bytes of a contiguous 1 KB per instruction.  (With plain rows every quarter-wave
// touched 16 different cache lines, and the block map spent half its time in the L1's tag
// lookups.)  Rows past nb in the last tile are never written; nothing that is kept depends on them.
__device__ inline size_t means_tiles(int nb) { return (size_t)((nb + 15) / 16); }

__device__ inline void store_split(float *means_head, int R, int d, float x) {
  const __bf16 hi = (__bf16)x;
  const __bf16 lo = (__bf16)(x - (float)hi);
  uint16_t *tile = (uint16_t *)means_head + (size_t)(R >> 4) * 4096;
  const int o = (d >> 5) * 512 + ((d >> 3) & 3) * 128 + (R & 15) * 8 + (d & 7);
  tile[o] = __builtin_bit_cast(uint16_t, hi);
  tile[2048 + o] = __builtin_bit_cast(uint16_t, lo);
}

// ------------------------------------------------------------------ Q block means
// grid (nb, Hq), 256 threads: thread = (row group of 16, 16-byte column); all RPT = b/16 loads of
// a thread are in flight before the first sum.  The kernel is pure HBM streaming and runs beside
// the window passes (vector ALU bound): it is launched with kQMeanLdsPad* bytes of unused dynamic
// LDS so that it never holds more than a few wave slots of a compute unit.
constexpr int kQMeanLdsPad128 = 32 * 1024, kQMeanLdsPad64 = 32 * 1024;  // measured best (16-96 KB swept)

template <int RPT>
__global__ __launch_bounds__(256) void q_block_mean_kernel(const uint16_t *__restrict__ Q, Shape sh,
                                                           float *__restrict__ qblk,
                                                           const int32_t *__restrict__ only_bc) {
  __shared__ float red[16][kHeadDim + 4];
  const int R = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  if (only_bc && only_bc[h] != SA_BLOCK_CLUSTER) return;  // this head's block map is not wanted
  const uint16_t *src = Q + (size_t)h * sh.q_hs + (size_t)R * sh.b * sh.q_rs;
  const int cc = tid & 15, rg = tid >> 4;
  uint4 x[RPT];
#pragma unroll
  for (int n = 0; n < RPT; ++n) {
    // read once: a streaming (non-temporal) load leaves the caches to K, which the second window
    // pass reads again
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t *)(src + (size_t)(rg + 16 * n) * sh.q_rs + cc * 8));
    x[n] = make_uint4(v.x, v.y, v.z, v.w);
  }
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int n = 0; n < RPT; ++n) {
    const uint32_t wds[4] = {x[n].x, x[n].y, x[n].z, x[n].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] += bf16_bits_to_f32(wds[e] & 0xFFFFu);
      acc[2 * e + 1] += bf16_bits_to_f32(wds[e] >> 16);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rg][cc * 8 + e] = acc[e];
  __syncthreads();
  if (tid < kHeadDim) {
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += red[r][tid];
    store_split(qblk + (size_t)h * means_tiles(sh.nb) * 2048, R, tid, sum * (1.0f / (float)sh.b));
  }
}

// ------------------------------------------------------------------ window passes
// Q window fragments of one head: lane (q = lane%32, gg = lane/32) holds window row
// 32*qh + q, elements d = 16*ks + 8*gg .. +7.  The same registers serve as the B operand
// of K Q^T (pass 1) and as the A operand of Q K^T (pass 2).
__device__ inline void load_qwin(const uint16_t *__restrict__ Q, const Shape &sh, int hq, int lane,
                                 bf16x8 (&qf)[2][8]) {
  const int q = lane & 31, gg = lane >> 5;
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    int i = 32 * qh + q;
    if (i >= sh.w) i = sh.w - 1;  // rows past the window are computed and ignored
    const uint16_t *row = Q + (size_t)hq * sh.q_hs + (size_t)(sh.N - sh.w + i) * sh.q_rs;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[qh][ks] = *(const bf16x8 *)(row + 16 * ks + 8 * gg);
  }
}

// A K tile is 64 keys x 256 B in LDS, the 16-byte chunks of a row XOR-swizzled with the row
// number (chunk c of row r sits at chunk c ^ (r & 15)): the b128 fragment reads of 32 rows are
// conflict-free without padding.  The swizzle is applied on the global side of the copy: the
// lane that owns physical chunk pc of row r fetches logical chunk pc ^ (r & 15).  One
// instruction moves four rows (16 bytes per lane, LDS address = M0 + 16*lane); wave w moves rows
// 4w..4w+3 (+16n, n = 0..3).
#define SA_DMA16(gptr, voff, ldsb)                                                                    \
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(gptr), \
               "s"(ldsb)                                                                              \
               : "memory")

// The window passes keep kStages K tiles in LDS: tile t is multiplied while the copies of the
// next kStages - 2 tiles are in flight (one tile of lead per workgroup left the passes waiting for
// memory latency most of the time: a workgroup only had 16 KB on its way).
constexpr int kStages = 3;

// Wait until this wave's copies of tile t have landed while up to `ahead` younger tiles (four copy
// instructions each) may still be in flight.  Vector memory operations of a kind retire in issue
// order, so at most 4 * ahead outstanding operations means the older copies are complete.
__device__ inline void wait_tile(int ahead) {
  if (ahead >= 2) __builtin_amdgcn_s_waitcnt(0x0F78);       // vmcnt(8)
  else if (ahead == 1) __builtin_amdgcn_s_waitcnt(0x0F74);  // vmcnt(4)
  else __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
}

struct KTileCopy {
  unsigned voff;   // per-lane byte offset inside a 16-row slab of K
  unsigned lds0;   // LDS byte address of this wave's first row in buffer 0
  size_t row16;    // elements between the rows of consecutive instructions
  __device__ inline void init(const uint16_t *ks0, int wv, int lane, int64_t kv_rs) {
    const int rl = 4 * wv + (lane >> 4);
    voff = (unsigned)(rl * (int)kv_rs * 2 + (((lane & 15) ^ rl) << 4));
    lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const uint16_t *)ks0 + 4 * wv * 256;
    row16 = 16 * (size_t)kv_rs;
  }
  __device__ inline void issue(const uint16_t *kb, int buf) const {
    const unsigned l = lds0 + buf * (64 * 256);
    SA_DMA16(kb, voff, l);
    SA_DMA16(kb + row16, voff, l + 16 * 256);
    SA_DMA16(kb + 2 * row16, voff, l + 32 * 256);
    SA_DMA16(kb + 3 * row16, voff, l + 48 * 256);
  }
};

// fragment (rows 32*kh + q, logical chunk 2*ks + gg) of a swizzled tile
__device__ inline bf16x8 k_frag(const uint16_t *tile, unsigned kbase, int gg, int kh, int ks) {
  return *(const bf16x8 *)((const char *)tile + ((kbase ^ (unsigned)((2 * ks + gg) << 4)) + kh * 32 * 256));
}

// pass 1: grid (nchunks, Hkv, ceil(g/4)), 256 threads.
__global__ __launch_bounds__(256, 2) void window_stats_kernel(const uint16_t *__restrict__ Q,
                                                           const uint16_t *__restrict__ K, Shape sh,
                                                           float c, float2 *__restrict__ part,
                                                           float *__restrict__ s_out,
                                                           float *__restrict__ kblk) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kStages][64 * 128];
  __shared__ float ksum[2][4][kHeadDim];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane & 31, gg = lane >> 5;
  const int chunk = blockIdx.x, kvh = blockIdx.y;
  const int hsub = 4 * blockIdx.z + wv;
  const bool head_ok = hsub < sh.g;
  const int hq = kvh * sh.g + (head_ok ? hsub : 0);
  const int jc0 = chunk * sh.chunk;
  const int jc1 = min(jc0 + sh.chunk, sh.N);
  const int nt = (jc1 - jc0) >> 6;  // N is a multiple of 64: whole tiles only
  const uint16_t *Kh = K + (size_t)kvh * sh.kv_hs + (size_t)jc0 * sh.kv_rs;
  const bool do_means = blockIdx.z == 0;

  KTileCopy cp;
  cp.init(&Ks[0][0], wv, lane, sh.kv_rs);
  cp.issue(Kh, 0);

  // the slash scores are accumulated with atomics in pass 2: clear this chunk's share now
  if (head_ok)
    for (int j = jc0 + lane; j < jc1; j += 64) s_out[(size_t)hq * sh.N + j] = 0.f;

  bf16x8 qf[2][8];
  load_qwin(Q, sh, hq, lane, qf);
#pragma unroll
  for (int s2 = 1; s2 < kStages - 1; ++s2)
    if (s2 < nt) cp.issue(Kh + (size_t)s2 * 64 * sh.kv_rs, s2);
  float m[2] = {-INFINITY, -INFINITY}, z[2] = {0.f, 0.f};
  const unsigned kbase = (unsigned)(q * 256) | (unsigned)((q & 15) << 4);

  // block sums of K: thread = (dword column cd of the 256-byte rows, rows 16*wv .. 16*wv+15)
  const int cd = tid & 63;
  const int tpb = sh.b >> 6;  // tiles per block: 1 or 2
  float ks_lo = 0.f, ks_hi = 0.f;
  int pending = -1;           // block whose four partial sums wait in ksum[pending & 1]

  for (int t = 0; t < nt; ++t) {
    const int cur = t % kStages;
    wait_tile(min(nt - 1 - t, kStages - 2));  // this wave's share of tile t has landed
    __syncthreads();                          // ... and everybody's; tile t-1 has been read by all
    if (t + kStages - 1 < nt)
      cp.issue(Kh + (size_t)(t + kStages - 1) * 64 * sh.kv_rs, (t + kStages - 1) % kStages);
    const uint16_t *Kt = Ks[cur];
    const int j0 = jc0 + 64 * t;

    if (do_means) {
      if (pending >= 0 && tid < kHeadDim) {
        const float(*ps)[kHeadDim] = ksum[pending & 1];
        store_split(kblk + (size_t)kvh * means_tiles(sh.nb) * 2048, pending, tid,
                    ((ps[0][tid] + ps[1][tid]) + (ps[2][tid] + ps[3][tid])) * (1.0f / (float)sh.b));
      }
      pending = -1;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 16 * wv + r;
        const uint32_t x = *(const uint32_t *)((const char *)Kt + row * 256 +
                                               ((((cd >> 2) ^ r) << 4) | ((cd & 3) << 2)));
        ks_lo += bf16_bits_to_f32(x & 0xFFFFu);
        ks_hi += bf16_bits_to_f32(x >> 16);
      }
      if ((t + 1) % tpb == 0) {
        const int C = j0 / sh.b;
        *(float2 *)&ksum[C & 1][wv][2 * cd] = make_float2(ks_lo, ks_hi);
        ks_lo = 0.f; ks_hi = 0.f;
        pending = C;
      }
    }

    // One 32-key half of the tile at a time: its scores are reduced to (max, sum) before the next
    // half is multiplied, so only 32 accumulator registers are live (two waves per SIMD fit).
    // lane = query 32qh+q ; acc[qh][r] <-> key j0 + 32kh + 8(r/4) + 4gg + r%4
    const bool tail = j0 + 63 > sh.N - sh.w;  // causal masking only in the last tile of the sequence
#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
      f32x16 acc[2];  // [query half]
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[qh][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = k_frag(Kt, kbase, gg, kh, ks);
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
          acc[qh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qh][ks], acc[qh], 0, 0, 0);
      }
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) {
        float tmax = -INFINITY;
        if (tail) {
          const int jmax = sh.N - sh.w + 32 * qh + q;  // last visible key of this window row
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = j0 + 32 * kh + 8 * (r / 4) + 4 * gg + (r % 4);
            if (j > jmax) acc[qh][r] = -INFINITY;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, acc[qh][r]);
        // the reference moves only when a row's maximum grew by more than 2^8 (terms stay <= 256)
        const float m_new = fmaxf(m[qh], tmax * c);
        if (__any(m_new - m[qh] > 8.f)) {
          z[qh] *= __builtin_amdgcn_exp2f(m[qh] - ((m_new == -INFINITY) ? 0.f : m_new));
          m[qh] = m_new;
        }
        const float m_ref = (m[qh] == -INFINITY) ? 0.f : m[qh];
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[qh][r], c, -m_ref));
        z[qh] += sum;
      }
    }
  }
  if (do_means) {
    __syncthreads();
    if (pending >= 0 && tid < kHeadDim) {
      const float(*ps)[kHeadDim] = ksum[pending & 1];
      store_split(kblk + (size_t)kvh * means_tiles(sh.nb) * 2048, pending, tid,
                  ((ps[0][tid] + ps[1][tid]) + (ps[2][tid] + ps[3][tid])) * (1.0f / (float)sh.b));
    }
  }
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    const float mp = __shfl_xor(m[qh], 32), zp = __shfl_xor(z[qh], 32);
    const float M = fmaxf(m[qh], mp);
    float Z = 0.f;
    if (M != -INFINITY) {
      if (m[qh] != -INFINITY) Z += z[qh] * __builtin_amdgcn_exp2f(m[qh] - M);
      if (mp != -INFINITY) Z += zp * __builtin_amdgcn_exp2f(mp - M);
    }
    const int i = 32 * qh + q;
    if (head_ok && gg == 0 && i < sh.w)
      part[((size_t)hq * sh.nchunks + chunk) * kWin + i] = make_float2(M, Z);
  }
}

// combine the per-chunk partials into bias[i] = max_i + log2(sum_i) (log2 domain), so that a
// window weight is exp2(logit * scale * log2e - bias).  Rows past the window get +inf (weight 0).
// grid (Hq, 4), 1024 threads = 64 chunk slices x 16 window rows.
__global__ __launch_bounds__(1024) void window_stats_reduce_kernel(const float2 *__restrict__ part,
                                                                  int nchunks, int w,
                                                                  float *__restrict__ bias) {
  __shared__ float red[64][17];
  const int hq = blockIdx.x, il = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int i = 16 * blockIdx.y + il;
  const float2 *p = part + (size_t)hq * nchunks * kWin + i;
  float M = -INFINITY;
  if (i < w)
    for (int cidx = sl; cidx < nchunks; cidx += 64) M = fmaxf(M, p[(size_t)cidx * kWin].x);
  red[sl][il] = M;
  __syncthreads();
  float Mt = -INFINITY;
#pragma unroll 16
  for (int k = 0; k < 64; ++k) Mt = fmaxf(Mt, red[k][il]);
  __syncthreads();
  float Z = 0.f;
  if (i < w)
    for (int cidx = sl; cidx < nchunks; cidx += 64) {
      const float2 e = p[(size_t)cidx * kWin];
      if (e.x != -INFINITY) Z += e.y * __builtin_amdgcn_exp2f(e.x - Mt);
    }
  red[sl][il] = Z;
  __syncthreads();
  if (sl == 0) {
    float Zt = 0.f;
#pragma unroll 16
    for (int k = 0; k < 64; ++k) Zt += red[k][il];
    bias[(size_t)hq * kWin + i] = i < w ? Mt + __builtin_amdgcn_logf(Zt) : INFINITY;  // v_log_f32 = log2
  }
}

// Lane shifts of a whole wavefront (DPP wave_shl:1 / wave_shr:1): lane l takes lane l+1 (l-1);
// the lane without a source gets 0.
__device__ inline float wave_shl1(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x130, 0xF, 0xF, true));
}
__device__ inline float wave_shr1(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x138, 0xF, 0xF, true));
}

// Weights of one 64-key tile (pass 2).  After the MFMAs lane l holds key 32kh + l%32 and
// register r of acc[kh][qh] window row 32qh + 8(r/4) + 4(l/32) + r%4.  v_permlane32_swap of
// the two key halves turns that into "register = one window row, lane = key 0..63": the row
// constants are wave-uniform and the column sum stays in the lane.
//
// Diagonal sums without LDS: the rows are taken in DESCENDING order, step tau = 64*tile + 63 - i,
// so that the offset of element (i, lane l) is A - (tau + l) for a chunk constant A.  `run`
// shifts one lane down per step (run[l] <- run[l+1] + weight): a slot then collects exactly one
// offset over 64 consecutive steps, is complete when it reaches lane 0, and `done` picks it up
// there while shifting the other way, so that after the 64 rows of a tile done[l] is the finished
// sum of offset (N - w - j0) + l.  Sums that straddle a chunk boundary are the only partial ones.
template <bool TAIL>
__device__ inline float scores_tile(const f32x16 (&acc)[2][2], const float (&bias)[kWin], float c,
                                    int lim0, bool lane0, float &run, float &done) {
  float colsum = 0.f;
#pragma unroll
  for (int qh = 1; qh >= 0; --qh)
#pragma unroll
    for (int rq = 3; rq >= 0; --rq) {
      float x[2][4];
#pragma unroll
      for (int rm = 0; rm < 4; ++rm) {
        const auto pr = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[0][qh][4 * rq + rm]),
                                                         __float_as_uint(acc[1][qh][4 * rq + rm]), false, false);
        x[0][rm] = __uint_as_float(pr[0]);
        x[1][rm] = __uint_as_float(pr[1]);
      }
#pragma unroll
      for (int u = 1; u >= 0; --u)
#pragma unroll
        for (int rm = 3; rm >= 0; --rm) {
          const int i = 32 * qh + 8 * rq + 4 * u + rm;
          float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x[u][rm], c, -bias[i]));
          if (TAIL) e = (lim0 + i >= 0) ? e : 0.f;  // key j0 + lane visible to row i iff j <= N-w+i
          colsum += e;
          run = wave_shl1(run) + e;
          const float up = wave_shr1(done);  // a cross-lane move: never under a lane condition
          done = lane0 ? run : up;
        }
    }
  return colsum;
}

// pass 2: grid (nchunks, Hkv, ceil(g/4)), 256 threads.  Chunks are walked in the reverse order
// of pass 1, so that the most recently streamed part of K is re-read first.
__global__ __launch_bounds__(256) void window_scores_kernel(const uint16_t *__restrict__ Q,
                                                            const uint16_t *__restrict__ K, Shape sh,
                                                            float c, const float *__restrict__ bias_g,
                                                            float *__restrict__ v_out,
                                                            float *__restrict__ s_out) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kStages][64 * 128];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane & 31, gg = lane >> 5;
  const int chunk = sh.nchunks - 1 - (int)blockIdx.x, kvh = sh.Hkv - 1 - (int)blockIdx.y;
  const int hsub = 4 * blockIdx.z + wv;
  const bool head_ok = hsub < sh.g;
  const int hq = kvh * sh.g + (head_ok ? hsub : 0);
  const int jc0 = chunk * sh.chunk;
  const int jc1 = min(jc0 + sh.chunk, sh.N);
  const int nt = (jc1 - jc0) >> 6;
  const uint16_t *Kh = K + (size_t)kvh * sh.kv_hs + (size_t)jc0 * sh.kv_rs;

  KTileCopy cp;
  cp.init(&Ks[0][0], wv, lane, sh.kv_rs);
  cp.issue(Kh, 0);

  bf16x8 qf[2][8];
  load_qwin(Q, sh, hq, lane, qf);
  float bias[kWin];  // wave-uniform: lives in scalar registers
#pragma unroll
  for (int i = 0; i < kWin; ++i)
    bias[i] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(bias_g[(size_t)hq * kWin + i])));
#pragma unroll
  for (int s2 = 1; s2 < kStages - 1; ++s2)
    if (s2 < nt) cp.issue(Kh + (size_t)s2 * 64 * sh.kv_rs, s2);
  const unsigned kbase = (unsigned)(q * 256) | (unsigned)((q & 15) << 4);
  float *srow = s_out + (size_t)hq * sh.N;
  float run = 0.f, done = 0.f;
  float cv = c;  // in a vector register: an FMA takes only one scalar operand, and that is the row's bias
  asm volatile("" : "+v"(cv));

  for (int t = 0; t < nt; ++t) {
    const int cur = t % kStages;
    // the stores of the previous tiles count like the copies: they only make the wait longer
    wait_tile(min(nt - 1 - t, kStages - 2));
    __syncthreads();
    if (t + kStages - 1 < nt)
      cp.issue(Kh + (size_t)(t + kStages - 1) * 64 * sh.kv_rs, (t + kStages - 1) % kStages);
    const uint16_t *Kt = Ks[cur];
    const int j0 = jc0 + 64 * t;

    f32x16 acc[2][2];  // [key half][query half]
#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[kh][qh][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = k_frag(Kt, kbase, gg, kh, ks);
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
          acc[kh][qh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[qh][ks], kf, acc[kh][qh], 0, 0, 0);
      }
    }
    float colsum;
    if (j0 + 63 > sh.N - sh.w)
      colsum = scores_tile<true>(acc, bias, cv, sh.N - sh.w - j0 - lane, lane == 0, run, done);
    else
      colsum = scores_tile<false>(acc, bias, cv, 0, lane == 0, run, done);
    if (head_ok) {
      v_out[(size_t)hq * sh.N + j0 + lane] = colsum;
      // The first tile's sums lack the previous chunk's rows (all but lane 0): they are added to
      // the zeroed slot, as is that chunk's remainder below.  Every offset so receives at most
      // two partial sums, so the result does not depend on the order of the atomics.
      const int o = sh.N - sh.w - j0 + lane;
      if (o < sh.N) {
        if (t == 0) atomicAdd(&srow[o], done);
        else srow[o] = done;
      }
    }
  }
  // what is left in `run` belongs to the next chunk's first tile: lane l holds offset
  // (N - w - jc1) + 64 - l, l = 1..63
  if (head_ok && lane > 0) {
    const int o = sh.N - sh.w - jc1 + 64 - lane;
    if (o >= 0 && o < sh.N) atomicAdd(&srow[o], run);
  }
}

// ------------------------------------------------------------------ block map
// blk[h][R][C] = softmax over C <= R of scale * Qblk[R].Kblk[C]; entries C > R are 0.
// One workgroup = 16 rows of one head.  The means arrive split into bf16 head + remainder (see
// store_split), and v_mfma_f32_16x16x32_bf16 forms the 16x16 logit tiles from head x head and the
// two cross products: fp32-grade logits (a bf16 product alone would break the 1e-3 tolerance of
// blk) at a fifth of the cycles of the fp32 matrix instruction.  Lane l of a tile: column l%16,
// rows 4(l/16) + r.  The column tiles of the strip go round-robin to the eight waves and stay in
// registers (MT tiles per wave) until the row maxima and sums are known, so blk is written exactly
// once.  Eight waves (and few registers each) rather than four: the operand reads come from
// another XCD's writes, and only occupancy hides them.
// grid ceil(nb/16) * Hq, 512 threads; strips are taken longest first.
constexpr int kMapWaves = 8;

template <int MT>
__global__ __launch_bounds__(64 * kMapWaves, (MT <= 8 ? 4 : 2)) void block_map_kernel(const float *__restrict__ qblk,
                                                                   const float *__restrict__ kblk,
                                                                   Shape sh, float c2,
                                                                   float *__restrict__ blk,
                                                                   const int32_t *__restrict__ only_bc) {
  __shared__ float red[2][kMapWaves][16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int nb = sh.nb;
  // Consecutive workgroup ids land on consecutive XCDs.  While Hkv is a multiple of 8, KV head k
  // is served by XCD k % 8 only, so that the L2 of an XCD holds the block means of one KV head at
  // a time instead of all of them.
  const int nstrips = (nb + 15) / 16;
  const int L = blockIdx.x;
  int strip, h;
  if (sh.Hkv % 8 == 0) {
    const int x = L & 7, s = L >> 3, hx = sh.Hq / 8;  // hx heads per XCD
    const int hl = s % hx;
    strip = nstrips - 1 - s / hx;
    h = (x + 8 * (hl / sh.g)) * sh.g + hl % sh.g;
  } else {
    strip = nstrips - 1 - L % nstrips;
    h = L / nstrips;
  }
  if (only_bc && only_bc[h] != SA_BLOCK_CLUSTER) return;  // uniform over the workgroup, before any barrier
  const int R0 = 16 * strip;
  const int T = strip + 1;  // column tiles 0..strip hold every C <= R of this strip
  // tile t of a means array: 8 KB = [part][st][lane][16 bytes]
  const uint16_t *qsrc = (const uint16_t *)(qblk + (size_t)h * means_tiles(nb) * 2048) + 8 * lane;
  const uint16_t *ksrc = (const uint16_t *)(kblk + (size_t)(h / sh.g) * means_tiles(nb) * 2048) + 8 * lane;

  // operands of v_mfma_f32_16x16x32_bf16: lane (n = row of A / column of B, g) holds elements
  // 32 st + 8 g .. + 7 of its mean, st = 0..3: 16 bytes of heads and 16 bytes of remainders per step,
  // which is the order the means are stored in
  bf16x8 ah[4], al[4];
  {
    const uint16_t *ap = qsrc + (size_t)strip * 4096;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      ah[st] = *(const bf16x8 *)(ap + 512 * st);
      al[st] = *(const bf16x8 *)(ap + 2048 + 512 * st);
    }
  }
  f32x4 acc[MT];
  bf16x8 bh[4], bl[4];
#pragma unroll
  for (int k = 0; k < MT; ++k) {
    const int tc = kMapWaves * k + wv;
    if (tc < T) {
      {
        const uint16_t *bp = ksrc + (size_t)tc * 4096;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          bh[st] = *(const bf16x8 *)(bp + 512 * st);
          bl[st] = *(const bf16x8 *)(bp + 2048 + 512 * st);
        }
      }
      // three independent chains: heads x heads, and the two cross terms (remainder x remainder,
      // about 2^-18 of the product, is dropped)
      f32x4 dhh = {0.f, 0.f, 0.f, 0.f}, dhl = dhh, dlh = dhh;
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        dhh = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[st], bh[st], dhh, 0, 0, 0);
        dhl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[st], bl[st], dhl, 0, 0, 0);
        dlh = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[st], bh[st], dlh, 0, 0, 0);
      }
      const f32x4 d = dhh + (dhl + dlh);
      const int C = 16 * tc + n;
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[k][r] = (C <= R0 + 4 * g + r) ? d[r] * c2 : -INFINITY;
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[k][r] = -INFINITY;
    }
  }
  // row maxima: over this lane's tiles, the 16 lanes of a group, the eight waves
  float mx[4], sm[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float v = -INFINITY;
#pragma unroll
    for (int k = 0; k < MT; ++k) v = fmaxf(v, acc[k][r]);
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
    mx[r] = v;
  }
  if (n == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[0][wv][4 * g + r] = mx[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float v = red[0][0][4 * g + r];
#pragma unroll
    for (int k = 1; k < kMapWaves; ++k) v = fmaxf(v, red[0][k][4 * g + r]);
    mx[r] = v;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < MT; ++k) {
      acc[k][r] = __builtin_amdgcn_exp2f(acc[k][r] - mx[r]);  // column 0 is kept in every row: mx is finite
      v += acc[k][r];
    }
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    sm[r] = v;
  }
  if (n == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) red[1][wv][4 * g + r] = sm[r];
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float v = red[1][0][4 * g + r];
#pragma unroll
    for (int k = 1; k < kMapWaves; ++k) v += red[1][k][4 * g + r];
    sm[r] = 1.0f / v;
  }
  float *dst = blk + (size_t)h * nb * nb;
#pragma unroll
  for (int k = 0; k < MT; ++k) {
    const int tc = kMapWaves * k + wv;
    if (tc < T) {
      const int C = 16 * tc + n;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int R = R0 + 4 * g + r;
        if (R < nb && C < nb) dst[(size_t)R * nb + C] = acc[k][r] * sm[r];
      }
    }
  }
  // zeros right of the strip's last tile (16 bytes per lane where the rows allow it)
  const int c0 = 16 * T;
  if ((nb & 3) == 0) {
    const int n4 = (nb - c0) >> 2, rows = min(16, nb - R0);
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = tid; i < rows * n4; i += 64 * kMapWaves) {
      const int r = i / n4, c4 = i - r * n4;
      *(float4 *)(dst + (size_t)(R0 + r) * nb + c0 + 4 * c4) = z4;
    }
  } else {
    for (int r = 0; r < 16; ++r) {
      const int R = R0 + r;
      if (R >= nb) break;
      for (int C = c0 + tid; C < nb; C += 64 * kMapWaves) dst[(size_t)R * nb + C] = 0.f;
    }
  }
}

}  // namespace

namespace {

void launch_q_block_mean(const Shape &sh, const Workspace &ws, const uint16_t *Q, const int32_t *only_bc,
                         hipStream_t sq) {
  if (sh.b == 128)
    q_block_mean_kernel<8><<<dim3(sh.nb, sh.Hq), 256, kQMeanLdsPad128, sq>>>(Q, sh, ws.qblk, only_bc);
  else
    q_block_mean_kernel<4><<<dim3(sh.nb, sh.Hq), 256, kQMeanLdsPad64, sq>>>(Q, sh, ws.qblk, only_bc);
}

void launch_block_map(const Shape &sh, const Workspace &ws, float c, float *blk, const int32_t *only_bc,
                      hipStream_t sq) {
  const dim3 bgrid((sh.nb + 15) / 16 * sh.Hq);
  const int tiles_per_wave = ((sh.nb + 15) / 16 + kMapWaves - 1) / kMapWaves;
  if (tiles_per_wave <= 8)
    block_map_kernel<8><<<bgrid, 64 * kMapWaves, 0, sq>>>(ws.qblk, ws.kblk, sh, c, blk, only_bc);
  else if (tiles_per_wave <= 16)
    block_map_kernel<16><<<bgrid, 64 * kMapWaves, 0, sq>>>(ws.qblk, ws.kblk, sh, c, blk, only_bc);
  else
    block_map_kernel<32><<<bgrid, 64 * kMapWaves, 0, sq>>>(ws.qblk, ws.kblk, sh, c, blk, only_bc);
}

}  // namespace

hipError_t launch_estimate_part(const Shape &sh, const Workspace &ws, const uint16_t *Q, const uint16_t *K,
                                sa_scores out, EstimatePart part, const int32_t *only_block_cluster,
                                hipStream_t st) {
  const float c = sh.scale * kLog2e;
  float *bias = (float *)ws.stats;
  if (part != EstimatePart::QChain) {
    const dim3 wgrid(sh.nchunks, sh.Hkv, (sh.g + 3) / 4);
    window_stats_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, ws.part, out.s, ws.kblk);
    window_stats_reduce_kernel<<<dim3(sh.Hq, kWin / 16), 1024, 0, st>>>(ws.part, sh.nchunks, sh.w, bias);
    window_scores_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, bias, out.v, out.s);
  }
  if (part != EstimatePart::KChain) {
    launch_q_block_mean(sh, ws, Q, only_block_cluster, st);
    launch_block_map(sh, ws, c, out.blk, only_block_cluster, st);
  }
  return hipGetLastError();
}

hipError_t launch_estimate(const Shape &sh, const Workspace &ws, const uint16_t *Q,
                           const uint16_t *K, sa_scores out, hipStream_t st, const Fork &fk,
                           bool join_back) {
  const float c = sh.scale * kLog2e;
  float *bias = (float *)ws.stats;
  // Two chains with complementary limits run side by side: the Q chain (block means of Q: HBM
  // bandwidth; block map: latency of many small L2 reads) on the context's side stream, the K
  // chain (both window passes: exp and vector ALU work on a quarter of the bytes) on the caller's
  // stream.  The side stream forks from the caller's stream at entry and joins it at exit, so
  // towards the caller the call behaves like a sequence of kernels on the given stream
  // (join_back == false: the caller of this function goes on using both streams and joins them
  // itself).
  hipStream_t sq = st;
  hipError_t e = hipSuccess;
  bool forked = false;
  if (fk.aux) {
    if ((e = hipEventRecord(fk.fork, st)) != hipSuccess) return e;
    if ((e = hipStreamWaitEvent(fk.aux, fk.fork, 0)) != hipSuccess) return e;
    sq = fk.aux;
    forked = true;
  }
  // From here on the side stream depends on the caller's stream: whatever fails below, it is joined
  // back before the call returns, so that no later call (or an active capture) sees it dangling.
  launch_q_block_mean(sh, ws, Q, nullptr, sq);
  const dim3 wgrid(sh.nchunks, sh.Hkv, (sh.g + 3) / 4);
  window_stats_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, ws.part, out.s, ws.kblk);
  if (forked) {  // the block map needs the K block means of the stats pass
    e = hipEventRecord(fk.mid, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(fk.aux, fk.mid, 0);
  }
  if (e == hipSuccess) {
    launch_block_map(sh, ws, c, out.blk, nullptr, sq);
    window_stats_reduce_kernel<<<dim3(sh.Hq, kWin / 16), 1024, 0, st>>>(ws.part, sh.nchunks, sh.w, bias);
    window_scores_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, bias, out.v, out.s);
  }
  if (forked && (join_back || e != hipSuccess)) {
    hipError_t j = hipEventRecord(fk.join, fk.aux);
    if (j == hipSuccess) j = hipStreamWaitEvent(st, fk.join, 0);
    if (e == hipSuccess) e = j;
  }
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace sa
