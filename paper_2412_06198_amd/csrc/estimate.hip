// Pattern estimator for gfx950.
//
//  * window scores (Alg. 2 "Compute Dense Attention Scores" on the last w query
//    rows only, then SumRows -> v and SumDiagonals -> s).  The softmax of a
//    window row needs its maximum and normaliser over ALL keys before any
//    column can be summed, so K is streamed twice:
//      pass 1  S^T = K Qwin^T  (lane = query)  -> per-chunk (max, sum) partials
//      pass 2  S   = Qwin K^T  (lane = key)    -> normalised weights, column sums,
//                                                 diagonal sums through LDS
//    The 4 query heads of a GQA group ride on one K stream: wave w = head w.
//  * block map (Alg. 3 "Compute Blocked Representation"): fp32 block means of Q
//    and K, an fp32 register-tiled GEMM for the block logits, a row softmax.
#include "sa_internal.h"

namespace sa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KS = 136;  // LDS row stride (16-bit elements) of a K tile

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// ------------------------------------------------------------------ block means
// grid (nb, Hq + Hkv), 256 threads: thread = (row group of 16, 16-byte column).
__global__ __launch_bounds__(256) void block_mean_kernel(const uint16_t *Q, const uint16_t *K,
                                                         Shape sh, float *qblk, float *kblk) {
  __shared__ float red[16][kHeadDim + 4];
  const int R = blockIdx.x, hh = blockIdx.y, tid = threadIdx.x;
  const bool isq = hh < sh.Hq;
  const int64_t rs = isq ? sh.q_rs : sh.kv_rs;
  const uint16_t *src = isq ? Q + (size_t)hh * sh.q_hs : K + (size_t)(hh - sh.Hq) * sh.kv_hs;
  src += (size_t)R * sh.b * rs;
  const int cc = tid & 15, rg = tid >> 4;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int r = rg; r < sh.b; r += 16) {
    const uint4 x = *(const uint4 *)(src + (size_t)r * rs + cc * 8);
    const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
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
    float *dst = isq ? qblk + ((size_t)hh * sh.nb + R) * kHeadDim
                     : kblk + ((size_t)(hh - sh.Hq) * sh.nb + R) * kHeadDim;
    dst[tid] = sum * (1.0f / (float)sh.b);
  }
}

// ------------------------------------------------------------------ window passes
// Q window fragments of one head: lane (q = lane%32, gg = lane/32) holds window row
// 32*qh + q, elements d = 16*ks + 8*gg .. +7.  The same registers serve as the B operand
// of K Q^T (pass 1) and as the A operand of Q K^T (pass 2).
__device__ inline void load_qwin(const uint16_t *Q, const Shape &sh, int hq, int lane,
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

// 64 keys x 128 d of K into LDS (rows past N are clamped; callers mask them).
__device__ inline void stage_k_tile(const uint16_t *Kh, const Shape &sh, int j0, int tid,
                                    uint16_t *Ks) {
  const int lrow = tid >> 4, lcc = tid & 15;
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    const int row = lrow + 16 * n;
    const int src = min(j0 + row, sh.N - 1);
    *(uint4 *)&Ks[row * KS + lcc * 8] = *(const uint4 *)(Kh + (size_t)src * sh.kv_rs + lcc * 8);
  }
}

// pass 1: grid (nchunks, Hkv, ceil(g/4)), 256 threads.
__global__ __launch_bounds__(256) void window_stats_kernel(const uint16_t *Q, const uint16_t *K,
                                                           Shape sh, float c, float2 *part,
                                                           float *s_out) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * KS];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int q = lane & 31, gg = lane >> 5;
  const int chunk = blockIdx.x, kvh = blockIdx.y;
  const int hsub = 4 * blockIdx.z + wv;
  const bool head_ok = hsub < sh.g;
  const int hq = kvh * sh.g + (head_ok ? hsub : 0);
  const int jc0 = chunk * kChunk;
  const int jc1 = min(jc0 + kChunk, sh.N);
  const uint16_t *Kh = K + (size_t)kvh * sh.kv_hs;

  // the slash scores are accumulated with atomics in pass 2: clear this chunk's share now
  if (head_ok)
    for (int j = jc0 + lane; j < jc1; j += 64) s_out[(size_t)hq * sh.N + j] = 0.f;

  bf16x8 qf[2][8];
  load_qwin(Q, sh, hq, lane, qf);
  float m[2] = {-INFINITY, -INFINITY}, z[2] = {0.f, 0.f};

  for (int j0 = jc0; j0 < jc1; j0 += 64) {
    __syncthreads();
    stage_k_tile(Kh, sh, j0, tid, Ks);
    __syncthreads();
    f32x16 acc[2][2];  // [key half][query half]
#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[kh][qh][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *(const bf16x8 *)&Ks[(32 * kh + q) * KS + 16 * ks + 8 * gg];
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
          acc[kh][qh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qh][ks], acc[kh][qh], 0, 0, 0);
      }
    }
    // lane = query 32qh+q ; acc[kh][qh][r] <-> key j0 + 32kh + 8(r/4) + 4gg + r%4
    const bool tail = j0 + 63 > sh.N - sh.w;  // causal / end-of-sequence masking only near the end
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      const int jmax = sh.N - sh.w + 32 * qh + q;  // last visible key of this window row
      float tmax = -INFINITY;
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (tail) {
            const int j = j0 + 32 * kh + 8 * (r / 4) + 4 * gg + (r % 4);
            if (j > jmax) acc[kh][qh][r] = -INFINITY;
          }
          tmax = fmaxf(tmax, acc[kh][qh][r]);
        }
      const float m_new = fmaxf(m[qh], tmax * c);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      float sum = 0.f;
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[kh][qh][r], c, -m_safe));
      z[qh] = z[qh] * __builtin_amdgcn_exp2f(m[qh] - m_safe) + sum;
      m[qh] = m_new;
    }
  }
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    const float mp = __shfl_xor(m[qh], 32), zp = __shfl_xor(z[qh], 32);
    const float M = fmaxf(m[qh], mp);
    float Z = 0.f;
    if (M != -INFINITY) Z = z[qh] * __builtin_amdgcn_exp2f(m[qh] - M) + zp * __builtin_amdgcn_exp2f(mp - M);
    const int i = 32 * qh + q;
    if (head_ok && gg == 0 && i < sh.w)
      part[((size_t)hq * sh.nchunks + chunk) * kWin + i] = make_float2(M, Z);
  }
}

// combine the per-chunk partials: grid Hq, 1024 threads = 16 chunk slices x 64 window rows.
__global__ __launch_bounds__(1024) void window_stats_reduce_kernel(const float2 *part, int nchunks,
                                                                  int w, float2 *stats) {
  __shared__ float2 red[16][kWin];
  const int hq = blockIdx.x, i = threadIdx.x & 63, sl = threadIdx.x >> 6;
  const float2 *p = part + (size_t)hq * nchunks * kWin + i;
  float M = -INFINITY, Z = 0.f;
  if (i < w)
    for (int cidx = sl; cidx < nchunks; cidx += 16) {
      const float2 e = p[(size_t)cidx * kWin];
      if (e.x == -INFINITY) continue;
      const float Mn = fmaxf(M, e.x);
      Z = Z * __builtin_amdgcn_exp2f(M - Mn) + e.y * __builtin_amdgcn_exp2f(e.x - Mn);
      M = Mn;
    }
  red[sl][i] = make_float2(M, Z);
  __syncthreads();
  if (sl == 0) {
    if (i >= w) { stats[(size_t)hq * kWin + i] = make_float2(INFINITY, 0.f); return; }
    float Mt = -INFINITY;
    for (int k = 0; k < 16; ++k) Mt = fmaxf(Mt, red[k][i].x);
    float Zt = 0.f;
    for (int k = 0; k < 16; ++k)
      if (red[k][i].x != -INFINITY) Zt += red[k][i].y * __builtin_amdgcn_exp2f(red[k][i].x - Mt);
    stats[(size_t)hq * kWin + i] = make_float2(Mt, 1.0f / Zt);
  }
}

// pass 2: grid (nchunks, Hkv, ceil(g/4)), 256 threads.
__global__ __launch_bounds__(256) void window_scores_kernel(const uint16_t *Q, const uint16_t *K,
                                                            Shape sh, float c, const float2 *stats,
                                                            float *v_out, float *s_out) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * KS];
  __shared__ float sdiag[4][kChunk + kWin];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int q = lane & 31, gg = lane >> 5;
  const int chunk = blockIdx.x, kvh = blockIdx.y;
  const int hsub = 4 * blockIdx.z + wv;
  const bool head_ok = hsub < sh.g;
  const int hq = kvh * sh.g + (head_ok ? hsub : 0);
  const int jc0 = chunk * kChunk;
  const int jc1 = min(jc0 + kChunk, sh.N);
  const uint16_t *Kh = K + (size_t)kvh * sh.kv_hs;

  for (int i = lane; i < kChunk + kWin; i += 64) sdiag[wv][i] = 0.f;

  bf16x8 qf[2][8];
  load_qwin(Q, sh, hq, lane, qf);
  // this lane's window rows: i(qh,r) = 32qh + 8(r/4) + 4gg + r%4
  float mrow[2][16], zinv[2][16];
#pragma unroll
  for (int qh = 0; qh < 2; ++qh)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 32 * qh + 8 * (r / 4) + 4 * gg + (r % 4);
      const float2 st = stats[(size_t)hq * kWin + i];
      mrow[qh][r] = st.x;
      zinv[qh][r] = i < sh.w ? st.y : 0.f;  // rows past the window contribute nothing
    }

  for (int j0 = jc0; j0 < jc1; j0 += 64) {
    __syncthreads();
    stage_k_tile(Kh, sh, j0, tid, Ks);
    __syncthreads();
#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
      f32x16 acc[2];
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[qh][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = *(const bf16x8 *)&Ks[(32 * kh + q) * KS + 16 * ks + 8 * gg];
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
          acc[qh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[qh][ks], kf, acc[qh], 0, 0, 0);
      }
      // lane = key j ; acc[qh][r] <-> window row i(qh,r)
      const int j = j0 + 32 * kh + q;
      float colsum = 0.f;
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 32 * qh + 8 * (r / 4) + 4 * gg + (r % 4);
          float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[qh][r], c, -mrow[qh][r])) * zinv[qh][r];
          if (j > sh.N - sh.w + i || j >= sh.N) pe = 0.f;
          colsum += pe;
          // diagonal offset o = (N-w+i) - j ; slot = o - (N-w - (jc0+kChunk-1)) = i + jc0+kChunk-1 - j.
          // Lanes (q,0) and (q+4,1) hold the same offset: fold the partner in first, so that
          // every lane that writes owns its slot and the summation order is fixed.
          const float partner = __shfl(pe, 32 + ((q + 4) & 31));
          const int slot = i + (jc0 + kChunk - 1 - j);
          if (gg == 0) sdiag[wv][slot] += (q < 28) ? pe + partner : pe;
          else if (q < 4) sdiag[wv][slot] += pe;
        }
      colsum += __shfl_xor(colsum, 32);
      if (head_ok && gg == 0 && j < sh.N) v_out[(size_t)hq * sh.N + j] = colsum;
    }
  }
  // every offset receives at most two partial sums (this chunk and one neighbour), so the
  // floating-point result does not depend on the order of the atomics
  if (head_ok) {
    const int obase = sh.N - sh.w - (jc0 + kChunk - 1);
    for (int i = lane; i < kChunk + kWin; i += 64) {
      const int o = obase + i;
      const float val = sdiag[wv][i];
      if (o >= 0 && o < sh.N && val != 0.f) atomicAdd(&s_out[(size_t)hq * sh.N + o], val);
    }
  }
}

// ------------------------------------------------------------------ block map
// raw block logits scale * Qblk[R].Kblk[C] for the tiles on or below the diagonal.
// grid (nb/64 rounded up, nb/64 rounded up, Hq), 256 threads, 4x4 outputs per thread.
__global__ __launch_bounds__(256) void block_logits_kernel(const float *qblk, const float *kblk,
                                                           Shape sh, float *blk) {
  __shared__ __attribute__((aligned(16))) float Qt[64][68];  // [k][row]
  __shared__ __attribute__((aligned(16))) float Kt[64][68];  // [k][col]
  const int tc = blockIdx.x, tr = blockIdx.y, h = blockIdx.z;
  if (tc > tr) return;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int nb = sh.nb;
  const float *qsrc = qblk + (size_t)h * nb * kHeadDim;
  const float *ksrc = kblk + (size_t)(h / sh.g) * nb * kHeadDim;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < kHeadDim; k0 += 64) {
    __syncthreads();
    // 64 rows x 64 k = 1024 float4 per matrix; thread moves 4 of each
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const int idx = tid + 256 * n;
      const int row = idx >> 4, kq = (idx & 15) * 4;
      const int R = min(tr * 64 + row, nb - 1), C = min(tc * 64 + row, nb - 1);
      const float4 a = *(const float4 *)(qsrc + (size_t)R * kHeadDim + k0 + kq);
      const float4 b = *(const float4 *)(ksrc + (size_t)C * kHeadDim + k0 + kq);
      Qt[kq + 0][row] = a.x; Qt[kq + 1][row] = a.y; Qt[kq + 2][row] = a.z; Qt[kq + 3][row] = a.w;
      Kt[kq + 0][row] = b.x; Kt[kq + 1][row] = b.y; Kt[kq + 2][row] = b.z; Kt[kq + 3][row] = b.w;
    }
    __syncthreads();
#pragma unroll 8
    for (int k = 0; k < 64; ++k) {
      const float4 a = *(const float4 *)&Qt[k][ty * 4];
      const float4 b = *(const float4 *)&Kt[k][tx * 4];
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(av[i], bv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int R = tr * 64 + ty * 4 + i;
    if (R >= nb) continue;
    const int C = tc * 64 + tx * 4;
    float *dst = blk + ((size_t)h * nb + R) * nb + C;
    if ((nb & 3) == 0 && C + 3 < nb) {
      *(float4 *)dst = make_float4(acc[i][0] * sh.scale, acc[i][1] * sh.scale, acc[i][2] * sh.scale,
                                   acc[i][3] * sh.scale);
    } else {
      for (int j = 0; j < 4 && C + j < nb; ++j) dst[j] = acc[i][j] * sh.scale;
    }
  }
}

// in-place causal row softmax of the block logits; entries C > R become 0.
// grid (nb, Hq), 256 threads; rows hold at most kMaxSeq/64 = 4096 blocks.
__global__ __launch_bounds__(256) void block_softmax_kernel(Shape sh, float *blk) {
  __shared__ float red[4];
  const int R = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int nb = sh.nb;
  float *row = blk + ((size_t)h * nb + R) * nb;
  constexpr int PER = 16;
  constexpr float LOG2E = 1.4426950408889634f;
  float x[PER];
  float mx = -INFINITY;
#pragma unroll
  for (int n = 0; n < PER; ++n) {
    const int C = tid + 256 * n;
    x[n] = (C <= R && C < nb) ? row[C] * LOG2E : -INFINITY;
    mx = fmaxf(mx, x[n]);
  }
  for (int d = 32; d >= 1; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
  if (lane == 0) red[wv] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
#pragma unroll
  for (int n = 0; n < PER; ++n) {
    x[n] = __builtin_amdgcn_exp2f(x[n] - mx);
    sum += x[n];
  }
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d);
  if (lane == 0) red[wv] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int n = 0; n < PER; ++n) {
    const int C = tid + 256 * n;
    if (C < nb) row[C] = (C <= R) ? x[n] * inv : 0.f;
  }
}

}  // namespace

hipError_t launch_estimate(const Shape &sh, const Workspace &ws, const uint16_t *Q,
                           const uint16_t *K, sa_scores out, hipStream_t st) {
  const float c = sh.scale * 1.4426950408889634f;
  const dim3 wgrid(sh.nchunks, sh.Hkv, (sh.g + 3) / 4);
  window_stats_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, ws.part, out.s);
  window_stats_reduce_kernel<<<sh.Hq, 1024, 0, st>>>(ws.part, sh.nchunks, sh.w, ws.stats);
  window_scores_kernel<<<wgrid, 256, 0, st>>>(Q, K, sh, c, ws.stats, out.v, out.s);
  block_mean_kernel<<<dim3(sh.nb, sh.Hq + sh.Hkv), 256, 0, st>>>(Q, K, sh, ws.qblk, ws.kblk);
  const int nt = (sh.nb + 63) / 64;
  block_logits_kernel<<<dim3(nt, nt, sh.Hq), 256, 0, st>>>(ws.qblk, ws.kblk, sh, out.blk);
  block_softmax_kernel<<<dim3(sh.nb, sh.Hq), 256, 0, st>>>(sh, out.blk);
  return hipGetLastError();
}

}  // namespace sa
