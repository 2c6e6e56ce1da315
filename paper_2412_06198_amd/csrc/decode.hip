// One decode step over the prefill index (the paper names gains in the decoding phase without a
// method; problem statement: decode queries are [B, 1, H]).  The query at position pos >= N
// attends, per query head, the union of the generated keys N..pos, the selected key columns, the
// keys pos - o of the selected diagonal offsets and the keys of the key blocks kept for the last
// row block of the prompt, each key once.  A pure gather: 512 bytes of K and V per kept key and
// head, nothing reused, so the kernel is laid out for HBM: every key is read by 16 lanes as one
// 256-byte row of K and one of V, sixteen keys per workgroup step, the key list of a head split
// over several workgroups whose partial (max, sum, output) triples a second kernel merges.
#include <mutex>

#include "sa_internal.h"

namespace sa {
namespace {

constexpr int kPartStride = 132;  // floats per partial: max, sum, 2 unused, 128 outputs

// Partials of the variant that allocates nothing (sa_sparse_decode_static): room for the largest
// head count x split count the launcher ever picks (Hq * splits <= 512), 270336 bytes on every GPU
// the library runs on, held until the process ends.  In host code this name is only a stand-in for
// the symbol: the device address comes from hipGetSymbolAddress, once per device.
constexpr int kStaticPartials = 512;
static __device__ __align__(256) float scratch[kStaticPartials * kPartStride];
constexpr int kMaxDevices = 64;

struct DecArgs {
  const uint16_t *q, *K, *V;
  uint16_t *o;
  const int32_t *n_cols, *cols, *n_offs, *offs, *rowptr, *blkcols;
  float *part;
  int Hq, g, N, b, nb, k_v, k_s, cap_b, S, pos;
  int64_t kv_hs, kv_rs;
  float c;  // softmax scale * log2(e)
};

__device__ inline void unpack8(const uint4 x, float (&f)[8]) {
  const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = __uint_as_float(w[e] << 16);
    f[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
  }
}

// grid (S, Hq), 256 threads = 16 key slots of 16 lanes; lane ln of a slot owns elements 8 ln .. 8 ln + 7.
__global__ __launch_bounds__(256) void decode_partial_kernel(DecArgs p) {
  __shared__ uint32_t blkbm[kMaxSeq / 64 / 32];  // key blocks kept for the last row block
  __shared__ uint32_t colbm[kMaxSeq / 32];       // selected key columns
  __shared__ float sm[16], sl[16], so[16][kHeadDim];
  const int sp = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int N = p.N, nb = p.nb, b = p.b;
  const int32_t *rp = p.rowptr + (size_t)h * (nb + 1);
  const int32_t *bc = p.blkcols + (size_t)h * p.cap_b;
  const int32_t *colp = p.cols + (size_t)h * p.k_v;
  const int32_t *offp = p.offs + (size_t)h * p.k_s;
  const int e0 = min(max(rp[nb - 1], 0), p.cap_b), e1 = min(max(rp[nb], e0), p.cap_b);
  const int nblk = e1 - e0;
  const int nc = min(max(p.n_cols[h], 0), p.k_v), no = min(max(p.n_offs[h], 0), p.k_s);
  const int ns = p.pos - N + 1;
  const bool need_cols = no > 0 && nc > 0;  // the column bitmap only screens diagonal keys
  for (int i = tid; i < (nb + 31) / 32; i += 256) blkbm[i] = 0u;
  if (need_cols)
    for (int i = tid; i < N / 32; i += 256) colbm[i] = 0u;
  __syncthreads();
  for (int e = tid; e < nblk; e += 256) {
    const int C = bc[e0 + e];
    if (C >= 0 && C < nb) atomicOr(&blkbm[C >> 5], 1u << (C & 31));
  }
  if (need_cols)
    for (int i = tid; i < nc; i += 256) {
      const int c = colp[i];
      if (c >= 0 && c < N) atomicOr(&colbm[c >> 5], 1u << (c & 31));
    }
  __syncthreads();
  // the head's key list: block keys, columns, diagonal keys, generated keys; this workgroup's share
  const int n0 = nblk * b, n1 = n0 + nc, n2 = n1 + no, total = n2 + ns;
  const int chunk = ((total + p.S - 1) / p.S + 15) / 16 * 16;
  const int t_begin = min(sp * chunk, total), t_end = min(t_begin + chunk, total);
  const int slot = tid >> 4, ln = tid & 15;
  float qv[8];
  unpack8(*(const uint4 *)(p.q + (size_t)h * kHeadDim + ln * 8), qv);
  const uint16_t *Kh = p.K + (size_t)(h / p.g) * p.kv_hs + ln * 8;
  const uint16_t *Vh = p.V + (size_t)(h / p.g) * p.kv_hs + ln * 8;
  float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int t0 = t_begin; t0 < t_end; t0 += 16) {
    const int t = t0 + slot;
    int j = -1;  // a key counts where it first appears in the list
    if (t < t_end) {
      if (t < n0) {
        const int C = bc[e0 + t / b];
        if (C >= 0 && C < nb) j = C * b + t % b;
      } else if (t < n1) {
        const int c = colp[t - n0];
        if (c >= 0 && c < N && !((blkbm[(c / b) >> 5] >> ((c / b) & 31)) & 1u)) j = c;
      } else if (t < n2) {
        const int o = offp[t - n1];
        const int jj = p.pos - o;
        if (o >= 0 && jj >= 0 && jj < N && !((blkbm[(jj / b) >> 5] >> ((jj / b) & 31)) & 1u) &&
            !(need_cols && ((colbm[jj >> 5] >> (jj & 31)) & 1u)))
          j = jj;
      } else {
        j = N + (t - n2);
      }
    }
    if (j >= 0) {  // uniform over the 16 lanes of a slot
      float kf[8], vf[8];
      const uint4 kx = *(const uint4 *)(Kh + (size_t)j * p.kv_rs);
      const uint4 vx = *(const uint4 *)(Vh + (size_t)j * p.kv_rs);
      unpack8(kx, kf);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = __builtin_fmaf(kf[e], qv[e], dot);
#pragma unroll
      for (int d = 1; d < 16; d <<= 1) dot += __shfl_xor(dot, d);
      const float s = dot * p.c;
      const float m_new = fmaxf(m, s);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new), pv = __builtin_amdgcn_exp2f(s - m_new);
      unpack8(vx, vf);
      l = l * alpha + pv;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(acc[e], alpha, pv * vf[e]);
      m = m_new;
    }
  }
  if (ln == 0) { sm[slot] = m; sl[slot] = l; }
#pragma unroll
  for (int e = 0; e < 8; ++e) so[slot][ln * 8 + e] = acc[e];
  __syncthreads();
  if (tid < kHeadDim) {
    float M = -INFINITY;
#pragma unroll
    for (int k = 0; k < 16; ++k) M = fmaxf(M, sm[k]);
    float L = 0.f, O = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const float wgt = __builtin_amdgcn_exp2f(sm[k] - M);  // 0 for an empty slot
        L += sl[k] * wgt;
        O += so[k][tid] * wgt;
      }
    }
    float *dst = p.part + ((size_t)h * p.S + sp) * kPartStride;
    if (tid == 0) { dst[0] = M; dst[1] = L; }
    dst[4 + tid] = O;
  }
}

// grid Hq, 128 threads: merge the S <= 64 partials of a head, normalise, round to bf16.  The
// (max, sum) pairs are read by one lane each and all output reads of a thread are independent.
__global__ __launch_bounds__(kHeadDim) void decode_merge_kernel(DecArgs p) {
  __shared__ float wgt[64];
  __shared__ float s_L;
  const int h = blockIdx.x, tid = threadIdx.x;
  const float *src = p.part + (size_t)h * p.S * kPartStride;
  if (tid < 64) {
    const float mk = tid < p.S ? src[(size_t)tid * kPartStride] : -INFINITY;
    const float lk = tid < p.S ? src[(size_t)tid * kPartStride + 1] : 0.f;
    float M = mk;
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    const float w = mk == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mk - M);
    float L = lk * w;
    for (int d = 32; d >= 1; d >>= 1) L += __shfl_xor(L, d);
    wgt[tid] = w;
    if (tid == 0) s_L = L;
  }
  __syncthreads();
  float O = 0.f;
#pragma unroll 8
  for (int k = 0; k < p.S; ++k) O = __builtin_fmaf(src[(size_t)k * kPartStride + 4 + tid], wgt[k], O);
  const float L = s_L;
  const __bf16 r = (__bf16)(L > 0.f ? O / L : 0.f);
  p.o[(size_t)h * kHeadDim + tid] = __builtin_bit_cast(uint16_t, r);
}

}  // namespace

int decode_splits(const Shape &sh) {
  const int s = 512 / (sh.Hq > 0 ? sh.Hq : 1);  // about two workgroups per compute unit in all
  return s < 1 ? 1 : (s > 64 ? 64 : s);
}

size_t decode_partial_bytes(const Shape &sh) { return (size_t)sh.Hq * decode_splits(sh) * kPartStride * 4; }

size_t decode_static_bytes() { return sizeof(float) * kStaticPartials * kPartStride; }

// Device address of `scratch` on the current device: asked for once per device (each GPU holds its
// own copy of the array at its own address) and kept.
hipError_t decode_static_scratch(float **out) {
  static std::mutex mu;
  static float *ptr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    float *d = nullptr;
    e = hipGetSymbolAddress((void **)&d, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!d) return hipErrorInvalidSymbol;
    ptr[dev] = d;
  }
  *out = ptr[dev];
  return hipSuccess;
}

hipError_t launch_sparse_decode(const Shape &sh, float *partials, const uint16_t *q, const uint16_t *K,
                                const uint16_t *V, sa_index idx, int pos, uint16_t *o, hipStream_t st) {
  DecArgs a;
  a.q = q; a.K = K; a.V = V; a.o = o;
  a.n_cols = idx.n_cols; a.cols = idx.cols; a.n_offs = idx.n_offs; a.offs = idx.offs;
  a.rowptr = idx.rowptr; a.blkcols = idx.blkcols;
  a.part = partials;
  a.Hq = sh.Hq; a.g = sh.g; a.N = sh.N; a.b = sh.b; a.nb = sh.nb; a.k_v = sh.k_v; a.k_s = sh.k_s;
  a.cap_b = sh.cap_b; a.S = decode_splits(sh); a.pos = pos;
  a.kv_hs = sh.kv_hs; a.kv_rs = sh.kv_rs;
  a.c = sh.scale * 1.4426950408889634f;
  decode_partial_kernel<<<dim3(a.S, sh.Hq), 256, 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  decode_merge_kernel<<<sh.Hq, kHeadDim, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace sa
