// Index builder for gfx950: per-head pattern choice and top-k selection
// (Main Idea "Categorization of Attention Heads"; Alg. 2 TopK / CombineIndices;
// Alg. 3 TopKBlocks).
//
// Integer work only: scores are compared through their fp32 bit patterns (all
// scores are >= +0, so the unsigned order is the numeric order), ties go to the
// lower index, and the pattern rule sums floor(score * 2^30) in 64-bit integers.
// One workgroup of 1024 threads per head:
//   radix select (4 passes of 8 bits, LDS histogram) -> threshold key and the
//   number of threshold-valued candidates to take, then an ordered compaction
//   (wave ballots over index-ordered segments) that emits the selection
//   ascending by index - no sort anywhere.
#include "sa_internal.h"

namespace sa {
namespace {

constexpr int NT = 1024;
constexpr int NWAVE = NT / 64;
constexpr int kMaxNb = kMaxSeq / 64;

struct IdxArgs {
  const float *v, *s, *blk;
  Shape sh;
  Override ov;
  sa_index out;
};

struct Smem {
  unsigned hist[256];
  unsigned wave_a[NWAVE], wave_b[NWAVE];
  unsigned long long red64[NWAVE];
  unsigned sel_prefix, sel_remaining;
  unsigned rowgt[kMaxNb], roweq[kMaxNb];
};

// floor(x * 2^30) of a finite fp32 x >= 0 given by its bits.
__device__ inline unsigned long long fx30(unsigned bits) {
  const int e = (int)(bits >> 23) & 0xFF;
  if (e == 0) return 0ull;  // denormals are far below 2^-30
  const unsigned long long m = (unsigned long long)((bits & 0x7FFFFFu) | 0x800000u);
  const int sh = e - 120;   // (e - 127) - 23 + 30
  if (sh >= 0) return sh < 40 ? (m << sh) : ~0ull;
  return (-sh) < 64 ? (m >> (-sh)) : 0ull;
}

__device__ inline unsigned long long block_sum_u64(unsigned long long x, Smem &sm) {
  for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.red64[threadIdx.x >> 6] = x;
  __syncthreads();
  unsigned long long t = 0;
  for (int w = 0; w < NWAVE; ++w) t += sm.red64[w];
  return t;
}

// exclusive prefix sums of two per-thread counters over the 1024 threads
__device__ inline void block_scan2(unsigned a, unsigned b, unsigned &ea, unsigned &eb, Smem &sm) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned ia = a, ib = b;
  for (int d = 1; d < 64; d <<= 1) {
    const unsigned oa = __shfl_up(ia, d), ob = __shfl_up(ib, d);
    if (lane >= d) { ia += oa; ib += ob; }
  }
  __syncthreads();
  if (lane == 63) { sm.wave_a[wv] = ia; sm.wave_b[wv] = ib; }
  __syncthreads();
  unsigned ba = 0, bb = 0;
  for (int w = 0; w < wv; ++w) { ba += sm.wave_a[w]; bb += sm.wave_b[w]; }
  ea = ba + ia - a;
  eb = bb + ib - b;
}

// Radix select: finds the k-th largest key T among the candidates and how many candidates
// equal to T belong to the k best (the ones with the lowest indices).  for_each(fn) must call
// fn(key) once for every candidate this thread is responsible for; k <= number of candidates.
template <class ForEach>
__device__ inline void radix_select(ForEach for_each, int k, unsigned &thr, unsigned &need_eq,
                                    Smem &sm) {
  if (k <= 0) { thr = 0xFFFFFFFFu; need_eq = 0; return; }
  unsigned prefix = 0, mask = 0, remaining = (unsigned)k;
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    __syncthreads();
    if (threadIdx.x < 256) sm.hist[threadIdx.x] = 0;
    __syncthreads();
    for_each([&](unsigned kk) {
      if ((kk & mask) == prefix) atomicAdd(&sm.hist[(kk >> shift) & 255u], 1u);
    });
    __syncthreads();
    if (threadIdx.x < 64) {
      // lane l owns bins 4l..4l+3; suffix sums from the top bin down
      const int l = threadIdx.x;
      const unsigned b0 = sm.hist[4 * l], b1 = sm.hist[4 * l + 1], b2 = sm.hist[4 * l + 2],
                     b3 = sm.hist[4 * l + 3];
      const unsigned tot = b0 + b1 + b2 + b3;
      unsigned incl = tot;  // inclusive suffix sum over lanes >= l
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned o = __shfl_down(incl, d);
        if (l + d < 64) incl += o;
      }
      // the bin that holds the remaining-th largest: above < remaining <= above + count
      unsigned ab = incl - tot;
      const unsigned bins[4] = {b3, b2, b1, b0};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (ab < remaining && remaining <= ab + bins[j]) {
          sm.sel_prefix = prefix | ((unsigned)(4 * l + 3 - j) << shift);
          sm.sel_remaining = remaining - ab;
        }
        ab += bins[j];
      }
    }
    __syncthreads();
    prefix = sm.sel_prefix;
    remaining = sm.sel_remaining;
    mask |= 255u << shift;
  }
  thr = prefix;
  need_eq = remaining;
}

// sum of fx30 over the `probe` largest keys (ties do not matter for a sum)
template <class KeyFn>
__device__ inline unsigned long long top_sum(KeyFn key, int n, int probe, Smem &sm) {
  probe = min(probe, n);
  if (probe <= 0) return 0ull;
  unsigned thr, need;
  radix_select([&](auto fn) { for (int i = threadIdx.x; i < n; i += NT) fn(key(i)); }, probe, thr,
               need, sm);
  unsigned long long acc = 0;
  for (int i = threadIdx.x; i < n; i += NT) {
    const unsigned kk = key(i);
    if (kk > thr) acc += fx30(kk);
  }
  acc = block_sum_u64(acc, sm);
  return acc + (unsigned long long)need * fx30(thr);
}

// Ordered compaction of a 1-D candidate list: out[0..k) = selected indices ascending,
// out[k..cap) = -1.  Each wave owns a contiguous, 64-aligned range of indices.
template <class KeyFn>
__device__ inline void select_1d(KeyFn key, int n, int k, int32_t *out, int cap, int32_t *count,
                                 Smem &sm) {
  k = min(k, n);
  unsigned thr, need;
  radix_select([&](auto fn) { for (int i = threadIdx.x; i < n; i += NT) fn(key(i)); }, k, thr, need,
               sm);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int seg = ((n + NWAVE - 1) / NWAVE + 63) / 64 * 64;
  const int lo = wv * seg, hi = min(lo + seg, n);
  unsigned gt = 0, eq = 0;
  for (int i = lo + lane; i < hi; i += 64) {
    const unsigned kk = key(i);
    gt += kk > thr;
    eq += kk == thr;
  }
  for (int d = 32; d >= 1; d >>= 1) { gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); }
  __syncthreads();
  if (lane == 0) { sm.wave_a[wv] = gt; sm.wave_b[wv] = eq; }
  __syncthreads();
  unsigned grun = 0, erun = 0;
  for (int w = 0; w < wv; ++w) { grun += sm.wave_a[w]; erun += sm.wave_b[w]; }
  for (int i0 = lo; i0 < hi; i0 += 64) {
    const int i = i0 + lane;
    const unsigned kk = i < hi ? key(i) : 0u;
    const bool isgt = i < hi && kk > thr, iseq = i < hi && kk == thr;
    const unsigned long long bg = __ballot(isgt), be = __ballot(iseq);
    const unsigned long long below = (1ull << lane) - 1ull;
    const unsigned G = grun + __popcll(bg & below), E = erun + __popcll(be & below);
    if (k > 0 && (isgt || (iseq && E < need))) out[G + min(E, need)] = i;
    grun += __popcll(bg);
    erun += __popcll(be);
  }
  for (int i = k + threadIdx.x; i < cap; i += NT) out[i] = -1;
  if (threadIdx.x == 0) *count = k;
}

__global__ __launch_bounds__(NT) void build_index_kernel(IdxArgs a) {
  __shared__ Smem sm;
  const Shape &sh = a.sh;
  const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int N = sh.N, nb = sh.nb, b = sh.b;
  const unsigned *vb = (const unsigned *)(a.v + (size_t)h * N);
  const unsigned *sb = (const unsigned *)(a.s + (size_t)h * N);
  const unsigned *bb = (const unsigned *)(a.blk + (size_t)h * nb * nb);
  auto vkey = [&](int i) { return vb[i]; };
  auto skey = [&](int i) { return sb[i]; };

  // ---- pattern ---------------------------------------------------------------------------
  int pat = a.ov.pat[h];
  if (pat < 0) {
    long long sbnd = (long long)sh.sink * b;
    if (sbnd > N) sbnd = N;
    long long lb0 = (long long)(nb - sh.local) * b;
    if (lb0 < sbnd) lb0 = sbnd;
    unsigned long long vt = 0, ct = 0;
    for (int j = tid; j < N; j += NT) {
      const unsigned long long f = fx30(vb[j]);
      vt += f;
      if (j < sbnd || j >= lb0) ct += f;
    }
    vt = block_sum_u64(vt, sm);
    ct = block_sum_u64(ct, sm);
    unsigned long long E = 0, ET = 0;
    for (int i = 0; i < sh.w; ++i) {
      const long long qi1 = (long long)N - sh.w + i + 1;
      E += (unsigned long long)qi1;
      ET += (unsigned long long)(qi1 < sbnd ? qi1 : sbnd);
      if (qi1 > lb0) ET += (unsigned long long)(qi1 - lb0);
    }
    typedef unsigned __int128 u128;
    if ((u128)sh.lift_den * ct * E >= (u128)sh.lift_num * vt * ET) {
      pat = SA_TRIANGULAR;
    } else {
      const unsigned long long sv = top_sum(vkey, N, sh.probe_v, sm);
      const unsigned long long ss = top_sum(skey, N, sh.probe_s, sm);
      if ((u128)sh.lift_den * (sv + ss) * E >=
          (u128)sh.lift_num * vt * (unsigned long long)(sh.probe_v + sh.probe_s) *
              (unsigned long long)sh.w)
        pat = SA_INTERVAL_SLASH;
      else
        pat = SA_BLOCK_CLUSTER;
    }
  }
  if (tid == 0) a.out.pattern[h] = pat;

  // ---- columns and diagonals (Interval-Slash only) ------------------------------------------
  int32_t *cols = a.out.cols + (size_t)h * sh.k_v;
  int32_t *offs = a.out.offs + (size_t)h * sh.k_s;
  if (pat == SA_INTERVAL_SLASH) {
    select_1d(vkey, N, sh.k_v, cols, sh.k_v, a.out.n_cols + h, sm);
    select_1d(skey, N, sh.k_s, offs, sh.k_s, a.out.n_offs + h, sm);
  } else {
    for (int i = tid; i < sh.k_v; i += NT) cols[i] = -1;
    for (int i = tid; i < sh.k_s; i += NT) offs[i] = -1;
    if (tid == 0) { a.out.n_cols[h] = 0; a.out.n_offs[h] = 0; }
  }

  // ---- block CSR ---------------------------------------------------------------------------
  int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
  int32_t *bc = a.out.blkcols + (size_t)h * sh.cap_b;
  int total;
  if (pat == SA_BLOCK_CLUSTER) {
    const long long ncand = (long long)nb * (nb - 1) / 2;
    int k = sh.k_b - nb;
    if (k < 0) k = 0;
    if (k > ncand) k = (int)ncand;
    // candidates: the entries C < R of the nb x nb map, one wave per row (coalesced reads)
    unsigned thr, need;
    radix_select(
        [&](auto fn) {
          for (int R = wv; R < nb; R += NWAVE)
            for (int C = lane; C < R; C += 64) fn(bb[(size_t)R * nb + C]);
        },
        k, thr, need, sm);
    // per-row counts (wave per row, coalesced), then a scan over rows
    for (int R = wv; R < nb; R += NWAVE) {
      unsigned gt = 0, eq = 0;
      for (int C = lane; C < R; C += 64) {
        const unsigned kk = bb[(size_t)R * nb + C];
        gt += kk > thr;
        eq += kk == thr;
      }
      for (int d = 32; d >= 1; d >>= 1) { gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); }
      if (lane == 0) { sm.rowgt[R] = gt; sm.roweq[R] = eq; }
    }
    __syncthreads();
    // exclusive scan over rows: thread t owns rows 4t..4t+3 (nb <= 4096)
    {
      unsigned g4[4], e4[4], gs = 0, es = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int R = 4 * tid + j;
        g4[j] = R < nb ? sm.rowgt[R] : 0u;
        e4[j] = R < nb ? sm.roweq[R] : 0u;
        gs += g4[j];
        es += e4[j];
      }
      unsigned eg, ee;
      block_scan2(gs, es, eg, ee, sm);
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int R = 4 * tid + j;
        if (R < nb) { sm.rowgt[R] = eg; sm.roweq[R] = ee; }
        eg += g4[j];
        ee += e4[j];
      }
    }
    __syncthreads();
    for (int R = wv; R < nb; R += NWAVE) {
      unsigned grun = sm.rowgt[R], erun = sm.roweq[R];
      const unsigned start = grun + min(erun, need) + (unsigned)R;  // R forced diagonals above
      if (lane == 0) rp[R] = (int)start;
      for (int C0 = 0; C0 < R; C0 += 64) {
        const int C = C0 + lane;
        const unsigned kk = C < R ? bb[(size_t)R * nb + C] : 0u;
        const bool isgt = C < R && kk > thr, iseq = C < R && kk == thr;
        const unsigned long long bg = __ballot(isgt), be = __ballot(iseq);
        const unsigned long long below = (1ull << lane) - 1ull;
        const unsigned G = grun + __popcll(bg & below), E = erun + __popcll(be & below);
        if (k > 0 && (isgt || (iseq && E < need))) bc[G + min(E, need) + R] = C;
        grun += __popcll(bg);
        erun += __popcll(be);
      }
      // the forced diagonal block closes the row
      if (lane == 0) bc[grun + min(erun, need) + R] = R;
    }
    total = k + nb;
    if (tid == 0) rp[nb] = total;
  } else if (pat == SA_TRIANGULAR) {
    // row R keeps C < min(sink, band start) and the band [max(R-L+1,0), R]
    unsigned c4[4], cs = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int R = 4 * tid + j;
      const int bs = max(R - sh.local + 1, 0);
      c4[j] = R < nb ? (unsigned)(min(sh.sink, bs) + (R - bs + 1)) : 0u;
      cs += c4[j];
    }
    unsigned ex, dummy;
    block_scan2(cs, 0u, ex, dummy, sm);
    unsigned run = ex;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int R = 4 * tid + j;
      if (R < nb) {
        rp[R] = (int)run;
        const int bs = max(R - sh.local + 1, 0);
        const int ns = min(sh.sink, bs);
        for (int C = 0; C < ns; ++C) bc[run + C] = C;
        for (int C = bs; C <= R; ++C) bc[run + ns + (C - bs)] = C;
        run += c4[j];
        if (R == nb - 1) { rp[nb] = (int)run; sm.sel_remaining = run; }
      }
    }
    __syncthreads();
    total = (int)sm.sel_remaining;
  } else {
    for (int R = tid; R < nb; R += NT) { rp[R] = R; bc[R] = R; }
    if (tid == 0) rp[nb] = nb;
    total = nb;
  }
  for (int i = total + tid; i < sh.cap_b; i += NT) bc[i] = -1;
}

}  // namespace

hipError_t launch_build_index(const Shape &sh, const Workspace &, sa_scores in, const Override &ov,
                              sa_index out, hipStream_t st) {
  IdxArgs a;
  a.v = in.v; a.s = in.s; a.blk = in.blk;
  a.sh = sh; a.ov = ov; a.out = out;
  build_index_kernel<<<sh.Hq, NT, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace sa
