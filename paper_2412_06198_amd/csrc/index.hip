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
  unsigned whist[NWAVE][256];  // one private histogram per wave: no cross-wave contention
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

// ---- candidate walks ---------------------------------------------------------------------------
// Score arrays are read four keys per lane (16-byte loads when the segment start is 16-byte
// aligned) with several independent loads in flight per thread: these loops are latency-bound.
// fn(k, i0, lim) receives keys k[0..3] of indices i0..i0+3; entries with i0 + j >= lim are padding.
struct Keys4 { unsigned k[4]; };

__device__ inline Keys4 load4(const unsigned *p, int i, int lim, bool vec) {
  Keys4 r;
  if (i + 3 < lim && vec) {
    const uint4 v = *(const uint4 *)(p + i);
    r.k[0] = v.x; r.k[1] = v.y; r.k[2] = v.z; r.k[3] = v.w;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) r.k[j] = (i + j < lim) ? p[i + j] : 0u;
  }
  return r;
}

// whole block, order irrelevant: group g of 4 keys goes to thread g % NT
template <class Fn>
__device__ inline void block_visit4(const unsigned *p, int n, bool vec, Fn fn) {
  constexpr int U = 4;
  for (int b0 = 0; b0 < n; b0 += NT * 4 * U) {
    Keys4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load4(p, b0 + (u * NT + (int)threadIdx.x) * 4, n, vec);
#pragma unroll
    for (int u = 0; u < U; ++u) fn(v[u], b0 + (u * NT + (int)threadIdx.x) * 4, n);
  }
}

// one wave, indices [lo,hi) in increasing groups of 256: lane l holds lo + 256g + 4l .. +3
template <class Fn>
__device__ inline void wave_visit4(const unsigned *p, int lo, int hi, bool vec, Fn fn) {
  constexpr int U = 4;
  const int lane = threadIdx.x & 63;
  for (int g0 = lo; g0 < hi; g0 += 256 * U) {
    Keys4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load4(p, g0 + 256 * u + 4 * lane, hi, vec);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (g0 + 256 * u < hi) fn(v[u], g0 + 256 * u + 4 * lane, hi);
  }
}

// The strictly-lower part (C < R) of every row this wave owns (R = wave, wave+16, ...), walked in
// units of 1024 keys with the next unit's loads issued before the current one is processed:
// short rows would otherwise expose one memory round trip each.  begin(R) / end(R) bracket a row.
template <class Begin, class Fn, class End>
__device__ inline void wave_rows_visit4(const unsigned *blk, int nb, bool vec, Begin begin, Fn fn, End end) {
  constexpr int U = 4;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int R = wv, c0 = 0;          // unit being processed
  int Rn = wv, cn = 0;         // unit being loaded
  Keys4 cur[U], nxt[U];
  auto load_unit = [&](Keys4 (&dst)[U], int row, int col) {
    const unsigned *p = blk + (size_t)row * nb;
#pragma unroll
    for (int u = 0; u < U; ++u) dst[u] = load4(p, col + 256 * u + 4 * lane, row, vec);
  };
  auto advance = [&](int &row, int &col) {
    col += 256 * U;
    if (col >= row) { row += NWAVE; col = 0; }
  };
  if (Rn < nb) load_unit(nxt, Rn, cn);
  while (R < nb) {
#pragma unroll
    for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    advance(Rn, cn);
    if (Rn < nb) load_unit(nxt, Rn, cn);
    if (c0 == 0) begin(R);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (c0 + 256 * u < R) fn(cur[u], c0 + 256 * u + 4 * lane, R);
    if (c0 + 256 * U >= R) end(R);
    advance(R, c0);
  }
}

// Ordered emission for one 256-key group of a wave: an element is selected if its key is above the
// threshold, or equal to it and among the first `need` such elements in index order.  put(pos, idx)
// stores the selection; grun / erun count the greater / equal elements seen so far.
template <class Put>
__device__ inline void emit_group(const Keys4 &v, int i0, int lim, unsigned thr, unsigned need,
                                  unsigned &grun, unsigned &erun, Put put) {
  const int lane = threadIdx.x & 63;
  const unsigned long long below = (1ull << lane) - 1ull;
  unsigned gl = 0, el = 0, gtot = 0, etot = 0;
  bool isgt[4], iseq[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    isgt[j] = i0 + j < lim && v.k[j] > thr;
    iseq[j] = i0 + j < lim && v.k[j] == thr;
    const unsigned long long bg = __ballot(isgt[j]), be = __ballot(iseq[j]);
    gl += __popcll(bg & below); el += __popcll(be & below);
    gtot += __popcll(bg); etot += __popcll(be);
  }
  unsigned G = grun + gl, E = erun + el;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (isgt[j] || (iseq[j] && E < need)) put(G + min(E, need), i0 + j);
    G += isgt[j];
    E += iseq[j];
  }
  grun += gtot;
  erun += etot;
}

// Adds one count per valid lane to a wave-private LDS histogram.  Same-address LDS atomics are
// serialised lane by lane, and the scores of a head share their leading bits, so the bin of the
// first valid lane is added once with its lane count (twice: two peels); what is left goes one
// atomic per lane.  Must be called by all 64 lanes.
__device__ inline void hist_add(unsigned *wh, unsigned bin, bool valid) {
#pragma unroll
  for (int peel = 0; peel < 2; ++peel) {
    const unsigned long long mv = __ballot(valid);
    if (mv == 0) return;
    const int first = __ffsll((long long)mv) - 1;
    const unsigned b0 = __builtin_amdgcn_readlane(bin, first);  // bin of the first valid lane
    const bool same = valid && bin == b0;
    const unsigned long long ms = __ballot(same);
    if ((int)(threadIdx.x & 63) == first) atomicAdd(&wh[b0], (unsigned)__popcll(ms));
    valid = valid && !same;
  }
  if (valid) atomicAdd(&wh[bin], 1u);
}

// Radix select: finds the k-th largest key T among the candidates and how many candidates
// equal to T belong to the k best (the ones with the lowest indices).  for_each(fn) must call
// fn(keys, i0, lim) in wave-uniform loops for every group of four candidates this thread is
// responsible for; k <= number of candidates.
template <class ForEach>
__device__ inline void radix_select(ForEach for_each, int k, unsigned &thr, unsigned &need_eq,
                                    Smem &sm) {
  if (k <= 0) { thr = 0xFFFFFFFFu; need_eq = 0; return; }
  unsigned prefix = 0, mask = 0, remaining = (unsigned)k;
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    __syncthreads();
    for (int i = threadIdx.x; i < NWAVE * 256; i += NT) (&sm.whist[0][0])[i] = 0;
    __syncthreads();
    unsigned *wh = sm.whist[threadIdx.x >> 6];
    for_each([&](const Keys4 &v, int i0, int lim) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        hist_add(wh, (v.k[j] >> shift) & 255u, i0 + j < lim && (v.k[j] & mask) == prefix);
    });
    __syncthreads();
    if (threadIdx.x < 256) {
      unsigned t = 0;
#pragma unroll
      for (int w = 0; w < NWAVE; ++w) t += sm.whist[w][threadIdx.x];
      sm.hist[threadIdx.x] = t;
    }
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
__device__ inline unsigned long long top_sum(const unsigned *p, int n, int probe, Smem &sm) {
  probe = min(probe, n);
  if (probe <= 0) return 0ull;
  unsigned thr, need;
  radix_select([&](auto fn) { block_visit4(p, n, true, fn); }, probe, thr, need, sm);
  unsigned long long acc = 0;
  block_visit4(p, n, true, [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i0 + j < lim && v.k[j] > thr) acc += fx30(v.k[j]);
  });
  acc = block_sum_u64(acc, sm);
  return acc + (unsigned long long)need * fx30(thr);
}

// Ordered compaction of a 1-D candidate list: out[0..k) = selected indices ascending,
// out[k..cap) = -1.  Each wave owns a contiguous range of indices (a multiple of 256 long).
__device__ inline void select_1d(const unsigned *p, int n, int k, int32_t *out, int cap,
                                 int32_t *count, Smem &sm) {
  k = min(k, n);
  unsigned thr, need;
  radix_select([&](auto fn) { block_visit4(p, n, true, fn); }, k, thr, need, sm);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int seg = ((n + NWAVE - 1) / NWAVE + 255) / 256 * 256;
  const int lo = min(wv * seg, n), hi = min(lo + seg, n);
  unsigned gt = 0, eq = 0;
  wave_visit4(p, lo, hi, true, [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      gt += i0 + j < lim && v.k[j] > thr;
      eq += i0 + j < lim && v.k[j] == thr;
    }
  });
  for (int d = 32; d >= 1; d >>= 1) { gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); }
  __syncthreads();
  if (lane == 0) { sm.wave_a[wv] = gt; sm.wave_b[wv] = eq; }
  __syncthreads();
  unsigned grun = 0, erun = 0;
  for (int w = 0; w < wv; ++w) { grun += sm.wave_a[w]; erun += sm.wave_b[w]; }
  if (k > 0)
    wave_visit4(p, lo, hi, true, [&](const Keys4 &v, int i0, int lim) {
      emit_group(v, i0, lim, thr, need, grun, erun, [&](unsigned pos, int idx) { out[pos] = idx; });
    });
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

  // ---- pattern ---------------------------------------------------------------------------
  int pat = a.ov.pat[h];
  if (pat < 0) {
    long long sbnd = (long long)sh.sink * b;
    if (sbnd > N) sbnd = N;
    long long lb0 = (long long)(nb - sh.local) * b;
    if (lb0 < sbnd) lb0 = sbnd;
    unsigned long long vt = 0, ct = 0;
    block_visit4(vb, N, true, [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int j = i0 + jj;
        if (j < lim) {
          const unsigned long long f = fx30(v.k[jj]);
          vt += f;
          if (j < sbnd || j >= lb0) ct += f;
        }
      }
    });
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
      const unsigned long long sv = top_sum(vb, N, sh.probe_v, sm);
      const unsigned long long ss = top_sum(sb, N, sh.probe_s, sm);
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
    select_1d(vb, N, sh.k_v, cols, sh.k_v, a.out.n_cols + h, sm);
    select_1d(sb, N, sh.k_s, offs, sh.k_s, a.out.n_offs + h, sm);
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
    const bool rowvec = (nb & 3) == 0;  // rows start 16-byte aligned
    unsigned thr, need;
    radix_select(
        [&](auto fn) {
          wave_rows_visit4(bb, nb, rowvec, [](int) {}, fn, [](int) {});
        },
        k, thr, need, sm);
    // per-row counts (wave per row, coalesced), then a scan over rows
    {
      unsigned gt = 0, eq = 0;
      wave_rows_visit4(
          bb, nb, rowvec, [&](int) { gt = 0; eq = 0; },
          [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              gt += i0 + j < lim && v.k[j] > thr;
              eq += i0 + j < lim && v.k[j] == thr;
            }
          },
          [&](int R) {
            unsigned g2 = gt, e2 = eq;
            for (int d = 32; d >= 1; d >>= 1) { g2 += __shfl_xor(g2, d); e2 += __shfl_xor(e2, d); }
            if (lane == 0) { sm.rowgt[R] = g2; sm.roweq[R] = e2; }
          });
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
    {
      unsigned grun = 0, erun = 0;
      wave_rows_visit4(
          bb, nb, rowvec,
          [&](int R) {
            grun = sm.rowgt[R];
            erun = sm.roweq[R];
            if (lane == 0) rp[R] = (int)(grun + min(erun, need) + (unsigned)R);  // R forced diagonals above
          },
          [&](const Keys4 &v, int i0, int lim) {
            // lim is the row index R: a selected entry lands after the R diagonals of the rows above
            if (k > 0)
              emit_group(v, i0, lim, thr, need, grun, erun,
                         [&](unsigned pos, int C) { bc[pos + lim] = C; });
          },
          [&](int R) {
            // the forced diagonal block closes the row
            if (lane == 0) bc[grun + min(erun, need) + R] = R;
          });
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
