// Index builder for gfx950: per-head pattern choice and top-k selection
// (Main Idea "Categorization of Attention Heads"; Alg. 2 TopK / CombineIndices;
// Alg. 3 TopKBlocks).
//
// Integer work only: scores are compared through their fp32 bit patterns (all
// scores are >= +0, so the unsigned order is the numeric order), ties go to the
// lower index, and the pattern rule sums floor(score * 2^30) in 64-bit integers.
//
// Five selections run side by side for every head, so that nothing waits on the
// pattern decision: the probe_v / probe_s best of v and s (pattern rule), the
// k_v best columns, the k_s best diagonals, the k_b - nb best blocks.  Each is a
// radix select in three levels (11 + 10 + 10 key bits; the sign bit is clear).  Every level is a
// launch of P workgroups per head (LDS histograms, flushed to global memory with
// integer atomics) followed by a one-workgroup-per-head launch that reads the
// merged histogram and fixes the next digit: kernel boundaries are the only
// synchronisation between workgroups, no fences or spin waits.  Two more
// launches count and then emit the selected entries in index order (wave
// ballots), so the result is sorted without any sort.
//
// With the per-row block rule (every row block of a Block-Cluster head keeps the
// same fraction of its causal blocks) the fifth selection is switched off and
// one more launch selects inside each row instead: one wave per row, keys in
// registers, the threshold found bit by bit.
//
// With block-granular diagonals four launches after the emission turn the selected
// offsets of the Interval-Slash heads into rows of the block CSR (bitmap per row,
// count, prefix, ordered write) and empty the offset list.
#include <cstddef>

#include "sa_internal.h"

namespace sa {
namespace {

constexpr int BT = 256;            // threads per workgroup
constexpr int WPB = BT / 64;       // waves per workgroup
constexpr int kMaxParts = 64;      // workgroups per head
constexpr int kMaxPW = kMaxParts * WPB;
constexpr int kMaxNb = kMaxSeq / 64;
constexpr int NSEL = 5;            // 0: v probe, 1: s probe, 2: v top k_v, 3: s top k_s, 4: blk top k_b - nb
constexpr int L1BINS = 2048, L2BINS = 1024, L3BINS = 1024;  // 11 + 10 + 10 key bits below the sign bit

// per-head scratch in the workspace
struct IdxScratch {
  alignas(16) unsigned hist1[3][L1BINS];  // level 1 per array: v, s, blk
  alignas(16) unsigned hist2[NSEL][L2BINS];
  alignas(16) unsigned hist3[NSEL][L3BINS];
  unsigned long long vtot, ct, topsum[2];
  // everything above is zeroed at the start of a call
  unsigned prefix[NSEL], remaining[NSEL];
  unsigned thr[NSEL], need[NSEL];
  unsigned wgt[2][kMaxPW], weq[2][kMaxPW];  // v / s: counts per wave part, then exclusive prefixes
  unsigned rowgt[kMaxNb], roweq[kMaxNb];    // blk: counts per row, then exclusive prefixes
  int pattern;
};
constexpr size_t kZeroWords = offsetof(IdxScratch, prefix) / 4;

struct IdxArgs {
  const unsigned *v, *s, *blk;     // fp32 scores as bit patterns
  IdxScratch *scratch;
  Shape sh;
  Override ov;
  sa_index out;
  int P, PW, seg;                  // workgroups per head, wave parts per head, keys of v / s per wave part
  int ksel[NSEL];                  // clamped k of every selection
  // Which part of the work a launch does: bit 0 = the selections on v and s, bit 1 = the selection
  // on the block map (the two parts touch disjoint fields of the scratch and may run side by side).
  int mask;
  // Heads (bit h) whose pattern override makes the v/s selections, or the block selection, unnecessary.
  uint32_t skip_vs[kMaxHeads / 32], skip_blk[kMaxHeads / 32];
  // Not null: the patterns an earlier launch decided ([Hq], device); the block-map part of the work
  // is then done for the Block-Cluster heads only (the block map of the others was never computed).
  const int32_t *decided;
};

// Whether a launch has to touch one part of a head's work (the selections on v and s, or the one on
// the block map): with a pattern override only the overridden pattern's own selection is needed,
// none for Triangular.  (Skipping the rest of a head as soon as it passes the Triangular test was
// tried too: the flag costs every later workgroup one more dependent read, more than it saves.)
__device__ inline bool head_wants(const IdxArgs &a, int h, bool blk_part) {
  const int w = h >> 5;  // four words: selected without indexing the argument block dynamically
  const uint32_t *m = blk_part ? a.skip_blk : a.skip_vs;
  const uint32_t bits = w == 0 ? m[0] : w == 1 ? m[1] : w == 2 ? m[2] : m[3];
  if ((bits >> (h & 31)) & 1u) return false;
  return !(blk_part && a.decided) || a.decided[h] == SA_BLOCK_CLUSTER;
}

// floor(x * 2^30) of a finite fp32 x >= 0 given by its bits.
__device__ inline unsigned long long fx30(unsigned bits) {
  const int e = (int)(bits >> 23) & 0xFF;
  if (e == 0) return 0ull;  // denormals are far below 2^-30
  const unsigned long long m = (unsigned long long)((bits & 0x7FFFFFu) | 0x800000u);
  const int sh = e - 120;   // (e - 127) - 23 + 30
  if (sh >= 0) return sh < 40 ? (m << sh) : ~0ull;
  return (-sh) < 64 ? (m >> (-sh)) : 0ull;
}

// The Triangular test of the pattern rule on the sums of the level-1 histogram launch; E receives
// the number of causal window entries.
__device__ inline bool triangular_test(const IdxArgs &a, const IdxScratch *G, unsigned long long &E) {
  const Shape &sh = a.sh;
  const int N = sh.N, nb = sh.nb;
  long long sbnd = (long long)sh.sink * sh.b;
  if (sbnd > N) sbnd = N;
  long long lb0 = (long long)(nb - sh.local) * sh.b;
  if (lb0 < sbnd) lb0 = sbnd;
  unsigned long long ET = 0;
  E = 0;
  for (int i = 0; i < sh.w; ++i) {
    const long long qi1 = (long long)N - sh.w + i + 1;
    E += (unsigned long long)qi1;
    ET += (unsigned long long)(qi1 < sbnd ? qi1 : sbnd);
    if (qi1 > lb0) ET += (unsigned long long)(qi1 - lb0);
  }
  typedef unsigned __int128 u128;
  return (u128)sh.lift_den * G->ct * E >= (u128)sh.lift_num * G->vtot * ET;
}

// Pattern of head h: the caller's override, else the integer lift tests on the sums that the level-1
// histogram launch (vtot, ct) and the counting launch (topsum) left in the scratch.
__device__ inline int decide_pattern(const IdxArgs &a, const IdxScratch *G, int h) {
  const Shape &sh = a.sh;
  const int pat = a.ov.pat[h];
  if (pat >= 0) return pat;
  unsigned long long E;
  if (triangular_test(a, G, E)) return SA_TRIANGULAR;
  typedef unsigned __int128 u128;
  // sum over the probe best = sum over keys above the threshold + ties at the threshold
  const unsigned long long sv =
      a.ksel[0] > 0 ? G->topsum[0] + (unsigned long long)G->need[0] * fx30(G->thr[0]) : 0ull;
  const unsigned long long ss =
      a.ksel[1] > 0 ? G->topsum[1] + (unsigned long long)G->need[1] * fx30(G->thr[1]) : 0ull;
  if ((u128)sh.lift_den * (sv + ss) * E >=
      (u128)sh.lift_num * G->vtot * (unsigned long long)(sh.probe_v + sh.probe_s) * (unsigned long long)sh.w)
    return SA_INTERVAL_SLASH;
  return SA_BLOCK_CLUSTER;
}

// Blocks that row block R keeps under the per-row rule: the same fraction k_b / (nb (nb+1) / 2) of
// its R + 1 causal blocks, rounded up (the diagonal block is one of them).
__device__ inline int row_share(const Shape &sh, int R) {
  const long long all = (long long)sh.nb * (sh.nb + 1) / 2;
  const long long k = ((long long)sh.k_b * (R + 1) + all - 1) / all;
  return (int)(k < R + 1 ? k : R + 1);
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

// The strictly-lower part (C < R) of the rows R = first, first + stride, ... of the nb x nb block
// map, walked by one wave in units of 1024 keys with the next unit's loads issued before the
// current one is processed: short rows would otherwise expose one memory round trip each.
// begin(R) / end(R) bracket a row.
// With scale_rows the key of an entry of row R is its value times R + 1 (one fp32 multiplication;
// all values are >= +0, so the products order like their bit patterns too).
template <class Begin, class Fn, class End>
__device__ inline void wave_rows_visit4(const unsigned *blk, int nb, int first, int stride, bool vec,
                                        bool scale_rows, Begin begin, Fn fn, End end) {
  constexpr int U = 4;
  const int lane = threadIdx.x & 63;
  int R = first, c0 = 0;    // unit being processed
  int Rn = first, cn = 0;   // unit being loaded
  Keys4 cur[U], nxt[U];
  auto load_unit = [&](Keys4 (&dst)[U], int row, int col) {
    const unsigned *p = blk + (size_t)row * nb;
#pragma unroll
    for (int u = 0; u < U; ++u) dst[u] = load4(p, col + 256 * u + 4 * lane, row, vec);
  };
  auto advance = [&](int &row, int &col) {
    col += 256 * U;
    if (col >= row) { row += stride; col = 0; }
  };
  if (Rn < nb) load_unit(nxt, Rn, cn);
  while (R < nb) {
#pragma unroll
    for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    advance(Rn, cn);
    if (Rn < nb) load_unit(nxt, Rn, cn);
    if (c0 == 0) begin(R);
    if (scale_rows) {
      const float len = (float)(R + 1);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[u].k[j] = __float_as_uint(__uint_as_float(cur[u].k[j]) * len);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (c0 + 256 * u < R) fn(cur[u], c0 + 256 * u + 4 * lane, R);
    if (c0 + 256 * U >= R) end(R);
    advance(R, c0);
  }
}

// Adds one count per valid lane to an LDS histogram.  Same-address LDS atomics are serialised
// lane by lane, and the scores of a head share their leading bits, so the bin of the first valid
// lane is added once with its lane count (two such peels); what is left goes one atomic per lane.
// Must be called by all 64 lanes.
__device__ inline void hist_add(unsigned *h, unsigned bin, bool valid) {
#pragma unroll
  for (int peel = 0; peel < 2; ++peel) {
    const unsigned long long mv = __ballot(valid);
    if (mv == 0) return;
    const int first = __ffsll((long long)mv) - 1;
    const unsigned b0 = __builtin_amdgcn_readlane(bin, first);
    const bool same = valid && bin == b0;
    const unsigned long long ms = __ballot(same);
    if ((int)(threadIdx.x & 63) == first) atomicAdd(&h[b0], (unsigned)__popcll(ms));
    valid = valid && !same;
  }
  if (valid) atomicAdd(&h[bin], 1u);
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

// In a histogram of nbins (a multiple of 64) counts held in LDS, the bin that holds the k-th key
// counted from the top bin down (1 <= k <= total), and the rank of that key inside the bin.
// One wave.
__device__ inline void wave_find_kth(const unsigned *hist, int nbins, unsigned k, unsigned &bin,
                                     unsigned &rank) {
  const int lane = threadIdx.x & 63;
  const int per = nbins / 64;  // lane l owns bins [l*per, (l+1)*per)
  unsigned tot = 0;
  for (int i = 0; i < per; ++i) tot += hist[lane * per + i];
  unsigned incl = tot;  // inclusive suffix sum over lanes >= l
  for (int d = 1; d < 64; d <<= 1) {
    const unsigned o = __shfl_down(incl, d);
    if (lane + d < 64) incl += o;
  }
  const unsigned above = incl - tot;
  const bool mine = above < k && k <= above + tot;
  const unsigned long long m = __ballot(mine);
  const int owner = m ? __ffsll((long long)m) - 1 : 0;
  unsigned b = 0, r = 0;
  if (lane == owner) {
    unsigned ab = above;
    for (int i = per - 1; i >= 0; --i) {
      const unsigned c = hist[lane * per + i];
      if (ab < k && k <= ab + c) { b = (unsigned)(lane * per + i); r = k - ab; break; }
      ab += c;
    }
  }
  bin = __shfl(b, owner);
  rank = __shfl(r, owner);
}

// Exclusive prefixes of two values per thread over the BT threads of a workgroup: shuffles inside
// the waves, the wave totals through LDS (wsum: 2 * WPB words).  Called by all threads.
__device__ inline void block_exclusive_scan2(unsigned &a, unsigned &b, unsigned *wsum) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned ia = a, ib = b;
  for (int d = 1; d < 64; d <<= 1) {
    const unsigned oa = __shfl_up(ia, d), ob = __shfl_up(ib, d);
    if (lane >= d) { ia += oa; ib += ob; }
  }
  if (lane == 63) { wsum[wv] = ia; wsum[WPB + wv] = ib; }
  __syncthreads();
  unsigned ba = 0, bb = 0;
  for (int w = 0; w < wv; ++w) { ba += wsum[w]; bb += wsum[WPB + w]; }
  __syncthreads();
  a = ba + ia - a;
  b = bb + ib - b;
}

__global__ void idx_zero_kernel(IdxScratch *scratch) {
  unsigned *p = (unsigned *)(scratch + blockIdx.x);
  for (size_t i = threadIdx.x; i < kZeroWords; i += blockDim.x) p[i] = 0u;
}

// ---- level histograms ------------------------------------------------------------------------------
// LEVEL 1: bits 30..20 of every key (scores are >= +0: bit 31 is clear), one histogram per array.
// LEVEL 2: bits 19..10 of the keys whose bits 30..20 equal the selection's prefix.
// LEVEL 3: bits  9..0 of the keys whose bits 31..10 equal the selection's prefix.
template <int LEVEL>
__global__ __launch_bounds__(BT) void idx_hist_kernel(IdxArgs a) {
  constexpr int NH = LEVEL == 1 ? 3 : NSEL;
  constexpr int BINS = LEVEL == 1 ? L1BINS : L2BINS;
  // levels 2 and 3: 20 KB, nothing else in LDS, so that eight workgroups (every wave slot) fit a CU
  __shared__ __attribute__((aligned(16))) unsigned hist[NH][BINS];
  const Shape &sh = a.sh;
  const int p = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int N = sh.N, nb = sh.nb;
  IdxScratch *G = a.scratch + h;
  const bool do_vs = (a.mask & 1) && head_wants(a, h, false);
  const bool do_blk = (a.mask & 2) && a.ksel[4] > 0 && head_wants(a, h, true);
  if (!do_vs && !do_blk) return;
  const unsigned *vb = a.v + (size_t)h * N, *sb = a.s + (size_t)h * N;
  const unsigned *bb = a.blk + (size_t)h * nb * nb;
  for (int i = tid; i < NH * BINS; i += BT) (&hist[0][0])[i] = 0u;
  unsigned pre[NSEL];
  bool act[NSEL];
#pragma unroll
  for (int q = 0; q < NSEL; ++q) {
    pre[q] = LEVEL == 1 ? 0u : G->prefix[q];
    act[q] = a.ksel[q] > 0;
  }
  __syncthreads();
  const int gw = p * WPB + wv;
  const int lo = min(gw * a.seg, N), hi = min(lo + a.seg, N);
  unsigned long long vt = 0, ct = 0;
  long long sbnd = (long long)sh.sink * sh.b;
  if (sbnd > N) sbnd = N;
  long long lb0 = (long long)(nb - sh.local) * sh.b;
  if (lb0 < sbnd) lb0 = sbnd;

  auto visit = [&](const Keys4 &v, int i0, int lim, int arr) {
    // arr 0: v (selections 0, 2), 1: s (selections 1, 3), 2: blk (selection 4)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool ok = i0 + j < lim;
      const unsigned key = v.k[j];
      if (LEVEL == 1) {
        hist_add(hist[arr], min(key >> 20, (unsigned)L1BINS - 1u), ok);  // the sign bit of a score is 0
      } else {
        const unsigned hi_bits = LEVEL == 2 ? key >> 20 : key >> 10;
        const unsigned bin = LEVEL == 2 ? (key >> 10) & 1023u : key & 1023u;
        if (arr == 2) {
          hist_add(hist[NH - 1], bin, ok && act[4] && hi_bits == pre[4]);
        } else {
          hist_add(hist[arr % NH], bin, ok && act[arr] && hi_bits == pre[arr]);
          hist_add(hist[(arr + 2) % NH], bin, ok && act[arr + 2] && hi_bits == pre[arr + 2]);
        }
      }
    }
  };
  if (do_vs) wave_visit4(vb, lo, hi, true, [&](const Keys4 &v, int i0, int lim) {
    visit(v, i0, lim, 0);
    if (LEVEL == 1) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i0 + j < lim) {
          const unsigned long long f = fx30(v.k[j]);
          vt += f;
          if (i0 + j < sbnd || i0 + j >= lb0) ct += f;
        }
    }
  });
  if (do_vs) wave_visit4(sb, lo, hi, true, [&](const Keys4 &v, int i0, int lim) { visit(v, i0, lim, 1); });
  if (do_blk)
    wave_rows_visit4(bb, nb, gw, a.PW, (nb & 3) == 0, sh.row_norm != 0, [](int) {},
                     [&](const Keys4 &v, int i0, int lim) { visit(v, i0, lim, 2); }, [](int) {});
  __syncthreads();
  unsigned *gh = LEVEL == 1 ? &G->hist1[0][0] : (LEVEL == 2 ? &G->hist2[0][0] : &G->hist3[0][0]);
  for (int i = tid; i < NH * BINS; i += BT) {
    const unsigned c = (&hist[0][0])[i];
    if (c) atomicAdd(&gh[i], c);
  }
  if (LEVEL == 1 && do_vs) {
    // the two 64-bit sums of the workgroup, through the histogram's LDS once it is flushed
    for (int d = 32; d >= 1; d >>= 1) { vt += __shfl_xor(vt, d); ct += __shfl_xor(ct, d); }
    unsigned long long *red64 = (unsigned long long *)&hist[0][0];
    __syncthreads();
    if (lane == 0) { red64[wv] = vt; red64[WPB + wv] = ct; }
    __syncthreads();
    if (tid == 0) {
      unsigned long long tv = 0, tc = 0;
      for (int w = 0; w < WPB; ++w) { tv += red64[w]; tc += red64[WPB + w]; }
      atomicAdd(&G->vtot, tv);
      atomicAdd(&G->ct, tc);
    }
  }
}

// One workgroup per head: fixes the next digit of every selection from the merged histograms.
template <int LEVEL>
__global__ __launch_bounds__(BT) void idx_select_kernel(IdxArgs a) {
  constexpr int NH = LEVEL == 1 ? 3 : NSEL;
  constexpr int BINS = LEVEL == 1 ? L1BINS : L2BINS;
  __shared__ __attribute__((aligned(16))) unsigned hist[NH][BINS];
  const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  IdxScratch *G = a.scratch + h;
  const unsigned *gh = LEVEL == 1 ? &G->hist1[0][0] : (LEVEL == 2 ? &G->hist2[0][0] : &G->hist3[0][0]);
  for (int i = tid * 4; i < NH * BINS; i += BT * 4)
    *(uint4 *)&(&hist[0][0])[i] = *(const uint4 *)&gh[i];
  __syncthreads();
  for (int q = wv; q < NSEL; q += WPB) {  // wave w takes selections w and w + 4
    if (!(a.mask & (q < 4 ? 1 : 2)) || !head_wants(a, h, q == 4)) continue;
    if (a.ksel[q] <= 0) {
      if (LEVEL == 3 && lane == 0) { G->thr[q] = 0xFFFFFFFFu; G->need[q] = 0u; }
      continue;
    }
    const unsigned *hsel = LEVEL == 1 ? hist[(q == 4 ? 2 : (q & 1)) % NH] : hist[q % NH];
    const unsigned pre = LEVEL == 1 ? 0u : G->prefix[q];
    const unsigned k = LEVEL == 1 ? (unsigned)a.ksel[q] : G->remaining[q];
    unsigned bin, rank;
    wave_find_kth(hsel, BINS, k, bin, rank);
    if (lane == 0) {
      if (LEVEL == 1) {
        G->prefix[q] = bin;
        G->remaining[q] = rank;
      } else if (LEVEL == 2) {
        G->prefix[q] = (pre << 10) | bin;
        G->remaining[q] = rank;
      } else {
        G->thr[q] = (pre << 10) | bin;
        G->need[q] = rank;
      }
    }
  }
}

// ---- counts, pattern, prefixes ---------------------------------------------------------------------
__global__ __launch_bounds__(BT) void idx_count_kernel(IdxArgs a) {
  __shared__ unsigned long long red64[2][WPB];
  const Shape &sh = a.sh;
  const int p = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int N = sh.N, nb = sh.nb;
  IdxScratch *G = a.scratch + h;
  const unsigned *vb = a.v + (size_t)h * N, *sb = a.s + (size_t)h * N;
  const unsigned *bb = a.blk + (size_t)h * nb * nb;
  unsigned thr[NSEL], need[NSEL];
#pragma unroll
  for (int q = 0; q < NSEL; ++q) { thr[q] = G->thr[q]; need[q] = G->need[q]; }
  const int gw = p * WPB + wv;
  const int lo = min(gw * a.seg, N), hi = min(lo + a.seg, N);
  const bool do_vs = (a.mask & 1) && head_wants(a, h, false);
  for (int arr = 0; arr < 2 && do_vs; ++arr) {
    unsigned gt = 0, eq = 0;
    unsigned long long ts = 0;
    const unsigned tp = thr[arr], tk = thr[arr + 2];
    wave_visit4(arr ? sb : vb, lo, hi, true, [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i0 + j < lim) {
          gt += v.k[j] > tk;
          eq += v.k[j] == tk;
          if (v.k[j] > tp) ts += fx30(v.k[j]);
        }
    });
    for (int d = 32; d >= 1; d >>= 1) {
      gt += __shfl_xor(gt, d); eq += __shfl_xor(eq, d); ts += __shfl_xor(ts, d);
    }
    if (lane == 0) { G->wgt[arr][gw] = gt; G->weq[arr][gw] = eq; red64[arr][wv] = ts; }
  }
  if (!sh.row_select && (a.mask & 2) && head_wants(a, h, true)) {
    unsigned gt = 0, eq = 0;
    wave_rows_visit4(
        bb, nb, gw, a.PW, (nb & 3) == 0, sh.row_norm != 0, [&](int) { gt = 0; eq = 0; },
        [&](const Keys4 &v, int i0, int lim) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            gt += i0 + j < lim && v.k[j] > thr[4];
            eq += i0 + j < lim && v.k[j] == thr[4];
          }
        },
        [&](int R) {
          unsigned g2 = gt, e2 = eq;
          for (int d = 32; d >= 1; d >>= 1) { g2 += __shfl_xor(g2, d); e2 += __shfl_xor(e2, d); }
          if (lane == 0) { G->rowgt[R] = g2; G->roweq[R] = e2; }
        });
  }
  __syncthreads();
  if (tid < 2 && do_vs) {
    unsigned long long t = 0;
    for (int w = 0; w < WPB; ++w) t += red64[tid][w];
    atomicAdd(&G->topsum[tid], t);
  }
}

// The pattern decision by itself, one thread per head, for a caller that needs it before the block
// map exists (the scan launch below takes the same decision again from the same sums).
__global__ void idx_decide_kernel(IdxArgs a) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h < a.sh.Hq) a.out.pattern[h] = decide_pattern(a, a.scratch + h, h);
}

// One workgroup per head: pattern decision, prefixes of the per-part and per-row counts, rowptr.
__global__ __launch_bounds__(BT) void idx_scan_kernel(IdxArgs a) {
  __shared__ unsigned s_wsum[2 * WPB];
  __shared__ int s_pat;
  const Shape &sh = a.sh;
  const int h = blockIdx.x, tid = threadIdx.x;
  const int N = sh.N, nb = sh.nb;
  IdxScratch *G = a.scratch + h;
  unsigned thr[NSEL], need[NSEL];
#pragma unroll
  for (int q = 0; q < NSEL; ++q) { thr[q] = G->thr[q]; need[q] = G->need[q]; }
  // ---- pattern of the head --------------------------------------------------------------------------
  if (tid == 0) {
    const int pat = decide_pattern(a, G, h);
    G->pattern = pat;
    a.out.pattern[h] = pat;
    s_pat = pat;
  }
  // ---- exclusive prefixes of the wave-part counts of v and s (PW <= 256 = one per thread) --------
  for (int arr = 0; arr < 2; ++arr) {
    unsigned pg = tid < a.PW ? G->wgt[arr][tid] : 0u, pe = tid < a.PW ? G->weq[arr][tid] : 0u;
    block_exclusive_scan2(pg, pe, s_wsum);
    if (tid < a.PW) { G->wgt[arr][tid] = pg; G->weq[arr][tid] = pe; }
  }
  const int pat = s_pat;  // written before the barriers of the scans above
  const bool bc_global = pat == SA_BLOCK_CLUSTER && !sh.row_select;
  // ---- row prefixes: thread t owns RP consecutive rows (nb <= kMaxNb) ------------------------------
  constexpr int RP = kMaxNb / BT;
  unsigned g16[RP], e16[RP], gs = 0, es = 0;
#pragma unroll
  for (int j = 0; j < RP; ++j) {
    const int R = RP * tid + j;
    unsigned g = 0, e = 0;
    if (R < nb) {
      if (bc_global) {
        g = G->rowgt[R];
        e = G->roweq[R];
      } else if (pat == SA_BLOCK_CLUSTER) {
        g = (unsigned)row_share(sh, R);
      } else if (pat == SA_TRIANGULAR) {
        const int bs = max(R - sh.local + 1, 0);  // row R keeps C < min(sink, band start) and the band
        g = (unsigned)(min(sh.sink, bs) + (R - bs + 1));
      } else {
        g = 1u;
      }
    }
    g16[j] = g; e16[j] = e;
    gs += g; es += e;
  }
  unsigned eg = gs, ee = es;
  block_exclusive_scan2(eg, ee, s_wsum);
  int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
#pragma unroll
  for (int j = 0; j < RP; ++j) {
    const int R = RP * tid + j;
    if (R < nb) {
      if (bc_global) {
        G->rowgt[R] = eg;
        G->roweq[R] = ee;
        rp[R] = (int)(eg + min(ee, need[4]) + (unsigned)R);  // R forced diagonals above this row
      } else {
        rp[R] = (int)eg;
      }
    }
    eg += g16[j];
    ee += e16[j];
    if (R == nb - 1) rp[nb] = bc_global ? a.ksel[4] + nb : (int)eg;
  }
}

// ---- emission ------------------------------------------------------------------------------------------
// Per-row block rule, one wave per row: out[0..kr) = the kr candidates C < R with the largest keys
// (ties to the lower C) in ascending order, out[kr] = R (the forced diagonal block).  Lane l holds
// the keys of the candidates l, l + 64, ... in registers (T of them, R <= 64 T); slots past the
// row hold key 0, which no counting step below can reach.
template <int T>
__device__ inline void emit_row_select(const unsigned *row, int R, int kr, int32_t *out) {
  const int lane = threadIdx.x & 63;
  if (kr > 0) {
    unsigned key[T];
#pragma unroll
    for (int t = 0; t < T; ++t) key[t] = (64 * t + lane < R) ? row[64 * t + lane] : 0u;
    auto count_ge = [&](unsigned c) {  // c >= 1
      unsigned n = 0;
#pragma unroll
      for (int t = 0; t < T; ++t)
        if (64 * t < R) n += __popcll(__ballot(key[t] >= c));
      return n;
    };
    // the kr-th largest key: the largest t with at least kr keys >= t, found bit by bit
    unsigned thr = 0u;
    for (int bit = 31; bit >= 0; --bit) {
      const unsigned c = thr | (1u << bit);
      if (count_ge(c) >= (unsigned)kr) thr = c;
    }
    const unsigned gt = thr == 0xFFFFFFFFu ? 0u : count_ge(thr + 1u);
    const unsigned need = (unsigned)kr - gt;  // ties at the threshold, taken in index order
    const unsigned long long below = (1ull << lane) - 1ull;
    unsigned grun = 0, erun = 0;
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (64 * t < R) {
        const bool ok = 64 * t + lane < R;
        const bool isgt = ok && key[t] > thr, iseq = ok && key[t] == thr;
        const unsigned long long bg = __ballot(isgt), be = __ballot(iseq);
        const unsigned gb = grun + __popcll(bg & below), eb = erun + __popcll(be & below);
        if (isgt || (iseq && eb < need)) out[gb + min(eb, need)] = 64 * t + lane;
        grun += __popcll(bg);
        erun += __popcll(be);
      }
  }
  if (lane == 0) out[kr] = R;
}

__global__ __launch_bounds__(BT) void idx_emit_kernel(IdxArgs a) {
  const Shape &sh = a.sh;
  const int p = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int N = sh.N, nb = sh.nb;
  IdxScratch *G = a.scratch + h;
  const int pat = G->pattern;
  const int gw = p * WPB + wv;
  const int gtid = p * BT + tid, gthreads = a.P * BT;
  int32_t *cols = a.out.cols + (size_t)h * sh.k_v, *offs = a.out.offs + (size_t)h * sh.k_s;
  int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
  int32_t *bc = a.out.blkcols + (size_t)h * sh.cap_b;
  // columns and diagonals (Interval-Slash only)
  const int kv = pat == SA_INTERVAL_SLASH ? a.ksel[2] : 0, ks = pat == SA_INTERVAL_SLASH ? a.ksel[3] : 0;
  if (pat == SA_INTERVAL_SLASH) {
    const int lo = min(gw * a.seg, N), hi = min(lo + a.seg, N);
    for (int arr = 0; arr < 2; ++arr) {
      const unsigned thr = G->thr[arr + 2], need = G->need[arr + 2];
      unsigned grun = G->wgt[arr][gw], erun = G->weq[arr][gw];
      int32_t *out = arr ? offs : cols;
      if (a.ksel[arr + 2] > 0)
        wave_visit4((arr ? a.s : a.v) + (size_t)h * N, lo, hi, true, [&](const Keys4 &v, int i0, int lim) {
          emit_group(v, i0, lim, thr, need, grun, erun, [&](unsigned pos, int idx) { out[pos] = idx; });
        });
    }
  }
  for (int i = kv + gtid; i < sh.k_v; i += gthreads) cols[i] = -1;
  for (int i = ks + gtid; i < sh.k_s; i += gthreads) offs[i] = -1;
  if (gtid == 0) { a.out.n_cols[h] = kv; a.out.n_offs[h] = ks; }
  // block CSR
  int total;
  if (pat == SA_BLOCK_CLUSTER && sh.row_select) {
    total = rp[nb];  // the rows themselves are written by idx_emit_rows_kernel
  } else if (pat == SA_BLOCK_CLUSTER) {
    const unsigned thr = G->thr[4], need = G->need[4];
    unsigned grun = 0, erun = 0;
    wave_rows_visit4(
        a.blk + (size_t)h * nb * nb, nb, gw, a.PW, (nb & 3) == 0, sh.row_norm != 0,
        [&](int R) { grun = G->rowgt[R]; erun = G->roweq[R]; },
        [&](const Keys4 &v, int i0, int lim) {
          // lim is the row index R: a selected entry lands after the R diagonals of the rows above
          if (a.ksel[4] > 0)
            emit_group(v, i0, lim, thr, need, grun, erun, [&](unsigned pos, int C) { bc[pos + lim] = C; });
        },
        [&](int R) {
          if (lane == 0) bc[grun + min(erun, need) + R] = R;  // the forced diagonal block closes the row
        });
    total = a.ksel[4] + nb;
  } else if (pat == SA_TRIANGULAR) {
    for (int R = gtid; R < nb; R += gthreads) {
      const int run = rp[R];
      const int bs = max(R - sh.local + 1, 0);
      const int ns = min(sh.sink, bs);
      for (int C = 0; C < ns; ++C) bc[run + C] = C;
      for (int C = bs; C <= R; ++C) bc[run + ns + (C - bs)] = C;
    }
    total = rp[nb];
  } else {
    for (int R = gtid; R < nb; R += gthreads) bc[R] = R;
    total = nb;
  }
  for (int i = total + gtid; i < sh.cap_b; i += gthreads) bc[i] = -1;
}

// Per-row block rule: the rows of the Block-Cluster heads, wave gw of a head taking the rows
// gw, gw + PW, ...  T = 64-key slices a row can have (nb <= 64 T).
template <int T>
__global__ __launch_bounds__(BT) void idx_emit_rows_kernel(IdxArgs a) {
  const Shape &sh = a.sh;
  const int h = blockIdx.y, nb = sh.nb;
  if ((a.scratch + h)->pattern != SA_BLOCK_CLUSTER) return;
  const int gw = blockIdx.x * WPB + (threadIdx.x >> 6);
  const unsigned *hb = a.blk + (size_t)h * nb * nb;
  const int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
  int32_t *bc = a.out.blkcols + (size_t)h * sh.cap_b;
  for (int R = gw; R < nb; R += a.PW)
    emit_row_select<T>(hb + (size_t)R * nb, R, row_share(sh, R) - 1, bc + rp[R]);
}

// ---- diagonals at block granularity -----------------------------------------------------------------
// Interval-Slash heads when the selected diagonals are kept as whole blocks.  Runs after the
// emission, which has left the selected offsets in the index: one wave per row block R collects the
// key blocks that hold a key i - o of a query i of the row (at most two per offset) and the diagonal
// block in a bitmap (the wave's own LDS slice).  PASS 0 stores the number of blocks of the row,
// PASS 1 writes them in ascending order behind the row pointer.
template <int PASS>
__global__ __launch_bounds__(BT) void idx_diag_rows_kernel(IdxArgs a) {
  __shared__ unsigned bm[WPB][kMaxNb / 32];
  const Shape &sh = a.sh;
  const int h = blockIdx.y, nb = sh.nb, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  IdxScratch *G = a.scratch + h;
  if (G->pattern != SA_INTERVAL_SLASH) return;
  const int gw = blockIdx.x * WPB + wv;
  const int n_offs = a.out.n_offs[h];
  const int32_t *offs = a.out.offs + (size_t)h * sh.k_s;
  const int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
  int32_t *bc = a.out.blkcols + (size_t)h * sh.cap_b;
  const int shift = sh.b == 128 ? 7 : 6;
  unsigned *w = bm[wv];
  for (int R = gw; R < nb; R += a.PW) {
    const int words = (R >> 5) + 1;  // bits 0..R
    for (int i = lane; i < words; i += 64) w[i] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const long long first = (long long)R << shift, last = first + sh.b - 1;  // queries of the row
    for (int t = lane; t < n_offs; t += 64) {
      const long long o = offs[t];
      if (last - o < 0) continue;  // the diagonal starts below this row
      const int c0 = (int)((first - o > 0 ? first - o : 0) >> shift), c1 = (int)((last - o) >> shift);
      atomicOr(&w[c0 >> 5], 1u << (c0 & 31));
      if (c1 != c0) atomicOr(&w[c1 >> 5], 1u << (c1 & 31));
    }
    if (lane == 0) atomicOr(&w[R >> 5], 1u << (R & 31));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    int run = PASS == 1 ? rp[R] : 0;
    for (int i0 = 0; i0 < words; i0 += 64) {
      unsigned bits = i0 + lane < words ? w[i0 + lane] : 0u;
      const int pc = __popc(bits);
      int incl = pc;  // inclusive prefix over the lanes
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
      }
      if (PASS == 1) {
        int pos = run + incl - pc;
        while (bits) {
          const int bit = __ffs(bits) - 1;
          bits &= bits - 1;
          bc[pos++] = (i0 + lane) * 32 + bit;
        }
      }
      run += __shfl(incl, 63);
    }
    if (PASS == 0 && lane == 0) G->rowgt[R] = (unsigned)run;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the slice is cleared again for the next row
  }
}

// One workgroup per head: row pointers of the Interval-Slash heads from the per-row counts above.
__global__ __launch_bounds__(BT) void idx_diag_scan_kernel(IdxArgs a) {
  __shared__ unsigned s_wsum[2 * WPB];
  const int h = blockIdx.x, tid = threadIdx.x, nb = a.sh.nb;
  IdxScratch *G = a.scratch + h;
  if (G->pattern != SA_INTERVAL_SLASH) return;
  constexpr int RP = kMaxNb / BT;
  unsigned g[RP], sum = 0;
#pragma unroll
  for (int j = 0; j < RP; ++j) {
    const int R = RP * tid + j;
    g[j] = R < nb ? G->rowgt[R] : 0u;
    sum += g[j];
  }
  unsigned run = sum, unused = 0;
  block_exclusive_scan2(run, unused, s_wsum);
  int32_t *rp = a.out.rowptr + (size_t)h * (nb + 1);
#pragma unroll
  for (int j = 0; j < RP; ++j) {
    const int R = RP * tid + j;
    if (R < nb) rp[R] = (int)run;
    run += g[j];
    if (R == nb - 1) rp[nb] = (int)run;
  }
}

// The offsets are part of the block CSR now: hand back an empty list.
__global__ void idx_diag_done_kernel(IdxArgs a) {
  const int h = blockIdx.x;
  if ((a.scratch + h)->pattern != SA_INTERVAL_SLASH) return;
  int32_t *offs = a.out.offs + (size_t)h * a.sh.k_s;
  for (int i = threadIdx.x; i < a.sh.k_s; i += blockDim.x) offs[i] = -1;
  if (threadIdx.x == 0) a.out.n_offs[h] = 0;
}

}  // namespace

size_t index_scratch_bytes(int n_heads) { return sizeof(IdxScratch) * (size_t)n_heads; }

namespace {

IdxArgs index_args(const Shape &sh, const Workspace &ws, sa_scores in, const Override &ov, sa_index out) {
  IdxArgs a;
  a.v = (const unsigned *)in.v; a.s = (const unsigned *)in.s; a.blk = (const unsigned *)in.blk;
  a.scratch = (IdxScratch *)ws.idx;
  a.sh = sh; a.ov = ov; a.out = out;
  // Workgroups per head.  Every launch is a chain of dependent memory round trips per wave, so more,
  // shorter waves win until the per-workgroup costs (clearing and flushing the LDS histograms) take
  // over: measured best at 32 per head up to 64K tokens and 64 at 128K, 256 keys per wave at least.
  int P = sh.N / 256;
  const int pmax = sh.N <= 65536 ? 32 : kMaxParts;
  if (P < 1) P = 1;
  if (P > pmax) P = pmax;
  a.P = P; a.PW = P * WPB;
  a.seg = ((sh.N + a.PW - 1) / a.PW + 255) / 256 * 256;
  const long long ncand = (long long)sh.nb * (sh.nb - 1) / 2;
  long long kb = (long long)sh.k_b - sh.nb;
  if (kb < 0) kb = 0;
  if (kb > ncand) kb = ncand;
  a.ksel[0] = sh.probe_v < sh.N ? sh.probe_v : sh.N;
  a.ksel[1] = sh.probe_s < sh.N ? sh.probe_s : sh.N;
  a.ksel[2] = sh.k_v < sh.N ? sh.k_v : sh.N;
  a.ksel[3] = sh.k_s < sh.N ? sh.k_s : sh.N;
  a.ksel[4] = sh.row_select ? 0 : (int)kb;   // per-row rule: selected row by row while emitting
  a.mask = 3;
  a.decided = nullptr;
  static_assert(kMaxHeads == 128, "four mask words");
  for (int w = 0; w < kMaxHeads / 32; ++w) a.skip_vs[w] = a.skip_blk[w] = 0u;
  for (int h = 0; h < sh.Hq; ++h) {
    const int p = ov.pat[h];
    if (p >= 0 && p != SA_INTERVAL_SLASH) a.skip_vs[h >> 5] |= 1u << (h & 31);
    if (p >= 0 && p != SA_BLOCK_CLUSTER) a.skip_blk[h >> 5] |= 1u << (h & 31);
  }
  return a;
}

void launch_levels(const IdxArgs &a, hipStream_t st) {
  const dim3 grid(a.P, a.sh.Hq);
  idx_hist_kernel<1><<<grid, BT, 0, st>>>(a);
  idx_select_kernel<1><<<a.sh.Hq, BT, 0, st>>>(a);
  idx_hist_kernel<2><<<grid, BT, 0, st>>>(a);
  idx_select_kernel<2><<<a.sh.Hq, BT, 0, st>>>(a);
  idx_hist_kernel<3><<<grid, BT, 0, st>>>(a);
  idx_select_kernel<3><<<a.sh.Hq, BT, 0, st>>>(a);
  idx_count_kernel<<<grid, BT, 0, st>>>(a);
}

void launch_finish(const IdxArgs &a, hipStream_t st) {
  const dim3 grid(a.P, a.sh.Hq);
  idx_scan_kernel<<<a.sh.Hq, BT, 0, st>>>(a);
  idx_emit_kernel<<<grid, BT, 0, st>>>(a);
  if (a.sh.row_select) {
    if (a.sh.nb <= 256) idx_emit_rows_kernel<4><<<grid, BT, 0, st>>>(a);
    else if (a.sh.nb <= 1024) idx_emit_rows_kernel<16><<<grid, BT, 0, st>>>(a);
    else idx_emit_rows_kernel<kMaxNb / 64><<<grid, BT, 0, st>>>(a);
  }
  if (a.sh.diag_blocks) {
    idx_diag_rows_kernel<0><<<grid, BT, 0, st>>>(a);
    idx_diag_scan_kernel<<<a.sh.Hq, BT, 0, st>>>(a);
    idx_diag_rows_kernel<1><<<grid, BT, 0, st>>>(a);
    idx_diag_done_kernel<<<a.sh.Hq, BT, 0, st>>>(a);
  }
}

}  // namespace

hipError_t launch_build_index(const Shape &sh, const Workspace &ws, sa_scores in, const Override &ov,
                              sa_index out, hipStream_t st) {
  const IdxArgs a = index_args(sh, ws, in, ov, out);
  idx_zero_kernel<<<sh.Hq, 256, 0, st>>>(a.scratch);
  launch_levels(a, st);
  launch_finish(a, st);
  return hipGetLastError();
}

// The same work in parts, so that it can run beside the estimator: the selections on v and s as
// soon as the window passes are done, the block-map selection as soon as the block map is (on
// another stream), and the emission once both are.  Decide (after ColumnsDiagonals) writes the
// patterns early, for a caller that computes the block map only where it is needed.
hipError_t launch_index_stage(const Shape &sh, const Workspace &ws, sa_scores in, const Override &ov,
                              sa_index out, IndexStage stage, hipStream_t st, bool lazy) {
  IdxArgs a = index_args(sh, ws, in, ov, out);
  if (lazy) a.decided = out.pattern;
  switch (stage) {
    case IndexStage::Zero:
      idx_zero_kernel<<<sh.Hq, 256, 0, st>>>(a.scratch);
      break;
    case IndexStage::ColumnsDiagonals:
      a.mask = 1;
      launch_levels(a, st);
      break;
    case IndexStage::Decide:
      idx_decide_kernel<<<(sh.Hq + 63) / 64, 64, 0, st>>>(a);
      break;
    case IndexStage::Blocks:
      a.mask = 2;
      if (!sh.row_select) launch_levels(a, st);
      break;
    case IndexStage::Emit:
      launch_finish(a, st);
      break;
  }
  return hipGetLastError();
}

}  // namespace sa
