// Sparse causal prefill attention for gfx950 (Alg. 2 / Alg. 3 "Compute Sparse
// Attention": softmax over the kept keys only, then the product with V).
//
// One workgroup = 128 query rows of one head (4 waves x 32 rows), two workgroups
// per compute unit, fed from work queues.  A (head, row block) item has two phases:
//   * tiles of 64 keys through LDS, shared by the four waves:
//       range tiles  - aligned key tiles of the key blocks the CSR keeps;
//       gather tiles - 64 selected key columns, gathered once per call into
//                      contiguous buffers, so that they are read like any tile;
//   * selected diagonals, one 32-key tile per wave and offset, without barriers.
// A key is counted once: selected columns are masked out of range tiles and
// diagonal entries whose key is a selected column or lies in a kept block are
// dropped.  Per tile each wave computes S^T = K Q^T (keys x queries) with
// v_mfma_f32_32x32x16_bf16, so that one lane owns one query: the online softmax
// needs a single cross-lane exchange, and the probabilities are already laid out
// as the B operand of O^T += V^T P^T.
#include "sa_internal.h"

namespace sa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int BQ = 128;           // query rows per workgroup
constexpr int BK = 64;            // keys per tile
constexpr int NWORDS = kMaxSeq / BK / 32;

struct AttnArgs {
  const uint16_t *Q, *K, *V;
  uint16_t *O;
  const int32_t *n_cols, *cols, *n_offs, *offs, *rowptr, *blkcols;
  const uint32_t *colbits;   // [Hq][N/32] membership bitmap of the selected columns
  const int32_t *colprefix;  // [Hq][N/32] selected columns before each word of colbits
  uint16_t *Kg, *Vg;  // [Hq][kvg_rows][kv_rs] selected key columns, gathered once per call
  int kvg_rows;
  int Hq, Hkv, g, N, b, nb, nT, k_v, k_s, cap_b;
  int64_t q_hs, q_rs, kv_hs, kv_rs;
  float c;  // softmax scale * log2(e)
  unsigned int *queue;           // [8] work-queue heads, zeroed by index_prepare_kernel
  int n_items;  // (head, row block) items in all
  int xs;       // queues (XCDs) that share one KV head at a time: 1, 2, 4 or 8
  int qcap;     // tickets per queue, holes of the id space included
  unsigned long long *counters;  // instrumentation only: {32x32 sub-tiles multiplied, kept (query,key) pairs}
  // Per KV head, written by index_prepare_kernel: [0] = number c of its query heads without
  // selected diagonals, [1..g] = the query heads of the group (0..g-1), those c first.
  int32_t *hperm;
};

// Read-only words at a wave-uniform address: through the constant address space these become
// scalar loads, which neither occupy the vector memory path nor count in vmcnt.
typedef const uint32_t __attribute__((address_space(4))) *const_u32p;
__device__ inline uint32_t uload(const void *p, int idx) { return ((const_u32p)(uintptr_t)p)[idx]; }

// 32 bits of a bitmap starting at bit `pos` (may be negative or run past the end); pos wave-uniform.
__device__ inline uint32_t bits_window32(const uint32_t *bm, int nw, int pos) {
  const int wi = pos >> 5, sh = pos & 31;  // arithmetic shift: floor for negatives
  uint32_t lo = uload(bm, min(max(wi, 0), nw - 1)), hi = uload(bm, min(max(wi + 1, 0), nw - 1));
  lo = (wi >= 0 && wi < nw) ? lo : 0u;
  hi = (wi + 1 >= 0 && wi + 1 < nw) ? hi : 0u;
  return (uint32_t)(((uint64_t)lo | ((uint64_t)hi << 32)) >> sh);
}

// What the attention kernel needs from the index before it starts, in one launch of 256-thread
// blocks.  Blocks 0 .. Hq-1: membership bitmap of a head's selected columns and the running count
// of selected columns before each bitmap word (built in LDS, written out once); block 0 also
// resets the work-queue heads.  The other blocks, (gather tile g, head h) = Hq + h * ntile + g:
// the selected key columns of every head are copied once into contiguous [k][d] buffers so that
// the attention kernel reads gather tiles like any other tile.
__global__ __launch_bounds__(256) void index_prepare_kernel(AttnArgs p, unsigned int *queue) {
  __shared__ uint32_t bm[kMaxSeq / 32];
  __shared__ int wsum[4];
  const int tid = threadIdx.x;
  if ((int)blockIdx.x < p.Hq) {
    const int h = blockIdx.x, nw = p.N / 32, lane = tid & 63, wv = tid >> 6;
    if (h == 0 && tid < 8) queue[tid] = 0u;
    if (h < p.Hkv && tid == 0) {  // the order in which the attention kernel walks the heads of KV head h
      int32_t *pm = p.hperm + (size_t)h * (p.g + 1);
      int c = 0;
      for (int j = 0; j < p.g; ++j)
        if (p.n_offs[h * p.g + j] <= 0) pm[1 + c++] = j;
      pm[0] = c;
      for (int j = 0; j < p.g; ++j)
        if (p.n_offs[h * p.g + j] > 0) pm[1 + c++] = j;
    }
    for (int i = tid; i < nw; i += 256) bm[i] = 0u;
    __syncthreads();
    const int nc = min(max(p.n_cols[h], 0), p.k_v);
    for (int i = tid; i < nc; i += 256) {
      const int c = p.cols[(size_t)h * p.k_v + i];
      if (c >= 0 && c < p.N) atomicOr(&bm[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    // exclusive prefix popcount: thread t owns a contiguous run of words
    const int per = (nw + 255) / 256;
    const int w0 = min(tid * per, nw), w1 = min(w0 + per, nw);
    int mine = 0;
    for (int w = w0; w < w1; ++w) mine += __popc(bm[w]);
    int incl = mine;
    for (int dd = 1; dd < 64; dd <<= 1) {
      const int o = __shfl_up(incl, dd);
      if (lane >= dd) incl += o;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int run = incl - mine;
    for (int k = 0; k < wv; ++k) run += wsum[k];
    uint32_t *cb = const_cast<uint32_t *>(p.colbits) + (size_t)h * nw;
    int32_t *cp = const_cast<int32_t *>(p.colprefix) + (size_t)h * nw;
    for (int w = w0; w < w1; ++w) {
      const uint32_t word = bm[w];
      cb[w] = word;
      cp[w] = run;
      run += __popc(word);
    }
    return;
  }
  const int ntile = p.kvg_rows / BK;
  const int h = ((int)blockIdx.x - p.Hq) / ntile, g = ((int)blockIdx.x - p.Hq) % ntile;
  const int nc = min(max(p.n_cols[h], 0), p.k_v);
  if (g * BK >= nc) return;
  const int kvh = h / p.g;
  const int lrow = tid >> 4, lcc = tid & 15;
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    const int ci = g * BK + lrow + 16 * n;
    int src = ci < nc ? p.cols[(size_t)h * p.k_v + ci] : 0;
    src = min(max(src, 0), p.N - 1);
    const size_t so = (size_t)kvh * p.kv_hs + (size_t)src * p.kv_rs + lcc * 8;
    const size_t dofs = ((size_t)h * p.kvg_rows + ci) * p.kv_rs + lcc * 8;  // same row stride as K / V
    *(uint4 *)(p.Kg + dofs) = *(const uint4 *)(p.K + so);
    *(uint4 *)(p.Vg + dofs) = *(const uint4 *)(p.V + so);
  }
}

// LDS tiles are 64 rows x 256 B with the 16-byte chunks of a row XOR-swizzled (no padding):
//   K: chunk c of row r sits at chunk c ^ (r & 15)      -> b128 reads of 16 rows hit 64 banks
//   V: chunk c of row r sits at chunk c ^ ((r & 3) << 2) -> the transposing b64 reads do
__device__ inline int vswz(int row, int chunk) { return row * 128 + ((chunk ^ ((row & 3) << 2)) << 3); }

template <bool STATS>
__global__ __launch_bounds__(256, 2) void sparse_prefill_kernel(AttnArgs p) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][BK * 128];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][BK * 128];
  __shared__ uint32_t need[NWORDS], kept0[NWORDS], kept1[NWORDS];
  __shared__ uint16_t tlist[kMaxSeq / BK];
  __shared__ int s_ntiles;
  __shared__ int s_cmax[4];

  const int wv = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);  // wave-uniform for the compiler too

  // Persistent workgroups pull (head, row block) items from eight queues, one per XCD
  // (consecutive workgroup ids land on consecutive XCDs).  xs queues share one KV head at a time
  // and 8/xs KV heads are in progress together: with xs = 1 a KV head lives in a single L2, with
  // larger xs fewer KV heads are live at once, so that the rows the diagonal phase fetches (no
  // reuse inside an L2) come out of the memory-side cache instead of HBM.  Ticket k of queue qn:
  // phase k / per_q selects the KV head, the rest walks the row blocks qn % xs, qn % xs + xs, ...
  // from the last (longest) one down: first for the query heads of the group that have no
  // selected diagonals, side by side per row block, then for each head with diagonals by itself
  // (the order index_prepare_kernel left in hperm).  A
  // workgroup whose own queue is empty takes from the others, then exits.  The ticket for the
  // next item of the home queue is drawn while the current item finishes, so its round trip is
  // off the critical path.
  __shared__ int s_item;
  const int home = blockIdx.x & 7;
  int ticket = 0;            // thread 0 only: position drawn from the home queue
  bool have_ticket = false;  // thread 0 only: ticket was drawn ahead and is not used yet
  bool home_open = true;     // thread 0 only: the home queue still had items at the last draw
  for (;;) {
  // Lane-derived constants are recomputed per item from an opaque copy of the thread id:
  // hoisted out of this loop they would stay live across every phase and spill.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, q = lane & 31, gg = lane >> 5;
  __syncthreads();  // previous item fully retired: LDS work lists and tiles may be reused
  if (tid == 0) {
    int item = -1;
    if (home_open) {
      if (!have_ticket) ticket = (int)atomicAdd(&p.queue[home], 1u);
      have_ticket = false;
      if (ticket < p.qcap) item = home + 8 * ticket;
      else home_open = false;
    }
    for (int qq = 1; qq < 8 && item < 0; ++qq) {
      const int qn = (home + qq) & 7;
      if ((int)__hip_atomic_load(&p.queue[qn], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= p.qcap)
        continue;
      const int k = (int)atomicAdd(&p.queue[qn], 1u);
      if (k < p.qcap) item = qn + 8 * k;
    }
    s_item = item;
  }
  __syncthreads();
  const int id = __builtin_amdgcn_readfirstlane(s_item);
  if (id < 0) break;
  int kvh, h, t128;
  {
    const int qn = id & 7, k = id >> 3;
    const int nslots = 8 / p.xs, slot = qn / p.xs, sub = qn % p.xs;
    const int per_q = (p.nT + p.xs - 1) / p.xs * p.g;
    const int r = k % per_q;
    kvh = k / per_q * nslots + slot;
    if (kvh >= p.Hkv) continue;  // a hole of the id space
    // Heads without selected diagonals walk a row block side by side (their tiles overlap: the
    // band of Triangular heads is the same for all of them); heads with diagonals follow one at a
    // time (their diagonal phase re-reads nothing, and one head's gathered columns stay in L2).
    const int rows_q = per_q / p.g;
    const int32_t *pm = p.hperm + (size_t)kvh * (p.g + 1);
    const int c = min(max((int)uload(pm, 0), 0), p.g);
    int slot_h, trow;
    if (r < c * rows_q) {
      slot_h = r % c; trow = r / c;
    } else {
      const int r2 = r - c * rows_q;
      slot_h = c + r2 / rows_q; trow = r2 % rows_q;
    }
    const int tidx = trow * p.xs + sub;
    if (tidx >= p.nT) continue;  // a hole of the id space
    h = kvh * p.g + min(max((int)uload(pm, 1 + slot_h), 0), p.g - 1);
    t128 = p.nT - 1 - tidx;
  }
  const int i0 = t128 * BQ;
  const int r0 = i0 + 32 * wv;
  const int iq = r0 + q;  // this lane's query row
  const int N = p.N;
  const int ilast = min(i0 + BQ, N) - 1;

  // long-latency reads first: they overlap the construction of the tile list
  bf16x8 qf[8];  // Q^T fragments: B operand, lane = query, 8 consecutive d per k-step half
  {
    const uint16_t *qrow = p.Q + (size_t)h * p.q_hs + (size_t)min(iq, N - 1) * p.q_rs;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8 *)(qrow + 16 * ks + 8 * gg);
  }
  // the item's small reads sit at wave-uniform addresses: scalar loads, all in flight together
  const int nc = min(max((int)uload(p.n_cols, h), 0), p.k_v);
  const bool has_offs = (int)uload(p.n_offs, h) > 0;
  // CSR entry ranges of the row blocks of this item: one at block 128, two (2*t128 for waves 0,1
  // and 2*t128+1 for waves 2,3) at block 64
  const int32_t *rp = p.rowptr + (size_t)h * (p.nb + 1);
  const int Ra = p.b == BQ ? t128 : 2 * t128;
  const bool two = p.b != BQ && Ra + 1 < p.nb;
  const int ea0 = max((int)uload(rp, Ra), 0), ea1 = min((int)uload(rp, Ra + 1), p.cap_b);
  const int eb0 = max((int)uload(rp, min(Ra + 1, p.nb)), 0), eb1 = min((int)uload(rp, min(Ra + 2, p.nb)), p.cap_b);
  const int na = max(ea1 - ea0, 0), nbk = two ? max(eb1 - eb0, 0) : 0;
  // selected columns visible to this query = those up to its own position: the running count
  // before its bitmap word plus the bits of that word up to the position (the list is ascending
  // and without repeats, so this is also the query's cut in the gathered list)
  int cle;
  {
    const int key = min(iq, N - 1), wi = key >> 5;
    const size_t bo = (size_t)h * (N / 32) + wi;
    cle = p.colprefix[bo] + __popc(p.colbits[bo] & (0xFFFFFFFFu >> (31 - (key & 31))));
    cle = nc > 0 ? cle : 0;
  }

  // ---- tile list of this row block -------------------------------------------------------
  const int nwords = ((ilast / BK + 1) + 31) / 32;
  for (int i = tid; i < nwords; i += 256) { need[i] = 0u; kept0[i] = 0u; kept1[i] = 0u; }
  __syncthreads();
  {
    // one pass over the entries of both row blocks, so that their reads are in flight together
    const int32_t *bc = p.blkcols + (size_t)h * p.cap_b;
    const int tpb = p.b / BK;  // key tiles per key block: their bits are adjacent in one word
    const uint32_t tbits = tpb == 2 ? 3u : 1u;
    for (int e = tid; e < na + nbk; e += 256) {
      const bool second = e >= na;
      const int C = bc[second ? eb0 + (e - na) : ea0 + e];
      if (C >= 0 && C <= Ra + (second ? 1 : 0)) {
        const int kt = C * tpb;
        atomicOr(&need[kt >> 5], tbits << (kt & 31));
        if (!second) atomicOr(&kept0[kt >> 5], tbits << (kt & 31));
        if (second || p.b == BQ) atomicOr(&kept1[kt >> 5], tbits << (kt & 31));
      }
    }
  }
  __syncthreads();
  if (wv == 0) {  // ordered compaction of the set bits into tlist
    int base = 0;
    for (int w0 = 0; w0 < nwords; w0 += 64) {
      const uint32_t word = (w0 + lane < nwords) ? need[w0 + lane] : 0u;
      const int cnt = __popc(word);
      int incl = cnt;
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
      }
      int pos = base + incl - cnt;
      uint32_t wbits = word;
      // the keep words are read once: the loop below then has no LDS read to wait for
      const uint32_t k0 = (w0 + lane < nwords) ? kept0[w0 + lane] : 0u, k1 = (w0 + lane < nwords) ? kept1[w0 + lane] : 0u;
      while (wbits) {
        const int bit = __ffs(wbits) - 1;
        wbits &= wbits - 1;
        // entry: key tile (bits 0..11), kept by waves 0,1 (bit 14) / by waves 2,3 (bit 15)
        tlist[pos++] = (uint16_t)(((w0 + lane) * 32 + bit) | (((k0 >> bit) & 1u) << 14) | (((k1 >> bit) & 1u) << 15));
      }
      base += __shfl(incl, 63);
    }
    if (lane == 0) s_ntiles = base;
  }

  int cmax = cle, cmin = cle;  // gather tiles this wave needs: up to its last query's cut; its first query's cut
  for (int d = 32; d >= 1; d >>= 1) {
    cmax = max(cmax, __shfl_xor(cmax, d));
    cmin = min(cmin, __shfl_xor(cmin, d));
  }
  if (lane == 0) s_cmax[wv] = cmax;
  __syncthreads();
  const int ntr = __builtin_amdgcn_readfirstlane(s_ntiles);
  const int cwave = __builtin_amdgcn_readfirstlane(cmax), cwmin = __builtin_amdgcn_readfirstlane(cmin);
  const int call = __builtin_amdgcn_readfirstlane(max(max(s_cmax[0], s_cmax[1]), max(s_cmax[2], s_cmax[3])));
  const int ng = (call + BK - 1) / BK;
  const int ntot = ntr + ng;
  const bool has_cols = nc > 0;

  // ---- operands ------------------------------------------------------------------------------
  const uint16_t *__restrict__ Kh = p.K + (size_t)kvh * p.kv_hs;
  const uint16_t *__restrict__ Vh = p.V + (size_t)kvh * p.kv_hs;
  const uint16_t *__restrict__ Kgh = p.Kg + (size_t)h * p.kvg_rows * p.kv_rs;
  const uint16_t *__restrict__ Vgh = p.Vg + (size_t)h * p.kvg_rows * p.kv_rs;
  const uint32_t *__restrict__ colbm = p.colbits + (size_t)h * (N / 32);

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 lacc[2] = {};  // the tile loop's share of the normaliser (every register of a lane holds the same sum)
  unsigned st_kept = 0u, st_tiles = 0u;  // counted variant: this lane's kept pairs, this wave's sub-tiles

  // ---- global -> LDS pipeline -----------------------------------------------------------------
  // K and V tiles go straight from global memory into LDS (global_load_lds_dwordx4: 16 bytes per
  // lane, LDS address = M0 + 16*lane, so one instruction fills four 256-byte rows).  The XOR
  // swizzle is applied on the global side: the lane that owns physical chunk pc of row r fetches
  // logical chunk pc ^ swz(r).  Wave w moves rows 4w..4w+3 (+16n, n = 0..3) of both tiles.
  const int rl = 4 * wv + (lane >> 4);  // (row & 15) of the rows this lane moves; (row & 3) = lane >> 4
  const unsigned dmaK = (unsigned)(rl * (int)p.kv_rs * 2 + (((lane & 15) ^ rl) << 4));
  const unsigned dmaV = (unsigned)(rl * (int)p.kv_rs * 2 + (((lane & 15) ^ ((lane >> 4) << 2)) << 4));
  const unsigned ldsK0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)&Ks[0][0] + 4 * wv * 256;
  const unsigned ldsV0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)&Vs[0][0] + 4 * wv * 256;
  const size_t row16 = 16 * (size_t)p.kv_rs;  // elements between the rows of consecutive instructions
#define SA_DMA16(gptr, voff, ldsb)                                                                    \
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(gptr), \
               "s"(ldsb)                                                                              \
               : "memory")
#define SA_ISSUE_TILE(t, buf, ent)                                                                  \
  {                                                                                              \
    const uint16_t *kb, *vb;                                                                     \
    if ((t) < ntr) {                                                                             \
      const size_t j0_ = (size_t)((ent) & 0xFFF) * BK * p.kv_rs;                                 \
      kb = Kh + j0_; vb = Vh + j0_;                                                              \
    } else {                                                                                     \
      const size_t g0_ = (size_t)((t) - ntr) * BK * p.kv_rs;                                     \
      kb = Kgh + g0_; vb = Vgh + g0_;                                                            \
    }                                                                                            \
    const unsigned lk = ldsK0 + (buf) * (BK * 256), lv = ldsV0 + (buf) * (BK * 256);             \
    SA_DMA16(kb, dmaK, lk); SA_DMA16(kb + row16, dmaK, lk + 16 * 256);                           \
    SA_DMA16(kb + 2 * row16, dmaK, lk + 32 * 256); SA_DMA16(kb + 3 * row16, dmaK, lk + 48 * 256); \
    SA_DMA16(vb, dmaV, lv); SA_DMA16(vb + row16, dmaV, lv + 16 * 256);                           \
    SA_DMA16(vb + 2 * row16, dmaV, lv + 32 * 256); SA_DMA16(vb + 3 * row16, dmaV, lv + 48 * 256); \
  }

  // per-lane LDS byte offsets of the operand reads.  The swizzles only touch address bits 4..7,
  // so every access is (one per-lane base) XOR (a compile-time constant):
  //   K (A of S^T): row 32hf + q, chunk 2ks + gg -> b128 at kbase ^ ((2ks + gg) << 4) + 32hf*256
  //   V (A of O^T, transposing read): within 16 lanes, source lane r supplies the 8-byte piece
  //   (key r/4, d 4(r%4)..+3) and receives (keys 0..3, d r); lanes 16..31 take d 16..31:
  //   row 4gg + r/4 (+ multiples of 4), chunk 4db + 2grp + (r%4)/2 -> b64 at vbase ^ (db << 6)
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const unsigned kbase = (unsigned)(q * 256) | (unsigned)((q & 15) << 4);
  unsigned vbase;
  {
    const int r = lane & 15, grp = (lane >> 4) & 1;
    const int row = 4 * gg + (r >> 2);
    vbase = (unsigned)(row * 256) | (unsigned)(((2 * grp + ((r & 3) >> 1)) ^ ((row & 3) << 2)) << 4) |
            (unsigned)((r & 1) << 3);
  }
#define SA_KFRAG(tile, hf, ks) \
  (*(const bf16x8 *)((const char *)(tile) + ((kbase ^ (unsigned)((2 * (ks) + gg) << 4)) + (hf) * 32 * 256)))
#define SA_VTR(tile, db, key0) \
  __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)((const char *)(tile) + ((vbase ^ (unsigned)((db) << 6)) + (key0) * 256)))

  // list entries travel one tile ahead in scalar registers, so that neither the copy of the next
  // tile nor this tile's keep test waits for an LDS read behind the barrier
  int e_cur = __builtin_amdgcn_readfirstlane((int)tlist[0]);
  int r_nxt = (int)tlist[1];  // raw LDS value: made scalar only where it is used, a tile later
  if (ntot > 0) SA_ISSUE_TILE(0, 0, e_cur);

  for (int t = 0; t < ntot; ++t) {
    const int cur = t & 1;
    // this wave's share of tile t has landed (nothing else is in flight); after the barrier the
    // whole tile is in LDS[cur] and every wave has finished reading LDS[cur^1] (tile t-1)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    const int e_nxt = __builtin_amdgcn_readfirstlane(r_nxt);
    if (t + 1 < ntot) SA_ISSUE_TILE(t + 1, cur ^ 1, e_nxt);
    const int e_this = e_cur;
    e_cur = e_nxt;
    r_nxt = (int)tlist[min(t + 2, kMaxSeq / BK - 1)];

    // ---- what this wave keeps of the tile: a 64-bit mask per lane over the key slots ---------
    // slot c (0..59 used) stands for key_local = c + 4*gg; see the accumulator layout below.
    // Without selected columns inside the tile the mask is a threshold (slot c kept iff c <= lim),
    // applied with one compare per element; km is then only needed by the counted variant.
    bool active, needmask, bits = false;
    uint64_t km;
    int lim = 63;
    if (t < ntr) {
      const int kt = e_this & 0xFFF;
      const int j0 = kt * BK;
      const bool bk = ((e_this >> (wv < 2 ? 14 : 15)) & 1) != 0;
      const bool beyond = j0 > min(r0 + 31, N - 1);
      active = !beyond && bk;
      const uint64_t vm = has_cols ? ((uint64_t)uload(colbm, 2 * kt) | ((uint64_t)uload(colbm, 2 * kt + 1) << 32)) : 0ull;
      needmask = !(vm == 0 && j0 + 63 <= r0);
      km = ~0ull;
      bits = vm != 0;
      if (active && needmask) {
        lim = iq - j0 - 4 * gg;  // causal: slot c kept iff c <= lim
        const uint64_t cm = lim < 0 ? 0ull : (lim >= 63 ? ~0ull : ((2ull << lim) - 1ull));
        km = cm & ~(vm >> (4 * gg));  // selected columns are served by the gather tiles
      }
    } else {
      const int gi = t - ntr;
      active = cwave > gi * BK;
      needmask = cwmin < (gi + 1) * BK;  // some query of the wave sees only a part of this tile
      km = ~0ull;
      if (needmask) {
        lim = cle - gi * BK - 1 - 4 * gg;  // visible columns of this tile for this query, as a slot limit
        km = lim < 0 ? 0ull : (lim >= 63 ? ~0ull : ((2ull << lim) - 1ull));
      }
    }
    if (!active) continue;
    if constexpr (STATS) {
      // slots this lane owns: c = 32hf + 8(r/4) + r%4
      st_kept += iq < N ? (unsigned)__popcll(km & 0x0F0F0F0F0F0F0F0Full) : 0u;
      st_tiles += 2u;
    }

    // ---- S^T = K Q^T : lane = query (q), accumulator r of half hf <-> key 32hf + 8(r/4) + 4gg + r%4
    const uint16_t *Kt = Ks[cur];
    f32x16 sacc[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[hf][r] = 0.f;
    {
      // the 16 K fragments go through a ring of four registers: the LDS read of fragment i+4 is
      // issued right after the MFMA that consumed fragment i, so reads stay 3-4 deep in flight
      bf16x8 kf[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) kf[i] = SA_KFRAG(Kt, 0, i);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int hf = i >> 3, ks = i & 7;
        sacc[hf] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i & 3], qf[ks], sacc[hf], 0, 0, 0);
        if (i + 4 < 16) kf[i & 3] = SA_KFRAG(Kt, (i + 4) >> 3, (i + 4) & 7);
      }
      // keep that order through instruction scheduling: 4 LDS reads, then MFMA / LDS read pairs
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int i = 0; i < 12; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    if (needmask) {
      if (bits) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * hf + 8 * (r / 4) + (r % 4);
            if (!((km >> c) & 1ull)) sacc[hf][r] = -INFINITY;
          }
      } else {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * hf + 8 * (r / 4) + (r % 4);
            if (c > lim) sacc[hf][r] = -INFINITY;
          }
      }
    }
    // ---- online softmax (log2 domain) -----------------------------------------------------------
    // a wave in its matrix phases (from here on: P V, the wait for the next tile, K Q^T) is issued ahead of
    // the other wave of the SIMD while that one does softmax arithmetic: measured 1-2 % on the tile loop
    __builtin_amdgcn_s_setprio(0);
    float tmax = -INFINITY;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[hf][r]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_new = fmaxf(m_run, tmax * p.c);
    // The reference maximum moves only when some row's maximum grew by more than 2^8: until
    // then probabilities may exceed 1 (by at most 256x), which fp32 sums and bf16 P hold easily,
    // and the 64 accumulator registers are not rescaled.
    if (__any(m_new - m_run > 8.f)) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
      m_run = m_new;
      lacc[0] *= alpha;
      lacc[1] *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    const float m_ref = (m_run == -INFINITY) ? 0.f : m_run;
    // Probabilities of key step g (8 of this lane's 32 entries, the B operand of that step's four
    // MFMAs), one pair at a time: exp2 of the pair j of step g, and its conversion to packed bf16.
    auto soft2 = [&](int g, int j) {
#pragma unroll
      for (int e = 2 * j; e < 2 * j + 2; ++e)
        sacc[g >> 1][8 * (g & 1) + e] =
            __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[g >> 1][8 * (g & 1) + e], p.c, -m_ref));
    };
    u32x4 pbuf[2];  // packed bf16 pairs of two consecutive steps
    auto cvt2 = [&](int g, int j) {
      const bf16x2 pr = {(__bf16)sacc[g >> 1][8 * (g & 1) + 2 * j], (__bf16)sacc[g >> 1][8 * (g & 1) + 2 * j + 1]};
      pbuf[g & 1][j] = __builtin_bit_cast(uint32_t, pr);
    };
    // The normaliser sums the probabilities as the matrix pipe sees them, rounded to bf16: the weights
    // p~ / sum p~ then add up to one exactly and a row's output stays a convex combination of its V
    // rows whatever the rounding of the individual p (with an fp32 sum of the unrounded p, a row with
    // a handful of kept keys shows the rounding of its dominant weight at full size).
    // v_mfma_f32_4x4x4_16b_bf16 with an all-ones A operand leaves, in every output register of a
    // lane, the sum of the four bf16 values the lane passed as B: two of them per key step
    // (2 passes each) replace eight additions on the vector ALU.
    const s16x4 ones4 = {0x3f80, 0x3f80, 0x3f80, 0x3f80};
    // ---- O^T += V^T P^T : k-slot (gg,e) of step (hf,u) <-> key 32hf + 16u + 8(e/4) + 4gg + e%4 ----
    const uint16_t *Vt = Vs[cur];
    {
      // 16 V^T fragments (4 key steps x 4 d blocks), each two transposing reads; same ring of four
      s16x4 vlo[4], vhi[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) soft2(0, j);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        vlo[i] = SA_VTR(Vt, i & 3, 16 * (i >> 2));
        vhi[i] = SA_VTR(Vt, i & 3, 16 * (i >> 2) + 8);
      }
#pragma unroll
      for (int j = 0; j < 3; ++j) cvt2(0, j);
      __builtin_amdgcn_s_setprio(1);
      // One slot per MFMA, in program order and fenced: the product, the two LDS reads that refill
      // its V fragment, a quarter of the next step's exponentials and the conversion of the quarter
      // before.  Vector-ALU and matrix instructions of one wave overlap only when they alternate
      // in its instruction stream.
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int g = i >> 2, db = i & 3;  // key step g = 2*hf + u covers keys 16g .. 16g+15
        if (db == 0) {
          cvt2(g, 3);
          asm("" : "+v"(pbuf[g & 1]));  // opaque from here on: halves are sub-registers, not new conversions
        }
        const bf16x8 pb = __builtin_bit_cast(bf16x8, pbuf[g & 1]);
        const s16x8 av = __builtin_shufflevector(vlo[i & 3], vhi[i & 3], 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, oacc[db], 0, 0, 0);
        {  // the step's row sums: low half in the first slot, high half in the last (placement swept: flat)
          const s16x8 ps = __builtin_bit_cast(s16x8, pb);
          if (db == 0)
            lacc[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ones4, __builtin_shufflevector(ps, ps, 0, 1, 2, 3), lacc[0], 0, 0, 0);
          if (db == 3)
            lacc[1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ones4, __builtin_shufflevector(ps, ps, 4, 5, 6, 7), lacc[1], 0, 0, 0);
        }
        if (i + 4 < 16) {
          vlo[i & 3] = SA_VTR(Vt, (i + 4) & 3, 16 * ((i + 4) >> 2));
          vhi[i & 3] = SA_VTR(Vt, (i + 4) & 3, 16 * ((i + 4) >> 2) + 8);
        }
        if (g + 1 < 4) {
          soft2(g + 1, db);
          if (db > 0) cvt2(g + 1, db - 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  l_run = lacc[0][0] + lacc[1][0];

  // ---- selected diagonals: one 32-key tile per (wave, offset), no workgroup barriers -----------
  // For offset o the 32 queries of this wave need the 32 keys r0-o .. r0-o+31, and in
  // S^T = K Q^T (32 keys x 32 queries) the wanted entries are the main diagonal.  K and V are
  // copied by the LDS DMA into a wave-private K tile and V tile (8 KB each, swizzled like the
  // shared tiles) and read from there like any tile.  An entry is dropped when its key block is
  // kept by the CSR or its key is a selected column: those tiles already counted it.
  // Nothing here is reused, so the phase lives on the memory path: the next offset's K is
  // requested as soon as S^T has read this offset's K tile, its V as soon as the PV product has
  // read this offset's V tile, so each copy has half an offset to land.
  __builtin_amdgcn_s_setprio(0);
  if (tid == 0 && home_open) {  // used at the next item
    ticket = (int)atomicAdd(&p.queue[home], 1u);
    have_ticket = true;
  }
  if (has_offs) __syncthreads();  // all waves are done with the shared tiles: reuse them as private V tiles
  if (has_offs && r0 < N) {
    const int32_t *__restrict__ offp = p.offs + (size_t)h * p.k_s;
    const int no = min(max(p.n_offs[h], 0), p.k_s);
    const int rmax = min(r0 + 31, N - 1);
    int dl = lane;
    asm volatile("" : "+v"(dl));  // this phase's lane constants are born here, not before the tile loop
    const int q = dl & 31, gg = dl >> 5, lane = dl;
    int nd = 0;  // offsets are ascending: the usable ones (0 <= o <= last row of the wave) come first
    for (int base = 0; base < no; base += 64) {
      const int i = base + lane;
      const int ov = i < no ? offp[i] : -1;
      const unsigned long long bad = ~__ballot(i < no && ov >= 0 && ov <= rmax);
      const int run = bad ? __ffsll(bad) - 1 : 64;
      nd += run;
      if (run < 64) break;
    }
    nd = __builtin_amdgcn_readfirstlane(nd);
    // one 8 KB K tile and one 8 KB V tile per wave: waves 0, 1 in the V buffers, waves 2, 3 in the K buffers
    uint16_t *Kw = (wv < 2 ? &Vs[0][0] : &Ks[0][0]) + (wv & 1) * (2 * 32 * 128);
    uint16_t *Vw = Kw + 32 * 128;
    const unsigned ldsKw = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)Kw;
    const unsigned ldsVw = ldsKw + 32 * 256;
    const int rstar = 4 * (q >> 3) + (q & 3);        // register of S^T that holds key_local == q
    const bool holder = gg == ((q >> 2) & 1);        // ... in this half of the lane pair
    const int vrow = lane >> 4;                      // copies: one instruction moves rows 4n + vrow
    const unsigned vchunk = (unsigned)(((lane & 15) ^ (vrow << 2)) << 4);  // swizzles applied on the global side
    // K rows are swizzled by (row & 15) = (4n & 15) ^ vrow: four per-lane offsets serve the eight copies
    const unsigned kchunk = (unsigned)(((lane & 15) ^ vrow) << 4);
    const unsigned krow = (unsigned)(vrow * (int)p.kv_rs * 2);
    const uint32_t *kw = wv < 2 ? kept0 : kept1;
    uint32_t cw = 0u;
    // The copies of one offset: 32 K rows and 32 V rows, both global -> LDS.  (K used to be read
    // straight into the operand registers, one row per lane: every quarter-wave of such a read
    // touches 16 different cache lines, and the L1's tag lookups, 512 per wave and offset, were what
    // this phase waited for.)
#define SA_DIAG_COPY(src, o, fastv, chunkv, swzn, ldsb)                                           \
  {                                                                                              \
    const int jb_ = r0 - (o);                                                                    \
    if (jb_ >= 0 && jb_ + 31 < N) {                                                              \
      const uint16_t *b_ = (src) + (size_t)jb_ * p.kv_rs;                                        \
      _Pragma("unroll") for (int n_ = 0; n_ < 8; ++n_)                                           \
        SA_DMA16(b_ + (size_t)(4 * n_) * p.kv_rs, (fastv) + ((chunkv) ^ (unsigned)(swzn)), (ldsb) + n_ * 1024); \
    } else { /* rows outside the sequence: clamped copies, masked out by the validity test */    \
      _Pragma("unroll") for (int n_ = 0; n_ < 8; ++n_) {                                         \
        const int rb_ = min(max(jb_ + 4 * n_, 0), N - 1);                                        \
        const int dr_ = min(max(jb_ + 4 * n_ + vrow, 0), N - 1) - rb_; /* >= 0 */                \
        SA_DMA16((src) + (size_t)rb_ * p.kv_rs,                                                  \
                 (unsigned)(dr_ * (int)p.kv_rs * 2) + ((chunkv) ^ (unsigned)(swzn)), (ldsb) + n_ * 1024); \
      }                                                                                          \
    }                                                                                            \
  }
#define SA_DIAG_ISSUE_K(o)                                                                       \
  {                                                                                              \
    if (has_cols) cw = bits_window32(colbm, N / 32, r0 - (o));                                   \
    SA_DIAG_COPY(Kh, o, krow, kchunk, ((4 * n_) & 15) << 4, ldsKw)                               \
  }
#define SA_DIAG_ISSUE_V(o) SA_DIAG_COPY(Vh, o, (unsigned)(vrow * (int)p.kv_rs * 2), vchunk, 0, ldsVw)
    // An offset whose (at most two) key tiles are both kept by the CSR contributes nothing here -
    // every one of its entries was counted by those tiles - so it is skipped before any copy is
    // issued.  The test is wave-uniform; `e` walks the offsets that are left.
    auto dead = [&](int o_) {
      const int jb_ = r0 - o_;
      const int kta_ = max(jb_, 0) >> 6, ktb_ = max(jb_ + 31, 0) >> 6;
      return (((kw[kta_ >> 5] >> (kta_ & 31)) & (kw[ktb_ >> 5] >> (ktb_ & 31))) & 1u) != 0u;
    };
    auto next_live = [&](int e_) {
      while (e_ < nd && __builtin_amdgcn_readfirstlane((int)dead((int)uload(offp, e_)))) ++e_;
      return e_;
    };
    int e = next_live(0);
    if (e < nd) {
      const int o0 = (int)uload(offp, e);
      SA_DIAG_ISSUE_K(o0);
      SA_DIAG_ISSUE_V(o0);
    }
    while (e < nd) {
      const int o = (int)uload(offp, e);
      const int e_nxt = next_live(e + 1);
      const int onext = (int)uload(offp, min(e_nxt, nd - 1));
      const int jb = r0 - o;
      f32x16 sd;
#pragma unroll
      for (int r = 0; r < 16; ++r) sd[r] = 0.f;
      // K of this offset has landed once only the 8 copies of its V, issued after it, are outstanding
      __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        sd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(SA_KFRAG(Kw, 0, ks), qf[ks], sd, 0, 0, 0);
      float sv = sd[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) sv = (r == rstar) ? sd[r] : sv;
      const bool cbit = (cw >> q) & 1u;
      // the K tile has been read into the matrix pipe: the next offset's K may land
      if (e_nxt < nd) SA_DIAG_ISSUE_K(onext);
      // validity of (query iq, key iq - o)
      const int j = iq - o;
      bool valid = holder && j >= 0 && iq < N;
      {
        const int kta = max(jb, 0) >> 6, ktb = max(jb + 31, 0) >> 6;  // the (at most two) key tiles touched
        const bool ba = (kw[kta >> 5] >> (kta & 31)) & 1u, bb = (kw[ktb >> 5] >> (ktb & 31)) & 1u;
        if (((max(j, 0) >> 6) == kta) ? ba : bb) valid = false;
        if (has_cols && cbit) valid = false;
      }
      if constexpr (STATS) {
        st_kept += valid ? 1u : 0u;
        st_tiles += 1u;
      }
      float sm = valid ? sv : -INFINITY;
      sm = fmaxf(sm, __shfl_xor(sm, 32));  // both lanes of the pair know the row's score
      const float m_new = fmaxf(m_run, sm * p.c);
      if (__any(m_new - m_run > 8.f)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
      }
      const float m_ref = (m_run == -INFINITY) ? 0.f : m_run;
      const float pv = valid ? __builtin_amdgcn_exp2f(__builtin_fmaf(sv, p.c, -m_ref)) : 0.f;
      const __bf16 pvb = (__bf16)pv, zb = (__bf16)0.f;
      l_run += (float)pvb;  // the weight as the matrix pipe sees it (see the tile loop's normaliser)
      // V of this offset has landed once only the 8 copies of the next K, issued after it, are
      // outstanding
      if (e_nxt < nd) __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8)
      else __builtin_amdgcn_s_waitcnt(0x0F70);                       // vmcnt(0)
      // P^T is diagonal: slot e2 of k-step u is register 8u+e2
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8 pb;
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) pb[e2] = (8 * u + e2 == rstar) ? pvb : zb;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const s16x4 lo = SA_VTR(Vw, db, 16 * u);
          const s16x4 hi = SA_VTR(Vw, db, 16 * u + 8);
          const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb,
                                                             oacc[db], 0, 0, 0);
        }
      }
      // the V tile has been read: the next offset's V may land
      if (e_nxt < nd) SA_DIAG_ISSUE_V(onext);
      e = e_nxt;
    }
#undef SA_DIAG_ISSUE_K
#undef SA_DIAG_ISSUE_V
#undef SA_DIAG_COPY
  }

  if constexpr (STATS) {  // one pair of atomics per wave and item
    unsigned long long kept_n = st_kept;
    for (int d = 32; d >= 1; d >>= 1) kept_n += __shfl_xor(kept_n, d);
    if (lane == 0) {
      atomicAdd(&p.counters[0], (unsigned long long)st_tiles);
      atomicAdd(&p.counters[1], kept_n);
    }
  }
  // ---- epilogue: O[iq][32db + 8(r/4) + 4gg + r%4] = oacc / l -------------------------------------
  // A lane holds 16 separate 8-byte pieces of its row.  They go through an 8 KB LDS tile of the
  // wave's own (swizzled like a K tile) and leave as whole 256-byte rows, 16 bytes per lane: 64
  // cache lines per wave instead of 1024 partial writes.
  const float ltot = l_run + __shfl_xor(l_run, 32);
  const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
  if (!has_offs) __syncthreads();  // the shared tiles are free (with diagonals, that barrier has been passed)
  {
    char *ow = (char *)((wv < 2 ? &Vs[0][0] : &Ks[0][0]) + (wv & 1) * (2 * 32 * 128));
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        union { __bf16 b[4]; uint2 u; } o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o.b[e] = (__bf16)(oacc[db][4 * rb + e] * inv);
        *(uint2 *)(ow + q * 256 + (((4 * db + rb) ^ (q & 15)) << 4) + 8 * gg) = o.u;
      }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int rr = lane >> 4, pc = lane & 15;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int r = 4 * n + rr;
      const uint4 v = *(const uint4 *)(ow + r * 256 + (pc << 4));
      if (r0 + r < N)
        *(uint4 *)(p.O + (size_t)h * p.q_hs + (size_t)(r0 + r) * p.q_rs + ((pc ^ (r & 15)) << 3)) = v;
    }
  }
  }  // work-queue loop
}

#undef SA_KFRAG
#undef SA_VTR
#undef SA_ISSUE_TILE
#undef SA_DMA16

}  // namespace

hipError_t launch_sparse_prefill(const Shape &sh, const Workspace &ws, const uint16_t *Q,
                                 const uint16_t *K, const uint16_t *V, sa_index idx, uint16_t *O,
                                 unsigned long long *counters, hipStream_t st) {
  AttnArgs a = {};
  a.Q = Q; a.K = K; a.V = V; a.O = O;
  a.n_cols = idx.n_cols; a.cols = idx.cols; a.n_offs = idx.n_offs; a.offs = idx.offs;
  a.rowptr = idx.rowptr; a.blkcols = idx.blkcols;
  a.colbits = ws.colbits; a.colprefix = ws.colprefix;
  a.Hq = sh.Hq; a.Hkv = sh.Hkv; a.g = sh.g; a.N = sh.N; a.b = sh.b; a.nb = sh.nb;
  a.nT = (sh.N + BQ - 1) / BQ;
  a.k_v = sh.k_v; a.k_s = sh.k_s; a.cap_b = sh.cap_b;
  a.q_hs = sh.q_hs; a.q_rs = sh.q_rs; a.kv_hs = sh.kv_hs; a.kv_rs = sh.kv_rs;
  a.c = sh.scale * 1.4426950408889634f;
  a.counters = counters;
  a.hperm = ws.hperm;
  a.Kg = ws.kg; a.Vg = ws.vg; a.kvg_rows = (sh.k_v + BK - 1) / BK * BK;
  index_prepare_kernel<<<sh.Hq + a.kvg_rows / BK * sh.Hq, 256, 0, st>>>(a, ws.queue);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  a.queue = ws.queue;
  a.n_items = a.nT * sh.Hq;
  // KV heads in progress together: as many as there are queues, unless their K and V rows
  // (what the diagonal phase streams) exceed the 256 MiB memory-side cache
  a.xs = 1;
  while (a.xs < 8 && 8 / a.xs > sh.Hkv) a.xs *= 2;  // fewer than 8 KV heads: no idle queues
  while (a.xs < 8 && (size_t)(8 / a.xs) * sh.N * kHeadDim * 2 * 2 > ((size_t)256 << 20)) a.xs *= 2;
  a.qcap = (a.nT + a.xs - 1) / a.xs * sh.g * ((sh.Hkv + 8 / a.xs - 1) / (8 / a.xs));
  const int grid = a.n_items < 2 * sh.n_cu ? a.n_items : 2 * sh.n_cu;  // two resident workgroups per CU
  if (counters)
    sparse_prefill_kernel<true><<<grid, 256, 0, st>>>(a);
  else
    sparse_prefill_kernel<false><<<grid, 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace sa
