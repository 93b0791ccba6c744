// Attention over the selected key clusters (Alg. 3 lines 9-10) and the dense branch.
//
// The label sort puts the keys in cluster order (a permutation, no copy for bf16: the planning step writes,
// per query cluster, the byte offset of every selected key row in K and V as they are, and the kernel loads
// its tiles through that table; fp32 gathers K and V into cluster order first and walks row ranges).  For
// every query cluster the selected key clusters form a short list of row ranges in that order; a
// query tile walks the concatenation of its ranges in full 64-key tiles, so cluster raggedness
// costs nothing but one masked tail tile.  The flash-style kernel keeps the S^T = K Q^T
// orientation: in the 32x32 MFMA accumulator a lane then owns one query and 16 keys, soft-max
// statistics are per-lane scalars, and the exponentiated block feeds the P V product as the B
// operand straight from registers.  K and V tiles both sit row-major in LDS; the A operand of that
// product (a column of V over 8 keys) is gathered by LDS transpose reads.
#include "common.h"
#include "launch.h"

#include <type_traits>

namespace adac {

static constexpr int TILE_REC = 6;       // ints per query-tile record
static constexpr int SPLIT_SLOTS = 128;  // partial slots per head for the chunks of cut key lists
static constexpr int KROW_PAD = 8 * 64;  // entries of the row-offset table a key list is padded by: the kernel reads up to 7 tiles ahead

// ------------------------------------------------------------------------------------------
// permutation of K and V rows (fp32 inputs)
// ------------------------------------------------------------------------------------------
// dst[h][i][:] = src[h][perm[h][i]][:], 16-byte pieces, one row per group of ROWB/16 lanes; a thread
// moves its piece of RPT rows of both tensors, all loads issued before the first store.
#ifndef GATHER_RPT
#define GATHER_RPT 4
#endif
template <int ROWB>
__global__ __launch_bounds__(256) void gather_rows2(const uint8_t* __restrict__ a, const uint8_t* __restrict__ b,
                                                    const int32_t* __restrict__ perm, int N,
                                                    uint8_t* __restrict__ ao, uint8_t* __restrict__ bo) {
  constexpr int LPR = ROWB / 16, RPB = 256 / LPR, RPT = GATHER_RPT;
  const int h = blockIdx.y;
  const int r0 = blockIdx.x * (RPB * RPT) + threadIdx.x / LPR;
  const int q = threadIdx.x % LPR;
  const int32_t* pm = perm + (size_t)h * N;
  int src[RPT];
#pragma unroll
  for (int k = 0; k < RPT; ++k) { const int r = r0 + k * RPB; src[k] = r < N ? pm[r] : 0; }
  uint4 va[RPT], vb[RPT];
#pragma unroll
  for (int k = 0; k < RPT; ++k) {
    const size_t so = ((size_t)h * N + src[k]) * ROWB + q * 16;
    va[k] = *reinterpret_cast<const uint4*>(a + so);
    vb[k] = *reinterpret_cast<const uint4*>(b + so);
  }
#pragma unroll
  for (int k = 0; k < RPT; ++k) {
    const int r = r0 + k * RPB;
    if (r >= N) continue;
    const size_t dd = ((size_t)h * N + r) * ROWB + q * 16;
    *reinterpret_cast<uint4*>(ao + dd) = va[k];
    *reinterpret_cast<uint4*>(bo + dd) = vb[k];
  }
}

int launch_permute_kv(hipStream_t s, int H, int N, int row_bytes, const void* K, const void* V,
                      const int32_t* perm, void* Kp, void* Vp) {
  auto A = (const uint8_t*)K; auto B = (const uint8_t*)V; auto Ao = (uint8_t*)Kp; auto Bo = (uint8_t*)Vp;
  const int rows_per_block = 256 / (row_bytes / 16) * GATHER_RPT;
  const dim3 g((N + rows_per_block - 1) / rows_per_block, H);
  if (row_bytes == 128) gather_rows2<128><<<g, 256, 0, s>>>(A, B, perm, N, Ao, Bo);
  else if (row_bytes == 256) gather_rows2<256><<<g, 256, 0, s>>>(A, B, perm, N, Ao, Bo);
  else if (row_bytes == 512) gather_rows2<512><<<g, 256, 0, s>>>(A, B, perm, N, Ao, Bo);
  else return ADACLUSTER_E_BADSHAPE;
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

// ------------------------------------------------------------------------------------------
// plan: per query cluster the merged key ranges; per head the list of query tiles
// ------------------------------------------------------------------------------------------
// rng_start [H][Cq][maxr]   first key row (in cluster order) of range r
// rng_pre   [H][Cq][maxr+1] keys before range r in the concatenation (last = total)
// rng_cnt   [H][Cq]
// tiles     [H][maxtiles] x {cluster, first sorted query position, rows, first key tile, end key
//           tile, partial slot or -1}; ntiles [H]
__global__ __launch_bounds__(256) void plan_sparse(int Cq, int cap, int maxr, int row_bytes,
                            const int32_t* __restrict__ k_offs, int k_offs_stride,
                            const int32_t* __restrict__ k_count,
                            const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_cnt,
                            int32_t* __restrict__ rng_start, int32_t* __restrict__ rng_pre,
                            int32_t* __restrict__ rng_cnt, int32_t* __restrict__ krow, size_t kstride,
                            const int32_t* __restrict__ perm_k, int N) {
  const int h = blockIdx.y, i = blockIdx.x, tid = threadIdx.x;
  int32_t* rs = rng_start + ((size_t)h * Cq + i) * maxr;
  int32_t* rp = rng_pre + ((size_t)h * Cq + i) * (maxr + 1);
  __shared__ int32_t s_nr, s_total;
  __shared__ int32_t s_we[4], s_wh[4], s_wlen[4], s_wst[4];
  {
    // The selected clusters in list order; a cluster whose rows follow the previous non-empty one's directly
    // extends its range.  256 entries per round: "end of the last non-empty entry before me" by a scan that
    // keeps the right operand when it is non-empty, then run starts and lengths by prefix sums; the state
    // after a round (last end, keys so far, ranges so far) is carried into the next.
    const int32_t* sel = sel_idx + ((size_t)h * Cq + i) * cap;
    const int cnt = sel_cnt[(size_t)h * Cq + i];
    const int32_t* ko = k_offs + (size_t)h * k_offs_stride;
    const int kc = k_count[h];
    const int lane = tid & 63, wave = tid >> 6;
    int carry_e = -1, carry_total = 0, carry_nr = 0;          // identical in every thread
    for (int base = 0; base < cnt; base += 256) {
      const int t = base + tid;
      int sk = 0, ek = 0;
      bool valid = false;
      if (t < cnt) {
        const int j = sel[t];
        if (j >= 0 && j < kc) { sk = ko[j]; ek = ko[j + 1]; valid = ek > sk; }
      }
      const int len = valid ? ek - sk : 0;
      // inclusive scans inside the wave
      int ie = valid ? ek : -1, ih = valid ? 1 : 0, il = len;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int oe = __shfl_up(ie, off), oh = __shfl_up(ih, off), ol = __shfl_up(il, off);
        if (lane >= off) { if (!ih) { ie = oe; ih = oh; } il += ol; }
      }
      if (lane == 63) { s_we[wave] = ie; s_wh[wave] = ih; s_wlen[wave] = il; }
      __syncthreads();
      // what precedes this thread: the carry, the earlier waves, the earlier lanes
      int pe = carry_e, ph = carry_e >= 0 ? 1 : 0, plen = carry_total;
      for (int w = 0; w < wave; ++w) { if (s_wh[w]) { pe = s_we[w]; ph = 1; } plen += s_wlen[w]; }
      const int le = __shfl_up(ie, 1), lh = __shfl_up(ih, 1);
      if (lane > 0 && lh) { pe = le; ph = 1; }
      plen += il - len;
      const bool start = valid && !(ph && pe == sk);
      int is = start ? 1 : 0;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) { const int o = __shfl_up(is, off); if (lane >= off) is += o; }
      if (lane == 63) s_wst[wave] = is;
      __syncthreads();
      int pst = carry_nr;
      for (int w = 0; w < wave; ++w) pst += s_wst[w];
      if (start) { const int r = pst + is - 1; rs[r] = sk; rp[r] = plen; }
      // the carry of the next round, the same in every thread
      for (int w = 0; w < 4; ++w) { if (s_wh[w]) carry_e = s_we[w]; carry_total += s_wlen[w]; carry_nr += s_wst[w]; }
      __syncthreads();                         // the wave totals are free again
    }
    if (tid == 0) {
      rp[carry_nr] = carry_total;
      rng_cnt[(size_t)h * Cq + i] = carry_nr;
      s_nr = carry_nr; s_total = carry_total;
    }
  }
  __syncthreads();        // the ranges are visible to the whole workgroup
  // Byte offset of every key row of the concatenation, in order: what a key tile of the attention kernel
  // loads its 64 rows by.  Entries past the end (up to the padding the kernel may read ahead) repeat the
  // first row: they are loaded and never used.
  if (!krow) return;       // (the fp32 kernel walks the ranges itself)
  const int nr = s_nr, total = s_total;
  int32_t* kr = krow + ((size_t)h * Cq + i) * kstride;
  const int32_t* pk = perm_k ? perm_k + (size_t)h * N : nullptr;      // sorted position -> token (rows stay where they are)
  const int first = nr > 0 ? (pk ? pk[rs[0]] : rs[0]) * row_bytes : 0;
  const int padded = (total + 63) / 64 * 64 + KROW_PAD;
  // the search runs on a copy of the range table in LDS when it fits: its steps depend on one another, and
  // from global memory each of them is a trip to the L2
  constexpr int LR = 512;
  __shared__ int32_t l_rs[LR], l_rp[LR];
  const bool in_lds = nr <= LR;
  if (in_lds) {
    for (int r = tid; r < nr; r += 256) { l_rs[r] = rs[r]; l_rp[r] = rp[r]; }
    __syncthreads();
  }
  auto fill = [&](const int32_t* srs, const int32_t* srp) __attribute__((always_inline)) {
    for (int p = tid; p < padded; p += 256) {
      int off = first;
      if (p < total) {
        int lo = 0, hi = nr - 1;                 // last range whose first position is <= p
        while (lo < hi) { const int mid = (lo + hi + 1) >> 1; if (srp[mid] <= p) lo = mid; else hi = mid - 1; }
        const int row = srs[lo] + (p - srp[lo]);
        off = (pk ? pk[row] : row) * row_bytes;
      }
      kr[p] = off;
    }
  };
  if (in_lds) fill(l_rs, l_rp); else fill(rs, rp);
}

// Query tiles of a head, cluster by cluster.  A query cluster whose key list is much longer than
// the head's average (top-p selections can be that skewed) would make its few workgroups the whole
// critical path of the launch, so such a list is cut into chunks of key tiles: each chunk is a
// workgroup of its own that leaves unnormalised (O, m, l) in a partial slot, and attn_merge
// combines the slots of a query tile.  merge [H][slots] x {first query position, rows, first slot,
// chunks}; a head has `slots` partial slots, and lists stay whole once they are used up.
__global__ __launch_bounds__(256) void plan_tiles(int Cq, int maxr, int maxtiles, int BM, int slots, int allow_split,
                                                  const int32_t* __restrict__ q_offs, int q_offs_stride,
                                                  const int32_t* __restrict__ rng_pre,
                                                  const int32_t* __restrict__ rng_cnt,
                                                  int32_t* __restrict__ tiles, int32_t* __restrict__ ntiles,
                                                  int32_t* __restrict__ merge, int32_t* __restrict__ nmerge) {
  constexpr int MAXC = 4096;                       // the largest q_clusters the library accepts
  const int h = blockIdx.x, tid = threadIdx.x;
  const int32_t* qo = q_offs + (size_t)h * q_offs_stride;
  int32_t* tl = tiles + (size_t)h * maxtiles * TILE_REC;
  int32_t* ml = merge + (size_t)h * slots * 4;
  __shared__ int32_t s_T[MAXC], s_nq[MAXC], s_pieces[MAXC], s_tile0[MAXC], s_slot0[MAXC], s_merge0[MAXC];
  __shared__ int32_t s_chunk;
  const int C = min(Cq, MAXC);
  for (int c = tid; c < C; c += 256) {
    s_nq[c] = (qo[c + 1] - qo[c] + BM - 1) / BM;
    const int tot = rng_pre[((size_t)h * Cq + c) * (maxr + 1) + rng_cnt[(size_t)h * Cq + c]];
    s_T[c] = (tot + 63) / 64;
  }
  __syncthreads();
  if (tid == 0) {
    // key tiles per chunk of a list that is cut: twice the average list of the head, at least 16
    long long work = 0; int qtiles = 0;
    for (int c = 0; c < C; ++c) { work += (long long)s_nq[c] * s_T[c]; qtiles += s_nq[c]; }
    const int mean_t = qtiles > 0 ? (int)((work + qtiles - 1) / qtiles) : 0;
    const int chunk = max(16, 2 * mean_t);
    s_chunk = chunk;
    // which lists are cut (in cluster order, while slots last), and where every cluster's records start
    int nt = 0, used = 0, nm = 0;
    for (int c = 0; c < C; ++c) {
      const int T = s_T[c];
      int pieces = 1;
      if (allow_split && T > 2 * chunk) {
        pieces = min(16, (T + chunk - 1) / chunk);
        if (used + pieces * s_nq[c] > slots) pieces = max(1, (slots - used) / max(s_nq[c], 1));   // fewer, longer chunks
      }
      if (pieces > 1) {
        const int per = (T + pieces - 1) / pieces;
        pieces = max(1, (T + per - 1) / max(per, 1));          // no empty chunk
      }
      s_pieces[c] = pieces; s_tile0[c] = nt; s_slot0[c] = used; s_merge0[c] = nm;
      nt += s_nq[c] * pieces;
      if (pieces > 1) { used += s_nq[c] * pieces; nm += s_nq[c]; }
    }
    ntiles[h] = nt;
    nmerge[h] = nm;
  }
  __syncthreads();
  // records of every cluster, one thread per cluster
  for (int c = tid; c < C; c += 256) {
    const int s0 = qo[c], e0 = qo[c + 1], T = s_T[c], pieces = s_pieces[c];
    const int per = (T + pieces - 1) / pieces;
    int nt = s_tile0[c], slot = s_slot0[c], nm = s_merge0[c];
    for (int r0 = s0; r0 < e0; r0 += BM) {
      const int rows = min(BM, e0 - r0);
      if (pieces > 1) {
        ml[nm * 4 + 0] = r0; ml[nm * 4 + 1] = rows; ml[nm * 4 + 2] = slot; ml[nm * 4 + 3] = pieces;
        ++nm;
      }
      for (int k = 0; k < pieces; ++k) {
        int32_t* t6 = tl + (size_t)nt * TILE_REC;
        t6[0] = c; t6[1] = r0; t6[2] = rows;
        t6[3] = pieces > 1 ? k * per : 0; t6[4] = pieces > 1 ? min(T, (k + 1) * per) : T;
        t6[5] = pieces > 1 ? slot + k : -1;
        ++nt;
      }
      if (pieces > 1) slot += pieces;
    }
  }
}

// dense: one query "cluster" over all rows, one key range [0,N)
__global__ void plan_dense(int N, int maxtiles, int BM, int row_bytes, int32_t* __restrict__ rng_start,
                           int32_t* __restrict__ rng_pre, int32_t* __restrict__ rng_cnt,
                           int32_t* __restrict__ tiles, int32_t* __restrict__ ntiles,
                           int32_t* __restrict__ krow, size_t kstride) {
  const int h = blockIdx.x;
  if (blockIdx.y > 0) {       // the other workgroups of a head fill its row-offset table (the identity)
    if (!krow) return;
    int32_t* kr = krow + (size_t)h * kstride;
    const int padded = (N + 63) / 64 * 64 + KROW_PAD;
    for (int p = (blockIdx.y - 1) * blockDim.x + threadIdx.x; p < padded; p += (gridDim.y - 1) * blockDim.x)
      kr[p] = p < N ? p * row_bytes : 0;
    return;
  }
  if (threadIdx.x == 0) {
    rng_start[h] = 0; rng_pre[(size_t)h * 2] = 0; rng_pre[(size_t)h * 2 + 1] = N; rng_cnt[h] = 1;
    ntiles[h] = (N + BM - 1) / BM;
  }
  int32_t* tl = tiles + (size_t)h * maxtiles * TILE_REC;
  for (int t = threadIdx.x; t * BM < N; t += blockDim.x) {
    int32_t* t6 = tl + (size_t)t * TILE_REC;
    t6[0] = 0; t6[1] = t * BM; t6[2] = min(BM, N - t * BM); t6[3] = 0; t6[4] = (N + 63) / 64; t6[5] = -1;
  }
}

// Per-head figures of the last clustering and the last attention plan on this workspace: |C|, F, stages and
// |U| per stage from the Algorithm 1 state, and the (query, key) pairs the attention launch covers: executed
// = rows x keys of every query tile, issued = the same with rows rounded up to whole 32-query waves and keys
// to whole 64-key tiles (what the matrix cores are actually fed).
__global__ __launch_bounds__(256) void attn_stats(int Cq, int maxr, int maxtiles, const KState* __restrict__ st,
                                                  const int32_t* __restrict__ tiles, const int32_t* __restrict__ ntiles,
                                                  const int32_t* __restrict__ rng_pre, const int32_t* __restrict__ rng_cnt,
                                                  adacluster_head_stats* __restrict__ out) {
  const int h = blockIdx.x, tid = threadIdx.x;
  const int nt = min(ntiles[h], maxtiles);
  const int32_t* tl = tiles + (size_t)h * maxtiles * TILE_REC;
  long long ex = 0, is = 0;
  for (int t = tid; t < nt; t += 256) {
    const int32_t* t6 = tl + (size_t)t * TILE_REC;
    const int c = t6[0], rows = t6[2], kt0 = t6[3], kt1 = t6[4];
    const int total = rng_pre[((size_t)h * Cq + c) * (maxr + 1) + rng_cnt[(size_t)h * Cq + c]];
    const long long keys = max(0, min(total, kt1 * 64) - kt0 * 64);
    ex += (long long)rows * keys;
    is += (long long)((rows + 31) / 32 * 32) * ((keys + 63) / 64 * 64);
  }
  __shared__ long long s_ex[256], s_is[256];
  s_ex[tid] = ex; s_is[tid] = is;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) { s_ex[tid] += s_ex[tid + o]; s_is[tid] += s_is[tid + o]; }
    __syncthreads();
  }
  if (tid == 0) {
    adacluster_head_stats r;
    const KState& k = st[h];
    r.k_count = k.ccount; r.full_flag = k.full; r.stages = k.stage; r.q_tiles = nt;
    for (int i = 0; i <= ADACLUSTER_MAX_STAGES; ++i) r.unassigned[i] = i <= k.stage ? k.u_hist[i] : 0;
    r.reserved = 0;
    r.executed_pairs = s_ex[0]; r.issued_pairs = s_is[0];
    out[h] = r;
  }
}

int launch_attn_stats(hipStream_t s, int H, int Cq, int maxr, int maxtiles, const KState* st, const int32_t* tiles,
                      const int32_t* ntiles, const int32_t* rng_pre, const int32_t* rng_cnt, adacluster_head_stats* out) {
  attn_stats<<<H, 256, 0, s>>>(Cq, maxr, maxtiles, st, tiles, ntiles, rng_pre, rng_cnt, out);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

struct AttnArgs {
  const void* Q; const void* Kp; const void* Vp; void* O;
  const int32_t* perm_q;        // sorted query position -> token (NULL: identity)
  const int32_t* tiles; const int32_t* ntiles;
  const int32_t* rng_start; const int32_t* rng_pre; const int32_t* rng_cnt;
  int N, Cq, maxtiles, maxr;
  float scale_log2e;            // softmax scale x log2(e)
  int head_major;               // workgroup -> (head, tile) mapping, see attn_mfma
  float* part_o; float* part_ml;   // partial slots of cut key lists: [H][slots][BM][d], [H][slots][BM][2]
  int slots, BM;
  const int32_t* krow; size_t kstride;   // byte offset of every key row of a query cluster's list: [H][Cq][kstride]
};

// position in the concatenation of ranges -> permuted key row; a cursor that only moves forward
template <typename PTR>
struct RangeCursorT {
  PTR rs; PTR rp; int nr; int r; int cur_end; int delta;
  __device__ __forceinline__ void init(PTR rs_, PTR rp_, int nr_) {
    rs = rs_; rp = rp_; nr = nr_; r = 0;
    cur_end = nr > 0 ? rp[1] : 0;
    delta = nr > 0 ? rs[0] - rp[0] : 0;
  }
  __device__ __forceinline__ int row(int p) {      // p is non-decreasing across calls
    while (r < nr && p >= cur_end) {
      ++r;
      if (r < nr) { cur_end = rp[r + 1]; delta = rs[r] - rp[r]; }
    }
    return r < nr ? p + delta : -1;
  }
};
typedef RangeCursorT<const int32_t*> RangeCursor;
typedef __attribute__((address_space(3))) const int32_t lds_ci32_t;

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;

// LDS transpose read (16-bit elements): inside each group of 16 lanes, lane r supplies the address
// of 4 consecutive elements and lane i receives element i%4 of the rows addressed by lanes
// i/4, i/4+4, i/4+8, i/4+12.
__device__ __forceinline__ s16x4_t lds_read_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p);
}

// Direct global -> LDS loads, written as inline assembly on purpose.  The compiler orders every LDS read
// behind an outstanding direct-to-LDS load that it cannot prove to touch another object (it then drains ALL
// loads in flight: vmcnt(0)), and its proof is fragile (it fails across the branches of a four-stage ring).
// The tile pipeline below keeps several tiles in flight and waits for exactly the one it needs, by count,
// before a workgroup barrier; hiding the loads from the compiler leaves that protocol in charge.  Each lane
// loads `bytes` at sbase + voff; the wave's data land at lds_addr + lane * bytes (M0 carries the LDS address).
__device__ __forceinline__ void dma_b128(uint32_t lds_addr, uint32_t voff, const void* sbase) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma_b32(uint32_t lds_addr, uint32_t voff, const void* sbase) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(sbase) : "memory", "m0");
}

// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt[3:0] and [15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() carries a release fence over global memory
// as well, which makes every wave drain all of its loads in flight (vmcnt(0)) at every barrier; the tile
// pipeline below waits for exactly the loads it needs by count and must keep the rest in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // this wave's LDS reads and writes are done
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");                         // nothing that touches memory moves across
}

// One workgroup = NW waves of 32 queries each; all waves share 64-key K and V tiles.  Tiles go global -> LDS
// directly (no register staging) as 16-byte chunks into a ring of NBUF stages, NBUF-1 tiles ahead of the
// arithmetic, one barrier per tile.  A tile row is unpadded and its 16-byte chunks are permuted by a row-dependent
// XOR that keeps the operand reads of either tile free of bank conflicts (see swz_k, swz_v).  The rows of a tile come
// from the row-offset table plan_sparse / plan_dense wrote: its 64 entries for a tile are themselves loaded
// global -> LDS, 2*(NBUF-1) tiles ahead, so that no wave walks a range list and no load waits on a register.
// LDS layout: [row offsets: NBUF x 64][K ring: NBUF tiles][V ring: NBUF tiles]; with the K tiles (and the V
// tiles) side by side, a stage is reached from one set of address registers by an immediate offset (< 64 KB;
// the start of the V ring is part of the V address registers).
template <int D, int NW, int NBUF, int MINB, int VPRE>
__global__ __launch_bounds__(NW * 64, MINB) void attn_mfma(AttnArgs a) {
  constexpr int BN = 64, NT = NW * 64, KS = D / 16, DB = D / 32, CH = D / 8, ROWB = D * 2;
  constexpr int ITEMS = BN * CH, PT = ITEMS / NT, TILEB = BN * ROWB, PD = NBUF - 1;
  constexpr int VM_STEP = 2 * PT + 1;             // vector-memory operations a wave issues per tile
  constexpr int ISSUE_J0 = D == 128 ? 2 : 3, ISSUE_STRIDE = (2 * KS - ISSUE_J0) / VM_STEP;     // the requests spread over the S products
  static_assert(ISSUE_STRIDE >= 1, "more requests than S products to put them behind");
  constexpr int RIDXB = NBUF * BN * 4;            // bytes of the row-offset slots at the start of LDS
  constexpr int KRING = NBUF * TILEB;             // bytes of the ring of K tiles (the ring of V tiles follows it)
  static_assert(ITEMS % NT == 0, "tile chunks must divide evenly over the threads");
  static_assert(NBUF == 2 || NBUF == 4, "two or four stages");
  static_assert(2 * PD + 1 <= KROW_PAD / 64, "the row-offset table is padded for the read-ahead");
  static_assert(64 % NW == 0, "every wave loads an equal share of a tile's row offsets");

  // Workgroups go to the 8 XCDs round-robin in launch order (gridDim.x is a multiple of 8, so
  // XCD = blockIdx.x % 8), and each XCD has its own L2.
  int h, tile;
  if (a.head_major) {
    // Heads are dealt to XCDs whole, eight at a time: all query tiles of a head then stream that
    // head's K/V rows behind one L2.  The H % 8 heads left over are split eight ways by tile.
    const int gx = gridDim.x, gx8 = gx >> 3;
    const int xcd = blockIdx.x & 7, slot = (blockIdx.y * gx + blockIdx.x) >> 3;
    const int Hfull = (gridDim.y >> 3) << 3, full_slots = (Hfull >> 3) * gx;
    if (slot < full_slots) {
      h = (slot / gx) * 8 + xcd; tile = slot % gx;
      if (tile >= a.ntiles[h]) return;
    } else {
      const int r = slot - full_slots, j = r % gx8;
      h = Hfull + r / gx8;
      const int nt = a.ntiles[h], per = (nt + 7) >> 3;    // eighths of the tiles the head has, not of the grid
      tile = xcd * per + j;
      if (j >= per || tile >= nt) return;
    }
  } else {
    // Every head is split eight ways: an XCD takes a contiguous run of its query tiles (the tiles
    // of one query cluster stream the same K/V rows, and so do it behind the same L2).  The runs
    // are eighths of the tiles the head has; the grid is sized for the most it could have.
    h = blockIdx.y;
    const int nt = a.ntiles[h], per = (nt + 7) >> 3, j = blockIdx.x >> 3;
    tile = (blockIdx.x & 7) * per + j;
    if (j >= per || tile >= nt) return;
  }
  const int32_t* tl = a.tiles + ((size_t)h * a.maxtiles + tile) * TILE_REC;
  const int qc = tl[0], row0 = tl[1], nrows = tl[2];
  const int kt0 = tl[3], kt1 = tl[4], pslot = tl[5];    // this workgroup's share of the key list
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;

  const int nr = a.rng_cnt[(size_t)h * a.Cq + qc];
  const int32_t* rp = a.rng_pre + ((size_t)h * a.Cq + qc) * (a.maxr + 1);
  // positions below are relative to the first key of the share
  const int pbase = kt0 * BN;
  const int total = max(0, min(rp[nr], kt1 * BN) - pbase);
  const int T = (total + BN - 1) / BN;
  const int32_t* krow = a.krow + ((size_t)h * a.Cq + qc) * a.kstride + pbase;   // byte offsets of the key rows

  const bf16raw* Qh = (const bf16raw*)a.Q + (size_t)h * a.N * D;
  const char* Kh = (const char*)a.Kp + (size_t)h * a.N * ROWB;
  const char* Vh = (const char*)a.Vp + (size_t)h * a.N * ROWB;
  bf16raw* Oh = (bf16raw*)a.O + (size_t)h * a.N * D;
  const int32_t* pq = a.perm_q ? a.perm_q + (size_t)h * a.N : nullptr;

  // query token of this lane and the B operand of S
  int qtok = -1;
  bf16x8_t qf[KS];
  const bool wave_has_rows = wave * 32 < nrows;
  {
    const int rr = wave * 32 + c;
    if (rr < nrows) qtok = pq ? pq[row0 + rr] : row0 + rr;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = {0, 0, 0, 0};
      if (qtok >= 0) raw = *reinterpret_cast<const uint4*>(Qh + (size_t)qtok * D + ks * 16 + hb * 8);
      qf[ks] = *reinterpret_cast<const bf16x8_t*>(&raw);
    }
  }

  f32x16_t oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  // Soft-max state of this lane's query: probabilities are taken relative to a reference mref that is only
  // moved when it has to be (see soft-max below); lrun is the sum of the probabilities so far.
  float mref = -INFINITY, lrun = 0.f;

  // Where a 16-byte chunk sits inside its (unpadded) tile row: chunk q of row r is in slot q ^ swz(r).  A row
  // is 256 B (d=128: every row starts at bank 0) or 128 B (d=64: rows two apart do), so the slot alone decides
  // the banks, and the two tiles are read in different shapes:
  //   K: a 16-byte operand read takes the same chunk of 16 consecutive rows per cycle -> 16 distinct slots
  //      (d=128), or 8 slots x the two row parities (d=64);
  //   V: a transpose read takes 64 contiguous bytes (4 slots) of 4 consecutive rows per cycle -> the rows
  //      must differ in the slot's upper bits; rows 8 apart share a swizzle, so the second half of an operand
  //      is a constant offset away.
  // Measured on the LDS alone: 3.7 and 2.2 cycles per read against 7.5 and 7.5 (3.9 at d=64) with q ^ (r & 7).
  auto swz_k = [](int r) __attribute__((always_inline)) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto swz_v = [](int r) __attribute__((always_inline)) { return D == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); };
  // thread -> (row, slot) of its PT chunks of a tile, and the global chunk that slot holds in either tile
  int lrow[PT], lswz_k[PT], lswz_v[PT];
#pragma unroll
  for (int i = 0; i < PT; ++i) {
    const int item = tid + i * NT;
    lrow[i] = item / CH;
    lswz_k[i] = ((item % CH) ^ swz_k(lrow[i])) * 16;
    lswz_v[i] = ((item % CH) ^ swz_v(lrow[i])) * 16;
  }
  __shared__ __attribute__((aligned(16))) char lds[RIDXB + 2 * KRING];
  char* const ldk = lds + RIDXB;                  // the K ring (compute_tile's V addresses carry KRING themselves)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t*)lds;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // the 64 row offsets of tile t go to the offsets slot of stage `st`, an equal share per wave
  const uint32_t ridx_voff = (uint32_t)((wave_u * (BN / NW) + (lane % (BN / NW))) * 4);
  auto issue_ridx = [&](int st, int t) __attribute__((always_inline)) {
    if (lane < BN / NW)
      dma_b32(lds0 + st * (BN * 4) + wave_u * (BN / NW) * 4, ridx_voff, krow + (size_t)t * BN);
  };
  auto issue_tile_op = [&](int st, const int32_t* off, int n) __attribute__((always_inline)) {     // operation n of issue_tile
    const int i = n >> 1;
    const uint32_t dst = lds0 + RIDXB + st * TILEB + (wave_u * 64 + i * NT) * 16;
    if ((n & 1) == 0) dma_b128(dst, (uint32_t)off[i] + (uint32_t)lswz_k[i], Kh);
    else dma_b128(dst + KRING, (uint32_t)off[i] + (uint32_t)lswz_v[i], Vh);
  };
  auto issue_tile = [&](int st, const int32_t* off) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const uint32_t dst = lds0 + RIDXB + st * TILEB + (wave_u * 64 + i * NT) * 16;     // wave-uniform; the lane offset is implicit
      dma_b128(dst, (uint32_t)off[i] + (uint32_t)lswz_k[i], Kh);
      dma_b128(dst + KRING, (uint32_t)off[i] + (uint32_t)lswz_v[i], Vh);
    }
  };

  // operand addresses inside a tile (bytes), fixed for the whole kernel
  int kaddr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kaddr[ks] = c * ROWB + (((ks * 2 + hb) ^ swz_k(c)) * 16);
  // The 8 accumulator values a lane feeds to one P V step are keys 4*hb + {0..3} and
  // 8 + 4*hb + {0..3} of a 16-key group; the V operand is gathered to match by two transpose
  // reads: this lane addresses key 4*hb + (lane%16)/4, columns 16*((lane/16)%2) + 4*(lane%4) .. +3
  // and receives column lane%32 of the four keys.
  int vaddr[DB];
  {
    const int i16 = lane & 15, blk = lane >> 4;
    const int vrow = 4 * hb + (i16 >> 2);
    const int gl = 2 * (blk & 1) + ((i16 & 3) >> 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) vaddr[db] = KRING + vrow * ROWB + (((db * 4 + gl) ^ swz_v(vrow)) * 16) + 8 * (i16 & 1);
  }       // (the offset of the V ring sits in the register: what an LDS read adds as an immediate must stay below 64 KB)
  const bf16x2_t ones2 = {(__bf16)1.0f, (__bf16)1.0f};   // row sums use the rounded probabilities P V uses
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float sc = a.scale_log2e;
  constexpr float P_LIMIT = 65536.f;      // a tile whose probabilities sum past this moves the reference

  // `prep` and `issue(n)`, n < ND: the requests of the tiles further ahead (row offsets out of LDS, then ND
  // direct-to-LDS loads), placed by compute_tile where they cost nothing: the offsets are read behind the K
  // operands, the loads are issued one by one between the S products, in the shadow of the matrix pipe.
  auto compute_tile = [&](const char* ks_, const char* vs_, int nvalid /* < BN only on a masked tail tile */,
                          auto masked, auto&& prep, auto&& issue, auto nd_) __attribute__((always_inline)) {
    constexpr bool MASK = decltype(masked)::value;
    constexpr int ND = decltype(nd_)::value;
    // All K operands of the tile are requested before the first product, and (below) the V operands before
    // the soft-max arithmetic: an LDS read takes a hundred cycles or more to come back, and the compiler, left
    // alone, requests an operand only one product ahead of its use.  The empty asm statements are fences for
    // memory operations (reads do not sink below them); the scheduling barrier behind each keeps the products
    // from rising above the reads that follow their own operands' (a product placed between two reads makes the
    // wave wait for its operand before the next read is even requested: measured, 5 % of the kernel at d=64).
    f32x16_t sacc[2];
    bf16x8_t ka[2][KS];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ka[kb][ks] = *reinterpret_cast<const bf16x8_t*>(ks_ + kb * 32 * ROWB + kaddr[ks]);
    asm volatile("" ::: "memory");
    prep();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kb][ks], qf[ks], ks == 0 ? zero16 : sacc[kb], 0, 0, 0);
        // request n goes behind product ISSUE_J0 + n * ISSUE_STRIDE
        const int j = kb * KS + ks;
        if (ND > 0 && j >= ISSUE_J0 && (j - ISSUE_J0) % ISSUE_STRIDE == 0 && (j - ISSUE_J0) / ISSUE_STRIDE < ND) {
          __builtin_amdgcn_sched_barrier(0);
          issue((j - ISSUE_J0) / ISSUE_STRIDE);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    static_assert(ND == 0 || ISSUE_J0 + (ND - 1) * ISSUE_STRIDE < 2 * KS, "every request finds a product to go behind");
    bf16x8_t va[VPRE > 0 ? VPRE : 1][2][2];
#pragma unroll
    for (int db = 0; db < VPRE; ++db)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const char* vp = vs_ + (kb * 32 + 16 * s2) * ROWB + vaddr[db];
          const s16x4_t lo = lds_read_tr16(vp), hi = lds_read_tr16(vp + 8 * ROWB);
          const s16x4_t both[2] = {lo, hi};
          va[db][kb][s2] = *reinterpret_cast<const bf16x8_t*>(both);
        }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    // accumulator value v of block kb is key  kb*32 + 8*(v/4) + 4*hb + v%4
    if (MASK) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = kb * 32 + 8 * (v >> 2) + 4 * hb + (v & 3);
          if (key >= nvalid) sacc[kb][v] = -INFINITY;
        }
    }
    // Soft-max.  p = 2^((s - mref) scale): any reference gives the same normalised result as long as nothing
    // overflows, so no maximum is taken per tile.  The row sum of the tile tells when the reference is too
    // low (or still -inf, on the first tile; a masked score against that gives NaN, caught by the same test):
    // only then is the tile's maximum taken, the reference moved up to it and the accumulator rescaled.
    bf16x8_t pf[2][2];
    float rsum;
    auto probabilities = [&]() __attribute__((always_inline)) {
      const float moff = mref * sc;
      float part[2][2];                    // four chains of sums, so that an add does not wait for the one before it
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          uint32_t w[4];
          part[kb][s2] = 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * s2 + 2 * j], sc, -moff));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][8 * s2 + 2 * j + 1], sc, -moff));
            w[j] = pack_bf16x2(p0, p1);
            part[kb][s2] = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w[j]), ones2, part[kb][s2], false);
          }
          const uint4 pk = {w[0], w[1], w[2], w[3]};
          pf[kb][s2] = *reinterpret_cast<const bf16x8_t*>(&pk);
        }
      rsum = (part[0][0] + part[0][1]) + (part[1][0] + part[1][1]);
    };
    probabilities();
    if (__any(!(rsum <= P_LIMIT))) {
      float tmax = sacc[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[kb][v]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));           // finite: every tile holds a valid key
      const float mnew = fmaxf(mref, tmax);
      const float alpha = __builtin_amdgcn_exp2f((mref - mnew) * sc);
      mref = mnew;
      lrun *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
      probabilities();
    }
    lrun += rsum;
    asm volatile("" ::: "memory");          // the V operands that were not requested ahead are requested from here on,
    bf16x8_t vb[DB - VPRE > 0 ? DB - VPRE : 1][2][2];      // ALL of them before the first product (second fence): left
#pragma unroll                                            // alone, the compiler requests an operand one product ahead
    for (int db = VPRE; db < DB; ++db)                     // of its use and every product then waits out an LDS read
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const char* vp = vs_ + (kb * 32 + 16 * s2) * ROWB + vaddr[db];
          const s16x4_t lo = lds_read_tr16(vp), hi = lds_read_tr16(vp + 8 * ROWB);
          const s16x4_t both[2] = {lo, hi};
          vb[db - VPRE][kb][s2] = *reinterpret_cast<const bf16x8_t*>(both);
        }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(db < VPRE ? va[db < VPRE ? db : 0][kb][s2] : vb[db >= VPRE ? db - VPRE : 0][kb][s2],
                                                             pf[kb][s2], oacc[db], 0, 0, 0);
    }
  };

  // Tile t lives in stage t % NBUF; the row offsets of tile t sit in the offsets slot of stage (t + 1) % NBUF,
  // the stage whose tile is being worked on when the loads of tile t are issued.  In step t:
  //   loads of tile t + PD          -> stage (t + PD) % NBUF (free since step t - 1), rows from the offsets slot
  //                                    of stage t % NBUF
  //   row offsets of tile t + 2 PD  -> the offsets slot of stage (t + PD) % NBUF
  //   arithmetic of tile t
  //   wait until this wave's loads of tile t + 1 have landed, barrier.
  // Loads are issued for tiles past the end too (the table is padded), so that the number of operations in
  // flight is the same in every step and one constant serves the wait.
  auto step = [&](auto stage, int t) __attribute__((always_inline)) {
    constexpr int U = decltype(stage)::value, G = (U + PD) % NBUF;
    int32_t off[PT];
    auto prep = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < PT; ++i) off[i] = reinterpret_cast<const int32_t*>(lds + U * (BN * 4))[lrow[i]];
    };
    auto issue = [&](int n) __attribute__((always_inline)) {
      if (n < 2 * PT) issue_tile_op(G, off, n); else issue_ridx(G, t + 2 * PD);
    };
    if (wave_has_rows) {
      compute_tile(ldk + U * TILEB, ldk + U * TILEB, BN, std::false_type{}, prep, issue, std::integral_constant<int, VM_STEP>{});
    } else {               // a wave without query rows still loads its share of the tiles
      prep();
#pragma unroll
      for (int n = 0; n < VM_STEP; ++n) issue(n);
    }
    wait_vmcnt<(PD - 1) * VM_STEP>();
    lds_barrier();
  };

  const int Tlast = T - 1;       // the loop takes tiles 0 .. Tlast-1; the last one, full or ragged, is peeled
  if (T > 0) {
    // tiles 0 .. PD-1: rows straight from the table; row offsets of tiles PD .. 2 PD - 1 to their slots
#pragma unroll
    for (int t = 0; t < PD; ++t) {
      int32_t off[PT];
#pragma unroll
      for (int i = 0; i < PT; ++i) off[i] = krow[(size_t)t * BN + lrow[i]];
      issue_tile(t, off);
    }
#pragma unroll
    for (int t = PD; t < 2 * PD; ++t) issue_ridx((t + 1) % NBUF, t);
    wait_vmcnt<0>();
    lds_barrier();
    if constexpr (NBUF == 2) {
      for (int t = 0; t < Tlast; t += 2) {
        step(std::integral_constant<int, 0>{}, t);
        if (t + 1 >= Tlast) break;
        step(std::integral_constant<int, 1>{}, t + 1);
      }
    } else {
      for (int t = 0; t < Tlast; t += 4) {
        step(std::integral_constant<int, 0>{}, t);
        if (t + 1 >= Tlast) break;
        step(std::integral_constant<int, 1>{}, t + 1);
        if (t + 2 >= Tlast) break;
        step(std::integral_constant<int, 2>{}, t + 2);
        if (t + 3 >= Tlast) break;
        step(std::integral_constant<int, 3>{}, t + 3);
      }
    }
    wait_vmcnt<0>();       // nothing of this wave is still on its way to LDS when it ends
    const int u = Tlast % NBUF;
    if (wave_has_rows) compute_tile(ldk + u * TILEB, ldk + u * TILEB, total - Tlast * BN, std::true_type{}, [] {}, [](int) {},
                                    std::integral_constant<int, 0>{});
  }

  // O^T accumulator value v of block db is column  db*32 + 8*(v/4) + 4*hb + v%4  of query c
  {
    const float l = lrun + __shfl_xor(lrun, 32);
    if (pslot >= 0) {
      // a chunk of a cut key list: leave the unnormalised accumulator, the reference and the
      // row sum in this chunk's slot; attn_merge combines the chunks of the query tile
      const int rr = wave * 32 + c;
      const size_t so = ((size_t)h * a.slots + pslot) * a.BM + rr;
      float* po = a.part_o + so * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 o = {oacc[db][4 * i], oacc[db][4 * i + 1], oacc[db][4 * i + 2], oacc[db][4 * i + 3]};
          *reinterpret_cast<float4*>(po + db * 32 + 8 * i + 4 * hb) = o;
        }
      if (hb == 0) { a.part_ml[so * 2] = mref; a.part_ml[so * 2 + 1] = l; }
      return;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    if (qtok < 0) return;
    bf16raw* orow = Oh + (size_t)qtok * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint2 o;
        o.x = pack_bf16x2(oacc[db][4 * i] * inv, oacc[db][4 * i + 1] * inv);
        o.y = pack_bf16x2(oacc[db][4 * i + 2] * inv, oacc[db][4 * i + 3] * inv);
        *reinterpret_cast<uint2*>(orow + db * 32 + 8 * i + 4 * hb) = o;
      }
  }
}

// ------------------------------------------------------------------------------------------
// fp32 kernel (the accuracy path of fp32 inputs): the same S^T = K Q^T / O^T += V^T P^T walk on the
// matrix cores with v_mfma_f32_32x32x2_f32 (fp32 products, fp32 accumulation)
// ------------------------------------------------------------------------------------------
// A workgroup is two waves of 32 queries; key tiles of 32 rows go through LDS.  In the 32x32 accumulator a
// lane (c = lane % 32, hb = lane / 32) owns query c and the keys 8*(v/4) + 4*hb + v%4 of the tile, v = 0..15.
// The two values a lane pair supplies per product step may be any pair of the contraction index as long as
// both operands agree: for S the pair is (dim ks, dim D/2 + ks), so a lane keeps one contiguous half of its
// query row; for P.V step j contracts exactly the keys of accumulator value j, so the probabilities are the
// B operand as they stand and no value crosses the half-waves.  K rows are padded to D + 1 floats and V rows
// to D + 8, which spreads the operand reads of a step over the banks.
template <int D>
__global__ __launch_bounds__(128) void attn_f32(AttnArgs a) {
  constexpr int BN = 32, HD = D / 2, KP = D + 1, VP = D + 8, DB = D / 32, NT = 128;
  const int h = blockIdx.y, tile = blockIdx.x;
  if (tile >= a.ntiles[h]) return;
  const int32_t* tl = a.tiles + ((size_t)h * a.maxtiles + tile) * TILE_REC;   // (key lists are never cut for fp32)
  const int qc = tl[0], row0 = tl[1], nrows = tl[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;
  const int nr = a.rng_cnt[(size_t)h * a.Cq + qc];
  const int32_t* rs = a.rng_start + ((size_t)h * a.Cq + qc) * a.maxr;
  const int32_t* rp = a.rng_pre + ((size_t)h * a.Cq + qc) * (a.maxr + 1);
  const int total = rp[nr];
  const float* Qh = (const float*)a.Q + (size_t)h * a.N * D;
  const float* Kh = (const float*)a.Kp + (size_t)h * a.N * D;
  const float* Vh = (const float*)a.Vp + (size_t)h * a.N * D;
  float* Oh = (float*)a.O + (size_t)h * a.N * D;
  __shared__ float Ks[BN * KP];
  __shared__ __attribute__((aligned(16))) float Vs[BN * VP];
  __shared__ int32_t ridx[BN];
  const int qrow = wave * 32 + c;
  int tok = -1;
  if (qrow < nrows) tok = a.perm_q ? a.perm_q[(size_t)h * a.N + row0 + qrow] : row0 + qrow;
  float q[HD];
#pragma unroll
  for (int j = 0; j < HD; j += 4) {
    float4 v = {0.f, 0.f, 0.f, 0.f};
    if (tok >= 0) v = *reinterpret_cast<const float4*>(Qh + (size_t)tok * D + hb * HD + j);
    q[j] = v.x; q[j + 1] = v.y; q[j + 2] = v.z; q[j + 3] = v.w;
  }
  f32x16_t o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  RangeCursor cur;
  if (tid < BN) cur.init(rs, rp, nr);
  for (int k0 = 0; k0 < total; k0 += BN) {
    __syncthreads();                                   // the previous tile has been consumed
    if (tid < BN) ridx[tid] = cur.row(k0 + tid);
    __syncthreads();
    for (int i = tid; i < BN * D / 4; i += NT) {
      const int r = i / (D / 4), qd = i % (D / 4);
      const int row = ridx[r];
      float4 kv = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (row >= 0) {
        kv = reinterpret_cast<const float4*>(Kh + (size_t)row * D)[qd];
        vv = reinterpret_cast<const float4*>(Vh + (size_t)row * D)[qd];
      }
      float* kd = &Ks[r * KP + 4 * qd];
      kd[0] = kv.x; kd[1] = kv.y; kd[2] = kv.z; kd[3] = kv.w;
      *reinterpret_cast<float4*>(&Vs[r * VP + 4 * qd]) = vv;
    }
    __syncthreads();
    f32x16_t sacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < HD; ++ks)
      sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(Ks[c * KP + hb * HD + ks], q[ks], sacc, 0, 0, 0);
    const int kn = total - k0;                          // keys of this tile that exist (>= 1)
    float tmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 8 * (v >> 2) + 4 * hb + (v & 3);
      sacc[v] = key < kn ? sacc[v] * a.scale_log2e : -INFINITY;
      tmax = fmaxf(tmax, sacc[v]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mnew = fmaxf(m, tmax);                  // finite: the tile holds at least one key
    const float alpha = exp2f(m - mnew);
    float lsum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sacc[v] = exp2f(sacc[v] - mnew); lsum += sacc[v]; }
    lsum += __shfl_xor(lsum, 32);
    l = l * alpha + lsum;
    m = mnew;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int key = 8 * (j >> 2) + 4 * hb + (j & 3);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(Vs[key * VP + db * 32 + c], sacc[j], o[db], 0, 0, 0);
      }
    }
  }
  // value v of dim block db is dim db*32 + 8*(v/4) + 4*hb + v%4 of query c
  if (tok >= 0) {
    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 o4 = {o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv};
        *reinterpret_cast<float4*>(Oh + (size_t)tok * D + db * 32 + 8 * g + 4 * hb) = o4;
      }
  }
}

// ------------------------------------------------------------------------------------------
// merge of the chunks of cut key lists
// ------------------------------------------------------------------------------------------
// One workgroup per cut query tile: O = sum_s 2^((m_s - m) scale) O_s / sum_s 2^((m_s - m) scale) l_s
// with m = max_s m_s; a chunk always holds at least one key, so every m_s is finite and l_s > 0.
template <int D>
__global__ __launch_bounds__(256) void attn_merge(AttnArgs a, const int32_t* __restrict__ merge,
                                                  const int32_t* __restrict__ nmerge) {
  // blockIdx.z takes every gridDim.z-th group of rows; the (at most 16) chunks of a row are loaded together,
  // not one after the other: the kernel is a handful of dependent round trips either way, so what counts is
  // how many of its loads are in flight at once.
  constexpr int MAXP = 16;                       // most chunks a list is cut into (plan_tiles)
  const int h = blockIdx.y, e = blockIdx.x;
  if (e >= nmerge[h]) return;
  const int32_t* ml = merge + ((size_t)h * a.slots + e) * 4;
  const int row0 = ml[0], nrows = ml[1], slot0 = ml[2], pieces = min(ml[3], MAXP);
  const int32_t* pq = a.perm_q ? a.perm_q + (size_t)h * a.N : nullptr;
  bf16raw* Oh = (bf16raw*)a.O + (size_t)h * a.N * D;
  constexpr int LPR = D / 4;                     // lanes per row, four columns each
  const int col = (threadIdx.x % LPR) * 4;
  for (int r = blockIdx.z * (256 / LPR) + threadIdx.x / LPR; r < nrows; r += gridDim.z * (256 / LPR)) {
    float ms[MAXP], ls[MAXP];
    float4 os[MAXP];
#pragma unroll
    for (int s = 0; s < MAXP; ++s) {
      const size_t so = ((size_t)h * a.slots + slot0 + min(s, pieces - 1)) * a.BM + r;
      ms[s] = a.part_ml[so * 2];
      ls[s] = a.part_ml[so * 2 + 1];
      os[s] = *reinterpret_cast<const float4*>(a.part_o + so * D + col);
    }
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < MAXP; ++s) if (s < pieces) m = fmaxf(m, ms[s]);
    float l = 0.f;
    float4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < MAXP; ++s) {
      if (s < pieces) {                          // in chunk order, as before: the sums are the same to the bit
        const float w = __builtin_amdgcn_exp2f((ms[s] - m) * a.scale_log2e);
        l = fmaf(w, ls[s], l);
        o.x = fmaf(w, os[s].x, o.x); o.y = fmaf(w, os[s].y, o.y); o.z = fmaf(w, os[s].z, o.z); o.w = fmaf(w, os[s].w, o.w);
      }
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    const int tok = pq ? pq[row0 + r] : row0 + r;
    uint2 out;
    out.x = pack_bf16x2(o.x * inv, o.y * inv);
    out.y = pack_bf16x2(o.z * inv, o.w * inv);
    *reinterpret_cast<uint2*>(Oh + (size_t)tok * D + col) = out;
  }
}

// ------------------------------------------------------------------------------------------
// tile shapes of the bf16 kernel: waves per workgroup NW (32 queries each), pipeline stages NBUF, and MINB = the
// waves per SIMD the register budget is set for (the second __launch_bounds__ argument)
#ifndef A64_NW
#define A64_NW 8
#endif
#ifndef A64_NBUF
#define A64_NBUF 4
#endif
#ifndef A64_MINB
#define A64_MINB 4
#endif
#ifndef A128_NW
#define A128_NW 8
#endif
#ifndef A128_NBUF
#define A128_NBUF 4
#endif
#ifndef A128_MINB
#define A128_MINB 2
#endif
// 32-column blocks of V whose operands are requested before the soft-max arithmetic (the rest follow it)
#ifndef A64_VPRE
#define A64_VPRE 0
#endif
#ifndef A128_VPRE
#define A128_VPRE 2
#endif

// Queries per workgroup.  The bf16 kernel comes in two shapes: eight waves (256 queries, a ring of four stages),
// and four waves (128 queries, two stages, twice the workgroups per CU) for query clusters too small to fill
// the first without long tails (a cluster of 273 queries is 256 + 17 in one shape, 128 + 128 + 17 in the other).
static bool attn_small_shape(int N, int Cq) { return Cq > 1 && N / Cq < 768; }
int attn_block_rows(int dtype, int d, int N, int Cq) {
  if (dtype != ADACLUSTER_BF16) return 64;
  if (attn_small_shape(N, Cq)) return 128;
  return d == 64 ? A64_NW * 32 : A128_NW * 32;
}
int attn_block_rows_min(int dtype) { return dtype == ADACLUSTER_BF16 ? 128 : 64; }
int attn_block_rows_max(int dtype) { return dtype == ADACLUSTER_BF16 ? 256 : 64; }

size_t attn_krow_stride(int N) { return (size_t)(N + 63) / 64 * 64 + KROW_PAD; }

int attn_split_slots() { return SPLIT_SLOTS; }

int launch_plan_sparse(hipStream_t s, int dtype, int H, int Cq, int cap, int maxr, int maxtiles, int BM,
                       const int32_t* q_offs, int q_offs_stride, const int32_t* k_offs, int k_offs_stride,
                       const int32_t* k_count, const int32_t* sel_idx, const int32_t* sel_cnt,
                       int32_t* rng_start, int32_t* rng_pre, int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles,
                       int32_t* merge, int32_t* nmerge, int row_bytes, int32_t* krow, size_t kstride,
                       const int32_t* perm_k, int N) {
  plan_sparse<<<dim3(Cq, H), 256, 0, s>>>(Cq, cap, maxr, row_bytes, k_offs, k_offs_stride, k_count, sel_idx, sel_cnt,
                                         rng_start, rng_pre, rng_cnt, krow, kstride, perm_k, N);
  plan_tiles<<<H, 256, 0, s>>>(Cq, maxr, maxtiles, BM, SPLIT_SLOTS, dtype == ADACLUSTER_BF16 ? 1 : 0, q_offs,
                              q_offs_stride, rng_pre, rng_cnt, tiles, ntiles, merge, nmerge);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

int launch_plan_dense(hipStream_t s, int H, int N, int maxtiles, int BM, int32_t* rng_start, int32_t* rng_pre,
                      int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles, int row_bytes, int32_t* krow, size_t kstride) {
  plan_dense<<<dim3(H, 9), 256, 0, s>>>(N, maxtiles, BM, row_bytes, rng_start, rng_pre, rng_cnt, tiles, ntiles, krow, kstride);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

int launch_attention(hipStream_t s, int dtype, int d, int H, int N, int Cq, int maxtiles, int maxr, float scale,
                     const void* Q, const void* Kp, const void* Vp, void* O, const int32_t* perm_q,
                     const int32_t* tiles, const int32_t* ntiles, const int32_t* rng_start,
                     const int32_t* rng_pre, const int32_t* rng_cnt, float* part_o, float* part_ml,
                     const int32_t* merge, const int32_t* nmerge, const int32_t* krow, size_t kstride) {
  AttnArgs a{Q, Kp, Vp, O, perm_q, tiles, ntiles, rng_start, rng_pre, rng_cnt, N, Cq, maxtiles, maxr,
             scale * 1.4426950408889634f,
             (Cq == 1 || (size_t)4 * N * d <= ((size_t)8 << 20)) ? 1 : 0,
             part_o, part_ml, SPLIT_SLOTS, attn_block_rows(dtype, d, N, Cq), krow, kstride};
  dim3 g((maxtiles + 7) / 8 * 8, H);
  if (dtype == ADACLUSTER_BF16) {
    if (attn_small_shape(N, Cq)) {
      if (d == 64) attn_mfma<64, 4, 2, 4, 0><<<g, 256, 0, s>>>(a);
      else attn_mfma<128, 4, 2, 2, 2><<<g, 256, 0, s>>>(a);
    } else {
      if (d == 64) attn_mfma<64, A64_NW, A64_NBUF, A64_MINB, A64_VPRE><<<g, A64_NW * 64, 0, s>>>(a);
      else attn_mfma<128, A128_NW, A128_NBUF, A128_MINB, A128_VPRE><<<g, A128_NW * 64, 0, s>>>(a);
    }
    if (merge) {      // the chunks of cut key lists (none for the dense branch)
      if (d == 64) attn_merge<64><<<dim3(SPLIT_SLOTS, H, 4), 256, 0, s>>>(a, merge, nmerge);
      else attn_merge<128><<<dim3(SPLIT_SLOTS, H, 4), 256, 0, s>>>(a, merge, nmerge);
    }
  } else {
    if (d == 64) attn_f32<64><<<g, 128, 0, s>>>(a);
    else attn_f32<128><<<g, 128, 0, s>>>(a);
  }
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

}  // namespace adac
