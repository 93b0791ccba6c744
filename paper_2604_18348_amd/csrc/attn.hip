// Attention over the selected key clusters (Alg. 3 lines 9-10) and the dense branch.
//
// Keys and values are first permuted cluster-contiguous (row gathers, HBM bound).  For every
// query cluster the selected key clusters then form a short list of row ranges in that order; a
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

// ------------------------------------------------------------------------------------------
// permutation of K and V rows
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
// rng_start [H][Cq][maxr]   first permuted key row of range r
// rng_pre   [H][Cq][maxr+1] keys before range r in the concatenation (last = total)
// rng_cnt   [H][Cq]
// tiles     [H][maxtiles] x {cluster, first sorted query position, rows, first key tile, end key
//           tile, partial slot or -1}; ntiles [H]
__global__ void plan_sparse(int Cq, int cap, int maxr,
                            const int32_t* __restrict__ k_offs, int k_offs_stride,
                            const int32_t* __restrict__ k_count,
                            const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_cnt,
                            int32_t* __restrict__ rng_start, int32_t* __restrict__ rng_pre,
                            int32_t* __restrict__ rng_cnt) {
  const int h = blockIdx.y, i = blockIdx.x;
  if (threadIdx.x != 0) return;
  const int32_t* sel = sel_idx + ((size_t)h * Cq + i) * cap;
  const int cnt = sel_cnt[(size_t)h * Cq + i];
  const int32_t* ko = k_offs + (size_t)h * k_offs_stride;
  const int kc = k_count[h];
  int32_t* rs = rng_start + ((size_t)h * Cq + i) * maxr;
  int32_t* rp = rng_pre + ((size_t)h * Cq + i) * (maxr + 1);
  int nr = 0, total = 0, cur_s = 0, cur_e = -1;
  for (int t = 0; t < cnt; ++t) {
    const int j = sel[t];
    if (j < 0 || j >= kc) continue;
    const int s = ko[j], e = ko[j + 1];
    if (e <= s) continue;
    if (s == cur_e) { cur_e = e; continue; }
    if (cur_e > cur_s) { rs[nr] = cur_s; rp[nr] = total; total += cur_e - cur_s; ++nr; }
    cur_s = s; cur_e = e;
  }
  if (cur_e > cur_s) { rs[nr] = cur_s; rp[nr] = total; total += cur_e - cur_s; ++nr; }
  rp[nr] = total;
  rng_cnt[(size_t)h * Cq + i] = nr;
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
__global__ void plan_dense(int N, int maxtiles, int BM, int32_t* __restrict__ rng_start,
                           int32_t* __restrict__ rng_pre, int32_t* __restrict__ rng_cnt,
                           int32_t* __restrict__ tiles, int32_t* __restrict__ ntiles) {
  const int h = blockIdx.x;
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

// One workgroup = NW waves, each owning QB blocks of 32 queries; all waves share 64-key K and V
// tiles.  Tiles go global -> LDS directly (no register staging) as 16-byte chunks, one tile
// ahead, double buffered.  A tile row is unpadded; chunk g of row r sits in slot g ^ (r & 7), which
// keeps the 16-byte operand reads and the transpose reads free of bank conflicts.
template <int D, int QB, int NW, int MINB>
__global__ __launch_bounds__(NW * 64, MINB) void attn_mfma(AttnArgs a) {
  constexpr int BN = 64, NT = NW * 64, KS = D / 16, DB = D / 32, CH = D / 8, ROWB = D * 2;
  constexpr int ITEMS = BN * CH, PT = ITEMS / NT, TILEB = BN * ROWB;
  static_assert(ITEMS % NT == 0, "tile chunks must divide evenly over the threads");

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
  const int32_t* rs = a.rng_start + ((size_t)h * a.Cq + qc) * a.maxr;
  const int32_t* rp = a.rng_pre + ((size_t)h * a.Cq + qc) * (a.maxr + 1);
  // positions below are relative to the first key of the share
  const int pbase = kt0 * BN;
  const int total = max(0, min(rp[nr], kt1 * BN) - pbase);
  const int T = (total + BN - 1) / BN;

  const bf16raw* Qh = (const bf16raw*)a.Q + (size_t)h * a.N * D;
  const char* Kh = (const char*)a.Kp + (size_t)h * a.N * ROWB;
  const char* Vh = (const char*)a.Vp + (size_t)h * a.N * ROWB;
  bf16raw* Oh = (bf16raw*)a.O + (size_t)h * a.N * D;
  const int32_t* pq = a.perm_q ? a.perm_q + (size_t)h * a.N : nullptr;

  // Every tile buffer is an LDS object of its own, and the tile loop below is unrolled so that each
  // access names its buffer at compile time: the compiler orders an LDS read behind an outstanding
  // direct-to-LDS load only when both may touch the same object, so this is what lets the load of
  // tile t+1 run under the arithmetic of tile t (with one array indexed by t & 1 it put a
  // vmcnt(0) wait in front of the first operand read of every tile).
  __shared__ __attribute__((aligned(16))) char K0[TILEB];
  __shared__ __attribute__((aligned(16))) char K1[TILEB];
  __shared__ __attribute__((aligned(16))) char V0[TILEB];
  __shared__ __attribute__((aligned(16))) char V1[TILEB];
  __shared__ int32_t ridx[4][BN];          // byte offset of each key row of a tile

  // query tokens of this lane and the B operand of S
  int qtok[QB];
  bf16x8_t qf[QB][KS];
  const bool wave_has_rows = wave * (32 * QB) < nrows;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int rr = wave * (32 * QB) + qb * 32 + c;
    qtok[qb] = -1;
    if (rr < nrows) qtok[qb] = pq ? pq[row0 + rr] : row0 + rr;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = {0, 0, 0, 0};
      if (qtok[qb] >= 0) raw = *reinterpret_cast<const uint4*>(Qh + (size_t)qtok[qb] * D + ks * 16 + hb * 8);
      qf[qb][ks] = *reinterpret_cast<const bf16x8_t*>(&raw);
    }
  }

  f32x16_t oacc[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][qb][v] = 0.f;
  float mrun[QB], lrun[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { mrun[qb] = -INFINITY; lrun[qb] = 0.f; }

  // thread -> (row, slot) of its PT chunks; the slot holds global chunk slot ^ (row & 7)
  auto issue_loads = [&](char* kdst, char* vdst, int rb) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = tid + i * NT;
      const int r = item / CH, q = item % CH;
      const uint32_t off = (uint32_t)ridx[rb][r] + (uint32_t)((q ^ (r & 7)) * 16);
      const int dst = (wave * 64 + i * NT) * 16;     // wave-uniform; the lane offset is implicit
      __builtin_amdgcn_global_load_lds(Kh + off, (lds_void_t*)(kdst + dst), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(Vh + off, (lds_void_t*)(vdst + dst), 16, 0, 0);
    }
  };

  // operand addresses inside a tile (bytes), fixed for the whole kernel
  int kaddr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kaddr[ks] = c * ROWB + (((ks * 2 + hb) ^ (c & 7)) * 16);
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
    for (int db = 0; db < DB; ++db) vaddr[db] = vrow * ROWB + (((db * 4 + gl) ^ (vrow & 7)) * 16) + 8 * (i16 & 1);
  }
  const bf16x2_t ones2 = {(__bf16)1.0f, (__bf16)1.0f};   // row sums use the rounded probabilities P V uses
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  auto compute_tile = [&](const char* ks_, const char* vs_, int nvalid /* < BN only on a masked tail tile */,
                          auto masked) {
    constexpr bool MASK = decltype(masked)::value;
    f32x16_t sacc[2][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      bf16x8_t ka[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        ka[ks] = *reinterpret_cast<const bf16x8_t*>(ks_ + kb * 32 * ROWB + kaddr[ks]);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          sacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[qb][ks], ks == 0 ? zero16 : sacc[kb][qb], 0, 0, 0);
    }
    // accumulator value v of block kb is key  kb*32 + 8*(v/4) + 4*hb + v%4
    if (MASK) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = kb * 32 + 8 * (v >> 2) + 4 * hb + (v & 3);
          if (key >= nvalid) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[kb][qb][v] = -INFINITY;
          }
        }
    }
    bf16x8_t pf[QB][2][2];
    float alpha[QB];
    bool need_rescale = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float tmax = sacc[0][qb][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[kb][qb][v]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float mnew = fmaxf(mrun[qb], tmax);           // finite: every tile holds a valid key
      alpha[qb] = __builtin_amdgcn_exp2f((mrun[qb] - mnew) * a.scale_log2e);
      need_rescale = need_rescale || (mnew != mrun[qb]);
      const float moff = mnew * a.scale_log2e;
      mrun[qb] = mnew;
      float rsum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          uint32_t w[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][8 * s2 + 2 * j], a.scale_log2e, -moff));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kb][qb][8 * s2 + 2 * j + 1], a.scale_log2e, -moff));
            w[j] = pack_bf16x2(p0, p1);
            rsum = __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<const bf16x2_t*>(&w[j]), ones2, rsum, false);
          }
          const uint4 pk = {w[0], w[1], w[2], w[3]};
          pf[qb][kb][s2] = *reinterpret_cast<const bf16x8_t*>(&pk);
        }
      lrun[qb] = lrun[qb] * alpha[qb] + rsum;
    }
    // the running maximum rarely moves after the first tiles: rescale only when some lane needs it
    if (__any(need_rescale)) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= alpha[qb];
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      bf16x8_t va[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const char* vp = vs_ + (kb * 32 + 16 * s2) * ROWB + vaddr[db];
          const s16x4_t lo = lds_read_tr16(vp), hi = lds_read_tr16(vp + 8 * ROWB);
          const s16x4_t both[2] = {lo, hi};
          va[kb][s2] = *reinterpret_cast<const bf16x8_t*>(both);
        }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[kb][s2], pf[qb][kb][s2], oacc[db][qb], 0, 0, 0);
    }
  };

  // prologue: row offsets of tiles 0..2 (a slot past the end repeats the first row: it is loaded
  // but masked), tile 0 into LDS
  // The range table of a query cluster is short (at most top-k entries): it is copied to LDS, so
  // that walking it issues no vector-memory load (those complete in order with the tile loads and
  // would make the walking wave wait for the tile just requested).  A longer table stays in HBM.
  constexpr int RNG_LDS = 256;
  __shared__ int32_t rng_s[RNG_LDS], rng_p[RNG_LDS + 1];
  const bool rng_in_lds = nr <= RNG_LDS;
  if (rng_in_lds) {
    for (int i = tid; i < nr; i += NT) rng_s[i] = rs[i];
    for (int i = tid; i <= nr; i += NT) rng_p[i] = rp[i];
  }
  __syncthreads();
  RangeCursor cur;
  RangeCursorT<lds_ci32_t*> cur_l;
  const int first_off = nr > 0 ? rs[0] * ROWB : 0;
  auto row_off = [&](int p) {
    const int r = rng_in_lds ? cur_l.row(p + pbase) : cur.row(p + pbase);
    return r < 0 ? first_off : r * ROWB;
  };
  if (tid < BN) {
    if (rng_in_lds) cur_l.init((lds_ci32_t*)rng_s, (lds_ci32_t*)rng_p, nr);
    else cur.init(rs, rp, nr);
    ridx[0][tid] = row_off(tid);
    ridx[1][tid] = row_off(BN + tid);
    ridx[2][tid] = row_off(2 * BN + tid);
  }
  __syncthreads();
  if (T > 0) issue_loads(K0, V0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's tile chunks have landed in LDS
  __syncthreads();

  // full tiles in the loop, two per trip (tile t lives in buffer t & 1); a ragged tail tile (the
  // only one that needs masking) after it
  const int Tfull = total / BN;
  auto step = [&](int t, const char* kc, const char* vc, char* kn, char* vn) {
    if (t + 1 < T) issue_loads(kn, vn, (t + 1) & 3);
    if (tid < BN && t + 3 < T) ridx[(t + 3) & 3][tid] = row_off((t + 3) * BN + tid);
    if (wave_has_rows) compute_tile(kc, vc, BN, std::false_type{});
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  };
  int t = 0;
  for (; t + 2 <= Tfull; t += 2) {
    step(t, K0, V0, K1, V1);
    step(t + 1, K1, V1, K0, V0);
  }
  if (t < Tfull) { step(t, K0, V0, K1, V1); ++t; }
  if (T > Tfull && wave_has_rows) {
    if (Tfull & 1) compute_tile(K1, V1, total - Tfull * BN, std::true_type{});
    else compute_tile(K0, V0, total - Tfull * BN, std::true_type{});
  }

  // O^T accumulator value v of block db is column  db*32 + 8*(v/4) + 4*hb + v%4  of query c
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l = lrun[qb] + __shfl_xor(lrun[qb], 32);
    if (pslot >= 0) {
      // a chunk of a cut key list: leave the unnormalised accumulator, the running maximum and the
      // row sum in this chunk's slot; attn_merge combines the chunks of the query tile
      const int rr = wave * (32 * QB) + qb * 32 + c;
      const size_t so = ((size_t)h * a.slots + pslot) * a.BM + rr;
      float* po = a.part_o + so * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 o = {oacc[db][qb][4 * i], oacc[db][qb][4 * i + 1], oacc[db][qb][4 * i + 2], oacc[db][qb][4 * i + 3]};
          *reinterpret_cast<float4*>(po + db * 32 + 8 * i + 4 * hb) = o;
        }
      if (hb == 0) { a.part_ml[so * 2] = mrun[qb]; a.part_ml[so * 2 + 1] = l; }
      continue;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    if (qtok[qb] < 0) continue;
    bf16raw* orow = Oh + (size_t)qtok[qb] * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint2 o;
        o.x = pack_bf16x2(oacc[db][qb][4 * i] * inv, oacc[db][qb][4 * i + 1] * inv);
        o.y = pack_bf16x2(oacc[db][qb][4 * i + 2] * inv, oacc[db][qb][4 * i + 3] * inv);
        *reinterpret_cast<uint2*>(orow + db * 32 + 8 * i + 4 * hb) = o;
      }
  }
}

// ------------------------------------------------------------------------------------------
// fp32 kernel: one query per thread, key tiles broadcast from LDS (accuracy path, small inputs)
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_f32(AttnArgs a) {
  constexpr int BN = 32;
  const int h = blockIdx.y, tile = blockIdx.x;
  if (tile >= a.ntiles[h]) return;
  const int32_t* tl = a.tiles + ((size_t)h * a.maxtiles + tile) * TILE_REC;   // (key lists are never cut for fp32)
  const int qc = tl[0], row0 = tl[1], nrows = tl[2];
  const int tid = threadIdx.x;
  const int nr = a.rng_cnt[(size_t)h * a.Cq + qc];
  const int32_t* rs = a.rng_start + ((size_t)h * a.Cq + qc) * a.maxr;
  const int32_t* rp = a.rng_pre + ((size_t)h * a.Cq + qc) * (a.maxr + 1);
  const int total = rp[nr];
  const float* Qh = (const float*)a.Q + (size_t)h * a.N * D;
  const float* Kh = (const float*)a.Kp + (size_t)h * a.N * D;
  const float* Vh = (const float*)a.Vp + (size_t)h * a.N * D;
  float* Oh = (float*)a.O + (size_t)h * a.N * D;
  __shared__ __attribute__((aligned(16))) float Ks[BN * D];
  __shared__ __attribute__((aligned(16))) float Vs[BN * D];
  __shared__ int32_t ridx[BN];
  int tok = -1;
  if (tid < nrows) tok = a.perm_q ? a.perm_q[(size_t)h * a.N + row0 + tid] : row0 + tid;
  float q[D], o[D];
#pragma unroll
  for (int j = 0; j < D; ++j) { q[j] = tok >= 0 ? Qh[(size_t)tok * D + j] : 0.f; o[j] = 0.f; }
  float m = -INFINITY, l = 0.f;
  RangeCursor cur;
  if (tid < BN) cur.init(rs, rp, nr);
  for (int k0 = 0; k0 < total; k0 += BN) {
    __syncthreads();
    if (tid < BN) ridx[tid] = cur.row(k0 + tid);
    __syncthreads();
    for (int i = tid; i < BN * D / 4; i += 64) {
      const int r = i / (D / 4), qd = i % (D / 4);
      const int row = ridx[r];
      float4 kv = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (row >= 0) {
        kv = reinterpret_cast<const float4*>(Kh + (size_t)row * D)[qd];
        vv = reinterpret_cast<const float4*>(Vh + (size_t)row * D)[qd];
      }
      reinterpret_cast<float4*>(Ks)[i] = kv;
      reinterpret_cast<float4*>(Vs)[i] = vv;
    }
    __syncthreads();
    const int kn = min(BN, total - k0);
    for (int r = 0; r < kn; ++r) {
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < D; j += 4) {
        const float4 kv = *reinterpret_cast<const float4*>(&Ks[r * D + j]);
        s = fmaf(q[j], kv.x, s); s = fmaf(q[j + 1], kv.y, s);
        s = fmaf(q[j + 2], kv.z, s); s = fmaf(q[j + 3], kv.w, s);
      }
      s *= a.scale_log2e;
      const float mnew = fmaxf(m, s);
      const float alpha = exp2f(m - mnew);
      const float p = exp2f(s - mnew);
      l = l * alpha + p;
#pragma unroll
      for (int j = 0; j < D; j += 4) {
        const float4 vv = *reinterpret_cast<const float4*>(&Vs[r * D + j]);
        o[j] = fmaf(o[j], alpha, p * vv.x); o[j + 1] = fmaf(o[j + 1], alpha, p * vv.y);
        o[j + 2] = fmaf(o[j + 2], alpha, p * vv.z); o[j + 3] = fmaf(o[j + 3], alpha, p * vv.w);
      }
      m = mnew;
    }
  }
  if (tok >= 0) {
    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int j = 0; j < D; ++j) Oh[(size_t)tok * D + j] = o[j] * inv;
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
  const int h = blockIdx.y, e = blockIdx.x;
  if (e >= nmerge[h]) return;
  const int32_t* ml = merge + ((size_t)h * a.slots + e) * 4;
  const int row0 = ml[0], nrows = ml[1], slot0 = ml[2], pieces = ml[3];
  const int32_t* pq = a.perm_q ? a.perm_q + (size_t)h * a.N : nullptr;
  bf16raw* Oh = (bf16raw*)a.O + (size_t)h * a.N * D;
  constexpr int LPR = D / 4;                     // lanes per row, four columns each
  for (int r = threadIdx.x / LPR; r < nrows; r += 256 / LPR) {
    const int col = (threadIdx.x % LPR) * 4;
    float m = -INFINITY;
    for (int s = 0; s < pieces; ++s)
      m = fmaxf(m, a.part_ml[(((size_t)h * a.slots + slot0 + s) * a.BM + r) * 2]);
    float l = 0.f;
    float4 o = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < pieces; ++s) {
      const size_t so = ((size_t)h * a.slots + slot0 + s) * a.BM + r;
      const float w = __builtin_amdgcn_exp2f((a.part_ml[so * 2] - m) * a.scale_log2e);
      l = fmaf(w, a.part_ml[so * 2 + 1], l);
      const float4 v = *reinterpret_cast<const float4*>(a.part_o + so * D + col);
      o.x = fmaf(w, v.x, o.x); o.y = fmaf(w, v.y, o.y); o.z = fmaf(w, v.z, o.z); o.w = fmaf(w, v.w, o.w);
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
// tile shapes of the bf16 kernel: queries per wave = 32*QB, waves per block NW, blocks per CU MINB
#ifndef A64_QB
#define A64_QB 1
#endif
#ifndef A64_NW
#define A64_NW 4
#endif
#ifndef A64_MINB
#define A64_MINB 4
#endif
#ifndef A128_QB
#define A128_QB 1
#endif
#ifndef A128_NW
#define A128_NW 4
#endif
#ifndef A128_MINB
#define A128_MINB 2
#endif

int attn_block_rows(int dtype, int d) {
  if (dtype != ADACLUSTER_BF16) return 64;
  return d == 64 ? A64_NW * 32 * A64_QB : A128_NW * 32 * A128_QB;
}

int attn_split_slots() { return SPLIT_SLOTS; }

int launch_plan_sparse(hipStream_t s, int dtype, int H, int Cq, int cap, int maxr, int maxtiles, int BM,
                       const int32_t* q_offs, int q_offs_stride, const int32_t* k_offs, int k_offs_stride,
                       const int32_t* k_count, const int32_t* sel_idx, const int32_t* sel_cnt,
                       int32_t* rng_start, int32_t* rng_pre, int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles,
                       int32_t* merge, int32_t* nmerge) {
  plan_sparse<<<dim3(Cq, H), 64, 0, s>>>(Cq, cap, maxr, k_offs, k_offs_stride, k_count, sel_idx, sel_cnt, rng_start,
                                        rng_pre, rng_cnt);
  plan_tiles<<<H, 256, 0, s>>>(Cq, maxr, maxtiles, BM, SPLIT_SLOTS, dtype == ADACLUSTER_BF16 ? 1 : 0, q_offs,
                              q_offs_stride, rng_pre, rng_cnt, tiles, ntiles, merge, nmerge);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

int launch_plan_dense(hipStream_t s, int H, int N, int maxtiles, int BM, int32_t* rng_start, int32_t* rng_pre,
                      int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles) {
  plan_dense<<<H, 256, 0, s>>>(N, maxtiles, BM, rng_start, rng_pre, rng_cnt, tiles, ntiles);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

int launch_attention(hipStream_t s, int dtype, int d, int H, int N, int Cq, int maxtiles, int maxr, float scale,
                     const void* Q, const void* Kp, const void* Vp, void* O, const int32_t* perm_q,
                     const int32_t* tiles, const int32_t* ntiles, const int32_t* rng_start,
                     const int32_t* rng_pre, const int32_t* rng_cnt, float* part_o, float* part_ml,
                     const int32_t* merge, const int32_t* nmerge) {
  AttnArgs a{Q, Kp, Vp, O, perm_q, tiles, ntiles, rng_start, rng_pre, rng_cnt, N, Cq, maxtiles, maxr,
             scale * 1.4426950408889634f,
             (Cq == 1 || (size_t)4 * N * d <= ((size_t)8 << 20)) ? 1 : 0,
             part_o, part_ml, SPLIT_SLOTS, attn_block_rows(dtype, d)};
  dim3 g((maxtiles + 7) / 8 * 8, H);
  if (dtype == ADACLUSTER_BF16) {
    if (d == 64) attn_mfma<64, A64_QB, A64_NW, A64_MINB><<<g, A64_NW * 64, 0, s>>>(a);
    else attn_mfma<128, A128_QB, A128_NW, A128_MINB><<<g, A128_NW * 64, 0, s>>>(a);
    if (merge) {      // the chunks of cut key lists (none for the dense branch)
      if (d == 64) attn_merge<64><<<dim3(SPLIT_SLOTS, H), 256, 0, s>>>(a, merge, nmerge);
      else attn_merge<128><<<dim3(SPLIT_SLOTS, H), 256, 0, s>>>(a, merge, nmerge);
    }
  } else {
    if (d == 64) attn_f32<64><<<g, 64, 0, s>>>(a);
    else attn_f32<128><<<g, 64, 0, s>>>(a);
  }
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

}  // namespace adac
