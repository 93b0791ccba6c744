// Stable label sort (LSD radix, 7-bit digits) and CSR offsets.
//
// The permutation that groups tokens by cluster label is what makes the centroid
// reduction atomic-free and the K/V gathers cluster-contiguous.  It must be
// deterministic, so ranks inside a segment are taken in item order (wave-wide
// match on the digit, never "who won the atomic").  All passes are bound by HBM
// traffic of 4-byte labels and indices.
#include "common.h"
#include "launch.h"
#include "small_head.h"

namespace adac {


struct SortArgs {
  const int32_t* n_dev;  int n_stride;  int n_const;
  const int32_t* active_dev; int active_stride;
};

__device__ __forceinline__ int head_items(const SortArgs& a, int h) {
  if (a.active_dev && !a.active_dev[(size_t)h * a.active_stride]) return 0;   // head not active
  return a.n_dev ? a.n_dev[(size_t)h * a.n_stride] : a.n_const;
}

// histogram of one digit per segment
__global__ __launch_bounds__(64) void radix_count(const int32_t* __restrict__ labels, int N, int shift,
                                                  SortArgs a, int nseg, int32_t* __restrict__ hist) {
  const int h = blockIdx.y, seg = blockIdx.x, lane = threadIdx.x;
  const int n = head_items(a, h);
  __shared__ int32_t cnt[RBINS];
  cnt[lane] = 0; cnt[lane + 64] = 0;
  __syncthreads();
  const int beg = seg * SEG;
  if (beg < n) {
    const int end = min(beg + SEG, n);
    const int32_t* lab = labels + (size_t)h * N;
    int lv[SEG / 64];
#pragma unroll
    for (int k = 0; k < SEG / 64; ++k) { const int p = beg + 64 * k + lane; lv[k] = p < end ? lab[p] : -1; }
#pragma unroll
    for (int k = 0; k < SEG / 64; ++k) if (lv[k] >= 0) atomicAdd(&cnt[(lv[k] >> shift) & (RBINS - 1)], 1);
  }
  __syncthreads();
  int32_t* out = hist + ((size_t)h * nseg + seg) * RBINS;
  out[lane] = cnt[lane]; out[lane + 64] = cnt[lane + 64];
}

// exclusive scan: bins major, segments minor -> first output position per (segment, bin).
// 8 groups of 128 threads each scan a contiguous eighth of the segments, then the groups are chained.
__global__ __launch_bounds__(8 * RBINS) void radix_scan(int nseg, int32_t* __restrict__ hist) {
  const int h = blockIdx.x, b = threadIdx.x & (RBINS - 1), g = threadIdx.x >> RBITS;
  int32_t* hh = hist + (size_t)h * nseg * RBINS;
  const int per = (nseg + 7) / 8;
  const int s0 = g * per, s1 = min(nseg, s0 + per);
  // The counts are read in batches of eight independent loads (a load per step behind the store of the step
  // before would make every segment a round trip of its own): first for the group's total, then again, once
  // the base is known, to write the running positions.
  constexpr int BATCH = 8;
  int run = 0;
  for (int sb = s0; sb < s1; sb += BATCH) {
    int c[BATCH];
#pragma unroll
    for (int k = 0; k < BATCH; ++k) c[k] = sb + k < s1 ? hh[(sb + k) * RBINS + b] : 0;
#pragma unroll
    for (int k = 0; k < BATCH; ++k) run += c[k];
  }
  __shared__ int32_t gsum[8][RBINS];
  __shared__ int32_t tot[RBINS];
  gsum[g][b] = run;
  __syncthreads();
  int before = 0, all = 0;
  for (int i = 0; i < 8; ++i) { const int v = gsum[i][b]; if (i < g) before += v; all += v; }
  if (g == 0) tot[b] = all;
  __syncthreads();
  int pos = before;
  for (int i = 0; i < b; ++i) pos += tot[i];
  for (int sb = s0; sb < s1; sb += BATCH) {
    int c[BATCH];
#pragma unroll
    for (int k = 0; k < BATCH; ++k) c[k] = sb + k < s1 ? hh[(sb + k) * RBINS + b] : 0;
#pragma unroll
    for (int k = 0; k < BATCH; ++k) {
      if (sb + k < s1) hh[(sb + k) * RBINS + b] = pos;
      pos += c[k];
    }
  }
}

// scatter one pass: (label, value) pairs move to their stable sorted position
__global__ __launch_bounds__(64) void radix_scatter(const int32_t* __restrict__ labels_in,
                                                    const int32_t* __restrict__ vals_in, int N, int shift,
                                                    SortArgs a, int nseg, const int32_t* __restrict__ hist,
                                                    int32_t* __restrict__ labels_out,
                                                    int32_t* __restrict__ vals_out) {
  const int h = blockIdx.y, seg = blockIdx.x, lane = threadIdx.x;
  const int n = head_items(a, h);
  const int beg = seg * SEG;
  if (beg >= n) return;
  const int end = min(beg + SEG, n);
  __shared__ int32_t base[RBINS];
  const int32_t* hb = hist + ((size_t)h * nseg + seg) * RBINS;
  base[lane] = hb[lane]; base[lane + 64] = hb[lane + 64];
  __syncthreads();
  const int32_t* lab = labels_in + (size_t)h * N;
  const int32_t* val = vals_in ? vals_in + (size_t)h * N : nullptr;
  int32_t* lo = labels_out + (size_t)h * N;
  int32_t* vo = vals_out + (size_t)h * N;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  // the segment's items, all loads in flight at once (a load per step of the loop below would leave
  // the wave waiting on memory eight times over)
  int lv[SEG / 64], vv[SEG / 64];
#pragma unroll
  for (int k = 0; k < SEG / 64; ++k) {
    const int p = beg + 64 * k + lane;
    lv[k] = p < end ? lab[p] : 0;
    vv[k] = p < end ? (val ? val[p] : p) : 0;
  }
#pragma unroll
  for (int k = 0; k < SEG / 64; ++k) {
    const int p = beg + 64 * k + lane;
    const bool valid = p < end;
    const int l = lv[k];
    const int v = vv[k];
    const int dig = (l >> shift) & (RBINS - 1);
    // lanes holding my digit: intersect, bit by bit, the ballots of lanes that agree with me
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RBITS; ++b) {
      const bool bit = (dig >> b) & 1;
      const uint64_t bal = __ballot(bit);
      same &= bit ? bal : ~bal;
    }
    const int rank = __popcll(same & lt_mask);
    const int cnt = __popcll(same);
    const bool leader = valid && rank == 0;
    int pos = 0;
    if (valid) pos = base[dig] + rank;
    __syncthreads();
    if (valid && leader) base[dig] += cnt;
    __syncthreads();
    if (valid) { lo[pos] = l; vo[pos] = v; }
  }
}

// offs[j] = number of sorted labels < j (j = 0..m), by binary search in the sorted labels
__global__ void label_offsets(const int32_t* __restrict__ sorted, int N, SortArgs a,
                              const int32_t* __restrict__ m_dev, int m_stride, int m_const,
                              int32_t* __restrict__ offs, int offs_stride) {
  const int h = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (a.active_dev && !a.active_dev[(size_t)h * a.active_stride]) return;
  const int m = m_dev ? m_dev[(size_t)h * m_stride] : m_const;
  if (j > m) return;
  const int n = head_items(a, h);
  const int32_t* s = sorted + (size_t)h * N;
  int lo = 0, hi = n;
  while (lo < hi) { int mid = (lo + hi) >> 1; if (s[mid] < j) lo = mid + 1; else hi = mid; }
  offs[(size_t)h * offs_stride + j] = lo;
}

// One workgroup per head: see sort_one_head.
__global__ __launch_bounds__(1024) void sort_small(const int32_t* __restrict__ labels, const int32_t* __restrict__ vals_in,
                                                   int N, int passes, SortArgs a, const int32_t* __restrict__ m_dev,
                                                   int m_stride, int m_const, int32_t* __restrict__ lab_a,
                                                   int32_t* __restrict__ val_a, int32_t* __restrict__ lab_b,
                                                   int32_t* __restrict__ perm, int32_t* __restrict__ offs,
                                                   int offs_stride, int32_t* __restrict__ poff, int part_rows) {
  const int h = blockIdx.x;
  if (a.active_dev && !a.active_dev[(size_t)h * a.active_stride]) return;
  const int n = head_items(a, h);
  const int m = m_dev ? m_dev[(size_t)h * m_stride] : m_const;
  const size_t o = (size_t)h * N;
  sort_one_head(labels + o, vals_in ? vals_in + o : nullptr, n, passes, m, lab_a + o, val_a + o, lab_b + o, perm + o,
                offs + (size_t)h * offs_stride, poff ? poff + (size_t)h * offs_stride : nullptr, part_rows);
}

int launch_sort(hipStream_t st, int H, int N, int n_bound, int m_bound,
                const int32_t* labels, const int32_t* ulist,
                const int32_t* n_dev, int n_stride, const int32_t* m_dev, int m_stride,
                const int32_t* active_dev, int active_stride,
                int32_t* perm, int32_t* offs, int offs_stride, const SortScratch& sc, int32_t* poff,
                int part_rows, int* poff_done) {
  SortArgs a{n_dev, n_stride, n_bound, active_dev, active_stride};
  const int nseg = (n_bound + SEG - 1) / SEG;
  int bits = 1;
  while ((1 << bits) < m_bound) ++bits;
  const int passes = (bits + RBITS - 1) / RBITS;
  if (poff_done) *poff_done = 0;
#ifndef SORT_SMALL_LIMIT
#define SORT_SMALL_LIMIT 32
#endif
  static_assert(SORT_SMALL_LIMIT <= SMALL_SEGS, "the one-workgroup sort holds SMALL_SEGS segments");
  if (nseg <= SORT_SMALL_LIMIT) {
    sort_small<<<H, 1024, 0, st>>>(labels, ulist, N, passes, a, m_dev, m_stride, m_bound, sc.lab_a, sc.val_a, sc.lab_b,
                                   perm, offs, offs_stride, poff, part_rows);
    if (poff_done && poff) *poff_done = 1;
    return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
  }
  dim3 g(nseg, H);
  const int32_t* lin = labels;
  const int32_t* vin = ulist;
  for (int ps = 0; ps < passes; ++ps) {
    const bool last = (ps == passes - 1);
    // ping-pong: the last pass writes sorted labels to lab_b and values to perm
    int32_t* lout = last ? sc.lab_b : sc.lab_a;
    int32_t* vout = last ? perm : sc.val_a;
    radix_count<<<g, 64, 0, st>>>(lin, N, ps * RBITS, a, nseg, sc.hist);
    radix_scan<<<H, 8 * RBINS, 0, st>>>(nseg, sc.hist);
    radix_scatter<<<g, 64, 0, st>>>(lin, vin, N, ps * RBITS, a, nseg, sc.hist, lout, vout);
    lin = lout; vin = vout;
  }
  dim3 go((m_bound + 1 + 255) / 256, H);
  label_offsets<<<go, 256, 0, st>>>(sc.lab_b, N, a, m_dev, m_stride, m_bound, offs, offs_stride);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

}  // namespace adac
