// Pieces shared by the label sort (sort.hip) and the clustering kernels (cluster.hip): the sort
// of one head by ONE workgroup of 1024 threads.
#pragma once
#include "common.h"

namespace adac {

static constexpr int SEG = 512;      // items per wave step of the label sort
static constexpr int RBITS = 7;
static constexpr int RBINS = 1 << RBITS;
static constexpr int SMALL_SEGS = 32;   // the one-workgroup sort holds at most this many segments

// The whole sort of one head's n <= SMALL_SEGS * SEG labels in one workgroup (all 1024 threads must
// call it): every radix pass, the label offsets offs[0..m] and, if poff is given, the part offsets
// of the centroid reduction, which otherwise take five launches per pass of a few microseconds
// each.  Same arithmetic and the same stable order as the multi-workgroup kernels: wave w takes
// segments w and w+16 and holds their items in registers for the whole pass; the per-(segment,
// digit) counts live in LDS.  All pointers are the head's own rows.  labels/vals_in are read,
// lab_a/val_a are scratch, lab_b receives the sorted labels and perm the sorted values (vals_in
// NULL: the item index).  Ends with every result written but NOT yet made visible to the other
// waves: the caller synchronises the workgroup before reading them.
__device__ __forceinline__ void sort_one_head(const int32_t* __restrict__ labels, const int32_t* __restrict__ vals_in,
                                              int n, int passes, int m, int32_t* __restrict__ lab_a_h,
                                              int32_t* __restrict__ val_a_h, int32_t* __restrict__ lab_b_h,
                                              int32_t* __restrict__ perm_h, int32_t* __restrict__ of,
                                              int32_t* __restrict__ po, int part_rows) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  n = min(n, SMALL_SEGS * SEG);
  const int nseg = (n + SEG - 1) / SEG;
  __shared__ int32_t hist[SMALL_SEGS][RBINS];
  __shared__ int32_t gsum[8][RBINS];
  __shared__ int32_t tot[RBINS];
  __shared__ int32_t sc[1024];
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const int32_t* lin = labels;
  const int32_t* vin = vals_in;
  for (int ps = 0; ps < passes; ++ps) {
    const bool last = ps == passes - 1;
    int32_t* lout = last ? lab_b_h : lab_a_h;
    int32_t* vout = last ? perm_h : val_a_h;
    const int shift = ps * RBITS;
    for (int i = tid; i < nseg * RBINS; i += 1024) (&hist[0][0])[i] = 0;
    // this wave's items of the pass, all loads in flight at once: segment wave + 16*i, item 64*k + lane
    int lab[SMALL_SEGS / 16][SEG / 64], val[SMALL_SEGS / 16][SEG / 64];
#pragma unroll
    for (int i = 0; i < SMALL_SEGS / 16; ++i)
#pragma unroll
      for (int k = 0; k < SEG / 64; ++k) {
        const int p = (wave + 16 * i) * SEG + 64 * k + lane;
        lab[i][k] = p < n ? lin[p] : 0;
        val[i][k] = p < n ? (vin ? vin[p] : p) : 0;
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SMALL_SEGS / 16; ++i)
#pragma unroll
      for (int k = 0; k < SEG / 64; ++k) {
        const int seg = wave + 16 * i, p = seg * SEG + 64 * k + lane;
        if (p < n) atomicAdd(&hist[seg][(lab[i][k] >> shift) & (RBINS - 1)], 1);
      }
    __syncthreads();
    {   // exclusive scan, bins major, segments minor (as radix_scan)
      const int b = tid & (RBINS - 1), g = tid >> RBITS;
      const int per = (nseg + 7) / 8;
      const int s0 = min(nseg, g * per), s1 = min(nseg, s0 + per);
      int run = 0;
      for (int sg = s0; sg < s1; ++sg) { const int c = hist[sg][b]; hist[sg][b] = run; run += c; }
      gsum[g][b] = run;
      __syncthreads();
      int before = 0, all = 0;
      for (int i = 0; i < 8; ++i) { const int v = gsum[i][b]; if (i < g) before += v; all += v; }
      // exclusive prefix of the bin totals: the first two waves scan 64 bins each by shuffles
      int incl = all;
      if (g == 0) {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
        tot[b] = incl - all;
        if (b == 63) sc[0] = incl;             // total of bins 0..63
      }
      __syncthreads();
      const int base = before + tot[b] + (b >= 64 ? sc[0] : 0);
      for (int sg = s0; sg < s1; ++sg) hist[sg][b] += base;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < SMALL_SEGS / 16; ++i) {
      const int seg = wave + 16 * i;
      if (seg >= nseg) break;                        // wave-uniform
      volatile int32_t* base = hist[seg];            // touched by this wave only, in program order
#pragma unroll
      for (int k = 0; k < SEG / 64; ++k) {
        const int p = seg * SEG + 64 * k + lane;
        const bool valid = p < n;
        const int l = lab[i][k], v = val[i][k];
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
        int pos = 0;
        if (valid) pos = base[dig] + rank;
        __builtin_amdgcn_wave_barrier();
        if (valid && rank == 0) base[dig] = base[dig] + cnt;
        __builtin_amdgcn_wave_barrier();
        if (valid) { lout[pos] = l; vout[pos] = v; }
      }
    }
    __syncthreads();        // the pass's output is read back by other waves of this workgroup
    lin = lout; vin = vout;
  }
  // offs[j] = number of sorted labels < j (j = 0..m)
  for (int j = tid; j <= m; j += 1024) {
    int lo = 0, hi = n;
    while (lo < hi) { const int mid = (lo + hi) >> 1; if (lin[mid] < j) lo = mid + 1; else hi = mid; }
    of[j] = lo;
  }
  if (!po) return;
  __syncthreads();
  // poff[j] = number of parts of the clusters before j (a cluster of c rows has ceil(c / part_rows) parts)
  const int per = (m + 1023) / 1024;
  const int j0 = min(m, tid * per), j1 = min(m, j0 + per);
  int run = 0;
  for (int j = j0; j < j1; ++j) run += (of[j + 1] - of[j] + part_rows - 1) / part_rows;
  int incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
  if (lane == 63) sc[wave] = incl;
  __syncthreads();
  int before = 0, total = 0;
  for (int w = 0; w < 16; ++w) { const int v = sc[w]; if (w < wave) before += v; total += v; }
  int base = before + incl - run;
  for (int j = j0; j < j1; ++j) { po[j] = base; base += (of[j + 1] - of[j] + part_rows - 1) / part_rows; }
  if (tid == 0) po[m] = total;
}

}  // namespace adac
