// Critical-cluster selection: centroid scores (Eq. 1 / Eq. 2, Algorithm 2), arg-top-k (Alg. 3
// line 8) and the top-p budget.
//
// The score matrix is tiny (Cq x Ck x d per head), so it is evaluated in fp64, term by term in ascending
// dimension order, with the bits a rounded multiply followed by a rounded add would give (score_kernel says
// why its fused multiply-adds do).  That makes every bit of a score, and therefore every selected index set,
// reproducible by a CPU implementation.  Floating-point contraction by the compiler is switched off for this
// file for the same reason.
#include "common.h"
#include "launch.h"

#include <atomic>

#pragma clang fp contract(off)

namespace adac {

struct SelectCfg {
  int Cq, cap, d, lds_cap;
  int score_mode, select_mode, topk;
  double top_p, scale;
};

// exp(x), x <= 0, from rounded +,* only: k = rint(x log2 e); r = (x - k ln2_hi) - k ln2_lo;
// degree-13 Taylor polynomial in Horner form; scaled by 2^k.  0 below -700.
__device__ double exp_det(double x) {
#pragma clang fp contract(off)
  if (x < -700.0) return 0.0;
  const double k = rint(x * 1.4426950408889634);
  const double r = (x - k * 0.693147180369123816490) - k * 1.90821492927058770002e-10;
  // 1/n!, each the correctly rounded quotient of 1 and the (exact) double n!; folded at compile time,
  // which rounds as the device would
  constexpr double c[14] = {1.0 / 1.0, 1.0 / 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0, 1.0 / 120.0, 1.0 / 720.0,
                            1.0 / 5040.0, 1.0 / 40320.0, 1.0 / 362880.0, 1.0 / 3628800.0, 1.0 / 39916800.0,
                            1.0 / 479001600.0, 1.0 / 6227020800.0};
  double p = c[13];
#pragma unroll
  for (int n = 12; n >= 0; --n) p = p * r + c[n];
  return ldexp(p, (int)k);
}

// monotone map double -> uint64 (larger double = larger key); -inf is the smallest key
__device__ __forceinline__ uint64_t order_key(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// Scores of every (query cluster, key cluster) pair: S[h][i][j], -inf for an empty key cluster, 0 for a head
// that attends to everything.  A thread owns SCORE_ROWS key clusters and reads their rows (16 bytes at a time,
// one step ahead) ONCE for SCORE_QG query clusters, whose centroids wait in LDS split by sign:
//   (q, 0) where q's sign bit is clear, (0, q) where it is set.
// Every score is the pair of chains  sp += q+ * k+,  sn += q- * k-  in ascending dimension order with
// k+/k- = max(c,0)/min(c,0) (Algorithm 2), box max/min (Eq. 1), or c itself with q- = 0 (plain dot product).
// The term of the sign q does not have is an exact zero, which leaves its chain as it was, so each chain sees
// exactly the terms it owns.  q and k are float values, so a product is exact in double (48 significant bits
// at most, exponents far inside the range) and the fused multiply-add rounds once, exactly where the add of a
// separately rounded product would: the same bits as multiply-then-add at twice the rate.
// (One workgroup per query cluster reading every key row itself, as the selection kernel did before, was bound
// by L2 traffic: 65 reads of a head's centroid table.)
// Measured at 1171 / 500 key clusters per head (24 / 30 heads, d = 128 / 64), (QG, rows): (13,1) 61 / 30 us,
// (7,1) 76 / 29, (13,2) 66 / 36, (9,2) 84 / 30, (7,2) 83 / 41, (5,2) 89 / 44; with one row the LDS pipe is the
// limit (a 16-byte broadcast read per two fused multiply-adds), with more rows the registers and the smaller
// number of waves are.  The query values as scalar operands (scalar loads from a table prepared by another
// kernel, no LDS) took 165 / 75 us: the scalar cache delivers far less than the LDS.
constexpr int SCORE_QG = 13;       // query clusters per thread (65 = 5 groups) ...
constexpr int SCORE_QG_SMALL = 5;  // ... or 5 (13 groups) when the launch would otherwise leave SIMDs without a wave
constexpr int SCORE_ROWS = 1;      // key clusters per thread
constexpr int SCORE_THREADS = 128;

template <int QG>
__global__ __launch_bounds__(SCORE_THREADS) void score_kernel(SelectCfg cfg, const float* __restrict__ q_cent,
                                                              const float* __restrict__ k_cent,
                                                              const float* __restrict__ k_bmin,
                                                              const float* __restrict__ k_bmax,
                                                              const int32_t* __restrict__ k_sizes,
                                                              const int32_t* __restrict__ k_count,
                                                              const int32_t* __restrict__ full_flag,
                                                              double* __restrict__ S) {
  constexpr int R = SCORE_ROWS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  double2* qs = reinterpret_cast<double2*>(smem);            // [QG][d]
  const int h = blockIdx.z, i0 = blockIdx.y * QG, tid = threadIdx.x;
  const int d = cfg.d;
  const int kc = min(k_count[h], cfg.lds_cap);
  if ((int)blockIdx.x * (R * SCORE_THREADS) >= kc) return;
  const bool dot = cfg.score_mode == ADACLUSTER_SCORE_DOT, box = cfg.score_mode == ADACLUSTER_SCORE_BOX;
  for (int e = tid; e < QG * d; e += SCORE_THREADS) {
    const int g = e / d, t = e - g * d;
    const int i = min(i0 + g, cfg.Cq - 1);        // (the last group repeats the last cluster; not stored)
    const float q = q_cent[((size_t)h * cfg.Cq + i) * d + t];
    const bool neg = (__float_as_uint(q) >> 31) != 0u;
    double2 v;
    v.x = (dot || !neg) ? (double)q : 0.0;
    v.y = (!dot && neg) ? (double)q : 0.0;
    qs[e] = v;
  }
  __syncthreads();
  // Row r of this thread is key cluster jb + r * SCORE_THREADS.  A row that needs no arithmetic (past the
  // count, empty, or in a head that attends to everything) runs on row jb's data all the same and stores its
  // fixed value instead.
  const int jb = blockIdx.x * (R * SCORE_THREADS) + tid;
  if (jb >= kc) return;
  const bool all = full_flag[h] != 0;
  bool live[R], any_live = false; double fixed[R];
  const float4* rpos[R]; const float4* rneg[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int j = jb + r * SCORE_THREADS;
    const int nj = j < kc ? k_sizes[(size_t)h * cfg.cap + j] : 0;
    live[r] = j < kc && nj > 0 && !all;
    any_live = any_live || live[r];
    fixed[r] = nj == 0 ? -INFINITY : 0.0;
    const int jl = live[r] ? j : jb;
    rpos[r] = reinterpret_cast<const float4*>((box ? k_bmax : k_cent) + ((size_t)h * cfg.cap + jl) * d);
    rneg[r] = reinterpret_cast<const float4*>((box ? k_bmin : k_cent) + ((size_t)h * cfg.cap + jl) * d);
  }
  double sp[R][QG], sn[R][QG];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int g = 0; g < QG; ++g) { sp[r][g] = 0.0; sn[r][g] = 0.0; }
  if (any_live) {
    constexpr int B4 = 4 / R > 0 ? 4 / R : 1;      // 16-byte pieces of a row per step
    float4 pb[R][B4], nb[R][B4];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int u4 = 0; u4 < B4; ++u4) { pb[r][u4] = rpos[r][u4]; nb[r][u4] = box ? rneg[r][u4] : pb[r][u4]; }
    for (int st = 0; st < d / (4 * B4); ++st) {
      float4 pc[R][B4], nc[R][B4];
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int u4 = 0; u4 < B4; ++u4) { pc[r][u4] = pb[r][u4]; nc[r][u4] = nb[r][u4]; }
      if (st + 1 < d / (4 * B4)) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int u4 = 0; u4 < B4; ++u4) {
            pb[r][u4] = rpos[r][(st + 1) * B4 + u4];
            nb[r][u4] = box ? rneg[r][(st + 1) * B4 + u4] : pb[r][u4];
          }
      }
#pragma unroll
      for (int u4 = 0; u4 < B4; ++u4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = (st * B4 + u4) * 4 + u;
          double kp[R], kn[R];
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const float pv = u == 0 ? pc[r][u4].x : u == 1 ? pc[r][u4].y : u == 2 ? pc[r][u4].z : pc[r][u4].w;
            const float nv = u == 0 ? nc[r][u4].x : u == 1 ? nc[r][u4].y : u == 2 ? nc[r][u4].z : nc[r][u4].w;
            kp[r] = (double)((box || dot) ? pv : fmaxf(pv, 0.f));
            kn[r] = (double)((box || dot) ? nv : fminf(nv, 0.f));
          }
#pragma unroll
          for (int g = 0; g < QG; ++g) {
            const double2 q2 = qs[g * d + t];
#pragma unroll
            for (int r = 0; r < R; ++r) {
              sp[r][g] = __fma_rn(q2.x, kp[r], sp[r][g]);
              sn[r][g] = __fma_rn(q2.y, kn[r], sn[r][g]);
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int j = jb + r * SCORE_THREADS;
    if (j >= kc) continue;
    double* out = S + ((size_t)h * cfg.Cq + i0) * cfg.cap + j;
#pragma unroll
    for (int g = 0; g < QG; ++g)
      if (i0 + g < cfg.Cq) out[(size_t)g * cfg.cap] = live[r] ? sp[r][g] + sn[r][g] : fixed[r];
  }
}

// One block per (query cluster, head).  Dynamic LDS: key[cap] (uint64) + flag[cap] (int).
__global__ __launch_bounds__(256) void select_kernel(SelectCfg cfg, const double* __restrict__ S,
                                                     const float* __restrict__ q_mean_norm,
                                                     const int32_t* __restrict__ k_sizes,
                                                     const int32_t* __restrict__ k_count,
                                                     const int32_t* __restrict__ full_flag,
                                                     int32_t* __restrict__ sel_idx, int32_t* __restrict__ sel_cnt) {
#pragma clang fp contract(off)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  double* sval = reinterpret_cast<double*>(smem);                        // [cap] score, then weight
  uint64_t* skey = reinterpret_cast<uint64_t*>(smem + (size_t)cfg.lds_cap * 8);   // [lds_cap]
  int32_t* sflag = reinterpret_cast<int32_t*>(smem + (size_t)cfg.lds_cap * 16);   // [lds_cap]
  __shared__ int32_t wsum[4], wsum2[4];
  __shared__ int32_t s_take, s_digit, s_krem, s_all;
  __shared__ int32_t hist[256];
  __shared__ double s_max;
  __shared__ double swmax[4];

  const int h = blockIdx.y, i = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  bool use_thr = false;          // top-k by threshold key: selected = key > thr_key, or == thr_key among the first thr_rem
  uint64_t thr_key = 0;
  int thr_rem = 0;
  const int kc = min(k_count[h], cfg.lds_cap);
  const bool all = full_flag[h] != 0;
  // ---- scores of this query cluster (score_kernel)
  {
    const double* sr = S + ((size_t)h * cfg.Cq + i) * cfg.cap;
    for (int j = tid; j < kc; j += 256) sval[j] = sr[j];
  }
  __syncthreads();

  const bool topp = cfg.select_mode == ADACLUSTER_SELECT_TOPP;
  if (all || (topp && cfg.top_p >= 1.0)) {
    for (int j = tid; j < kc; j += 256) sflag[j] = sval[j] > -INFINITY;
  } else if (!topp) {
    // The topk largest by (score desc, index asc).  No ranks are needed, only the key of the
    // topk-th largest: an MSB-first radix select over the 64-bit order keys (eight 8-bit digits, a
    // 256-bin histogram per digit).  Equal keys at the threshold are resolved by index in the
    // compaction below, which walks the clusters in ascending order anyway.
    int nv = 0;
    for (int j = tid; j < kc; j += 256) {
      const double v = sval[j];
      skey[j] = order_key(v);
      nv += v > -INFINITY;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) nv += __shfl_xor(nv, o);
    if (lane == 0) wsum[wave] = nv;
    __syncthreads();
    const int nvalid = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
    if (nvalid <= cfg.topk) {
      for (int j = tid; j < kc; j += 256) sflag[j] = sval[j] > -INFINITY;
    } else {
      use_thr = true;
      uint64_t prefix = 0;
      int krem = cfg.topk;
      for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < kc; j += 256) {
          const uint64_t k = skey[j];
          if (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(int)((k >> shift) & 255)], 1);
        }
        __syncthreads();
        // thread t owns bin 255 - t: an inclusive scan over t counts the keys in higher or equal bins
        const int bin = 255 - tid;
        const int cnt = hist[bin];
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) { const int u = __shfl_up(incl, o); if (lane >= o) incl += u; }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        for (int w = 0; w < wave; ++w) incl += wsum[w];
        const int excl = incl - cnt;
        if (excl < krem && krem <= incl) { s_digit = bin; s_krem = krem - excl; s_all = (krem == incl); }
        __syncthreads();
        prefix |= (uint64_t)s_digit << shift;
        krem = s_krem;
        // every key of the chosen bin is wanted: the threshold is the bin's lower edge, no ties to split
        if (s_all && prefix != 0) { prefix -= 1; krem = 0; break; }
      }
      thr_key = prefix; thr_rem = krem;
    }
  } else {
    // weights w_j = n_j exp(alpha (S_j - max S)); order by (w desc, j asc); shortest prefix
    // whose running sum reaches top_p * total
    {
      // the maximum does not depend on the order it is taken in
      double m = -INFINITY;
      for (int j = tid; j < kc; j += 256) m = fmax(m, sval[j]);
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) m = fmax(m, __shfl_xor(m, o));
      if (lane == 0) swmax[wave] = m;
      __syncthreads();
      if (tid == 0) s_max = fmax(fmax(swmax[0], swmax[1]), fmax(swmax[2], swmax[3]));
      __syncthreads();
    }
    const double alpha = (double)q_mean_norm[(size_t)h * cfg.Cq + i] * cfg.scale;
    const double mx = s_max;
    for (int j = tid; j < kc; j += 256) {
      const int nj = k_sizes[(size_t)h * cfg.cap + j];
      double w = 0.0;
      if (nj > 0) w = (double)nj * exp_det(alpha * (sval[j] - mx));
      const bool valid = sval[j] > -INFINITY;
      sval[j] = w;
      // invalid (empty) clusters sort after everything else
      skey[j] = valid ? order_key(w) : 0ull;
      sflag[j] = valid;
    }
    __syncthreads();
    // rank of every valid cluster, stored in place of the flag: sflag = rank+1, 0 = invalid
    // (a thread ranks its clusters two at a time, so that a key read serves both)
    for (int j = tid; j < kc; j += 512) {
      const int j2 = j + 256;
      const bool v1 = sflag[j] != 0, v2 = j2 < kc && sflag[j2] != 0;
      const uint64_t k1 = skey[j], k2 = j2 < kc ? skey[j2] : 0ull;
      int r1 = 0, r2 = 0;
      for (int t = 0; t < kc; ++t) {
        const uint64_t kt = skey[t];
        r1 += (kt > k1) || (kt == k1 && t < j);
        r2 += (kt > k2) || (kt == k2 && t < j2);
      }
      if (v1) sflag[j] = r1 + 1;
      if (v2) sflag[j2] = r2 + 1;
    }
    __syncthreads();
    // The weights in rank order go into skey (dead once the ranks are known), then one thread takes
    // the two sums, each a chain of rounded adds in a fixed order: the total in ascending index, the
    // running sum in rank order.  It reads eight values at a time, so that the LDS reads of a batch
    // are in flight together and only the adds wait for one another.
    double* sw = reinterpret_cast<double*>(skey);
    int nv_local = 0;
    for (int j = tid; j < kc; j += 256) nv_local += sflag[j] != 0;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) nv_local += __shfl_xor(nv_local, o);
    if (lane == 0) wsum[wave] = nv_local;
    __syncthreads();                // every thread has read its keys: skey may be overwritten
    for (int j = tid; j < kc; j += 256) if (sflag[j]) sw[sflag[j] - 1] = sval[j];
    __syncthreads();
    if (tid == 0) {
      const int nvalid = wsum[0] + wsum[1] + wsum[2] + wsum[3];
      double total = 0.0;
      int j = 0;
      for (; j + 8 <= kc; j += 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = sval[j + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) total = total + v[u];
      }
      for (; j < kc; ++j) total = total + sval[j];
      const double target = cfg.top_p * total;
      double cum = 0.0;
      int take = nvalid;
      bool found = false;
      int r = 0;
      for (; r + 8 <= nvalid && !found; r += 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = sw[r + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (!found) {
            cum = cum + v[u];
            if (cum >= target) { take = r + u + 1; found = true; }
          }
        }
      }
      for (; r < nvalid && !found; ++r) {
        cum = cum + sw[r];
        if (cum >= target) { take = r + 1; found = true; }
      }
      s_take = take;
    }
    __syncthreads();
    const int take = s_take;
    for (int j = tid; j < kc; j += 256) sflag[j] = sflag[j] != 0 && sflag[j] <= take;
  }
  __syncthreads();

  // ---- ascending compaction of the selected indices
  int32_t* out = sel_idx + ((size_t)h * cfg.Cq + i) * cfg.cap;
  int run = 0, run_eq = 0;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int j0 = 0; j0 < kc; j0 += 256) {
    const int j = j0 + tid;
    bool f;
    if (use_thr) {
      const bool valid = j < kc && sval[j] > -INFINITY;
      const uint64_t k = j < kc ? skey[j] : 0ull;
      const bool eq = valid && k == thr_key;
      const uint64_t bal_eq = __ballot(eq);
      __syncthreads();
      if (lane == 0) wsum2[wave] = __popcll(bal_eq);
      __syncthreads();
      int eq_before = run_eq + __popcll(bal_eq & lt_mask);
      for (int w = 0; w < wave; ++w) eq_before += wsum2[w];
      run_eq += wsum2[0] + wsum2[1] + wsum2[2] + wsum2[3];
      f = valid && (k > thr_key || (eq && eq_before < thr_rem));
    } else {
      f = j < kc && sflag[j] != 0;
    }
    const uint64_t bal = __ballot(f);
    __syncthreads();
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    if (f) out[run + before + __popcll(bal & lt_mask)] = j;
    run += wsum[0] + wsum[1] + wsum[2] + wsum[3];
  }
  if (tid == 0) sel_cnt[(size_t)h * cfg.Cq + i] = run;
}

int launch_select(hipStream_t s, int H, int Cq, int cap, int d, int score_mode, int select_mode, int topk,
                  float top_p, float scale, const float* q_cent, const float* q_mean_norm, const float* k_cent,
                  const float* k_bmin, const float* k_bmax, const int32_t* k_sizes, const int32_t* k_count,
                  const int32_t* full_flag, int32_t* sel_idx, int32_t* sel_cnt, int kc_max, double* scores) {
  // kc_max: an upper bound of k_count[h] known to the host; it sizes the LDS arrays (and with
  // them the number of workgroups a CU can hold)
  const int lds_cap = kc_max < cap ? (kc_max + 63) / 64 * 64 : cap;
  SelectCfg c{Cq, cap, d, lds_cap, score_mode, select_mode, topk, (double)top_p, (double)scale};
  const size_t shm = (size_t)lds_cap * 20;
  if (shm > 150 * 1024) return ADACLUSTER_E_BADSHAPE;
  // The kernel's dynamic-LDS limit is raised only when a launch needs more than any launch before it on this
  // device (a call that repeats an earlier shape then consists of launches only, which is what a caller that
  // captures it into a HIP graph needs).
  static std::atomic<int> granted[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return ADACLUSTER_E_INTERNAL;
  if ((int)shm > granted[dev].load()) {
    if (hipFuncSetAttribute((const void*)select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
      return ADACLUSTER_E_INTERNAL;
    granted[dev].store((int)shm);
  }
  const int kb = kc_max < cap ? kc_max : cap;
  const int kblocks = (kb + SCORE_ROWS * SCORE_THREADS - 1) / (SCORE_ROWS * SCORE_THREADS);
  // 1024 SIMDs: with fewer than two waves each the larger grid of the small group size is the faster one
  const bool small_groups = (long long)kblocks * ((Cq + SCORE_QG - 1) / SCORE_QG) * H * (SCORE_THREADS / 64) < 2048;
  if (small_groups)
    score_kernel<SCORE_QG_SMALL><<<dim3(kblocks, (Cq + SCORE_QG_SMALL - 1) / SCORE_QG_SMALL, H), SCORE_THREADS,
                                   (size_t)SCORE_QG_SMALL * d * sizeof(double2), s>>>(c, q_cent, k_cent, k_bmin, k_bmax, k_sizes,
                                                                                     k_count, full_flag, scores);
  else
    score_kernel<SCORE_QG><<<dim3(kblocks, (Cq + SCORE_QG - 1) / SCORE_QG, H), SCORE_THREADS,
                             (size_t)SCORE_QG * d * sizeof(double2), s>>>(c, q_cent, k_cent, k_bmin, k_bmax, k_sizes, k_count,
                                                                         full_flag, scores);
  select_kernel<<<dim3(Cq, H), 256, shm, s>>>(c, scores, q_mean_norm, k_sizes, k_count, full_flag, sel_idx, sel_cnt);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

}  // namespace adac
