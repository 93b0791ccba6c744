// Quest scores between query rows and key pages (Sec. 3.2.3): the upper bound of Eq. 1 evaluated
// with plain vector arithmetic, and its reformulation as two matrix products (Eq. 2, Algorithm 2)
// on the matrix cores.  Both take the per-dimension maxima R+ and minima R- of every page (for a
// single vector per page, e.g. a cluster centroid, Algorithm 2 uses R+ = max(k, 0), R- = min(k, 0):
// `clamp` does that on the fly from one tensor).
//   S[h, i, j] = sum_d max(q_d R+_jd, q_d R-_jd)                       (Eq. 1)
//              = sum_d max(q_d, 0) R+_jd + sum_d min(q_d, 0) R-_jd     (Eq. 2)
#include "common.h"
#include "launch.h"

namespace adac {

// ---- Eq. 1 with vector arithmetic: 64 x 64 outputs per workgroup, 4 x 4 per thread, operands staged through
// LDS 32 dimensions at a time
template <typename T>
__global__ __launch_bounds__(256) void quest_alu(int Lq, int Lk, int d, int clamp, const T* __restrict__ Q,
                                                 const T* __restrict__ Rp, const T* __restrict__ Rn,
                                                 float* __restrict__ S) {
  constexpr int TD = 32;
  __shared__ float qs[64][TD + 1], ps[64][TD + 1], ns[64][TD + 1];
  const int h = blockIdx.z, q0 = blockIdx.x * 64, k0 = blockIdx.y * 64, tid = threadIdx.x;
  const int tq = (tid >> 4) * 4, tk = (tid & 15) * 4;
  const T* Qh = Q + (size_t)h * Lq * d;
  const T* Ph = Rp + (size_t)h * Lk * d;
  const T* Nh = Rn + (size_t)h * Lk * d;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int d0 = 0; d0 < d; d0 += TD) {
    __syncthreads();
    for (int e = tid; e < 64 * TD; e += 256) {
      const int r = e / TD, cc = e % TD;
      qs[r][cc] = (q0 + r < Lq) ? Elem<T>::load(Qh + (size_t)(q0 + r) * d + d0 + cc) : 0.f;
      float p = 0.f, n = 0.f;
      if (k0 + r < Lk) {
        p = Elem<T>::load(Ph + (size_t)(k0 + r) * d + d0 + cc);
        n = Elem<T>::load(Nh + (size_t)(k0 + r) * d + d0 + cc);
        if (clamp) { p = fmaxf(p, 0.f); n = fminf(n, 0.f); }
      }
      ps[r][cc] = p; ns[r][cc] = n;
    }
    __syncthreads();
#pragma unroll 4
    for (int cc = 0; cc < TD; ++cc) {
      float qv[4], pv[4], nv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { qv[i] = qs[tq + i][cc]; pv[i] = ps[tk + i][cc]; nv[i] = ns[tk + i][cc]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += fmaxf(qv[i] * pv[j], qv[i] * nv[j]);
    }
  }
  float* Sh = S + (size_t)h * Lq * Lk;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (q0 + tq + i < Lq && k0 + tk + j < Lk) Sh[(size_t)(q0 + tq + i) * Lk + k0 + tk + j] = acc[i][j];
}

// ---- Eq. 2 on the matrix cores (bf16): S^T[32 pages x 32 queries] += R+[32 x 16] Q+^T[16 x 32] + R-[32 x 16] Q-^T.
// A wave keeps the positive and negative parts of its 32 query rows in registers as B operands; page
// rows are staged through LDS 64 at a time (clamped while staging when asked to) and are the A operands.
template <int D>
__global__ __launch_bounds__(256, 2) void quest_mfma(int Lq, int Lk, int clamp, const bf16raw* __restrict__ Q,
                                                     const bf16raw* __restrict__ Rp, const bf16raw* __restrict__ Rn,
                                                     float* __restrict__ S) {
  constexpr int CB = 64, LDW = D + 8, KS = D / 16;
  __shared__ __attribute__((aligned(16))) bf16raw ps[CB * LDW], ns[CB * LDW];
  __shared__ float ts[4][32 * 33];          // a wave's finished tile, for the turn before the store
  const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;
  const int q = blockIdx.x * 128 + wave * 32 + c;
  const bf16raw* Qh = Q + (size_t)h * Lq * D;
  bf16x8_t qp[KS], qn[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 raw = {0, 0, 0, 0};
    if (q < Lq) raw = *reinterpret_cast<const uint4*>(Qh + (size_t)q * D + ks * 16 + hb * 8);
    // bf16 pairs: keep the elements whose sign bit is clear (positive part) or set (negative part)
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    uint32_t wp[4], wn[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo_neg = (w[i] & 0x8000u) ? 0xFFFFu : 0u, hi_neg = (w[i] & 0x80000000u) ? 0xFFFF0000u : 0u;
      const uint32_t negmask = lo_neg | hi_neg;
      wn[i] = w[i] & negmask; wp[i] = w[i] & ~negmask;
    }
    const uint4 up = {wp[0], wp[1], wp[2], wp[3]}, un = {wn[0], wn[1], wn[2], wn[3]};
    qp[ks] = *reinterpret_cast<const bf16x8_t*>(&up);
    qn[ks] = *reinterpret_cast<const bf16x8_t*>(&un);
  }
  const bf16raw* Ph = Rp + (size_t)h * Lk * D;
  const bf16raw* Nh = Rn + (size_t)h * Lk * D;
  float* Sh = S + (size_t)h * Lq * Lk;
  for (int k0 = 0; k0 < Lk; k0 += CB) {
    __syncthreads();
    constexpr int CHUNKS = D / 8;
    for (int i = tid; i < CB * CHUNKS; i += 256) {
      const int r = i / CHUNKS, g = i % CHUNKS;
      uint4 vp = {0, 0, 0, 0}, vn = {0, 0, 0, 0};
      if (k0 + r < Lk) {
        vp = *reinterpret_cast<const uint4*>(Ph + (size_t)(k0 + r) * D + g * 8);
        vn = *reinterpret_cast<const uint4*>(Nh + (size_t)(k0 + r) * D + g * 8);
        if (clamp) {
          uint32_t* a = reinterpret_cast<uint32_t*>(&vp);
          uint32_t* b = reinterpret_cast<uint32_t*>(&vn);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t negmask = ((a[e] & 0x8000u) ? 0xFFFFu : 0u) | ((a[e] & 0x80000000u) ? 0xFFFF0000u : 0u);
            const uint32_t negmask_b = ((b[e] & 0x8000u) ? 0xFFFFu : 0u) | ((b[e] & 0x80000000u) ? 0xFFFF0000u : 0u);
            a[e] &= ~negmask; b[e] &= negmask_b;
          }
        }
      }
      *reinterpret_cast<uint4*>(&ps[r * LDW + g * 8]) = vp;
      *reinterpret_cast<uint4*>(&ns[r * LDW + g * 8]) = vn;
    }
    __syncthreads();
#pragma unroll
    for (int rb = 0; rb < CB / 32; ++rb) {
      if (k0 + rb * 32 >= Lk) break;
      f32x16_t acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t ap = *reinterpret_cast<const bf16x8_t*>(&ps[(rb * 32 + c) * LDW + ks * 16 + hb * 8]);
        const bf16x8_t an = *reinterpret_cast<const bf16x8_t*>(&ns[(rb * 32 + c) * LDW + ks * 16 + hb * 8]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap, qp[ks], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(an, qn[ks], acc, 0, 0, 0);
      }
      // value v of the tile is page k0 + rb*32 + 8*(v/4) + 4*hb + v%4 for query q: turned through LDS, so
      // that a half-wave writes 32 consecutive pages of one query row
      float* tw = &ts[wave][0];
#pragma unroll
      for (int v = 0; v < 16; ++v) tw[c * 33 + 8 * (v >> 2) + 4 * hb + (v & 3)] = acc[v];
      __builtin_amdgcn_wave_barrier();
      const int q_base = blockIdx.x * 128 + wave * 32;
      const int page = k0 + rb * 32 + c;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qq = 2 * r + hb;
        if (q_base + qq < Lq && page < Lk) Sh[(size_t)(q_base + qq) * Lk + page] = tw[qq * 33 + c];
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

int launch_quest_scores(hipStream_t s, int dtype, int form, int clamp, int H, int Lq, int Lk, int d, const void* Q,
                        const void* Rp, const void* Rn, float* S) {
  if (form == 0) {
    const dim3 g((Lq + 63) / 64, (Lk + 63) / 64, H);
    if (dtype == ADACLUSTER_BF16)
      quest_alu<bf16raw><<<g, 256, 0, s>>>(Lq, Lk, d, clamp, (const bf16raw*)Q, (const bf16raw*)Rp, (const bf16raw*)Rn, S);
    else
      quest_alu<float><<<g, 256, 0, s>>>(Lq, Lk, d, clamp, (const float*)Q, (const float*)Rp, (const float*)Rn, S);
  } else {
    if (dtype != ADACLUSTER_BF16) return ADACLUSTER_E_UNSUPPORTED;
    const dim3 g((Lq + 127) / 128, H);
    if (d == 64) quest_mfma<64><<<g, 256, 0, s>>>(Lq, Lk, clamp, (const bf16raw*)Q, (const bf16raw*)Rp, (const bf16raw*)Rn, S);
    else quest_mfma<128><<<g, 256, 0, s>>>(Lq, Lk, clamp, (const bf16raw*)Q, (const bf16raw*)Rp, (const bf16raw*)Rn, S);
  }
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

// ------------------------------------------------------------------------------------------
// Matrix-core probe: every wave runs four independent chains of v_mfma_f32_32x32x16_bf16 on operands that
// never leave its registers.  It moves no data, so the rate it reaches is the bf16 MFMA throughput the chip
// sustains at the clock it holds under that load: the yardstick quoted beside the published peak.
// ------------------------------------------------------------------------------------------
static constexpr int PROBE_BLOCKS = 2048, PROBE_THREADS = 256, PROBE_CHAINS = 4;
__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe(int iters, float* __restrict__ sink) {
  const int tid = threadIdx.x;
  bf16x8_t a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)((tid + i) & 3); b[i] = (__bf16)(float)((tid >> 2) & 1); }
  f32x16_t c[PROBE_CHAINS];
#pragma unroll
  for (int j = 0; j < PROBE_CHAINS; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < PROBE_CHAINS; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < PROBE_CHAINS; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c[j][v];
  if (blockIdx.x == 0) sink[tid] = s;
}

int launch_mfma_probe(hipStream_t s, int iters, float* sink, size_t sink_floats, double* flops) {
  if (sink_floats < (size_t)PROBE_THREADS) return ADACLUSTER_E_BADARG;
  mfma_probe<<<PROBE_BLOCKS, PROBE_THREADS, 0, s>>>(iters, sink);
  *flops = (double)PROBE_BLOCKS * (PROBE_THREADS / 64) * (double)iters * PROBE_CHAINS * (2.0 * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL;
}

}  // namespace adac
