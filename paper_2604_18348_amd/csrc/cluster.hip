// k-means building blocks for the query clustering (Sec. 3.1, Alg. 3 line 1) and the
// multi-stage key clustering (Algorithm 1):
//   * point-to-centre assignment as an MFMA GEMM  C . X^T  with an in-lane running arg-max
//     (bf16 I/O) or a plain fp32 kernel (fp32 I/O);
//   * atomic-free centroid update: segmented sums over the label-sorted token order;
//   * the stage bookkeeping of Algorithm 1 (centre count rule, threshold filter, compaction
//     of the unassigned set U), kept on the device.
#include "common.h"
#include "launch.h"

namespace adac {

// ------------------------------------------------------------------------------------------
// assignment
// ------------------------------------------------------------------------------------------
// modes: 0 = fixed (row_off 0, m = m_const, n = N, every head)
//        1 = stage (row_off = ccount, m = m_t, n = ucount, only active heads)
//        2 = final (row_off 0, m = ccount, n = N, every head)
//        3 = final, seeded (bf16): only the centres of the stages after the first are visited (row_off =
//            stage_offs[1], m = ccount - row_off); every point starts from its best first-stage centre, whose
//            label and score the last pass of stage 0 left in seed_lab / seed_score (that pass ran over all
//            points against exactly those centres).  Labels are indices into all centres, as in mode 2.
// keep_lab / keep_score (stage 0, last pass): a second copy of the labels and the best score, for mode 3.
struct AssignCfg {
  int mode; int m_const; int N; int cap;
  const KState* st; const int32_t* ulist;
  int32_t* keep_lab; float* keep_score;
  const int32_t* seed_lab; const float* seed_score;
};

__device__ __forceinline__ bool assign_setup(const AssignCfg& c, int h, int& n, int& m, int& row_off) {
  if (c.mode == 0) { n = c.N; m = c.m_const; row_off = 0; return true; }
  const KState& s = c.st[h];
  if (c.mode == 1) { n = s.ucount; m = s.m_t; row_off = s.ccount; return s.active != 0; }
  if (c.mode == 3) { n = c.N; row_off = s.stage_offs[1]; m = s.ccount - row_off; return true; }
  n = c.N; m = s.ccount; row_off = 0; return true;
}

// score(x, c) = x.c + bias(c), bias = -||c||^2/2 (Euclidean arg-min) or 0 (cosine arg-max);
// label = arg-max, ties to the lowest index;  dist2 = ||x||^2 - 2 score.
//
// MFMA formulation: D[32 centres x 32 points] += A[32 x 16] B[16 x 32] with A = centre rows from
// LDS and B = point rows held in registers for the whole kernel.  In the 32x32 accumulator a lane
// owns ONE point (column lane%32) and 16 centres, so the arg-max over centres runs in-lane; the
// two half-waves are merged once at the end.  Two workgroups per CU in the launch bounds keep the
// register budget at 256, so the accumulators are ordinary VGPRs that the arg-max reads directly (with
// 512 the compiler parks them in AGPRs and copies every value out first).
//
// ACC (small stages of Algorithm 1): the workgroup also leaves, per centre, the sum and the count of the
// points of its block that chose it, so that the centroid update needs neither a label sort nor a
// segmented reduction.  The sums are a second MFMA product, S^T[32 dims x 32 centres] +=
// X^T[32 dims x 16 points] . E[16 points x 32 centres] with E the one-hot label matrix: exact products,
// fp32 accumulation in a fixed order.  Block b of head h writes row j * nb_stride + b of the head's
// part-sum table and bcnt[(h * nb_stride + b) * ACC_MAXM + j].
struct AccumOut { float* psum; int32_t* bcnt; int P; int nb_stride; };
constexpr int ACC_MAXM = 128;          // most centres the block sums are kept for

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;

template <int D, bool ACC>
__global__ __launch_bounds__(256, (ACC && D == 128) ? 1 : 2) void assign_mfma(const bf16raw* __restrict__ X, AssignCfg cfg,
                                                                const bf16raw* __restrict__ cent,
                                                                const float* __restrict__ bias,
                                                                int32_t* __restrict__ labels, float* __restrict__ dist2,
                                                                AccumOut acc_out) {
  constexpr int CB = D == 128 ? 64 : 128;   // centres per LDS chunk (16 KB either way; larger chunks measured slower)
  constexpr int KS = D / 16;
  constexpr int PB = 2;                 // 32-point blocks per wave
  constexpr int CROWB = D * 2, CH = D / 8;  // bytes and 16-byte pieces of a centre row
  const int h = blockIdx.y;
  int n, m, row_off;
  if (!assign_setup(cfg, h, n, m, row_off)) return;
  const int base = blockIdx.x * (4 * PB * 32);
  if (base >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;

  // Centre chunks go global -> LDS directly (no registers), one chunk ahead, in two buffers that are LDS
  // objects of their own (the compiler orders an LDS read behind an outstanding direct load only when
  // both may touch the same object, so the load of chunk i+1 runs under the arithmetic of chunk i).
  // Rows are unpadded; piece g of row r sits in slot g ^ swz(r), which keeps the 16-byte operand
  // reads of 16 consecutive rows in 16 different bank groups.
  __shared__ __attribute__((aligned(16))) char cs0[CB * CROWB];
  __shared__ __attribute__((aligned(16))) char cs1[CB * CROWB];
  __shared__ __attribute__((aligned(16))) float bs0[CB];
  __shared__ __attribute__((aligned(16))) float bs1[CB];
  auto swz = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };

  // B operand: this lane's point rows
  bf16x8_t xf[PB][KS];
  float xn2[PB];
  int pos[PB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    pos[pb] = base + wave * (PB * 32) + pb * 32 + c;
    float ss = 0.f;
    if (pos[pb] < n) {
      const int tok = cfg.ulist ? cfg.ulist[(size_t)h * cfg.N + pos[pb]] : pos[pb];
      const bf16raw* row = X + ((size_t)h * cfg.N + tok) * D + hb * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 raw = *reinterpret_cast<const uint4*>(row + ks * 16);
        xf[pb][ks] = *reinterpret_cast<const bf16x8_t*>(&raw);
      }
      if (dist2) {                       // ||x||^2 is only needed for the distances
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint4 raw = *reinterpret_cast<const uint4*>(&xf[pb][ks]);
          const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float a = __uint_as_float(w[q] << 16), b = __uint_as_float(w[q] & 0xFFFF0000u);
            ss = fmaf(a, a, ss); ss = fmaf(b, b, ss);
          }
        }
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { const uint4 z = {0, 0, 0, 0}; xf[pb][ks] = *reinterpret_cast<const bf16x8_t*>(&z); }
    }
    xn2[pb] = ss + __shfl_xor(ss, 32);
  }

  // Running arg-max with the position inside a 32x32 accumulator tile carried in the low 4
  // mantissa bits of the score (a 2^-19 relative perturbation, far below the near-tie margin):
  // one and-or per value, then a max3 tree, then one compare per tile.
  float best[PB]; int btile[PB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) { best[pb] = -INFINITY; btile[pb] = 0; }
  // Seeded final pass: the half-wave that owns the seed centre's accumulator position starts from the seed,
  // in the packed form a visit of that centre would have left (score with the position code in the low bits);
  // a negative tile marks "still the seed".
  int slab[PB];
  const int label_base = cfg.mode == 3 ? row_off : 0;
  if (!ACC && cfg.seed_lab) {
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      slab[pb] = 0;
      if (pos[pb] < n) {
        const int j0 = cfg.seed_lab[(size_t)h * cfg.N + pos[pb]];
        const float s0 = cfg.seed_score[(size_t)h * cfg.N + pos[pb]];
        const int r = j0 & 31, v0 = ((r >> 3) << 2) | (r & 3);
        slab[pb] = j0;
        if (hb == ((r >> 2) & 1)) {
          best[pb] = __uint_as_float((__float_as_uint(s0) & 0xFFFFFFF0u) | (uint32_t)(15 - v0));
          btile[pb] = -1;
        }
      }
    }
    if (m <= 0) {                      // no later stage: the first-stage labels are final
#pragma unroll
      for (int pb = 0; pb < PB; ++pb)
        if (hb == 0 && pos[pb] < n) labels[(size_t)h * cfg.N + pos[pb]] = slab[pb];
      return;
    }
  }

  const bf16raw* ch = cent + ((size_t)h * cfg.cap + row_off) * D;
  const float* bh = bias + (size_t)h * cfg.cap + row_off;

  // operand addresses inside a chunk (bytes), fixed for the whole kernel
  int kaddr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kaddr[ks] = c * CROWB + (((ks * 2 + hb) ^ swz(c)) * 16);
  // thread -> (row, slot) of its pieces of a chunk; rows past m repeat the last centre (their bias never wins)
  constexpr int PT = CB * CH / 256;
  auto issue_chunk = [&](int c0, char* dst_base) {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int item = tid + i * 256;
      const int r = item / CH, sl = item % CH;
      const int row = min(c0 + r, m - 1);
      const char* src = reinterpret_cast<const char*>(ch) + (size_t)row * CROWB + ((sl ^ swz(r)) * 16);
      const int dst = (wave * 64 + i * 256) * 16;     // wave-uniform; the lane offset is implicit
      __builtin_amdgcn_global_load_lds(src, (lds_void_t*)(dst_base + dst), 16, 0, 0);
    }
  };
  auto load_bias = [&](int c0) { return (tid < CB && c0 + tid < m) ? bh[c0 + tid] : -3.0e38f; };   // finite: survives the bit packing
  auto compute_chunk = [&](int c0, const char* cs, const float* bs) {
    const int rbmax = min(CB / 32, (m - c0 + 31) / 32);
    for (int rb = 0; rb < rbmax; ++rb) {
      f32x16_t acc[PB];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 b4 = *reinterpret_cast<const float4*>(&bs[rb * 32 + 8 * i + 4 * hb]);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
          acc[pb][4 * i + 0] = b4.x; acc[pb][4 * i + 1] = b4.y;
          acc[pb][4 * i + 2] = b4.z; acc[pb][4 * i + 3] = b4.w;
        }
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(cs + rb * 32 * CROWB + kaddr[ks]);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
          acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xf[pb][ks], acc[pb], 0, 0, 0);
      }
      const int tile_id = (c0 >> 5) + rb;
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) {
        float pk[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) pk[v] = __uint_as_float((__float_as_uint(acc[pb][v]) & 0xFFFFFFF0u) | (uint32_t)(15 - v));
        float tm = fmaxf(fmaxf(pk[0], pk[1]), pk[2]);
#pragma unroll
        for (int v = 3; v < 15; v += 2) tm = fmaxf(fmaxf(tm, pk[v]), pk[v + 1]);
        tm = fmaxf(tm, pk[15]);
        if (tm > best[pb]) { best[pb] = tm; btile[pb] = tile_id; }
      }
    }
  };
  // one step: request the next chunk, work on this one, then let the request land
  auto step = [&](int c0, const char* cs, const float* bs, char* csn, float* bsn) {
    const bool more = c0 + CB < m;
    float bnext = 0.f;
    if (more) { bnext = load_bias(c0 + CB); issue_chunk(c0 + CB, csn); }
    compute_chunk(c0, cs, bs);
    if (more && tid < CB) bsn[tid] = bnext;
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's pieces of the next chunk are in LDS
    __syncthreads();
  };
  {
    const float b0 = load_bias(0);
    issue_chunk(0, cs0);
    if (tid < CB) bs0[tid] = b0;
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }
  for (int c0 = 0; c0 < m; c0 += 2 * CB) {
    step(c0, cs0, bs0, cs1, bs1);
    if (c0 + CB < m) step(c0 + CB, cs1, bs1, cs0, bs0);
  }
  int blab[PB];
#pragma unroll
  for (int pb = 0; pb < PB; ++pb) {
    // accumulator value v of a tile is centre  32*tile + 8*(v/4) + 4*hb + v%4
    const int v = 15 - (int)(__float_as_uint(best[pb]) & 15u);   // 15-v was packed: equal scores >= 0 go to the lowest centre
    int bidx = label_base + btile[pb] * 32 + 8 * (v >> 2) + 4 * hb + (v & 3);
    if (!ACC && cfg.seed_lab && btile[pb] < 0) bidx = slab[pb];
    float bv = __uint_as_float(__float_as_uint(best[pb]) & 0xFFFFFFF0u);
    const float ob = __shfl_xor(bv, 32);
    const int oi = __shfl_xor(bidx, 32);
    if (ob > bv || (ob == bv && oi < bidx)) { bv = ob; bidx = oi; }
    if (hb == 0 && pos[pb] < n) {
      labels[(size_t)h * cfg.N + pos[pb]] = bidx;
      if (dist2) dist2[(size_t)h * cfg.N + pos[pb]] = fmaxf(xn2[pb] - 2.f * bv, 0.f);
      if (!ACC && cfg.keep_lab) { cfg.keep_lab[(size_t)h * cfg.N + pos[pb]] = bidx; cfg.keep_score[(size_t)h * cfg.N + pos[pb]] = bv; }
    }
    if (ACC) blab[pb] = pos[pb] < n ? bidx : -1;
  }
  if constexpr (ACC) {
    constexpr int ROWB = D * 2, DT = D / 32;
    __shared__ __attribute__((aligned(16))) bf16raw xs[256 * D];     // the block's points, row-major
    __shared__ __attribute__((aligned(16))) int32_t lab_s[256];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int pr = wave * (PB * 32) + pb * 32 + c;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<bf16x8_t*>(&xs[pr * D + ks * 16 + hb * 8]) = xf[pb][ks];
      if (hb == 0) lab_s[pr] = blab[pb];
    }
    __syncthreads();
    const int b = blockIdx.x;
    // output tiles (centre tile ct, dim tile db) dealt to the four waves; one more "dim tile" per centre
    // tile has X^T replaced by ones, so that its rows are the member counts (exact: at most 256)
    const int CT = (m + 31) >> 5;
    // X^T operand by transpose reads (see the V operand of the attention kernel): this lane addresses
    // point 4*hb + (lane%16)/4 of a 16-point group, dims 16*((lane/16)%2) + 4*(lane%4) .. +3
    const int i16 = lane & 15, blk = lane >> 4;
    const int vrow = 4 * hb + (i16 >> 2);
    const int gl = 2 * (blk & 1) + ((i16 & 3) >> 1);
    const char* xsb = reinterpret_cast<const char*>(xs);
    if (CT >= 4) {
      // Many centre tiles: a wave takes whole centre tiles, so that the one-hot operand of a group of
      // 16 points (twenty vector instructions, more than the product it feeds) is built once and serves
      // every dim tile and the counting tile.
      const uint4 ones4 = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
      const bf16x8_t ones = *reinterpret_cast<const bf16x8_t*>(&ones4);
      for (int ct = wave; ct < CT; ct += 4) {
        const int cid = ct * 32 + c;
        f32x16_t sacc[DT + 1];
#pragma unroll
        for (int t = 0; t <= DT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) sacc[t][v] = 0.f;
        const int xoff = vrow * ROWB + gl * 16 + 8 * (i16 & 1);
#pragma unroll 4
        for (int g = 0; g < 16; ++g) {
          const int4 l0 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 4 * hb]);
          const int4 l1 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 8 + 4 * hb]);
          uint4 e;
          e.x = (l0.x == cid ? 0x3F80u : 0u) | (l0.y == cid ? 0x3F800000u : 0u);
          e.y = (l0.z == cid ? 0x3F80u : 0u) | (l0.w == cid ? 0x3F800000u : 0u);
          e.z = (l1.x == cid ? 0x3F80u : 0u) | (l1.y == cid ? 0x3F800000u : 0u);
          e.w = (l1.z == cid ? 0x3F80u : 0u) | (l1.w == cid ? 0x3F800000u : 0u);
          const bf16x8_t eb = *reinterpret_cast<const bf16x8_t*>(&e);
#pragma unroll
          for (int db = 0; db < DT; ++db) {
            const char* xp = xsb + g * 16 * ROWB + xoff + db * 64;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)xp);
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(xp + 8 * ROWB));
            const s16x4_t both[2] = {lo, hi};
            sacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(both), eb, sacc[db], 0, 0, 0);
          }
          sacc[DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, eb, sacc[DT], 0, 0, 0);
        }
        if (cid < m) {
          if (hb == 0) acc_out.bcnt[((size_t)h * acc_out.nb_stride + b) * ACC_MAXM + cid] = (int)sacc[DT][0];
#pragma unroll
          for (int db = 0; db < DT; ++db) {
            float* out = acc_out.psum + ((size_t)h * acc_out.P + (size_t)cid * acc_out.nb_stride + b) * D + db * 32 + 4 * hb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float4 o4 = {sacc[db][4 * i], sacc[db][4 * i + 1], sacc[db][4 * i + 2], sacc[db][4 * i + 3]};
              *reinterpret_cast<float4*>(out + 8 * i) = o4;
            }
          }
        }
      }
      return;
    }
    for (int t = wave; t < CT * (DT + 1); t += 4) {
      const int ct = t / (DT + 1), db = t % (DT + 1);
      const bool counting = db == DT;
      const int cid = ct * 32 + c;
      f32x16_t sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
      const int xoff = vrow * ROWB + ((counting ? 0 : db) * 4 + gl) * 16 + 8 * (i16 & 1);
#pragma unroll
      for (int g = 0; g < 16; ++g) {
        const char* xp = xsb + g * 16 * ROWB + xoff;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)xp);
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(xp + 8 * ROWB));
        const s16x4_t both[2] = {lo, hi};
        bf16x8_t xa = *reinterpret_cast<const bf16x8_t*>(both);
        if (counting) { const uint4 o = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u}; xa = *reinterpret_cast<const bf16x8_t*>(&o); }
        // one-hot rows of the points this lane's eight operand elements stand for
        const int4 l0 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 4 * hb]);
        const int4 l1 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 8 + 4 * hb]);
        uint4 e;
        e.x = (l0.x == cid ? 0x3F80u : 0u) | (l0.y == cid ? 0x3F800000u : 0u);
        e.y = (l0.z == cid ? 0x3F80u : 0u) | (l0.w == cid ? 0x3F800000u : 0u);
        e.z = (l1.x == cid ? 0x3F80u : 0u) | (l1.y == cid ? 0x3F800000u : 0u);
        e.w = (l1.z == cid ? 0x3F80u : 0u) | (l1.w == cid ? 0x3F800000u : 0u);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, *reinterpret_cast<const bf16x8_t*>(&e), sacc, 0, 0, 0);
      }
      if (counting) {
        if (cid < m && hb == 0) acc_out.bcnt[((size_t)h * acc_out.nb_stride + b) * ACC_MAXM + cid] = (int)sacc[0];
        continue;
      }
      // value v of the tile is dim db*32 + 8*(v/4) + 4*hb + v%4 of centre cid
      if (cid < m) {
        float* out = acc_out.psum + ((size_t)h * acc_out.P + (size_t)cid * acc_out.nb_stride + b) * D + db * 32 + 4 * hb;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 o4 = {sacc[4 * i], sacc[4 * i + 1], sacc[4 * i + 2], sacc[4 * i + 3]};
          *reinterpret_cast<float4*>(out + 8 * i) = o4;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// One pass of the query k-means in ONE read of the points: assignment and centroid sums together.
// ------------------------------------------------------------------------------------------
// A workgroup walks `subs` consecutive sub-blocks of 128 points.  Per sub-block every wave assigns its 32
// points to the nearest of the m <= 128 centres (all of them resident in LDS; the same MFMA product and in-lane
// arg-max as assign_mfma), then the sub-block's points, labels and weights go through LDS and every wave adds
//   S^T[32 dims x 32 centres] += X^T[32 dims x 16 points] . E[16 points x 32 centres]
// to the accumulator tiles it owns for the WHOLE walk (wave w: centre tile w in every dim tile).  E is the one-hot label matrix times the point's weight: 1 for Euclidean sums, and for the
// clustering by angle the bf16 value of 1/|x|, so that the tile holds the sum of the (almost) normalised
// members; the weight's rounding (2^-9 relative per member, of random sign) is far below the bf16 rounding the
// centres of the next assignment get anyway.  Products are exact, the accumulation is fp32 in a fixed order,
// so the pass is deterministic.  Walk b of head h leaves row j * NP + b of the head's part-sum table
// psum [H][m * NP][D] and pcnt[(h * NP + b) * ACC_MAXM + j]; finalize_centroids adds the walks in order.
// No label is written: only the last pass of a clustering needs labels, and that one takes the sorted path.
template <int D>
__global__ __launch_bounds__(256, 2) void qpass_mfma(const bf16raw* __restrict__ X, int N, int m, int cap, int subs,
                                                     int weighted, const bf16raw* __restrict__ cent,
                                                     const float* __restrict__ bias, float* __restrict__ psum,
                                                     int32_t* __restrict__ pcnt, int NP) {
  constexpr int KS = D / 16, DT = D / 32, ROWB = D * 2, CH = D / 8, SB = 128, MAXCT = ACC_MAXM / 32;
  const int h = blockIdx.y, b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;
  const int CT = (m + 31) >> 5;
  __shared__ __attribute__((aligned(16))) char cs[MAXCT * 32 * ROWB];     // the centres, rows permuted by chunk
  __shared__ __attribute__((aligned(16))) float bs[MAXCT * 32];
  __shared__ __attribute__((aligned(16))) bf16raw xs[SB * D];             // the sub-block's points, row-major
  __shared__ __attribute__((aligned(16))) int32_t lab_s[SB];
  __shared__ __attribute__((aligned(16))) uint32_t w_s[SB];               // weight of a point as bf16 bits
  __shared__ int32_t cnt_s[ACC_MAXM];
  auto swz = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  {
    const bf16raw* chh = cent + (size_t)h * cap * D;
    for (int item = tid; item < CT * 32 * CH; item += 256) {
      const int r = item / CH, sl = item % CH;
      const int row = min(r, m - 1);                                      // rows past m repeat the last centre under a bias that never wins
      *reinterpret_cast<uint4*>(cs + r * ROWB + ((sl ^ swz(r)) * 16)) =
          *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(chh) + (size_t)row * ROWB + sl * 16);
    }
    if (tid < MAXCT * 32) { bs[tid] = tid < m ? bias[(size_t)h * cap + tid] : -3.0e38f; cnt_s[tid] = 0; }
  }
  int kaddr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kaddr[ks] = c * ROWB + (((ks * 2 + hb) ^ swz(c)) * 16);
  // Wave w owns centre tile w (there are at most four) in all its dim tiles: the one-hot operand of a group
  // of 16 points (about twenty vector instructions, more than one product costs) is built once per group
  // and serves every dim tile.
  f32x16_t sacc[DT];
#pragma unroll
  for (int k = 0; k < DT; ++k)
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[k][v] = 0.f;
  // X^T operand by transpose reads (as the V operand of the attention kernel): this lane addresses point
  // 4*hb + (lane%16)/4 of a 16-point group, dims 16*((lane/16)%2) + 4*(lane%4) .. +3
  const int i16 = lane & 15, blk = lane >> 4;
  const int vrow = 4 * hb + (i16 >> 2);
  const int gl = 2 * (blk & 1) + ((i16 & 3) >> 1);
  // Piece q (16 bytes) of point row r sits in slot q ^ xswz(r): a bijection over 16 consecutive rows (the
  // row-wise 16-byte writes of 16 lanes fall into 16 different bank groups) that also sends the four rows
  // of one transpose read to four different 64-byte groups.
  auto xswz = [](int r) { return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : (((((r >> 1) & 7) & 1) << 2) | (((r >> 1) & 7) >> 1)); };
  int xlo[DT], xhi[DT];
#pragma unroll
  for (int db = 0; db < DT; ++db) {
    xlo[db] = vrow * ROWB + (((db * 4 + gl) ^ xswz(vrow)) * 16) + 8 * (i16 & 1);
    xhi[db] = (vrow + 8) * ROWB + (((db * 4 + gl) ^ xswz(vrow + 8)) * 16) + 8 * (i16 & 1);
  }
  const char* xsb = reinterpret_cast<const char*>(xs);

  const int p_begin = b * subs * SB;
  const bf16raw* Xh = X + (size_t)h * N * D;
  auto load_rows = [&](int base, bf16x8_t* xf) {
    const int pos = base + wave * 32 + c;
    if (pos < N) {
      const bf16raw* row = Xh + (size_t)pos * D + hb * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { const uint4 raw = *reinterpret_cast<const uint4*>(row + ks * 16); xf[ks] = *reinterpret_cast<const bf16x8_t*>(&raw); }
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { const uint4 z = {0, 0, 0, 0}; xf[ks] = *reinterpret_cast<const bf16x8_t*>(&z); }
    }
  };
  bf16x8_t xnext[KS];
  load_rows(p_begin, xnext);
  __syncthreads();                       // centres, bias and counters are in LDS
  for (int sb = 0; sb < subs; ++sb) {
    const int base = p_begin + sb * SB;
    if (base >= N) break;
    bf16x8_t xf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xf[ks] = xnext[ks];
    if (sb + 1 < subs) load_rows(base + SB, xnext);          // the next sub-block's rows travel under this one's arithmetic
    const int pos = base + wave * 32 + c;
    // squared norm of this lane's point (both half-waves hold half of the row)
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&xf[ks]);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(w[q] << 16), bb = __uint_as_float(w[q] & 0xFFFF0000u);
        ss = fmaf(a, a, ss); ss = fmaf(bb, bb, ss);
      }
    }
    ss += __shfl_xor(ss, 32);
    // assignment: arg-max of x.c + bias over the centre tiles, position in a tile carried in the low 4 mantissa bits
    float best = -INFINITY; int btile = 0;
    for (int ct = 0; ct < CT; ++ct) {
      f32x16_t acc;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 b4 = *reinterpret_cast<const float4*>(&bs[ct * 32 + 8 * i + 4 * hb]);
        acc[4 * i + 0] = b4.x; acc[4 * i + 1] = b4.y; acc[4 * i + 2] = b4.z; acc[4 * i + 3] = b4.w;
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(cs + ct * 32 * ROWB + kaddr[ks]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xf[ks], acc, 0, 0, 0);
      }
      float pk[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) pk[v] = __uint_as_float((__float_as_uint(acc[v]) & 0xFFFFFFF0u) | (uint32_t)(15 - v));
      float tm = fmaxf(fmaxf(pk[0], pk[1]), pk[2]);
#pragma unroll
      for (int v = 3; v < 15; v += 2) tm = fmaxf(fmaxf(tm, pk[v]), pk[v + 1]);
      tm = fmaxf(tm, pk[15]);
      if (tm > best) { best = tm; btile = ct; }
    }
    {
      const int v = 15 - (int)(__float_as_uint(best) & 15u);
      int bidx = btile * 32 + 8 * (v >> 2) + 4 * hb + (v & 3);
      float bv = __uint_as_float(__float_as_uint(best) & 0xFFFFFFF0u);
      const float ob = __shfl_xor(bv, 32);
      const int oi = __shfl_xor(bidx, 32);
      if (ob > bv || (ob == bv && oi < bidx)) { bv = ob; bidx = oi; }
      const int pr = wave * 32 + c;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        *reinterpret_cast<bf16x8_t*>(reinterpret_cast<char*>(xs) + pr * ROWB + (((ks * 2 + hb) ^ xswz(pr)) * 16)) = xf[ks];
      if (hb == 0) {
        const bool valid = pos < N;
        lab_s[pr] = valid ? bidx : -1;
        w_s[pr] = weighted ? (uint32_t)f32_to_bf16(1.0f / fmaxf(sqrtf(ss), 1e-12f)) : 0x3F80u;
        if (valid) atomicAdd(&cnt_s[bidx], 1);
      }
    }
    __syncthreads();
    // sums: the owned centre tile takes the eight 16-point groups of the sub-block
    if (wave < CT) {
      const int cid = wave * 32 + c;
#pragma unroll 2
      for (int g = 0; g < SB / 16; ++g) {
        const int4 l0 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 4 * hb]);
        const int4 l1 = *reinterpret_cast<const int4*>(&lab_s[g * 16 + 8 + 4 * hb]);
        const uint4 w0 = *reinterpret_cast<const uint4*>(&w_s[g * 16 + 4 * hb]);
        const uint4 w1 = *reinterpret_cast<const uint4*>(&w_s[g * 16 + 8 + 4 * hb]);
        uint4 e;
        e.x = (l0.x == cid ? w0.x : 0u) | (l0.y == cid ? w0.y << 16 : 0u);
        e.y = (l0.z == cid ? w0.z : 0u) | (l0.w == cid ? w0.w << 16 : 0u);
        e.z = (l1.x == cid ? w1.x : 0u) | (l1.y == cid ? w1.y << 16 : 0u);
        e.w = (l1.z == cid ? w1.z : 0u) | (l1.w == cid ? w1.w << 16 : 0u);
        const bf16x8_t eb = *reinterpret_cast<const bf16x8_t*>(&e);
#pragma unroll
        for (int db = 0; db < DT; ++db) {
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(xsb + g * 16 * ROWB + xlo[db]));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(xsb + g * 16 * ROWB + xhi[db]));
          const s16x4_t both[2] = {lo, hi};
          sacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(both), eb, sacc[db], 0, 0, 0);
        }
      }
    }
    __syncthreads();                     // the sub-block's points and labels may be overwritten
  }
  // value v of dim tile db is dim db*32 + 8*(v/4) + 4*hb + v%4 of centre cid
  if (wave < CT && wave * 32 + c < m) {
    const int cid = wave * 32 + c;
#pragma unroll
    for (int db = 0; db < DT; ++db) {
      float* out = psum + ((size_t)h * m * NP + (size_t)cid * NP + b) * D + db * 32 + 4 * hb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 o4 = {sacc[db][4 * i], sacc[db][4 * i + 1], sacc[db][4 * i + 2], sacc[db][4 * i + 3]};
        *reinterpret_cast<float4*>(out + 8 * i) = o4;
      }
    }
  }
  if (tid < m) pcnt[((size_t)h * NP + b) * ACC_MAXM + tid] = cnt_s[tid];
}

// fp32 I/O: one point per thread, centre chunks broadcast from LDS.
template <int D>
__global__ __launch_bounds__(128) void assign_f32(const float* __restrict__ X, AssignCfg cfg,
                                                  const float* __restrict__ cent,
                                                  const float* __restrict__ bias,
                                                  int32_t* __restrict__ labels, float* __restrict__ dist2) {
  constexpr int CB = 32;
  const int h = blockIdx.y;
  int n, m, row_off;
  if (!assign_setup(cfg, h, n, m, row_off)) return;
  const int base = blockIdx.x * 128;
  if (base >= n) return;
  const int tid = threadIdx.x;
  const int p = base + tid;
  __shared__ __attribute__((aligned(16))) float cs[CB * D];
  __shared__ float bs[CB];
  float x[D];
  float xn2 = 0.f;
  if (p < n) {
    const int tok = cfg.ulist ? cfg.ulist[(size_t)h * cfg.N + p] : p;
    const float4* row = reinterpret_cast<const float4*>(X + ((size_t)h * cfg.N + tok) * D);
#pragma unroll
    for (int q = 0; q < D / 4; ++q) {
      const float4 v = row[q];
      x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
    }
#pragma unroll
    for (int j = 0; j < D; ++j) xn2 = fmaf(x[j], x[j], xn2);
  } else {
#pragma unroll
    for (int j = 0; j < D; ++j) x[j] = 0.f;
  }
  const float* ch = cent + ((size_t)h * cfg.cap + row_off) * D;
  const float* bh = bias + (size_t)h * cfg.cap + row_off;
  float best = -INFINITY; int bidx = 0;
  for (int c0 = 0; c0 < m; c0 += CB) {
    __syncthreads();
    for (int i = tid; i < CB * D / 4; i += 128) {
      const int r = i / (D / 4);
      float4 v = {0.f, 0.f, 0.f, 0.f};
      if (c0 + r < m) v = reinterpret_cast<const float4*>(ch + (size_t)c0 * D)[i];
      reinterpret_cast<float4*>(cs)[i] = v;
    }
    if (tid < CB) bs[tid] = (c0 + tid < m) ? bh[c0 + tid] : -INFINITY;
    __syncthreads();
    const int rmax = min(CB, m - c0);
    for (int r = 0; r < rmax; ++r) {
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < D / 4; ++q) {
        const float4 v = *reinterpret_cast<const float4*>(&cs[r * D + 4 * q]);
        s = fmaf(x[4 * q], v.x, s); s = fmaf(x[4 * q + 1], v.y, s);
        s = fmaf(x[4 * q + 2], v.z, s); s = fmaf(x[4 * q + 3], v.w, s);
      }
      s += bs[r];
      if (s > best) { best = s; bidx = c0 + r; }
    }
  }
  if (p < n) {
    labels[(size_t)h * cfg.N + p] = bidx;
    if (dist2) dist2[(size_t)h * cfg.N + p] = fmaxf(xn2 - 2.f * best, 0.f);
  }
}

// ------------------------------------------------------------------------------------------
// centroid update: segmented sums over the sorted order (no atomics, fixed summation order)
// ------------------------------------------------------------------------------------------
struct ReduceCfg {
  int mode;            // same meaning as AssignCfg::mode (where m and activity come from)
  int m_const; int N; int P /* upper bound of parts per head = grid.x */; int m_bound;
  const KState* st;
  int normalize;       // rows are scaled to unit length before summing (query clustering)
  int want_box;
};

__device__ __forceinline__ bool reduce_setup(const ReduceCfg& c, int h, int& m) {
  if (c.mode == 0) { m = c.m_const; return true; }
  const KState& s = c.st[h];
  if (c.mode == 1) { m = s.m_t; return s.active != 0; }
  m = s.ccount; return true;
}

// One wave sums one part of one cluster with 16-byte loads: a row is covered by LPR lanes, the
// wave takes RPI = 64/LPR rows per step (two steps in flight), and the RPI row slots are merged
// at the end in a fixed order, so the result does not depend on scheduling.
// psum [H][m_bound][P][D]; pnorm [H][m_bound][P]; pmin/pmax like psum.
static constexpr int REDUCE_ROWS = 128;   // rows summed by one wave (64, 96 and 192 measured the same)

// poff[j] = number of parts of the clusters before j (a cluster of n rows has ceil(n/REDUCE_ROWS)
// parts), j = 0..m.  One block per head.
// pcl[b] = cluster of part b (written when there are more than 128 clusters: seg_reduce then reads its
// cluster instead of searching poff, ten dependent round trips at 1024 clusters).
__global__ __launch_bounds__(1024) void part_scan(ReduceCfg cfg, const int32_t* __restrict__ offs, int offs_stride,
                                                  int32_t* __restrict__ poff, int32_t* __restrict__ pcl) {
  const int h = blockIdx.x, tid = threadIdx.x;
  int m;
  if (!reduce_setup(cfg, h, m)) return;
  const int32_t* of = offs + (size_t)h * offs_stride;
  int32_t* po = poff + (size_t)h * offs_stride;
  const int per = (m + 1023) / 1024;
  const int j0 = tid * per, j1 = min(m, j0 + per);
  int run = 0;
  for (int j = j0; j < j1; ++j) run += (of[j + 1] - of[j] + REDUCE_ROWS - 1) / REDUCE_ROWS;
  // inclusive scan over the 1024 threads: inside a wave by shuffles, across the 16 waves through LDS
  const int lane = tid & 63, wave = tid >> 6;
  int incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
  __shared__ int32_t wtot[16];
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) { const int v = wtot[w]; if (w < wave) before += v; total += v; }
  int base = before + incl - run;
  int32_t* pc = (pcl && m > 128) ? pcl + (size_t)h * cfg.P : nullptr;
  for (int j = j0; j < j1; ++j) {
    po[j] = base;
    const int np = (of[j + 1] - of[j] + REDUCE_ROWS - 1) / REDUCE_ROWS;
    if (pc) for (int q = 0; q < np && base + q < cfg.P; ++q) pc[base + q] = j;
    base += np;
  }
  if (tid == 1023) po[m] = total;
}

template <typename T> struct Vec16;
template <> struct Vec16<bf16raw> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void decode(const uint4 r, float* x) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = __uint_as_float(w[i] << 16); x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
  }
};
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void decode(const uint4 r, float* x) {
    x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y); x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
  }
};

template <typename T, int D>
__global__ __launch_bounds__(64) void seg_reduce(const T* __restrict__ X, ReduceCfg cfg,
                                                 const int32_t* __restrict__ perm,
                                                 const int32_t* __restrict__ offs, int offs_stride,
                                                 const int32_t* __restrict__ poff, const int32_t* __restrict__ pcl,
                                                 float* __restrict__ psum, float* __restrict__ pnorm,
                                                 float* __restrict__ pmin, float* __restrict__ pmax) {
  constexpr int EV = Vec16<T>::N;     // elements per 16-byte load
  constexpr int LPR = D / EV;         // lanes per row
  constexpr int RPI = 64 / LPR;       // rows per wave step
  const int h = blockIdx.y;
  int m;
  if (!reduce_setup(cfg, h, m)) return;
  // part b of this head -> (cluster j, part index): parts of REDUCE_ROWS rows, clusters in order
  const int32_t* po = poff + (size_t)h * offs_stride;
  const int32_t* of = offs + (size_t)h * offs_stride;
  const int b = blockIdx.x;
  const int lane = threadIdx.x, slot = lane / LPR, cl = lane % LPR;
  int j, part, beg, end;
  if (m <= 128) {
    // few clusters: every lane takes two entries of both tables in one round trip and the
    // cluster of this part is found by a vote (j = number of clusters that start at or before b)
    const int a0 = lane, a1 = lane + 64;
    const int p0 = a0 <= m ? po[a0] : INT32_MAX, p1 = a1 <= m ? po[a1] : INT32_MAX;
    const int o0 = a0 <= m ? of[a0] : 0, o1 = a1 <= m ? of[a1] : 0;
    const int o2 = of[m], ptotal = po[m];
    if (b >= ptotal) return;
    // entries 0..m-1 are cluster starts, entry m is the total
    const int cnt = __popcll(__ballot(a0 < m && p0 <= b)) + __popcll(__ballot(a1 < m && p1 <= b));
    j = cnt - 1;
    const int pj = j < 64 ? __shfl(p0, j) : __shfl(p1, j - 64);
    part = b - pj;
    beg = j < 64 ? __shfl(o0, j) : __shfl(o1, j - 64);
    const int jn = j + 1;
    end = jn == m ? o2 : (jn < 64 ? __shfl(o0, jn) : __shfl(o1, jn - 64));
  } else {
    if (b >= po[m]) return;
    if (pcl) {
      j = pcl[(size_t)h * cfg.P + b];
    } else {
      int lo = 0, hi = m - 1;
      while (lo < hi) { const int mid = (lo + hi + 1) >> 1; if (po[mid] <= b) lo = mid; else hi = mid - 1; }
      j = lo;
    }
    part = b - po[j];
    beg = of[j]; end = of[j + 1];
  }
  const int mb = beg + part * REDUCE_ROWS;
  const int me = min(end, mb + REDUCE_ROWS);
  const int32_t* pm = perm + (size_t)h * cfg.N;
  const T* Xh = X + (size_t)h * cfg.N * D + cl * EV;
  float acc[EV], mn[EV], mx[EV];
#pragma unroll
  for (int e = 0; e < EV; ++e) { acc[e] = 0.f; mn[e] = INFINITY; mx[e] = -INFINITY; }
  float nsum = 0.f;
  auto add_row = [&](const float* x, bool valid) {
    float xs[EV];
#pragma unroll
    for (int e = 0; e < EV; ++e) xs[e] = x[e];
    if (cfg.normalize) {
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < EV; ++e) ss = fmaf(xs[e], xs[e], ss);
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o);
      const float nrm = sqrtf(ss);
      const float inv = 1.0f / fmaxf(nrm, 1e-12f);
#pragma unroll
      for (int e = 0; e < EV; ++e) xs[e] *= inv;
      if (valid) nsum += nrm;
    }
    if (valid) {
#pragma unroll
      for (int e = 0; e < EV; ++e) {
        acc[e] += xs[e];
        if (cfg.want_box) { mn[e] = fminf(mn[e], xs[e]); mx[e] = fmaxf(mx[e], xs[e]); }
      }
    }
  };
  // The wave fetches up to 64 row indices with one coalesced load (the next 64 while the current
  // rows are summed), then keeps UNR row gathers in flight per lane: small clusters are bound by
  // the number of dependent memory round trips, not by bytes.  Every lane runs the same number of
  // steps (the shuffles in add_row need all lanes of a row present); rows past the end contribute
  // nothing.  The order in which a lane adds its rows is ascending, whatever UNR is.
  // The rows wait in registers as loaded (16 bytes, four registers each) and are decoded one by one when
  // they are added, so that sixteen gathers per lane fit where eight decoded rows did.
  constexpr int UNR = (64 / RPI) < 16 ? (64 / RPI) : 16;
  int idx_next = (mb + lane < me) ? pm[mb + lane] : 0;
  for (int r0 = mb; r0 < me; r0 += 64) {
    const int idx = idx_next;
    if (r0 + 64 < me) idx_next = (r0 + 64 + lane < me) ? pm[r0 + 64 + lane] : 0;
    const int nhere = min(64, me - r0);
    for (int k0 = 0; k0 < nhere; k0 += UNR * RPI) {
      uint4 raw[UNR];
      bool valid[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int k = k0 + u * RPI + slot;            // < 64 + RPI*UNR, but only k < nhere is used
        valid[u] = k < nhere;
        const int tok = __shfl(idx, k & 63);
        raw[u] = uint4{0u, 0u, 0u, 0u};
        if (valid[u]) raw[u] = *reinterpret_cast<const uint4*>(Xh + (size_t)tok * D);
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        float x[EV];
        Vec16<T>::decode(raw[u], x);
        add_row(x, valid[u]);
      }
    }
  }
  // merge the row slots: slot s+o into slot s, o = RPI/2 ... 1
#pragma unroll
  for (int o = RPI / 2; o >= 1; o >>= 1) {
#pragma unroll
    for (int e = 0; e < EV; ++e) {
      acc[e] += __shfl_down(acc[e], o * LPR);
      mn[e] = fminf(mn[e], __shfl_down(mn[e], o * LPR));
      mx[e] = fmaxf(mx[e], __shfl_down(mx[e], o * LPR));
    }
    nsum += __shfl_down(nsum, o * LPR);
  }
  if (slot == 0) {
    const size_t o = (size_t)h * cfg.P + b;
#pragma unroll
    for (int e = 0; e < EV; ++e) {
      psum[o * D + cl * EV + e] = acc[e];
      if (cfg.want_box) { pmin[o * D + cl * EV + e] = mn[e]; pmax[o * D + cl * EV + e] = mx[e]; }
    }
    if (cfg.normalize && cl == 0) pnorm[o] = nsum;
  }
}

// Combine the parts and write centres.
//   update_assign = 1 (Lloyd step): non-empty clusters get master := mean (or unit mean), the
//     I/O-dtype copy used by the next assignment, its fp32 image and the arg-max bias.
//   update_assign = 0 (final): out_cent := mean / unit mean (empty: `fallback` row), sizes, mean
//     norms, boxes.  `master` is also refreshed when given (query clustering returns it).
struct FinalizeCfg {
  int mode; int m_const; int P; int m_bound; int cap; int master_stride;
  const KState* st;
  int spherical; int update_assign; int lp_is_bf16; int want_box;
  const int32_t* bcnt; int nb_stride;     // block sums of the assignment kernel instead of cluster parts (stage mode)
  int nb_const;                           // > 0: that many blocks (walks of the one-read query pass), whatever the state says
};

constexpr int FIN_ROWS = 4;           // clusters per workgroup, one wave each (no step needs the workgroup)
template <int D>
__global__ __launch_bounds__(64 * FIN_ROWS) void finalize_centroids(FinalizeCfg cfg, const int32_t* __restrict__ offs,
                                                         int offs_stride, const int32_t* __restrict__ poff,
                                                         const float* __restrict__ psum,
                                                         const float* __restrict__ pnorm,
                                                         const float* __restrict__ pmin,
                                                         const float* __restrict__ pmax,
                                                         float* __restrict__ master, void* __restrict__ assign_lp,
                                                         float* __restrict__ assign_f32, float* __restrict__ bias,
                                                         float* __restrict__ out_cent, const float* __restrict__ fallback,
                                                         int32_t* __restrict__ out_sizes, float* __restrict__ out_mean_norm,
                                                         float* __restrict__ out_bmin, float* __restrict__ out_bmax) {
  constexpr int CPL = D / 64;          // columns per lane
  const int h = blockIdx.y, j = blockIdx.x * FIN_ROWS + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  int m, row_off = 0;
  if (cfg.mode == 0) m = cfg.m_const;
  else {
    const KState& s = cfg.st[h];
    if (cfg.mode == 1) { if (!s.active) return; m = s.m_t; row_off = s.ccount; }
    else m = s.ccount;
  }
  if (j >= m) {
    if (!cfg.update_assign && out_sizes && j < cfg.cap) out_sizes[(size_t)h * cfg.cap + j] = 0;
    return;
  }
  int nj, p_beg, p_end;
  if (cfg.bcnt) {
    // the blocks of 256 points of the assignment kernel, in block order
    const int nb = cfg.nb_const > 0 ? cfg.nb_const : (cfg.st[h].ucount + 255) >> 8;
    nj = 0;
    for (int b = lane; b < nb; b += 64) nj += cfg.bcnt[((size_t)h * cfg.nb_stride + b) * ACC_MAXM + j];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) nj += __shfl_xor(nj, o);
    p_beg = j * cfg.nb_stride; p_end = p_beg + nb;
  } else {
    nj = offs[(size_t)h * offs_stride + j + 1] - offs[(size_t)h * offs_stride + j];
    p_beg = poff[(size_t)h * offs_stride + j]; p_end = poff[(size_t)h * offs_stride + j + 1];
  }
  const size_t pbase = (size_t)h * cfg.P;
  float s[CPL], mn[CPL], mx[CPL];
#pragma unroll
  for (int q = 0; q < CPL; ++q) { s[q] = 0.f; mn[q] = INFINITY; mx[q] = -INFINITY; }
  float ns = 0.f;
  int p = p_beg;
  if (!cfg.want_box && (!cfg.spherical || cfg.update_assign)) {
    // sums only: eight parts' loads in flight, added in part order all the same
    for (; p + 8 <= p_end; p += 8) {
      float t[8][CPL];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int q = 0; q < CPL; ++q) t[u][q] = psum[(pbase + p + u) * D + lane + 64 * q];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int q = 0; q < CPL; ++q) s[q] += t[u][q];
    }
  }
  for (; p < p_end; ++p) {
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
      s[q] += psum[(pbase + p) * D + lane + 64 * q];
      if (cfg.want_box) {
        mn[q] = fminf(mn[q], pmin[(pbase + p) * D + lane + 64 * q]);
        mx[q] = fmaxf(mx[q], pmax[(pbase + p) * D + lane + 64 * q]);
      }
    }
    if (cfg.spherical && !cfg.update_assign) ns += pnorm[pbase + p];     // (member norms matter to the final outputs only)
  }
  bool ok = nj > 0;
  float val[CPL];
  if (cfg.spherical) {
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < CPL; ++q) ss = fmaf(s[q], s[q], ss);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) ss += __shfl_xor(ss, o);
    const float nrm = sqrtf(ss);
    ok = ok && (nrm >= 1e-12f);
#pragma unroll
    for (int q = 0; q < CPL; ++q) val[q] = s[q] / fmaxf(nrm, 1e-30f);
  } else {
#pragma unroll
    for (int q = 0; q < CPL; ++q) val[q] = s[q] / (float)max(nj, 1);
  }
  if (cfg.update_assign) {
    if (!ok) return;
    float bsum = 0.f;
#pragma unroll
    for (int q = 0; q < CPL; ++q) {
      const int col = lane + 64 * q;
      master[((size_t)h * cfg.master_stride + j) * D + col] = val[q];
      const size_t ao = ((size_t)h * cfg.cap + row_off + j) * D + col;
      float img = val[q];
      if (cfg.lp_is_bf16) {
        const bf16raw r = f32_to_bf16(val[q]);
        reinterpret_cast<bf16raw*>(assign_lp)[ao] = r;
        img = bf16_to_f32(r);
      } else {
        reinterpret_cast<float*>(assign_lp)[ao] = img;
      }
      assign_f32[ao] = img;
      bsum = fmaf(img, img, bsum);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) bsum += __shfl_xor(bsum, o);
    if (lane == 0) bias[(size_t)h * cfg.cap + row_off + j] = cfg.spherical ? 0.f : -0.5f * bsum;
    return;
  }
  // final outputs
#pragma unroll
  for (int q = 0; q < CPL; ++q) {
    const int col = lane + 64 * q;
    const size_t oo = ((size_t)h * cfg.cap + j) * D + col;
    if (ok) {
      out_cent[oo] = val[q];
    } else if (fallback) {
      out_cent[oo] = fallback[oo];
    }
    if (cfg.want_box) {
      out_bmin[oo] = nj > 0 ? mn[q] : 0.f;
      out_bmax[oo] = nj > 0 ? mx[q] : 0.f;
    }
  }
  if (lane == 0) {
    if (out_sizes) out_sizes[(size_t)h * cfg.cap + j] = nj;
    // mean member norm, the factor that brings unit-centroid scores back to logits; 1 for raw centroids
    if (out_mean_norm) out_mean_norm[(size_t)h * cfg.cap + j] = nj > 0 ? (cfg.spherical ? ns / (float)nj : 1.f) : 0.f;
  }
}

// ------------------------------------------------------------------------------------------
// Centroid update of a stage with few points in ONE launch (fp32 inputs): the workgroup of a centre finds
// its members in the label list itself (an ordered compaction, so the member order is the list order),
// sums their rows in a fixed order and writes the new centre, its copies for the assignment kernel and
// the arg-max bias.  It stands for the label sort, the segmented reduction and the combining kernel,
// three launches that are each bound by latency at a few thousand points.
// ------------------------------------------------------------------------------------------
constexpr int DIRECT_ROUND = 4096;          // list positions scanned per round: 1024 per wave, 16 per lane
constexpr long long DIRECT_MAX_VISITS = 1 << 21;
constexpr int DIRECT_MAX_POINTS = 4 * DIRECT_ROUND;  // a workgroup scans the list alone: at most four rounds   // centres x points up to which every centre scans the whole list

template <int D>
__global__ __launch_bounds__(256) void update_direct_f32(const float* __restrict__ X, int N, int cap, int master_stride,
                                                         const KState* __restrict__ st,
                                                         const int32_t* __restrict__ labels,
                                                         const int32_t* __restrict__ ulist,
                                                         float* __restrict__ master, float* __restrict__ assign_lp,
                                                         float* __restrict__ assign_f32, float* __restrict__ bias) {
  constexpr int LPR = D / 4, G = 256 / LPR;   // lanes per row (16 bytes each), rows in flight per step
  const int h = blockIdx.y, j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const KState& s = st[h];
  if (!s.active) return;
  const int n = s.ucount, m = s.m_t, row_off = s.ccount;
  if (j >= m) return;
  __shared__ int32_t list[DIRECT_ROUND];
  __shared__ int32_t wcnt[4];
  __shared__ float4 red[256];
  const int32_t* lab = labels + (size_t)h * N;
  const int32_t* ul = ulist ? ulist + (size_t)h * N : nullptr;
  const float* Xh = X + (size_t)h * N * D;
  const int g = tid / LPR, cl = tid % LPR;
  const uint64_t below = (1ull << lane) - 1ull;
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  int total = 0;
  for (int r0 = 0; r0 < n; r0 += DIRECT_ROUND) {
    // wave w scans positions r0 + 1024 w ... in 16 steps of 64; members keep their list order
    int tok[16];
    uint32_t hit = 0;
    int mine = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int pos = r0 + wave * 1024 + i * 64 + lane;
      const bool in = pos < n;
      const int l = in ? lab[pos] : -1;
      tok[i] = in ? (ul ? ul[pos] : pos) : 0;
      if (l == j) hit |= 1u << i;
    }
    int woff[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint64_t b = __ballot((hit >> i) & 1u);
      woff[i] = mine + __popcll(b & below);
      mine += __popcll(b);
    }
    __syncthreads();                 // the list of the round before has been summed
    if (lane == 0) wcnt[wave] = mine;
    __syncthreads();
    int base = 0, cnt = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) { const int c = wcnt[w]; if (w < wave) base += c; cnt += c; }
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if ((hit >> i) & 1u) list[base + woff[i]] = tok[i];
    __syncthreads();
    // row i of the round goes to row group i % G; a group adds its rows in ascending order
    for (int i0 = g; i0 < cnt; i0 += 4 * G) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * G;
        v[u] = float4{0.f, 0.f, 0.f, 0.f};
        if (i < cnt) v[u] = *reinterpret_cast<const float4*>(Xh + (size_t)list[i] * D + cl * 4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    total += cnt;
  }
  if (total == 0) return;            // an empty cluster keeps its centre
  red[tid] = acc;
  __syncthreads();
  if (tid >= LPR) return;
  float4 sum = red[cl];
#pragma unroll
  for (int q = 1; q < G; ++q) {
    const float4 t = red[q * LPR + cl];
    sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
  }
  const float cntf = (float)total;
  const float4 val = {sum.x / cntf, sum.y / cntf, sum.z / cntf, sum.w / cntf};
  *reinterpret_cast<float4*>(master + ((size_t)h * master_stride + j) * D + cl * 4) = val;
  const size_t ao = ((size_t)h * cap + row_off + j) * D + cl * 4;
  *reinterpret_cast<float4*>(assign_lp + ao) = val;
  *reinterpret_cast<float4*>(assign_f32 + ao) = val;
  float bsum = fmaf(val.x, val.x, 0.f);
  bsum = fmaf(val.y, val.y, bsum); bsum = fmaf(val.z, val.z, bsum); bsum = fmaf(val.w, val.w, bsum);
#pragma unroll
  for (int o = 1; o < LPR; o <<= 1) bsum += __shfl_xor(bsum, o);
  if (cl == 0) bias[(size_t)h * cap + row_off + j] = -0.5f * bsum;
}

// Initial centres: strided sample of the current point list (or the rows of `master` as given).
//   source_master = 1: master already holds the centres (warm start)
template <typename T, int D>
__global__ __launch_bounds__(64) void init_centroids(const T* __restrict__ X, int N, int mode, int m_const,
                                                     const KState* __restrict__ st,
                                                     const int32_t* __restrict__ ulist, int spherical,
                                                     int source_master, int cap, int master_stride,
                                                     int lp_is_bf16, float* __restrict__ master,
                                                     void* __restrict__ assign_lp, float* __restrict__ assign_f32,
                                                     float* __restrict__ bias) {
  constexpr int CPL = D / 64;
  const int h = blockIdx.y, j = blockIdx.x, lane = threadIdx.x;
  int n = N, m = m_const, row_off = 0;
  if (mode == 1) {
    const KState& s = st[h];
    if (!s.active) return;
    n = s.ucount; m = s.m_t; row_off = s.ccount;
  }
  if (j >= m) return;
  float val[CPL];
  if (source_master) {
#pragma unroll
    for (int q = 0; q < CPL; ++q) val[q] = master[((size_t)h * master_stride + j) * D + lane + 64 * q];
  } else {
    const long long pos = ((2ll * j + 1) * (long long)n) / (2ll * m);
    const int tok = ulist ? ulist[(size_t)h * N + pos] : (int)pos;
    const T* row = X + ((size_t)h * N + tok) * D;
#pragma unroll
    for (int q = 0; q < CPL; ++q) val[q] = Elem<T>::load(row + lane + 64 * q);
    if (spherical) {
      float ss = 0.f;
#pragma unroll
      for (int q = 0; q < CPL; ++q) ss = fmaf(val[q], val[q], ss);
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) ss += __shfl_xor(ss, o);
      const float inv = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
#pragma unroll
      for (int q = 0; q < CPL; ++q) val[q] *= inv;
    }
  }
  float bsum = 0.f;
#pragma unroll
  for (int q = 0; q < CPL; ++q) {
    const int col = lane + 64 * q;
    master[((size_t)h * master_stride + j) * D + col] = val[q];
    const size_t ao = ((size_t)h * cap + row_off + j) * D + col;
    float img = val[q];
    if (lp_is_bf16) {
      const bf16raw r = f32_to_bf16(val[q]);
      reinterpret_cast<bf16raw*>(assign_lp)[ao] = r;
      img = bf16_to_f32(r);
    } else {
      reinterpret_cast<float*>(assign_lp)[ao] = img;
    }
    assign_f32[ao] = img;
    bsum = fmaf(img, img, bsum);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) bsum += __shfl_xor(bsum, o);
  if (lane == 0) bias[(size_t)h * cap + row_off + j] = spherical ? 0.f : -0.5f * bsum;
}

// ------------------------------------------------------------------------------------------
// Algorithm 1 bookkeeping
// ------------------------------------------------------------------------------------------
__global__ void kstate_init(KState* st, int H, int N) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= H) return;
  KState s;
  s.ucount = N; s.ccount = 0; s.m_t = 0; s.stage = 0; s.done = 0; s.full = 0; s.active = 0; s.pad = 0;
  for (int i = 0; i <= ADACLUSTER_MAX_STAGES; ++i) { s.stage_offs[i] = 0; s.u_hist[i] = 0; }
  s.u_hist[0] = N;
  st[h] = s;
}

// Warm start (Sec. 3.2.2, "Efficient initialization"): one stage over all tokens, centre count given.
__global__ void kstate_warm(KState* st, int H, int N, int cap, const int32_t* __restrict__ k_count,
                            const int32_t* __restrict__ full_flag) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= H) return;
  KState s;
  s.ucount = N; s.ccount = 0; s.m_t = max(1, min(min(k_count[h], cap), N)); s.stage = 0; s.done = 0;
  s.full = full_flag[h] != 0; s.active = 1; s.pad = 0;
  for (int i = 0; i <= ADACLUSTER_MAX_STAGES; ++i) { s.stage_offs[i] = 0; s.u_hist[i] = 0; }
  s.u_hist[0] = N;
  st[h] = s;
}
__global__ void kstate_commit(KState* st, int H) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= H) return;
  KState s = st[h];
  s.ccount = s.m_t; s.stage = 1; s.stage_offs[1] = s.ccount; s.ucount = 0; s.active = 0; s.done = 1;
  st[h] = s;
}

// Head of the while-loop of Algorithm 1: U empty? |C| >= N_max (flag F)?  stage / leftover limits?
// then the centre count m_t of the next stage.  summary = {active heads, max |U|, max m_t}.
__global__ void kstage_begin(KState* st, int H, int N, int n_max, int m0, int m_min, int max_stages,
                             int u_min, int32_t* summary) {
  __shared__ int32_t s_act, s_u, s_m;
  if (threadIdx.x == 0) { s_act = 0; s_u = 0; s_m = 0; }
  __syncthreads();
  for (int h = threadIdx.x; h < H; h += blockDim.x) {
    KState s = st[h];
    if (!s.done) {
      if (s.ucount == 0) s.done = 1;
      else if (s.ccount >= n_max) { s.full = 1; s.done = 1; }
      else if (s.stage >= max_stages || s.ucount <= u_min) s.done = 1;
    }
    s.active = !s.done;
    if (s.active) {
      long long mm = ((long long)m0 * s.ucount + N - 1) / N;
      int m = (int)mm;
      m = max(m_min, min(m0, m));
      m = min(m, s.ucount);
      s.m_t = m;
      atomicAdd(&s_act, 1); atomicMax(&s_u, s.ucount); atomicMax(&s_m, m);
    } else {
      s.m_t = 0;
    }
    st[h] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) { summary[0] = s_act; summary[1] = s_u; summary[2] = s_m; }
}

// tau = factor x mean first-stage distance over all heads and tokens (Sec. 4.1).
__global__ __launch_bounds__(256) void tau_partial(const float* __restrict__ dist2, int N, int nblk,
                                                   double* __restrict__ part) {
  const int h = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
  double s = 0.0;
  const int beg = b * 1024;
  for (int i = 0; i < 4; ++i) {
    const int p = beg + i * 256 + tid;
    if (p < N) s += (double)sqrtf(dist2[(size_t)h * N + p]);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) s += __shfl_xor(s, o);
  __shared__ double ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) part[(size_t)h * nblk + b] = (ws[0] + ws[1]) + (ws[2] + ws[3]);
}

__global__ __launch_bounds__(256) void tau_final(const double* __restrict__ part, int count, double denom, float factor,
                                                 float* __restrict__ tau_out /* [0]=tau, [1]=tau^2 */) {
  // fixed-order reduction: thread i takes elements i, i+256, ...; then a fixed tree
  const int tid = threadIdx.x;
  double s = 0.0;
  for (int i = tid; i < count; i += 256) s += part[i];
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) s += __shfl_xor(s, o);
  __shared__ double ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    const double tot = (ws[0] + ws[1]) + (ws[2] + ws[3]);
    const double tau = (double)factor * tot / denom;
    tau_out[0] = (float)tau;
    tau_out[1] = (float)tau * (float)tau;
  }
}

__global__ void tau_set(float tau, float* __restrict__ tau_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { tau_out[0] = tau; tau_out[1] = tau * tau; }
}

// threshold filter of Algorithm 1: tokens with d < tau leave U.  Three passes keep U ascending.
__global__ __launch_bounds__(256) void filter_count(const KState* __restrict__ st, const float* __restrict__ dist2,
                                                    int N, int nblk, const float* __restrict__ tau,
                                                    int32_t* __restrict__ blockcnt) {
  const int h = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
  const KState& s = st[h];
  if (!s.active) return;
  const int n = s.ucount;
  const float t2 = tau[1];
  int c = 0;
  for (int i = 0; i < 4; ++i) {
    const int p = b * 1024 + i * 256 + tid;
    if (p < n && !(dist2[(size_t)h * N + p] < t2)) ++c;
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) c += __shfl_xor(c, o);
  __shared__ int32_t ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = c;
  __syncthreads();
  if (tid == 0) blockcnt[(size_t)h * nblk + b] = ws[0] + ws[1] + ws[2] + ws[3];
}

__global__ __launch_bounds__(64) void filter_scan(KState* __restrict__ st, int nblk_used, int nblk,
                                                  int32_t* __restrict__ blockcnt, int32_t* __restrict__ u_prev) {
  // one wave per head: a lane takes a run of consecutive blocks, the runs are chained by a wave scan
  const int h = blockIdx.x, lane = threadIdx.x;
  KState s = st[h];
  if (!s.active) return;
  const int nb = min((s.ucount + 1023) / 1024, nblk_used);
  const int per = (nb + 63) / 64;
  const int b0 = min(lane * per, nb), b1 = min(b0 + per, nb);
  int32_t* bc = blockcnt + (size_t)h * nblk;
  int mine = 0;
  for (int b = b0; b < b1; ++b) mine += bc[b];
  int incl = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
  const int total = __shfl(incl, 63);
  int run = incl - mine;
  for (int b = b0; b < b1; ++b) { const int c = bc[b]; bc[b] = run; run += c; }
  if (lane != 0) return;
  u_prev[h] = s.ucount;
  s.ucount = total;
  s.ccount += s.m_t;
  s.stage += 1;
  s.stage_offs[s.stage] = s.ccount;
  s.u_hist[s.stage] = total;
  st[h] = s;
}

__global__ __launch_bounds__(256) void filter_scatter(const KState* __restrict__ st, const int32_t* __restrict__ u_prev,
                                                      const float* __restrict__ dist2, int N, int nblk,
                                                      const float* __restrict__ tau,
                                                      const int32_t* __restrict__ blockbase,
                                                      const int32_t* __restrict__ ulist_in,
                                                      int32_t* __restrict__ ulist_out,
                                                      int32_t* __restrict__ stage_of, int stage) {
  const int h = blockIdx.y, b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const KState& s = st[h];
  if (!s.active) return;
  const int n = u_prev[h];
  if (b * 1024 >= n) return;
  const float t2 = tau[1];
  int run = blockbase[(size_t)h * nblk + b];
  __shared__ int32_t ws[4];
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int i = 0; i < 4; ++i) {
    const int p = b * 1024 + i * 256 + tid;
    const bool valid = p < n;
    const bool keep = valid && !(dist2[(size_t)h * N + p] < t2);
    const int tok = valid ? (ulist_in ? ulist_in[(size_t)h * N + p] : p) : 0;
    const uint64_t bal = __ballot(keep);
    __syncthreads();
    if (lane == 0) ws[wave] = __popcll(bal);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += ws[w];
    const int total = ws[0] + ws[1] + ws[2] + ws[3];
    if (keep) ulist_out[(size_t)h * N + run + before + __popcll(bal & lt_mask)] = tok;
    if (valid && !keep && stage_of) stage_of[(size_t)h * N + tok] = stage;
    run += total;
  }
}

// The three filter passes in one workgroup per head, for heads whose |U| is small.  A thread takes
// four consecutive items per step (4096 per workgroup step), so most heads need one step.
__global__ __launch_bounds__(1024) void filter_small(KState* __restrict__ st, const float* __restrict__ dist2, int N,
                                                     const float* __restrict__ tau,
                                                     const int32_t* __restrict__ ulist_in,
                                                     int32_t* __restrict__ ulist_out, int32_t* __restrict__ stage_of,
                                                     int stage) {
  const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const KState s0 = st[h];
  if (!s0.active) return;
  const int n = min(s0.ucount, N);
  const float t2 = tau[1];
  __shared__ int32_t ws[16];
  const float* dh = dist2 + (size_t)h * N;
  const int32_t* uin = ulist_in ? ulist_in + (size_t)h * N : nullptr;
  int32_t* uout = ulist_out + (size_t)h * N;
  int32_t* sof = stage_of ? stage_of + (size_t)h * N : nullptr;
  int run = 0;
  for (int base = 0; base < n; base += 4096) {
    const int p0 = base + 4 * tid;
    bool keep[4]; int tok[4]; int c = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = p0 + i;
      const bool valid = p < n;
      keep[i] = valid && !(dh[p < n ? p : 0] < t2);
      tok[i] = valid ? (uin ? uin[p] : p) : -1;
      c += keep[i] ? 1 : 0;
    }
    // exclusive prefix of the per-thread counts: inside the wave by shuffles, across waves through LDS
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
    __syncthreads();
    if (lane == 63) ws[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
    for (int w = 0; w < 16; ++w) { const int v = ws[w]; if (w < wave) before += v; total += v; }
    int pos = run + before + incl - c;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (keep[i]) uout[pos++] = tok[i];
      else if (tok[i] >= 0 && sof) sof[tok[i]] = stage;
    }
    run += total;
  }
  __syncthreads();      // every thread has taken its copy of the state
  if (tid == 0) {
    KState s = s0;
    s.ucount = run;
    s.ccount += s.m_t;
    s.stage += 1;
    s.stage_offs[s.stage] = s.ccount;
    s.u_hist[s.stage] = run;
    st[h] = s;
  }
}

// ------------------------------------------------------------------------------------------
// The late stages of Algorithm 1 in one launch.
// ------------------------------------------------------------------------------------------
// Once every head has few unassigned points left (|U| <= SMALL_NU) and at most SMALL_M centres per
// stage, a stage is eight launches of a few microseconds each with next to no work in them, and
// Algorithm 1 may run ten such stages.  Heads are independent, so here ONE workgroup per head runs
// every remaining stage from the loop head to the threshold filter: strided initial sample, `iters`
// assignment passes with the centre update in between, filter and compaction of U, stage
// bookkeeping - the same arithmetic as the separate kernels (same scores, same arg-max, same
// distance, same centre rounding), with the centres, their bias and the member counts in LDS.
//   assignment: as assign_mfma, D[32 centres x 32 points]; a wave takes every NW-th tile of 32 points and
//               runs free of the other waves, with the rows of its next tile in flight;
//   update:     the wave stages its 32 points in LDS and adds S^T[32 dims x 32 centres] += X^T E for
//               them, E the one-hot labels (see assign_mfma<D, true>), into accumulators it keeps for
//               the whole pass; the waves' partial sums are then added in a fixed order, so the result
//               is deterministic;
//   filter:     squared distances of the last pass stay in LDS; U is compacted in ascending order.
constexpr int SMALL_NU = 8192;
constexpr int SMALL_M = 32;

struct SmallStageCfg {
  int N, cap, n_max, m0, m_min, max_stages, u_min, iters;
  const float* tau;               // [1] = tau^2
  int32_t* ulist[2];              // U of stage t is ulist[t & 1]
  bf16raw* cent_lp; float* assign_f32; float* bias;
  int32_t* stage_of;              // may be NULL
};

template <int D> struct SmallStage { static constexpr int NW = D == 64 ? 16 : 8; };   // waves (register budget 128 / 256)

template <int D>
__global__ __launch_bounds__(SmallStage<D>::NW * 64) void kstages_small(const bf16raw* __restrict__ X, KState* __restrict__ st,
                                                                       SmallStageCfg cfg) {
  constexpr int LDW = D + 8, KS = D / 16, DT = D / 32, CPL = D / 64;
  constexpr int NW = SmallStage<D>::NW, NT = NW * 64;
  constexpr int SROWB = D * 2 + 16;                  // staged row, padded: the 16-byte pieces of 8 rows fall in 8 bank groups
  constexpr int JPW = SMALL_M / NW;                  // centres a wave finalises
  const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hb = lane >> 5;
  // a wave's staged tile, row-major; between the tile loop and the next pass the partial centre sums of
  // GW waves at a time (rows padded by four floats: the float4 pieces of 8 centres fall in 8 bank groups)
  constexpr int GW = D == 64 ? 8 : 4, PROW = D + 4;
  __shared__ __attribute__((aligned(16))) char xs[NW][32 * SROWB];
  static_assert(sizeof(float) * GW * SMALL_M * PROW <= sizeof(char) * NW * 32 * SROWB, "the partial sums reuse the staging area");
  float* ps = reinterpret_cast<float*>(&xs[0][0]);
  __shared__ __attribute__((aligned(16))) int32_t lab_s[NW][32];
  __shared__ __attribute__((aligned(16))) float fs[SMALL_NU];       // squared distances of the last pass
  __shared__ __attribute__((aligned(16))) bf16raw cs[SMALL_M * LDW];
  __shared__ __attribute__((aligned(16))) float bs[SMALL_M];
  __shared__ int32_t cnt_s[SMALL_M];
  __shared__ int32_t ws[NW];
  __shared__ KState s_st;
  if (tid == 0) s_st = st[h];
  __syncthreads();
  if (!s_st.active) return;                 // the stage head that ran before this launch closed the head
  const float t2 = cfg.tau[1];
  // transpose-read addressing of the X^T operand (see assign_mfma<D, true>)
  const int i16 = lane & 15;
  const int vrow = 4 * hb + (i16 >> 2);
  const int gl = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);
  const char* xw = xs[wave] + vrow * SROWB + gl * 16 + 8 * (i16 & 1);

  for (bool first = true;; first = false) {
    if (!first) {
      // head of the while-loop of Algorithm 1 (as kstage_begin)
      if (tid == 0) {
        KState s = s_st;
        if (s.ucount == 0) s.done = 1;
        else if (s.ccount >= cfg.n_max) { s.full = 1; s.done = 1; }
        else if (s.stage >= cfg.max_stages || s.ucount <= cfg.u_min) s.done = 1;
        s.active = !s.done;
        if (s.active) {
          int m = (int)(((long long)cfg.m0 * s.ucount + cfg.N - 1) / cfg.N);
          m = max(cfg.m_min, min(cfg.m0, m));
          s.m_t = min(m, s.ucount);
        } else {
          s.m_t = 0;
        }
        s_st = s;
      }
      __syncthreads();
    }
    if (!s_st.active) break;
    const int n = min(s_st.ucount, SMALL_NU), m = min(s_st.m_t, SMALL_M), row_off = s_st.ccount, stage = s_st.stage;
    const int32_t* uin = cfg.ulist[stage & 1] + (size_t)h * cfg.N;
    int32_t* uout = cfg.ulist[(stage + 1) & 1] + (size_t)h * cfg.N;
    const bf16raw* Xh = X + (size_t)h * cfg.N * D;

    // initial centres: strided sample of U (as init_centroids); rows past m are zero with a bias that never wins
    if (tid < SMALL_M) cnt_s[tid] = 0;
    for (int j = wave; j < SMALL_M; j += NW) {
      if (j < m) {
        const long long pos = ((2ll * j + 1) * (long long)n) / (2ll * m);
        const int tok = uin[pos];
        const bf16raw* row = Xh + (size_t)tok * D;
        float bsum = 0.f;
#pragma unroll
        for (int q = 0; q < CPL; ++q) {
          const int col = lane + 64 * q;
          const bf16raw r = row[col];
          const float img = bf16_to_f32(r);
          cs[j * LDW + col] = r;
          const size_t ao = ((size_t)h * cfg.cap + row_off + j) * D + col;
          cfg.cent_lp[ao] = r;          // an empty cluster keeps this centre to the end of the stage
          cfg.assign_f32[ao] = img;
          bsum = fmaf(img, img, bsum);
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) bsum += __shfl_xor(bsum, o);
        if (lane == 0) { bs[j] = -0.5f * bsum; cfg.bias[(size_t)h * cfg.cap + row_off + j] = -0.5f * bsum; }
      } else {
#pragma unroll
        for (int q = 0; q < CPL; ++q) cs[j * LDW + lane + 64 * q] = 0;
        if (lane == 0) bs[j] = -3.0e38f;
      }
    }
    __syncthreads();

    const int ntiles = (n + 31) >> 5;
    // Rows of a tile: every lane loads its 16-byte pieces of point c.  Both loads are unconditional
    // (positions past the end are clamped to the last point, whose result is then ignored): a load
    // under a branch would make every later wait a wait for all loads in flight.
    auto load_tok = [&](int tile) { return uin[min(tile * 32 + c, n - 1)]; };
    auto load_rows = [&](int tok, bf16x8_t (&x)[KS]) {
      const bf16raw* row = Xh + (size_t)tok * D + hb * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 raw = *reinterpret_cast<const uint4*>(row + ks * 16);
        x[ks] = *reinterpret_cast<const bf16x8_t*>(&raw);
      }
    };

    for (int it = 0; it < cfg.iters; ++it) {
      const bool update = it < cfg.iters - 1;
      f32x16_t sacc[DT];
#pragma unroll
      for (int b = 0; b < DT; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[b][v] = 0.f;
      // One tile of 32 points: scores, arg-max, and in an update pass the tile's share of the centre sums.
      auto process = [&](int tile, const bf16x8_t (&x)[KS]) {
        const int p = tile * 32 + c;
        const bool valid = p < n;
        // scores against every centre, arg-max (as assign_mfma)
        f32x16_t acc;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 b4 = *reinterpret_cast<const float4*>(&bs[8 * i + 4 * hb]);
          acc[4 * i + 0] = b4.x; acc[4 * i + 1] = b4.y; acc[4 * i + 2] = b4.z; acc[4 * i + 3] = b4.w;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&cs[c * LDW + ks * 16 + hb * 8]);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, x[ks], acc, 0, 0, 0);
        }
        float pk[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) pk[v] = __uint_as_float((__float_as_uint(acc[v]) & 0xFFFFFFF0u) | (uint32_t)(15 - v));
        float best = fmaxf(fmaxf(pk[0], pk[1]), pk[2]);
#pragma unroll
        for (int v = 3; v < 15; v += 2) best = fmaxf(fmaxf(best, pk[v]), pk[v + 1]);
        best = fmaxf(best, pk[15]);
        const int v = 15 - (int)(__float_as_uint(best) & 15u);
        int bidx = 8 * (v >> 2) + 4 * hb + (v & 3);
        float bv = __uint_as_float(__float_as_uint(best) & 0xFFFFFFF0u);
        {
          const float ob = __shfl_xor(bv, 32);
          const int oi = __shfl_xor(bidx, 32);
          if (ob > bv || (ob == bv && oi < bidx)) { bv = ob; bidx = oi; }
        }
        if (!update) {
          // last pass: squared distance to the chosen centre, kept for the filter
          float ss = 0.f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const uint4 raw = *reinterpret_cast<const uint4*>(&x[ks]);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float a = __uint_as_float(w[q] << 16), b = __uint_as_float(w[q] & 0xFFFF0000u);
              ss = fmaf(a, a, ss); ss = fmaf(b, b, ss);
            }
          }
          const float xn2 = ss + __shfl_xor(ss, 32);
          if (hb == 0 && valid) fs[p] = fmaxf(xn2 - 2.f * bv, 0.f);
        } else {
          // update pass: stage the tile (this wave's own LDS, read back by this wave only), count the
          // members, add the tile's share of the centre sums
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<bf16x8_t*>(xs[wave] + c * SROWB + (ks * 16 + hb * 8) * 2) = x[ks];
          if (hb == 0) {
            lab_s[wave][c] = valid ? bidx : -1;
            if (valid) atomicAdd(&cnt_s[bidx], 1);
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
          for (int g = 0; g < 2; ++g) {
            const int4 l0 = *reinterpret_cast<const int4*>(&lab_s[wave][g * 16 + 4 * hb]);
            const int4 l1 = *reinterpret_cast<const int4*>(&lab_s[wave][g * 16 + 8 + 4 * hb]);
            uint4 e;
            e.x = (l0.x == c ? 0x3F80u : 0u) | (l0.y == c ? 0x3F800000u : 0u);
            e.y = (l0.z == c ? 0x3F80u : 0u) | (l0.w == c ? 0x3F800000u : 0u);
            e.z = (l1.x == c ? 0x3F80u : 0u) | (l1.y == c ? 0x3F800000u : 0u);
            e.w = (l1.z == c ? 0x3F80u : 0u) | (l1.w == c ? 0x3F800000u : 0u);
#pragma unroll
            for (int db = 0; db < DT; ++db) {
              const char* xp = xw + g * 16 * SROWB + db * 64;
              const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)xp);
              const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(xp + 8 * SROWB));
              const s16x4_t both[2] = {lo, hi};
              sacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(both),
                                                                 *reinterpret_cast<const bf16x8_t*>(&e), sacc[db], 0, 0, 0);
            }
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();      // the next tile overwrites the staged rows
        }
      };
      if constexpr (NW == 16) {
        // Four waves per SIMD hide the latency of the row loads between them, and 128 registers do not
        // hold a second row buffer: only the token ids run one tile ahead.
        bf16x8_t x0[KS];
        int tk = load_tok(wave);
        for (int tile = wave; tile < ntiles; tile += NW) {
          const int tkn = load_tok(tile + NW);
          load_rows(tk, x0);
          process(tile, x0);
          tk = tkn;
        }
      } else {
        // Software pipeline over this wave's tiles, unrolled twice so that the two row buffers keep
        // their names (a rotating copy would wait for the newest load): rows one tile ahead, token
        // ids two ahead, each token load issued before the row loads of its step.
        bf16x8_t x0[KS], x1[KS];
        int tk = load_tok(wave + NW);
        load_rows(load_tok(wave), x0);
        for (int tile = wave; tile < ntiles; tile += 2 * NW) {
          const int tkn = load_tok(tile + 2 * NW);
          load_rows(tk, x1);
          process(tile, x0);
          if (tile + NW >= ntiles) break;
          tk = load_tok(tile + 3 * NW);
          load_rows(tkn, x0);
          process(tile + NW, x1);
        }
      }
      if (!update) break;
      // The waves' partial sums, GW at a time through LDS, added in wave order by the thread that
      // finalises the element: wave w owns centres w, w+NW, ..., a lane the columns lane, lane+64.
      float tot[JPW][CPL];
#pragma unroll
      for (int a = 0; a < JPW; ++a)
#pragma unroll
        for (int q = 0; q < CPL; ++q) tot[a][q] = 0.f;
#pragma unroll
      for (int grp = 0; grp < NW / GW; ++grp) {
        __syncthreads();                     // the area is free (first group: every wave is out of its tile loop)
        if (wave / GW == grp) {
          // value v of tile db is dim db*32 + 8*(v/4) + 4*hb + v%4 of centre c
#pragma unroll
          for (int db = 0; db < DT; ++db) {
            float* out = ps + ((size_t)((wave % GW) * SMALL_M + c)) * PROW + db * 32 + 4 * hb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float4 o4 = {sacc[db][4 * i], sacc[db][4 * i + 1], sacc[db][4 * i + 2], sacc[db][4 * i + 3]};
              *reinterpret_cast<float4*>(out + 8 * i) = o4;
            }
          }
        }
        __syncthreads();
#pragma unroll
        for (int a = 0; a < JPW; ++a) {
          const int j = wave + NW * a;
#pragma unroll
          for (int u = 0; u < GW; ++u)
#pragma unroll
            for (int q = 0; q < CPL; ++q) tot[a][q] += ps[((size_t)(u * SMALL_M + j)) * PROW + lane + 64 * q];
        }
      }
      // new centres: member mean, rounded to the I/O type; an empty cluster keeps its centre.  Only the
      // centres of the stage's last assignment are its result: they alone go to global memory.
      const bool last_update = it == cfg.iters - 2;
#pragma unroll
      for (int a = 0; a < JPW; ++a) {
        const int j = wave + NW * a;
        if (j >= m) continue;
        const int nj = cnt_s[j];
        if (lane == 0) cnt_s[j] = 0;
        if (nj > 0) {
          float bsum = 0.f;
#pragma unroll
          for (int q = 0; q < CPL; ++q) {
            const bf16raw r = f32_to_bf16(tot[a][q] / (float)nj);
            const float img = bf16_to_f32(r);
            cs[j * LDW + lane + 64 * q] = r;
            bsum = fmaf(img, img, bsum);
          }
#pragma unroll
          for (int o = 1; o < 64; o <<= 1) bsum += __shfl_xor(bsum, o);
          if (lane == 0) bs[j] = -0.5f * bsum;
        }
        if (last_update) {
#pragma unroll
          for (int q = 0; q < CPL; ++q) {
            const int col = lane + 64 * q;
            const bf16raw r = cs[j * LDW + col];          // written by this lane, now or in an earlier pass
            const size_t ao = ((size_t)h * cfg.cap + row_off + j) * D + col;
            cfg.cent_lp[ao] = r;
            cfg.assign_f32[ao] = bf16_to_f32(r);
          }
          if (lane == 0) cfg.bias[(size_t)h * cfg.cap + row_off + j] = bs[j];
        }
      }
      __syncthreads();
    }

    // threshold filter: points with d < tau leave U; U stays ascending (as filter_small)
    __syncthreads();
    int run = 0;
    for (int base = 0; base < n; base += 4 * NT) {
      const int p0 = base + 4 * tid;
      bool keep[4]; int tok[4]; int cnt = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int p = p0 + i;
        const bool valid = p < n;
        keep[i] = valid && !(fs[valid ? p : 0] < t2);
        tok[i] = valid ? uin[p] : -1;
        cnt += keep[i] ? 1 : 0;
      }
      int incl = cnt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o); if (lane >= o) incl += v; }
      __syncthreads();
      if (lane == 63) ws[wave] = incl;
      __syncthreads();
      int before = 0, total = 0;
      for (int w = 0; w < NW; ++w) { const int v = ws[w]; if (w < wave) before += v; total += v; }
      int pos = run + before + incl - cnt;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (keep[i]) uout[pos++] = tok[i];
        else if (tok[i] >= 0 && cfg.stage_of) cfg.stage_of[(size_t)h * cfg.N + tok[i]] = stage;
      }
      run += total;
    }
    __syncthreads();          // U of the next stage is written, and nobody reads the state any more
    if (tid == 0) {
      s_st.ucount = run;
      s_st.ccount += m;
      s_st.stage += 1;
      s_st.stage_offs[s_st.stage] = s_st.ccount;
      s_st.u_hist[s_st.stage] = run;
    }
  }
  if (tid == 0) st[h] = s_st;
}

__global__ void fill_i32(int32_t* p, size_t n, int32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// k_count, full_flag and stage offsets out of the state; the threshold in use, if asked for
__global__ void kstate_export(const KState* __restrict__ st, int H, int32_t* k_count, int32_t* full_flag,
                              int32_t* stage_offs, const float* __restrict__ tau, float* __restrict__ tau_used) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h == 0 && tau_used) tau_used[0] = tau[0];
  if (h >= H) return;
  const KState& s = st[h];
  if (k_count) k_count[h] = s.ccount;
  if (full_flag) full_flag[h] = s.full;
  if (stage_offs)
    for (int i = 0; i <= ADACLUSTER_MAX_STAGES; ++i)
      stage_offs[(size_t)h * (ADACLUSTER_MAX_STAGES + 1) + i] = (i <= s.stage) ? s.stage_offs[i] : s.ccount;
}

// ------------------------------------------------------------------------------------------
// compactness (Sec. 3.2.1): MSE_h = mean_n || k_n - c(k_n) ||^2
// ------------------------------------------------------------------------------------------
// One row per group of LPR lanes (16-byte pieces), fp32 inside a row, fp64 across rows; block
// partials are merged by mse_final in a fixed order.
template <typename T, int D>
__global__ __launch_bounds__(256) void mse_partial(const T* __restrict__ X, const int32_t* __restrict__ labels,
                                                   const float* __restrict__ cent, int N, int cap, int nblk,
                                                   double* __restrict__ part) {
  constexpr int EV = Vec16<T>::N, LPR = D / EV, RPB = 256 / LPR;   // rows per block step
  const int h = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
  const int slot = tid / LPR, cl = tid % LPR;
  double acc = 0.0;
  const int beg = b * 1024, end = min(N, beg + 1024);
  for (int r0 = beg; r0 < end; r0 += RPB) {
    const int r = r0 + slot;
    float ss = 0.f;
    if (r < end) {
      const int j = labels[(size_t)h * N + r];
      float x[EV];
      Vec16<T>::decode(*reinterpret_cast<const uint4*>(X + ((size_t)h * N + r) * D + cl * EV), x);
      const float* c = cent + ((size_t)h * cap + j) * D + cl * EV;
#pragma unroll
      for (int e = 0; e < EV; ++e) { const float df = x[e] - c[e]; ss = fmaf(df, df, ss); }
    }
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o);
    if (cl == 0) acc += (double)ss;
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) acc += __shfl_xor(acc, o);
  __shared__ double ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) part[(size_t)h * nblk + b] = (ws[0] + ws[1]) + (ws[2] + ws[3]);
}

__global__ __launch_bounds__(256) void mse_final(const double* __restrict__ part, int nblk, int N,
                                                 float* __restrict__ mse) {
  const int h = blockIdx.x, tid = threadIdx.x;
  double s = 0.0;
  for (int i = tid; i < nblk; i += 256) s += part[(size_t)h * nblk + i];
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) s += __shfl_xor(s, o);
  __shared__ double ws[4];
  if ((tid & 63) == 0) ws[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) mse[h] = (float)(((ws[0] + ws[1]) + (ws[2] + ws[3])) / (double)N);
}

// ------------------------------------------------------------------------------------------
// host-side launchers
// ------------------------------------------------------------------------------------------
static inline int chk() { return hipGetLastError() == hipSuccess ? 0 : ADACLUSTER_E_INTERNAL; }

int reduce_part_rows() { return REDUCE_ROWS; }
int assign_block_sum_centres() { return ACC_MAXM; }

int launch_assign(hipStream_t s, int dtype, int d, int H, int N, int n_bound, int mode, int m_const, int cap,
                  const KState* st, const int32_t* ulist, const void* X, const void* cent_lp, const float* bias,
                  int32_t* labels, float* dist2, float* blk_sum, int32_t* blk_cnt, int P, int32_t* keep_lab,
                  float* keep_score, const int32_t* seed_lab, const float* seed_score) {
  if ((mode == 3 || keep_lab || seed_lab) && (dtype != ADACLUSTER_BF16 || blk_sum)) return ADACLUSTER_E_INTERNAL;
  AssignCfg c{mode, m_const, N, cap, st, ulist, keep_lab, keep_score, seed_lab, seed_score};
  if (dtype == ADACLUSTER_BF16) {
    dim3 g((n_bound + 255) / 256, H);
    const AccumOut ao{blk_sum, blk_cnt, P, (int)g.x};
    if (blk_sum) {
      if (d == 64) assign_mfma<64, true><<<g, 256, 0, s>>>((const bf16raw*)X, c, (const bf16raw*)cent_lp, bias, labels, dist2, ao);
      else assign_mfma<128, true><<<g, 256, 0, s>>>((const bf16raw*)X, c, (const bf16raw*)cent_lp, bias, labels, dist2, ao);
    } else {
      if (d == 64) assign_mfma<64, false><<<g, 256, 0, s>>>((const bf16raw*)X, c, (const bf16raw*)cent_lp, bias, labels, dist2, ao);
      else assign_mfma<128, false><<<g, 256, 0, s>>>((const bf16raw*)X, c, (const bf16raw*)cent_lp, bias, labels, dist2, ao);
    }
  } else {
    if (blk_sum) return ADACLUSTER_E_INTERNAL;     // block sums exist for bf16 only
    dim3 g((n_bound + 127) / 128, H);
    if (d == 64) assign_f32<64><<<g, 128, 0, s>>>((const float*)X, c, (const float*)cent_lp, bias, labels, dist2);
    else assign_f32<128><<<g, 128, 0, s>>>((const float*)X, c, (const float*)cent_lp, bias, labels, dist2);
  }
  return chk();
}

// one-read pass of the query clustering (bf16, at most assign_block_sum_centres() centres): NP = walks per head
int qpass_walks(int N) { const int sb = (N + 127) / 128; const int subs = (sb + 63) / 64; return (sb + subs - 1) / subs; }
int launch_qpass(hipStream_t s, int d, int H, int N, int m, int cap, int weighted, const void* X, const void* cent_lp,
                 const float* bias, float* psum, int32_t* pcnt) {
  const int sb = (N + 127) / 128, subs = (sb + 63) / 64, NP = (sb + subs - 1) / subs;
  dim3 g(NP, H);
  if (d == 64) qpass_mfma<64><<<g, 256, 0, s>>>((const bf16raw*)X, N, m, cap, subs, weighted, (const bf16raw*)cent_lp, bias, psum, pcnt, NP);
  else qpass_mfma<128><<<g, 256, 0, s>>>((const bf16raw*)X, N, m, cap, subs, weighted, (const bf16raw*)cent_lp, bias, psum, pcnt, NP);
  return chk();
}

int launch_seg_reduce(hipStream_t s, int dtype, int d, int H, int N, int mode, int m_const, int m_bound, int P,
                      const KState* st, int normalize, int want_box, const void* X, const int32_t* perm,
                      const int32_t* offs, int offs_stride, int32_t* poff, int32_t* pcl, float* psum, float* pnorm,
                      float* pmin, float* pmax, int poff_ready) {
  ReduceCfg c{mode, m_const, N, P, m_bound, st, normalize, want_box};
  // poff_ready: 0 the parts are cut here; 1 the one-launch sort of small heads has cut them (and left no part ->
  // cluster table); 2 launch_part_scan has
  if (!poff_ready) part_scan<<<H, 1024, 0, s>>>(c, offs, offs_stride, poff, pcl);
  else if (poff_ready == 1) pcl = nullptr;
  dim3 g(P, H);
  if (dtype == ADACLUSTER_BF16) {
    if (d == 64) seg_reduce<bf16raw, 64><<<g, 64, 0, s>>>((const bf16raw*)X, c, perm, offs, offs_stride, poff, pcl, psum, pnorm, pmin, pmax);
    else seg_reduce<bf16raw, 128><<<g, 64, 0, s>>>((const bf16raw*)X, c, perm, offs, offs_stride, poff, pcl, psum, pnorm, pmin, pmax);
  } else {
    if (d == 64) seg_reduce<float, 64><<<g, 64, 0, s>>>((const float*)X, c, perm, offs, offs_stride, poff, pcl, psum, pnorm, pmin, pmax);
    else seg_reduce<float, 128><<<g, 64, 0, s>>>((const float*)X, c, perm, offs, offs_stride, poff, pcl, psum, pnorm, pmin, pmax);
  }
  return chk();
}

int launch_part_scan(hipStream_t s, int H, int N, int mode, int m_const, int m_bound, int P, const KState* st,
                     const int32_t* offs, int offs_stride, int32_t* poff, int32_t* pcl) {
  ReduceCfg c{mode, m_const, N, P, m_bound, st, 0, 0};
  part_scan<<<H, 1024, 0, s>>>(c, offs, offs_stride, poff, pcl);
  return chk();
}

int launch_finalize(hipStream_t s, int dtype, int d, int H, int mode, int m_const, int m_bound, int P, int cap,
                    int master_stride, const KState* st, int spherical, int update_assign, int want_box,
                    const int32_t* offs, int offs_stride, const int32_t* poff, const float* psum, const float* pnorm,
                    const float* pmin, const float* pmax, float* master, void* assign_lp, float* assign_f32,
                    float* bias, float* out_cent, const float* fallback, int32_t* out_sizes,
                    float* out_mean_norm, float* out_bmin, float* out_bmax, const int32_t* blk_cnt, int nb_stride,
                    int nb_const) {
  FinalizeCfg c{mode, m_const, P, m_bound, cap, master_stride, st, spherical, update_assign,
                dtype == ADACLUSTER_BF16, want_box, blk_cnt, nb_stride, nb_const};
  // in final mode every row of the output (up to cap) gets a size, so cover cap rows
  dim3 g(((update_assign ? m_bound : cap) + FIN_ROWS - 1) / FIN_ROWS, H);
  if (d == 64)
    finalize_centroids<64><<<g, 64 * FIN_ROWS, 0, s>>>(c, offs, offs_stride, poff, psum, pnorm, pmin, pmax, master, assign_lp,
                                            assign_f32, bias, out_cent, fallback, out_sizes, out_mean_norm,
                                            out_bmin, out_bmax);
  else
    finalize_centroids<128><<<g, 64 * FIN_ROWS, 0, s>>>(c, offs, offs_stride, poff, psum, pnorm, pmin, pmax, master, assign_lp,
                                             assign_f32, bias, out_cent, fallback, out_sizes, out_mean_norm,
                                             out_bmin, out_bmax);
  return chk();
}

bool direct_update_fits(int dtype, int n_bound, int m_bound) {
  return dtype == ADACLUSTER_F32 && n_bound <= DIRECT_MAX_POINTS && (long long)n_bound * m_bound <= DIRECT_MAX_VISITS;
}
int launch_update_direct(hipStream_t s, int d, int H, int N, int m_bound, int cap, int master_stride, const KState* st,
                         const int32_t* labels, const int32_t* ulist, const void* X, float* master, void* assign_lp,
                         float* assign_f32, float* bias) {
  dim3 g(m_bound, H);
  if (d == 64) update_direct_f32<64><<<g, 256, 0, s>>>((const float*)X, N, cap, master_stride, st, labels, ulist, master, (float*)assign_lp, assign_f32, bias);
  else update_direct_f32<128><<<g, 256, 0, s>>>((const float*)X, N, cap, master_stride, st, labels, ulist, master, (float*)assign_lp, assign_f32, bias);
  return chk();
}

int launch_init_centroids(hipStream_t s, int dtype, int d, int H, int N, int mode, int m_const, int m_bound,
                          const KState* st, const int32_t* ulist, int spherical, int source_master, int cap,
                          int master_stride, const void* X, float* master, void* assign_lp, float* assign_f32,
                          float* bias) {
  dim3 g(m_bound, H);
  const int lp = dtype == ADACLUSTER_BF16;
  if (dtype == ADACLUSTER_BF16) {
    if (d == 64) init_centroids<bf16raw, 64><<<g, 64, 0, s>>>((const bf16raw*)X, N, mode, m_const, st, ulist, spherical, source_master, cap, master_stride, lp, master, assign_lp, assign_f32, bias);
    else init_centroids<bf16raw, 128><<<g, 64, 0, s>>>((const bf16raw*)X, N, mode, m_const, st, ulist, spherical, source_master, cap, master_stride, lp, master, assign_lp, assign_f32, bias);
  } else {
    if (d == 64) init_centroids<float, 64><<<g, 64, 0, s>>>((const float*)X, N, mode, m_const, st, ulist, spherical, source_master, cap, master_stride, lp, master, assign_lp, assign_f32, bias);
    else init_centroids<float, 128><<<g, 64, 0, s>>>((const float*)X, N, mode, m_const, st, ulist, spherical, source_master, cap, master_stride, lp, master, assign_lp, assign_f32, bias);
  }
  return chk();
}

int launch_kstate_init(hipStream_t s, KState* st, int H, int N) {
  kstate_init<<<(H + 63) / 64, 64, 0, s>>>(st, H, N);
  return chk();
}

int launch_kstate_warm(hipStream_t s, KState* st, int H, int N, int cap, const int32_t* k_count,
                       const int32_t* full_flag) {
  kstate_warm<<<(H + 63) / 64, 64, 0, s>>>(st, H, N, cap, k_count, full_flag);
  return chk();
}

int launch_kstate_commit(hipStream_t s, KState* st, int H) {
  kstate_commit<<<(H + 63) / 64, 64, 0, s>>>(st, H);
  return chk();
}

int launch_kstage_begin(hipStream_t s, KState* st, int H, int N, int n_max, int m0, int m_min, int max_stages,
                        int u_min, int32_t* summary) {
  kstage_begin<<<1, 256, 0, s>>>(st, H, N, n_max, m0, m_min, max_stages, u_min, summary);
  return chk();
}

int launch_tau(hipStream_t s, int H, int N, const float* dist2, double* part, float factor, float tau_abs,
               float* tau_out) {
  if (tau_abs > 0.f) {
    tau_set<<<1, 64, 0, s>>>(tau_abs, tau_out);
    return chk();
  }
  const int nblk = (N + 1023) / 1024;
  tau_partial<<<dim3(nblk, H), 256, 0, s>>>(dist2, N, nblk, part);
  tau_final<<<1, 256, 0, s>>>(part, nblk * H, (double)H * (double)N, factor, tau_out);
  return chk();
}

int launch_filter(hipStream_t s, KState* st, int H, int N, int n_bound, const float* dist2, const float* tau,
                  int32_t* blockcnt, int32_t* u_prev, const int32_t* ulist_in, int32_t* ulist_out,
                  int32_t* stage_of, int stage) {
#ifndef FILTER_SMALL_LIMIT
#define FILTER_SMALL_LIMIT 32768
#endif
  if (n_bound <= FILTER_SMALL_LIMIT) {
    filter_small<<<H, 1024, 0, s>>>(st, dist2, N, tau, ulist_in, ulist_out, stage_of, stage);
    return chk();
  }
  const int nblk = (N + 1023) / 1024;
  const int nb = (n_bound + 1023) / 1024;
  filter_count<<<dim3(nb, H), 256, 0, s>>>(st, dist2, N, nblk, tau, blockcnt);
  filter_scan<<<H, 64, 0, s>>>(st, nb, nblk, blockcnt, u_prev);
  filter_scatter<<<dim3(nb, H), 256, 0, s>>>(st, u_prev, dist2, N, nblk, tau, blockcnt, ulist_in, ulist_out,
                                             stage_of, stage);
  return chk();
}

int small_stage_points() { return SMALL_NU; }
int small_stage_centres() { return SMALL_M; }

int launch_kstages_small(hipStream_t s, int d, int H, int N, int cap, int n_max, int m0, int m_min, int max_stages,
                         int u_min, int iters, KState* st, const float* tau, int32_t* ulist0, int32_t* ulist1,
                         const void* X, void* cent_lp, float* assign_f32, float* bias, int32_t* stage_of) {
  SmallStageCfg cfg;
  cfg.N = N; cfg.cap = cap; cfg.n_max = n_max; cfg.m0 = m0; cfg.m_min = m_min; cfg.max_stages = max_stages;
  cfg.u_min = u_min; cfg.iters = iters; cfg.tau = tau; cfg.ulist[0] = ulist0; cfg.ulist[1] = ulist1;
  cfg.cent_lp = (bf16raw*)cent_lp; cfg.assign_f32 = assign_f32; cfg.bias = bias; cfg.stage_of = stage_of;
  if (d == 64) kstages_small<64><<<H, SmallStage<64>::NW * 64, 0, s>>>((const bf16raw*)X, st, cfg);
  else kstages_small<128><<<H, SmallStage<128>::NW * 64, 0, s>>>((const bf16raw*)X, st, cfg);
  return chk();
}

int launch_mse(hipStream_t s, int dtype, int d, int H, int N, int cap, const void* X, const int32_t* labels,
               const float* cent, double* part, float* mse) {
  const int nblk = (N + 1023) / 1024;
  dim3 g(nblk, H);
  if (dtype == ADACLUSTER_BF16) {
    if (d == 64) mse_partial<bf16raw, 64><<<g, 256, 0, s>>>((const bf16raw*)X, labels, cent, N, cap, nblk, part);
    else mse_partial<bf16raw, 128><<<g, 256, 0, s>>>((const bf16raw*)X, labels, cent, N, cap, nblk, part);
  } else {
    if (d == 64) mse_partial<float, 64><<<g, 256, 0, s>>>((const float*)X, labels, cent, N, cap, nblk, part);
    else mse_partial<float, 128><<<g, 256, 0, s>>>((const float*)X, labels, cent, N, cap, nblk, part);
  }
  mse_final<<<H, 256, 0, s>>>(part, nblk, N, mse);
  return chk();
}

int launch_fill_i32(hipStream_t s, int32_t* p, size_t n, int32_t v) {
  if (n == 0) return 0;
  fill_i32<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(p, n, v);
  return chk();
}

int launch_kstate_export(hipStream_t s, const KState* st, int H, int32_t* k_count, int32_t* full_flag,
                         int32_t* stage_offs, const float* tau, float* tau_used) {
  kstate_export<<<(H + 63) / 64, 64, 0, s>>>(st, H, k_count, full_flag, stage_offs, tau, tau_used);
  return chk();
}

}  // namespace adac
