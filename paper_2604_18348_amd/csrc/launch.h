// Host-side launchers of the kernels (each enqueues on the given stream and returns 0 or
// ADACLUSTER_E_INTERNAL).
#pragma once
#include "common.h"

namespace adac {

struct SortScratch {
  int32_t* hist;                     // [H][nseg][128]
  int32_t* lab_a; int32_t* val_a;    // [H][N] intermediate pass
  int32_t* lab_b;                    // [H][N] sorted labels
};

// Stable sort of the first n_h items of every head by label (labels are indexed by position in
// the item list; the items are token ids from `ulist`, or the positions themselves).
//   n_dev / m_dev: per-head item and label counts read on the device (NULL: n_bound / m_bound)
//   active_dev:    per-head flag; heads with 0 are skipped (NULL: all heads)
// Outputs: perm [H][N] token ids ordered by (label, position); offs [H][offs_stride] with
// offs[j] = first sorted position of label j for j = 0..m_h.
int launch_sort(hipStream_t st, int H, int N, int n_bound, int m_bound, const int32_t* labels,
                const int32_t* ulist, const int32_t* n_dev, int n_stride, const int32_t* m_dev, int m_stride,
                const int32_t* active_dev, int active_stride, int32_t* perm, int32_t* offs, int offs_stride,
                const SortScratch& sc, int32_t* poff = nullptr, int part_rows = 0, int* poff_done = nullptr);

int launch_assign(hipStream_t s, int dtype, int d, int H, int N, int n_bound, int mode, int m_const, int cap,
                  const KState* st, const int32_t* ulist, const void* X, const void* cent_lp, const float* bias,
                  int32_t* labels, float* dist2, float* blk_sum = nullptr, int32_t* blk_cnt = nullptr, int P = 0,
                  int32_t* keep_lab = nullptr, float* keep_score = nullptr, const int32_t* seed_lab = nullptr,
                  const float* seed_score = nullptr);
int assign_block_sum_centres();   // most centres the assignment kernel keeps block sums for
int launch_seg_reduce(hipStream_t s, int dtype, int d, int H, int N, int mode, int m_const, int m_bound, int P,
                      const KState* st, int normalize, int want_box, const void* X, const int32_t* perm,
                      const int32_t* offs, int offs_stride, int32_t* poff, int32_t* pcl, float* psum, float* pnorm, float* pmin,
                      float* pmax, int poff_ready = 0);
int reduce_part_rows();
// Cuts the clusters of a sorted head into reduction parts on its own (launch_seg_reduce then takes poff_ready = 2).
int launch_part_scan(hipStream_t s, int H, int N, int mode, int m_const, int m_bound, int P, const KState* st,
                     const int32_t* offs, int offs_stride, int32_t* poff, int32_t* pcl);
int launch_finalize(hipStream_t s, int dtype, int d, int H, int mode, int m_const, int m_bound, int P, int cap,
                    int master_stride, const KState* st, int spherical, int update_assign, int want_box,
                    const int32_t* offs, int offs_stride, const int32_t* poff, const float* psum, const float* pnorm,
                    const float* pmin, const float* pmax, float* master, void* assign_lp, float* assign_f32,
                    float* bias, float* out_cent, const float* fallback, int32_t* out_sizes,
                    float* out_mean_norm, float* out_bmin, float* out_bmax, const int32_t* blk_cnt = nullptr,
                    int nb_stride = 0, int nb_const = 0);
// Centroid update of a running stage (state mode 1) in one launch, fp32 inputs: every centre's workgroup scans the
// stage's label list (`ulist` NULL: positions are tokens), so it is for few points and centres only:
// direct_update_fits() says when.  Writes what launch_finalize(update_assign = 1) writes.
bool direct_update_fits(int dtype, int n_bound, int m_bound);
int launch_update_direct(hipStream_t s, int d, int H, int N, int m_bound, int cap, int master_stride, const KState* st,
                         const int32_t* labels, const int32_t* ulist, const void* X, float* master, void* assign_lp,
                         float* assign_f32, float* bias);
// One pass of a k-means with at most assign_block_sum_centres() centres in one read of the points (bf16):
// assignment and (weighted) centroid sums together.  psum [H][m * NP][d], pcnt [H][NP][assign_block_sum_centres()]
// with NP = qpass_walks(N); launch_finalize(..., blk_cnt = pcnt, nb_stride = NP, nb_const = NP) turns them into centres.
int qpass_walks(int N);
int launch_qpass(hipStream_t s, int d, int H, int N, int m, int cap, int weighted, const void* X, const void* cent_lp,
                 const float* bias, float* psum, int32_t* pcnt);
int launch_init_centroids(hipStream_t s, int dtype, int d, int H, int N, int mode, int m_const, int m_bound,
                          const KState* st, const int32_t* ulist, int spherical, int source_master, int cap,
                          int master_stride, const void* X, float* master, void* assign_lp, float* assign_f32,
                          float* bias);
int launch_kstate_init(hipStream_t s, KState* st, int H, int N);
int launch_kstate_warm(hipStream_t s, KState* st, int H, int N, int cap, const int32_t* k_count, const int32_t* full_flag);
int launch_kstate_commit(hipStream_t s, KState* st, int H);
int launch_kstage_begin(hipStream_t s, KState* st, int H, int N, int n_max, int m0, int m_min, int max_stages,
                        int u_min, int32_t* summary);
int launch_tau(hipStream_t s, int H, int N, const float* dist2, double* part, float factor, float tau_abs,
               float* tau_out);
int launch_filter(hipStream_t s, KState* st, int H, int N, int n_bound, const float* dist2, const float* tau,
                  int32_t* blockcnt, int32_t* u_prev, const int32_t* ulist_in, int32_t* ulist_out,
                  int32_t* stage_of, int stage);
// Every remaining stage of Algorithm 1 in one launch, one workgroup per head (bf16 only).  Valid once every
// active head has at most small_stage_points() unassigned points and small_stage_centres() centres per
// stage, and never for stage 0 (it needs a list of U and a known tau).
int small_stage_points();
int small_stage_centres();
int launch_kstages_small(hipStream_t s, int d, int H, int N, int cap, int n_max, int m0, int m_min, int max_stages,
                         int u_min, int iters, KState* st, const float* tau, int32_t* ulist0, int32_t* ulist1,
                         const void* X, void* cent_lp, float* assign_f32, float* bias, int32_t* stage_of);
int launch_mse(hipStream_t s, int dtype, int d, int H, int N, int cap, const void* X, const int32_t* labels,
               const float* cent, double* part, float* mse);
int launch_fill_i32(hipStream_t s, int32_t* p, size_t n, int32_t v);
int launch_kstate_export(hipStream_t s, const KState* st, int H, int32_t* k_count, int32_t* full_flag,
                         int32_t* stage_offs, const float* tau = nullptr, float* tau_used = nullptr);

int launch_select(hipStream_t s, int H, int Cq, int cap, int d, int score_mode, int select_mode, int topk,
                  float top_p, float scale, const float* q_cent, const float* q_mean_norm, const float* k_cent,
                  const float* k_bmin, const float* k_bmax, const int32_t* k_sizes, const int32_t* k_count,
                  const int32_t* full_flag, int32_t* sel_idx, int32_t* sel_cnt, int kc_max, double* scores);   // scores: scratch [H][Cq][cap]

int attn_block_rows(int dtype, int d, int N, int Cq);   // queries per workgroup of the attention launch
int attn_block_rows_min(int dtype);
int attn_block_rows_max(int dtype);
int launch_permute_kv(hipStream_t s, int H, int N, int row_bytes, const void* K, const void* V,
                      const int32_t* perm, void* Kp, void* Vp);
int launch_quest_scores(hipStream_t s, int dtype, int form, int clamp, int H, int Lq, int Lk, int d, const void* Q,
                        const void* Rp, const void* Rn, float* S);
// register-only loop of bf16 MFMAs on every SIMD of the chip (measures what the matrix cores sustain)
int launch_mfma_probe(hipStream_t s, int iters, float* sink, size_t sink_floats, double* flops);
int attn_split_slots();      // partial slots per head for the chunks of cut key lists (also extra tile records)
int launch_plan_sparse(hipStream_t s, int dtype, int H, int Cq, int cap, int maxr, int maxtiles, int BM,
                       const int32_t* q_offs, int q_offs_stride, const int32_t* k_offs, int k_offs_stride,
                       const int32_t* k_count, const int32_t* sel_idx, const int32_t* sel_cnt,
                       int32_t* rng_start, int32_t* rng_pre, int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles,
                       int32_t* merge, int32_t* nmerge, int row_bytes, int32_t* krow, size_t kstride, const int32_t* perm_k = nullptr, int N = 0);
int launch_plan_dense(hipStream_t s, int H, int N, int maxtiles, int BM, int32_t* rng_start, int32_t* rng_pre,
                      int32_t* rng_cnt, int32_t* tiles, int32_t* ntiles, int row_bytes, int32_t* krow, size_t kstride);
// entries per (head, query cluster) of the table of key-row byte offsets the bf16 attention kernel loads by
size_t attn_krow_stride(int N);
int launch_attn_stats(hipStream_t s, int H, int Cq, int maxr, int maxtiles, const KState* st, const int32_t* tiles,
                      const int32_t* ntiles, const int32_t* rng_pre, const int32_t* rng_cnt, adacluster_head_stats* out);
int launch_attention(hipStream_t s, int dtype, int d, int H, int N, int Cq, int maxtiles, int maxr, float scale,
                     const void* Q, const void* Kp, const void* Vp, void* O, const int32_t* perm_q,
                     const int32_t* tiles, const int32_t* ntiles, const int32_t* rng_start,
                     const int32_t* rng_pre, const int32_t* rng_cnt, float* part_o, float* part_ml,
                     const int32_t* merge /* NULL: no cut lists */, const int32_t* nmerge,
                     const int32_t* krow, size_t kstride);

}  // namespace adac
