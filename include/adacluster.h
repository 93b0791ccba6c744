/*
 * adacluster.h -- C ABI of the MI355X (gfx950) clustered sparse-attention library.
 *
 * The library implements the attention-layer replacement of AdaCluster
 * (Algorithm 3 of the paper): queries are clustered on the unit sphere, keys by
 * the multi-stage threshold-adaptive k-means of Algorithm 1, critical key
 * clusters are chosen per query cluster from centroid-level scores (Eq. 1 / Eq. 2,
 * Algorithm 2) and attention runs only over the selected clusters.
 *
 * General conventions
 *   - Every pointer named in a signature is a DEVICE pointer unless the comment
 *     says "host".  Tensors are contiguous, row-major.  Q, K, V, O are [H,N,d] in
 *     the dtype named by params.dtype; d is 64 or 128; N is arbitrary (>= 1).
 *   - The caller owns every buffer.  The library allocates no device memory: all
 *     scratch lives in the caller's workspace `ws` of at least
 *     adacluster_workspace_bytes() bytes, 256-byte aligned.  Workspace contents
 *     are undefined after a call.  Output buffers are fully overwritten.
 *   - All work is ordered by `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream): it is enqueued there, except that adacluster_attn puts
 *     the query clustering (and, for fp32 inputs, the K/V permutation) on a second, library-owned stream
 *     (one per calling thread and device, created on first use, default priority),
 *     forked from `stream` and joined back to it before the step that needs the
 *     result, so work queued on `stream` after the call still waits for all of it.
 *     Calls are asynchronous
 *     except adacluster_kcluster and adacluster_attn with k_init_mode 0, which block
 *     the calling thread once per clustering stage on an event, to read a few
 *     integers back through pinned host memory the library keeps per thread (the
 *     stage loop of Algorithm 1 has a data-dependent trip count; the host runs one
 *     stage behind the device, so the stream is not drained, except once, before the
 *     second stage, when the first stage's sizes would be a poor bound for it).
 *   - Every function returns 0 on success or a negative ADACLUSTER_E_* code.  On
 *     an argument error nothing is launched.  adacluster_last_error() returns a
 *     message for the calling thread's last failure.  No function throws, aborts
 *     or prints.
 *   - Calls that share a workspace must not overlap in time.
 */
#ifndef ADACLUSTER_H
#define ADACLUSTER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADACLUSTER_OK             0
#define ADACLUSTER_E_BADARG      -1   /* NULL pointer or value out of range          */
#define ADACLUSTER_E_BADSHAPE    -2   /* H, N, d or a cluster count is not supported */
#define ADACLUSTER_E_BADDTYPE    -3
#define ADACLUSTER_E_WORKSPACE   -4   /* workspace NULL, misaligned or too small     */
#define ADACLUSTER_E_UNSUPPORTED -5
#define ADACLUSTER_E_INTERNAL    -6   /* a HIP runtime call failed                   */

#define ADACLUSTER_F32  0
#define ADACLUSTER_BF16 1

#define ADACLUSTER_SCORE_TQ  0   /* Alg. 2 on centroids: Q+ (K+)^T + Q- (K-)^T            */
#define ADACLUSTER_SCORE_BOX 1   /* Eq. 1 on each cluster's per-dimension min/max box      */
#define ADACLUSTER_SCORE_DOT 2   /* plain centroid dot product (the "w/o Quest" ablation)  */

#define ADACLUSTER_SELECT_TOPK 0 /* Alg. 3 line 8 */
#define ADACLUSTER_SELECT_TOPP 1 /* smallest set of clusters holding a share top_p of the
                                    size-weighted softmax mass of the centroid scores     */

#define ADACLUSTER_MAX_STAGES 16

/* Problem and method parameters (Alg. 3 inputs: tau, topk, N_max; Sec. 4.1 settings). */
typedef struct adacluster_params {
  int32_t H, N, d;              /* heads, tokens, head width (64 or 128)                       */
  int32_t dtype;                /* ADACLUSTER_F32 or ADACLUSTER_BF16 (Q,K,V,O)                  */
  int32_t q_clusters;           /* number of query clusters (paper: 65); 1 <= q_clusters <= N   */
  int32_t q_iters;              /* assignment passes of the query k-means (>= 1)                */
  int32_t k_iters;              /* assignment passes of each key k-means stage (>= 1)           */
  int32_t q_init_mode;          /* 0: strided sample of the queries; 1: q_centroids passed in   */
  int32_t k_init_mode;          /* 0: Algorithm 1 from scratch; 1: warm start (Sec. 3.2.2,
                                   "Efficient initialization"): cluster count fixed, previous centres
                                   passed in k_centroids / k_count / full_flag, k_iters passes    */
  int32_t k_m0;                 /* key centres of the first stage ("Initial K", paper: 100)     */
  int32_t k_m_min;              /* floor for the centre count of later stages                   */
  int32_t k_max_clusters;       /* N_max of Alg. 1.  Centre buffers hold cap = N_max + k_m0 rows */
  int32_t k_max_stages;         /* at most this many stages (<= ADACLUSTER_MAX_STAGES)          */
  float   tau_abs;              /* > 0: absolute distance threshold tau                         */
  float   tau_factor;           /* used when tau_abs <= 0: tau = factor x mean first-stage
                                   token-to-centre distance over all heads (paper: 1.5)        */
  float   min_unassigned_frac;  /* stop staging once |U| <= floor(frac*N); 0 = Alg. 1 literally */
  int32_t score_mode;           /* ADACLUSTER_SCORE_*                                           */
  int32_t select_mode;          /* ADACLUSTER_SELECT_*                                          */
  int32_t topk;                 /* clusters kept per query cluster (top-k mode), >= 1           */
  float   top_p;                /* mass share (top-p mode), in (0,1]                            */
  float   softmax_scale;        /* <= 0 means 1/sqrt(d)                                         */
  int32_t q_no_norm;            /* 0 (the paper): queries are clustered by angle, as q/|q|;      */
                                /* 1: ablation "w/o Norm" (App. component ablation): Euclidean   */
                                /* k-means on the raw queries, scores from the raw centroids      */
} adacluster_params;

/* rows of every per-head key-centre buffer: k_max_clusters + k_m0 */
int adacluster_centroid_capacity(const adacluster_params* p);

/* Bytes of workspace any entry point needs for these parameters (host pointer out). */
int adacluster_workspace_bytes(const adacluster_params* p, size_t* bytes);

/* Copies the calling thread's last error message into buf (host), NUL-terminated. */
int adacluster_last_error(char* buf, size_t buf_bytes);

/*
 * Query clustering: KMeans(Normalize(Q)), Alg. 3 line 1 / Sec. 3.1.
 *   Q                  [H,N,d]   in
 *   q_labels           [H,N]     out  cluster of every query (arg-max cosine to q_assign_centroids)
 *   q_centroids        [H,Cq,d]  in (q_init_mode 1: initial centres) / out: unit-norm member means
 *                                under q_labels (empty cluster: previous centre)
 *   q_assign_centroids [H,Cq,d]  out  centres the last assignment pass used, as fp32 holding
 *                                values representable in the I/O dtype
 *   q_sizes            [H,Cq]    out  members per cluster
 *   q_mean_norm        [H,Cq]    out  mean ||q|| of the members (0 for an empty cluster)
 */
int adacluster_qcluster(const adacluster_params* p, const void* Q,
                        int32_t* q_labels, float* q_centroids, float* q_assign_centroids,
                        int32_t* q_sizes, float* q_mean_norm,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Key clustering: MultiStageClustering(K, tau, N_max), Algorithm 1.  cap = capacity above.
 *   K                  [H,N,d]    in
 *   k_labels           [H,N]      out  nearest centre among all stage centres (Alg. 1 last step)
 *   k_centroids        [H,cap,d]  out  member means under k_labels (rows >= k_count undefined;
 *                                 empty cluster: its stage centre)
 *   k_assign_centroids [H,cap,d]  out  the stage centres, in stage order (what k_labels is the
 *                                 arg-min of), fp32 holding I/O-dtype-representable values
 *   k_box_min,k_box_max[H,cap,d]  out  per-dimension member extremes; both may be NULL
 *   k_sizes            [H,cap]    out  members per cluster (0 beyond k_count)
 *   k_count            [H]        out  number of centres |C|
 *   full_flag          [H]        out  1 iff staging stopped on |C| >= N_max with tokens left (F)
 *   k_stage_offs       [H,ADACLUSTER_MAX_STAGES+1] out  running centre count after each stage,
 *                                 unused entries = k_count; may be NULL
 *   k_stage_of         [H,N]      out  stage at which a token fell within tau (-1: never); may be NULL
 *   tau_used           [1]        out  the threshold applied (tau_abs, or the derived value)
 * Warm start (k_init_mode 1): k_centroids (rows < k_count), k_count and full_flag are INPUTS as left
 * by a previous call; the centre count stays fixed, k_iters assignment passes start from those
 * centres, no token is staged (k_stage_of = 0 everywhere, one stage), full_flag and tau_used are
 * passed through unchanged; every other output is produced as above.
 */
int adacluster_kcluster(const adacluster_params* p, const void* K,
                        int32_t* k_labels, float* k_centroids, float* k_assign_centroids,
                        float* k_box_min, float* k_box_max,
                        int32_t* k_sizes, int32_t* k_count, int32_t* full_flag,
                        int32_t* k_stage_offs, int32_t* k_stage_of, float* tau_used,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Critical-cluster selection: centroid scores (Eq. 1 / Eq. 2, Alg. 2) and arg-top-k (Alg. 3
 * line 8) or the top-p budget.  Scores are evaluated in fp64 with the contraction summed in
 * ascending dimension order, so the index sets are reproducible bit for bit.
 *   q_centroids [H,Cq,d], q_mean_norm [H,Cq]              in (outputs of adacluster_qcluster)
 *   k_centroids, k_box_min, k_box_max [H,cap,d]           in (boxes only read in BOX mode)
 *   k_sizes [H,cap], k_count [H], full_flag [H]           in
 *   sel_idx [H,Cq,cap]  out  ascending key-cluster ids per query cluster (first sel_cnt entries)
 *   sel_cnt [H,Cq]      out
 * Empty key clusters are never selected; a head with full_flag set selects every non-empty one.
 */
int adacluster_select(const adacluster_params* p,
                      const float* q_centroids, const float* q_mean_norm,
                      const float* k_centroids, const float* k_box_min, const float* k_box_max,
                      const int32_t* k_sizes, const int32_t* k_count, const int32_t* full_flag,
                      int32_t* sel_idx, int32_t* sel_cnt,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * Attention over the selected clusters (Alg. 3 lines 9-10): for a query n in query cluster i,
 *   O_n = sum over keys m whose cluster is in sel(i) of softmax_m(scale * q_n . k_m) v_m,
 * with the raw (un-normalised) query.  A query cluster with an empty selection yields zeros.
 *   Q,K,V [H,N,d] in;  q_labels,k_labels [H,N] in (values in [0,Cq) and [0,k_count[h]));
 *   k_count [H] in;  sel_idx [H,Cq,cap], sel_cnt [H,Cq] in (ascending, distinct);
 *   O [H,N,d] out, original token order.
 */
int adacluster_sparse_attn(const adacluster_params* p,
                           const void* Q, const void* K, const void* V,
                           const int32_t* q_labels, const int32_t* k_labels, const int32_t* k_count,
                           const int32_t* sel_idx, const int32_t* sel_cnt,
                           void* O, void* ws, size_t ws_bytes, void* stream);

/*
 * The whole of Algorithm 3 in one call: query clustering, Algorithm 1, selection, attention
 * (heads whose flag F is set attend to every key).  Cluster outputs may each be NULL when the
 * caller does not need them (they then live in the workspace); shapes as above.
 */
typedef struct adacluster_outputs {
  int32_t* q_labels;  float* q_centroids;  float* q_assign_centroids;
  int32_t* q_sizes;   float* q_mean_norm;
  int32_t* k_labels;  float* k_centroids;  float* k_assign_centroids;
  float* k_box_min;   float* k_box_max;
  int32_t* k_sizes;   int32_t* k_count;    int32_t* full_flag;
  int32_t* k_stage_offs; int32_t* k_stage_of; float* tau_used;
  int32_t* sel_idx;   int32_t* sel_cnt;
} adacluster_outputs;

int adacluster_attn(const adacluster_params* p,
                    const void* Q, const void* K, const void* V, void* O,
                    const adacluster_outputs* outs /* host struct of device pointers, may be NULL */,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * Per-head figures of the last adacluster_attn call on a workspace (diagnostics; Alg. 1's stage loop and the
 * executed share of the score matrix that Alg. 3 lines 8-10 leave).  adacluster_stats_fetch must follow that
 * call with the same params and workspace, before any other call touches the workspace: it reduces what the
 * call left there with one small kernel on `stream`, copies H records to host_stats (HOST pointer) and waits
 * for `stream`.  After adacluster_kcluster alone the first five fields are valid, after adacluster_sparse_attn
 * alone the last three.
 */
typedef struct adacluster_head_stats {
  int32_t k_count;        /* |C|: key centres Algorithm 1 ended with                                   */
  int32_t full_flag;      /* F                                                                         */
  int32_t stages;         /* stages of Algorithm 1 that ran (1 for a warm start)                       */
  int32_t q_tiles;        /* workgroups of the attention launch (query tiles, cut key lists counted per chunk) */
  int32_t unassigned[ADACLUSTER_MAX_STAGES + 1]; /* |U| at the head of stage t for t < stages; entry
                             [stages] = keys still beyond tau of every centre when staging stopped      */
  int32_t reserved;
  int64_t executed_pairs; /* sum over query clusters i of n_q(i) * sum_{j in sel(i)} n_k(j)            */
  int64_t issued_pairs;   /* the same with the rows of every query tile rounded up to whole 32-query
                             waves and its keys to whole 64-key tiles: what the matrix cores are fed    */
} adacluster_head_stats;

int adacluster_stats_fetch(const adacluster_params* p, void* ws, size_t ws_bytes,
                           adacluster_head_stats* host_stats /* host, [H] */, void* stream);

/* Dense softmax attention on the same attention kernel (the F = True branch of Alg. 3 and the
 * timing baseline): every query attends to every key. */
int adacluster_dense_attn(const adacluster_params* p,
                          const void* Q, const void* K, const void* V, void* O,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * Compactness of a key clustering (Sec. 3.2.1): k_mse[h] = (1/N) sum_n || k_n - c(k_n) ||^2 with
 * c(k_n) = k_centroids[h, k_labels[h,n], :]; the paper's layer score is Comp = 1 / mean_h k_mse[h].
 *   K [H,N,d] in (dtype), k_labels [H,N] in (every label < capacity), k_centroids [H,cap,d] fp32 in,
 *   k_mse [H] fp32 out.  Squares are summed in fp32 inside a row and in fp64 across rows, in a fixed
 *   order.  Asynchronous on `stream`; reads no other state, so it may follow adacluster_kcluster or
 *   adacluster_attn (with those outputs requested) at any time.
 */
int adacluster_compactness(const adacluster_params* p, const void* K, const int32_t* k_labels,
                           const float* k_centroids, float* k_mse, void* ws, size_t ws_bytes, void* stream);

/*
 * adacluster_compactness for callers that cannot allocate device memory or size a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same result bit for bit.  The per-block partial sums go to a 512 KiB array that is part of the
 * library's device image (every GPU the library runs on holds its copy until the process ends); nothing is
 * allocated or freed by the call.  Limit: H * ceil(N / 1024) <= 65536 partial sums, else
 * ADACLUSTER_E_UNSUPPORTED and nothing is launched.  All calls on one GPU share that array: calls that
 * overlap in time on one GPU (different streams or threads) race and must be serialised by the caller.
 * Asynchronous on `stream`.
 */
int adacluster_compactness_noalloc(const adacluster_params* p, const void* K, const int32_t* k_labels,
                                   const float* k_centroids, float* k_mse, void* stream);

/*
 * Quest scores of query rows against key pages (Sec. 3.2.3), in either of the two forms whose speed the
 * paper compares (Sec. 4.3, "TensorQuest reformulation benefits"):
 *   form ADACLUSTER_QUEST_ALU   Eq. 1 as written, S[h,i,j] = sum_d max(q_d R+_jd, q_d R-_jd), fp32 vector
 *                               arithmetic (any dtype);
 *   form ADACLUSTER_QUEST_MFMA  Eq. 2 / Algorithm 2, S = Q+ (R+)^T + Q- (R-)^T with Q+ = max(Q,0),
 *                               Q- = min(Q,0), two matrix products on the matrix cores, fp32 accumulation
 *                               (bf16 inputs only: ADACLUSTER_E_UNSUPPORTED otherwise).
 * R_pos and R_neg [H,Lk,d] are the per-dimension maxima and minima of every page (Eq. 1); with clamp != 0
 * they are taken as max(R_pos, 0) and min(R_neg, 0) on the fly, which for R_pos == R_neg == a tensor of
 * single vectors per page (cluster centroids) is Algorithm 2 as written.  The two forms agree exactly in
 * real arithmetic whenever R_pos >= R_neg elementwise.
 *   Q [H,Lq,d], R_pos, R_neg in `dtype`; S [H,Lq,Lk] fp32 out, fully overwritten.  d is 64 or 128.
 * Device pointers; asynchronous on `stream`; needs no workspace.
 */
#define ADACLUSTER_QUEST_ALU  0
#define ADACLUSTER_QUEST_MFMA 1
int adacluster_quest_scores(int32_t H, int32_t Lq, int32_t Lk, int32_t d, int32_t dtype, int32_t form, int32_t clamp,
                            const void* Q, const void* R_pos, const void* R_neg, float* S, void* stream);

/*
 * Stage timing for benchmarks.  adacluster_profile_enable(1) creates HIP events; while enabled,
 * adacluster_attn, adacluster_sparse_attn and adacluster_dense_attn record them on the call's
 * stream at their stage boundaries (adacluster_qcluster and adacluster_kcluster record their own).
 * adacluster_profile_read waits for the last recorded call
 * and writes, to the HOST array ms[7], the milliseconds of: query clustering, Algorithm 1,
 * selection (stand-alone sparse_attn: the two label sorts), K/V permutation (fp32 inputs only: bf16
 * rows are read where they are, through the key permutation), planning, the
 * attention kernel, and the segmented reduction over all N keys that ends Algorithm 1 (one launch,
 * also counted inside Algorithm 1); -1 for a stage the call did not run.  In adacluster_attn the two clusterings
 * run side by side and each is timed from the start of the call, so their sum exceeds the time
 * the pair takes; the K/V permutation is timed from the final key sort, after which it runs on the
 * second stream beside the tail of Algorithm 1, the selection and the planning.  Not thread-safe.
 */
int adacluster_profile_enable(int on);

/*
 * Matrix-core yardstick for benchmarks: a register-only loop of bf16 MFMAs (v_mfma_f32_32x32x16_bf16, four
 * independent chains per wave, `iters` trips) on every SIMD of the chip, enqueued on `stream`.  *flops (HOST)
 * receives the floating-point operations of the launch; the caller times it.  sink: DEVICE, >= 256 floats.
 */
int adacluster_mfma_probe(int32_t iters, float* sink, size_t sink_floats, double* flops, void* stream);
int adacluster_profile_read(float* ms);

#ifdef __cplusplus
}
#endif
#endif /* ADACLUSTER_H */
