// C ABI of the clustered sparse-attention library: argument checks, workspace layout and the
// order in which the kernels of Algorithm 3 are enqueued.  No device memory is allocated here.
#include "common.h"
#include "launch.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

using namespace adac;

// Scratch memory that belongs to the library, for the one entry point that takes no workspace
// (adacluster_compactness_noalloc).  Every GPU the library runs on holds its own copy of the array until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels get the
// address that call returns for the current device, never the name.
constexpr size_t STATIC_SCRATCH_DOUBLES = 65536;                 // 512 KiB
static __device__ __align__(256) double scratch[STATIC_SCRATCH_DOUBLES];

namespace {

thread_local char g_err[256] = "";

// Optional stage timing: hipEvents recorded at the stage boundaries of a call.  A stage is timed
// from the event in from[] (default: the previous recorded stage boundary); the fused call runs
// the two clusterings side by side, so both of those are timed from the start of the call.
enum { EV_START = 0, EV_QCLUSTER, EV_KCLUSTER, EV_SELECT, EV_PERMUTE, EV_PLAN, EV_ATTN, EV_KREDUCE, EV_STAGES,
       EV_JOIN = EV_STAGES, EV_JOIN2, EV_KSORT, EV_COUNT };
struct Profiler {
  bool enabled = false;
  bool recorded[EV_COUNT] = {};
  int from[EV_COUNT] = {};
  hipEvent_t ev[EV_COUNT] = {};
} g_prof;

void prof_begin(hipStream_t st) {
  if (!g_prof.enabled) return;
  for (int i = 0; i < EV_COUNT; ++i) { g_prof.recorded[i] = false; g_prof.from[i] = -1; }
  (void)hipEventRecord(g_prof.ev[EV_START], st);
  g_prof.recorded[EV_START] = true;
}
void prof_mark(int which, hipStream_t st, int from = -1) {
  if (!g_prof.enabled) return;
  (void)hipEventRecord(g_prof.ev[which], st);
  g_prof.recorded[which] = true;
  g_prof.from[which] = from;
}

// A second stream per calling thread and device, for work of a call that does not depend on what
// the caller's stream is doing (default priority, like every stream here), and the events that fork
// it from and join it to the caller's stream.  Per thread, so that calls of different host threads
// on one device do not share events.
struct AuxStream {
  bool ready = false;
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr, join2 = nullptr;
};
thread_local AuxStream g_aux[64];

// Pinned host slots for the per-stage report of Algorithm 1 and two events to wait on, per thread.
struct StageReadback {
  bool ready = false;
  int device = -1;
  int32_t* host = nullptr;     // [ADACLUSTER_MAX_STAGES + 2][4], pinned and mapped
  int32_t* dev = nullptr;      // the same memory as the device sees it
  hipEvent_t ev[2] = {nullptr, nullptr};
};
thread_local StageReadback t_readback;

StageReadback* stage_readback() {
  StageReadback& r = t_readback;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  if (r.ready && r.device != dev) {        // events belong to the device they were created on
    for (int i = 0; i < 2; ++i) (void)hipEventDestroy(r.ev[i]);
    (void)hipHostFree(r.host);
    r.ready = false;
  }
  if (!r.ready) {
    r.device = dev;
    if (hipHostMalloc((void**)&r.host, (ADACLUSTER_MAX_STAGES + 2) * 4 * sizeof(int32_t), hipHostMallocMapped) != hipSuccess) return nullptr;
    if (hipHostGetDevicePointer((void**)&r.dev, r.host, 0) != hipSuccess) return nullptr;
    for (int i = 0; i < 2; ++i)
      if (hipEventCreateWithFlags(&r.ev[i], hipEventDisableTiming) != hipSuccess) return nullptr;
    r.ready = true;
  }
  return &r;
}

AuxStream* aux_stream() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  AuxStream& a = g_aux[dev];
  if (!a.ready) {
    if (hipStreamCreateWithFlags(&a.s, hipStreamNonBlocking) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&a.fork, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&a.join, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&a.join2, hipEventDisableTiming) != hipSuccess) return nullptr;
    a.ready = true;
  }
  return &a;
}

int fail(int code, const char* fmt, ...);

// Device address of `scratch` on the current device, looked up once per device.
std::mutex g_scratch_mu;
double* g_scratch_ptr[64] = {};
double* static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev] = (double*)ptr;
  }
  return g_scratch_ptr[dev];
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_params(const adacluster_params* p) {
  if (!p) return fail(ADACLUSTER_E_BADARG, "params is NULL");
  if (p->H < 1 || p->N < 1) return fail(ADACLUSTER_E_BADSHAPE, "H and N must be >= 1 (H=%d N=%d)", p->H, p->N);
  if (p->H > 65535) return fail(ADACLUSTER_E_BADSHAPE, "H must be <= 65535");
  if (p->d != 64 && p->d != 128) return fail(ADACLUSTER_E_BADSHAPE, "d must be 64 or 128 (d=%d)", p->d);
  if (p->dtype != ADACLUSTER_F32 && p->dtype != ADACLUSTER_BF16) return fail(ADACLUSTER_E_BADDTYPE, "unknown dtype %d", p->dtype);
  if ((long long)p->N * p->d * 4 >= (1ll << 40)) return fail(ADACLUSTER_E_BADSHAPE, "N too large");
  if (p->q_clusters < 1 || p->q_clusters > p->N) return fail(ADACLUSTER_E_BADSHAPE, "q_clusters must be in [1,N]");
  if (p->q_clusters > 4096) return fail(ADACLUSTER_E_BADSHAPE, "q_clusters must be <= 4096");
  if (p->q_iters < 1 || p->k_iters < 1) return fail(ADACLUSTER_E_BADARG, "q_iters and k_iters must be >= 1");
  if (p->q_init_mode != 0 && p->q_init_mode != 1) return fail(ADACLUSTER_E_BADARG, "q_init_mode must be 0 or 1");
  if (p->k_init_mode != 0 && p->k_init_mode != 1) return fail(ADACLUSTER_E_BADARG, "k_init_mode must be 0 or 1");
  if (p->k_m0 < 1 || p->k_m0 > p->N) return fail(ADACLUSTER_E_BADSHAPE, "k_m0 must be in [1,N]");
  if (p->k_m_min < 1 || p->k_m_min > p->k_m0) return fail(ADACLUSTER_E_BADARG, "k_m_min must be in [1,k_m0]");
  if (p->k_max_clusters < 1) return fail(ADACLUSTER_E_BADARG, "k_max_clusters must be >= 1");
  if (p->k_m0 > p->k_max_clusters) return fail(ADACLUSTER_E_BADARG, "k_m0 must not exceed k_max_clusters");
  if ((long long)p->k_max_clusters + p->k_m0 > 7168) return fail(ADACLUSTER_E_BADSHAPE, "k_max_clusters + k_m0 must be <= 7168");
  if (p->k_max_stages < 1 || p->k_max_stages > ADACLUSTER_MAX_STAGES) return fail(ADACLUSTER_E_BADARG, "k_max_stages must be in [1,%d]", ADACLUSTER_MAX_STAGES);
  if (!(p->tau_abs > 0.f) && !(p->tau_factor > 0.f)) return fail(ADACLUSTER_E_BADARG, "tau_abs or tau_factor must be > 0");
  if (!(p->min_unassigned_frac >= 0.f) || p->min_unassigned_frac > 1.f) return fail(ADACLUSTER_E_BADARG, "min_unassigned_frac must be in [0,1]");
  if (p->score_mode < 0 || p->score_mode > 2) return fail(ADACLUSTER_E_BADARG, "unknown score_mode %d", p->score_mode);
  if (p->select_mode < 0 || p->select_mode > 1) return fail(ADACLUSTER_E_BADARG, "unknown select_mode %d", p->select_mode);
  if (p->topk < 1) return fail(ADACLUSTER_E_BADARG, "topk must be >= 1");
  if (!(p->top_p > 0.f) || p->top_p > 1.f) return fail(ADACLUSTER_E_BADARG, "top_p must be in (0,1]");
  if (p->q_no_norm != 0 && p->q_no_norm != 1) return fail(ADACLUSTER_E_BADARG, "q_no_norm must be 0 or 1");
  return 0;
}

constexpr int STAGE_SUM_BLOCKS = 128;   // a stage of at most this many 256-point blocks may update from block sums

inline int capacity(const adacluster_params* p) { return p->k_max_clusters + p->k_m0; }
inline size_t esize(const adacluster_params* p) { return p->dtype == ADACLUSTER_BF16 ? 2 : 4; }
// upper bound of the number of 128-row parts of n rows in m clusters
inline int parts_for(int n, int m) { const int r = reduce_part_rows(); return m + (n + r - 1) / r + 1; }   // every cluster ends in at most one short part

// ---- workspace layout ----------------------------------------------------------------------
struct Layout {
  size_t total = 0;
  size_t take(size_t bytes) { size_t o = total; total += align_up(bytes, 256); return o; }
};

struct WS {
  unsigned char* base;
  KState* kstate; int32_t* summary; float* tau; int32_t* u_prev;
  void* cent_lp; float* bias; float* master;
  int32_t* labels_tmp; float* dist2; int32_t* ulist[2]; int32_t* blockcnt; double* tau_part;
  SortScratch sort; int32_t* perm_tmp; int32_t* offs_tmp; int32_t* poff; int32_t* pcl; int32_t* lab0; float* score0;
  float* psum; float* pnorm; float* pmin; float* pmax; int32_t* bcnt; float* bsum;
  int32_t* perm_q; int32_t* offs_q; int32_t* perm_k; int32_t* offs_k;
  // scratch of the query clustering (its own set: it runs beside the key clustering)
  void* q_cent_lp; float* q_bias; SortScratch q_sort; int32_t* q_poff; float* q_psum; float* q_pnorm;
  float* q_wsum; int32_t* q_wcnt;     // walk sums and counts of the one-read passes of the query clustering
  void* Kp; void* Vp;
  double* scores;       // [H][Cq][cap] centroid scores between the kernels of the selection step
  int32_t* rng_start; int32_t* rng_pre; int32_t* rng_cnt; int32_t* tiles; int32_t* ntiles;
  int32_t* merge; int32_t* nmerge; float* part_o; float* part_ml;   // cut key lists of the attention step
  int32_t* krow;        // [H][Cq][kstride] byte offset of every key row of a query cluster's list
  // homes for outputs of the fused call the caller did not ask for
  int32_t* q_labels; float* q_centroids; float* q_assign; int32_t* q_sizes; float* q_mean_norm;
  int32_t* k_labels; float* k_centroids; float* k_assign; float* k_bmin; float* k_bmax;
  int32_t* k_sizes; int32_t* k_count; int32_t* full_flag; int32_t* sel_idx; int32_t* sel_cnt;
  int32_t* one_count;   // [H] constant key-cluster count for the dense plan
  adacluster_head_stats* stats;   // [H] staging area of adacluster_stats_fetch
};

struct Dims {
  int H, N, d, Cq, cap, capmax, nblk, nseg, maxtiles, maxr, prow, brow, BM, BMmax;
};

Dims dims_of(const adacluster_params* p) {
  Dims D;
  D.H = p->H; D.N = p->N; D.d = p->d; D.Cq = p->q_clusters; D.cap = capacity(p);
  D.capmax = D.cap > D.Cq ? D.cap : D.Cq;
  D.nblk = (p->N + 1023) / 1024;
  D.nseg = (p->N + 511) / 512;
  D.BM = attn_block_rows(p->dtype, p->d, p->N, D.Cq);
  D.BMmax = attn_block_rows_max(p->dtype);
  D.maxtiles = p->N / attn_block_rows_min(p->dtype) + D.Cq + 1 + attn_split_slots();   // (sized for the smaller tile shape)
  D.maxr = D.cap;
  D.prow = p->N / reduce_part_rows() + D.capmax + 34;
  {  // rows of the block-sum table of small stages: (blocks of 256 points) x (centres), both capped
    const int nb = (p->N + 255) / 256, mb = p->k_m0 < assign_block_sum_centres() ? p->k_m0 : assign_block_sum_centres();
    D.brow = (nb < STAGE_SUM_BLOCKS ? nb : STAGE_SUM_BLOCKS) * mb;
  }
  return D;
}

// bf16: the attention kernel takes every key row by its byte offset, so K and V stay where they are and the
// row-offset table of a query cluster is written through the key permutation (no permuted copies; measured
// against gathering K and V into cluster order first: the same attention time, and the gather with its 4 bytes
// of HBM traffic per input byte gone).  fp32: the kernel walks row ranges of the permuted copies.
static bool rows_in_place(const adacluster_params* p) { return p->dtype == ADACLUSTER_BF16; }

size_t layout(const adacluster_params* p, WS* w, unsigned char* base) {
  const Dims D = dims_of(p);
  const size_t H = D.H, N = D.N, d = D.d, es = esize(p);
  Layout L;
#define TAKE(field, type, bytes) { size_t o_ = L.take(bytes); if (w) w->field = (type)(base + o_); }
  TAKE(kstate, KState*, H * sizeof(KState));
  TAKE(summary, int32_t*, 64);
  TAKE(tau, float*, 64);
  TAKE(u_prev, int32_t*, H * 4);
  TAKE(cent_lp, void*, H * D.capmax * d * es);
  TAKE(bias, float*, H * D.capmax * 4);
  TAKE(master, float*, H * (size_t)(p->k_m0 > D.Cq ? p->k_m0 : D.Cq) * d * 4);
  TAKE(labels_tmp, int32_t*, H * N * 4);
  TAKE(dist2, float*, H * N * 4);
  TAKE(ulist[0], int32_t*, H * N * 4);
  TAKE(ulist[1], int32_t*, H * N * 4);
  TAKE(blockcnt, int32_t*, H * D.nblk * 4);
  TAKE(tau_part, double*, H * D.nblk * 8);
  TAKE(sort.hist, int32_t*, H * D.nseg * 128 * 4);
  TAKE(sort.lab_a, int32_t*, H * N * 4);
  TAKE(sort.val_a, int32_t*, H * N * 4);
  TAKE(sort.lab_b, int32_t*, H * N * 4);
  TAKE(perm_tmp, int32_t*, H * N * 4);
  TAKE(offs_tmp, int32_t*, H * (size_t)(D.capmax + 1) * 4);
  TAKE(poff, int32_t*, H * (size_t)(D.capmax + 1) * 4);
  TAKE(pcl, int32_t*, H * (size_t)D.prow * 4);
  TAKE(lab0, int32_t*, p->dtype == ADACLUSTER_BF16 ? H * N * 4 : 256);
  TAKE(score0, float*, p->dtype == ADACLUSTER_BF16 ? H * N * 4 : 256);
  TAKE(psum, float*, H * (size_t)D.prow * d * 4);
  TAKE(bcnt, int32_t*, H * (size_t)STAGE_SUM_BLOCKS * assign_block_sum_centres() * 4);
  TAKE(bsum, float*, H * (size_t)D.brow * d * 4);
  TAKE(pnorm, float*, H * (size_t)D.prow * 4);
  TAKE(pmin, float*, H * (size_t)D.prow * d * 4);
  TAKE(pmax, float*, H * (size_t)D.prow * d * 4);
  TAKE(q_cent_lp, void*, H * (size_t)D.Cq * d * es);
  TAKE(q_bias, float*, H * (size_t)D.Cq * 4);
  TAKE(q_sort.hist, int32_t*, H * D.nseg * 128 * 4);
  TAKE(q_sort.lab_a, int32_t*, H * N * 4);
  TAKE(q_sort.val_a, int32_t*, H * N * 4);
  TAKE(q_sort.lab_b, int32_t*, H * N * 4);
  TAKE(q_poff, int32_t*, H * (size_t)(D.Cq + 1) * 4);
  TAKE(q_psum, float*, H * (size_t)(N / reduce_part_rows() + D.Cq + 34) * d * 4);
  TAKE(q_pnorm, float*, H * (size_t)(N / reduce_part_rows() + D.Cq + 34) * 4);
  {
    const bool one_read = p->dtype == ADACLUSTER_BF16 && D.Cq <= assign_block_sum_centres();
    TAKE(q_wsum, float*, one_read ? H * (size_t)D.Cq * qpass_walks(D.N) * d * 4 : 256);
    TAKE(q_wcnt, int32_t*, one_read ? H * (size_t)qpass_walks(D.N) * assign_block_sum_centres() * 4 : 256);
  }
  TAKE(perm_q, int32_t*, H * N * 4);
  TAKE(offs_q, int32_t*, H * (size_t)(D.Cq + 1) * 4);
  TAKE(perm_k, int32_t*, H * N * 4);
  TAKE(offs_k, int32_t*, H * (size_t)(D.cap + 1) * 4);
  TAKE(Kp, void*, rows_in_place(p) ? 256 : H * N * d * es);      // permuted copies: fp32 only
  TAKE(Vp, void*, rows_in_place(p) ? 256 : H * N * d * es);
  TAKE(scores, double*, H * (size_t)D.Cq * D.cap * 8);
  TAKE(rng_start, int32_t*, H * (size_t)D.Cq * D.maxr * 4);
  TAKE(rng_pre, int32_t*, H * (size_t)D.Cq * (D.maxr + 1) * 4);
  TAKE(rng_cnt, int32_t*, H * (size_t)D.Cq * 4);
  TAKE(tiles, int32_t*, H * (size_t)D.maxtiles * 6 * 4);
  TAKE(merge, int32_t*, H * (size_t)attn_split_slots() * 4 * 4);
  TAKE(nmerge, int32_t*, H * 4);
  TAKE(part_o, float*, H * (size_t)attn_split_slots() * D.BMmax * d * 4);
  TAKE(part_ml, float*, H * (size_t)attn_split_slots() * D.BMmax * 2 * 4);
  TAKE(ntiles, int32_t*, H * 4);
  TAKE(krow, int32_t*, p->dtype == ADACLUSTER_BF16 ? H * (size_t)D.Cq * attn_krow_stride(D.N) * 4 : 256);
  TAKE(q_labels, int32_t*, H * N * 4);
  TAKE(q_centroids, float*, H * (size_t)D.Cq * d * 4);
  TAKE(q_assign, float*, H * (size_t)D.Cq * d * 4);
  TAKE(q_sizes, int32_t*, H * (size_t)D.Cq * 4);
  TAKE(q_mean_norm, float*, H * (size_t)D.Cq * 4);
  TAKE(k_labels, int32_t*, H * N * 4);
  TAKE(k_centroids, float*, H * (size_t)D.cap * d * 4);
  TAKE(k_assign, float*, H * (size_t)D.cap * d * 4);
  TAKE(k_bmin, float*, H * (size_t)D.cap * d * 4);
  TAKE(k_bmax, float*, H * (size_t)D.cap * d * 4);
  TAKE(k_sizes, int32_t*, H * (size_t)D.cap * 4);
  TAKE(k_count, int32_t*, H * 4);
  TAKE(full_flag, int32_t*, H * 4);
  TAKE(sel_idx, int32_t*, H * (size_t)D.Cq * D.cap * 4);
  TAKE(sel_cnt, int32_t*, H * (size_t)D.Cq * 4);
  TAKE(one_count, int32_t*, H * 4);
  TAKE(stats, adacluster_head_stats*, H * sizeof(adacluster_head_stats));
#undef TAKE
  if (w) w->base = base;
  return L.total;
}

int check_ws(const adacluster_params* p, void* ws, size_t ws_bytes, WS* w) {
  if (!ws) return fail(ADACLUSTER_E_WORKSPACE, "workspace is NULL");
  if (((uintptr_t)ws) & 255) return fail(ADACLUSTER_E_WORKSPACE, "workspace must be 256-byte aligned");
  const size_t need = layout(p, nullptr, nullptr);
  if (ws_bytes < need) return fail(ADACLUSTER_E_WORKSPACE, "workspace too small: %zu < %zu bytes", ws_bytes, need);
  layout(p, w, (unsigned char*)ws);
  return 0;
}

#define RET_IF(expr) { int rc_ = (expr); if (rc_ != 0) return rc_ == ADACLUSTER_E_INTERNAL ? fail(rc_, "HIP launch failed: %s", hipGetErrorString(hipGetLastError())) : rc_; }

// ---- query clustering ----------------------------------------------------------------------
int run_qcluster(const adacluster_params* p, const WS& w, hipStream_t st, const void* Q, int32_t* q_labels,
                 float* q_centroids, float* q_assign, int32_t* q_sizes, float* q_mean_norm) {
  const Dims D = dims_of(p);
  const int P = parts_for(D.N, D.Cq);
  int poff_done = 0;   // set when the sort has already cut the clusters into reduction parts
  const int sph = p->q_no_norm ? 0 : 1;      // by angle on q/|q| (the paper), or Euclidean on raw queries (ablation)
  RET_IF(launch_init_centroids(st, p->dtype, D.d, D.H, D.N, 0, D.Cq, D.Cq, nullptr, nullptr, sph, p->q_init_mode,
                               D.Cq, D.Cq, Q, q_centroids, w.q_cent_lp, q_assign, w.q_bias));
  // A pass that only updates the centres reads the queries once: assignment and (normalised) sums in one
  // kernel.  The last pass needs the labels sorted (for the attention step) and exact member statistics, and
  // takes the sort and the segmented reduction.
  const bool one_read = p->dtype == ADACLUSTER_BF16 && D.Cq <= assign_block_sum_centres();
  for (int it = 0; it < p->q_iters; ++it) {
    if (one_read && it < p->q_iters - 1) {
      const int NP = qpass_walks(D.N);
      RET_IF(launch_qpass(st, D.d, D.H, D.N, D.Cq, D.Cq, sph, Q, w.q_cent_lp, w.q_bias, w.q_wsum, w.q_wcnt));
      RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 0, D.Cq, D.Cq, D.Cq * NP, D.Cq, D.Cq, nullptr, sph, 1, 0, nullptr, 0,
                             nullptr, w.q_wsum, w.q_pnorm, nullptr, nullptr, q_centroids, w.q_cent_lp, q_assign, w.q_bias,
                             nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.q_wcnt, NP, NP));
      continue;
    }
    RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, D.N, 0, D.Cq, D.Cq, nullptr, nullptr, Q, w.q_cent_lp, w.q_bias,
                         q_labels, nullptr));
    RET_IF(launch_sort(st, D.H, D.N, D.N, D.Cq, q_labels, nullptr, nullptr, 0, nullptr, 0, nullptr, 0, w.perm_q,
                       w.offs_q, D.Cq + 1, w.q_sort, w.q_poff, reduce_part_rows(), &poff_done));
    RET_IF(launch_seg_reduce(st, p->dtype, D.d, D.H, D.N, 0, D.Cq, D.Cq, P, nullptr, sph, 0, Q, w.perm_q, w.offs_q,
                             D.Cq + 1, w.q_poff, nullptr, w.q_psum, w.q_pnorm, nullptr, nullptr, poff_done));
    const bool last = it == p->q_iters - 1;
    if (!last) {
      RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 0, D.Cq, D.Cq, P, D.Cq, D.Cq, nullptr, sph, 1, 0, w.offs_q,
                             D.Cq + 1, w.q_poff, w.q_psum, w.q_pnorm, nullptr, nullptr, q_centroids, w.q_cent_lp, q_assign, w.q_bias,
                             nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
    } else {
      RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 0, D.Cq, D.Cq, P, D.Cq, D.Cq, nullptr, sph, 0, 0, w.offs_q,
                             D.Cq + 1, w.q_poff, w.q_psum, w.q_pnorm, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                             q_centroids, nullptr, q_sizes, q_mean_norm, nullptr, nullptr));
    }
  }
  return 0;
}

// ---- Algorithm 1 ---------------------------------------------------------------------------
int run_kcluster(const adacluster_params* p, const WS& w, hipStream_t st, const void* K, int32_t* k_labels,
                 float* k_centroids, float* k_assign, float* k_bmin, float* k_bmax, int32_t* k_sizes,
                 int32_t* k_count, int32_t* full_flag, int32_t* k_stage_offs, int32_t* k_stage_of,
                 float* tau_used, int* kc_bound_out, hipEvent_t sorted_ev = nullptr) {
  const Dims D = dims_of(p);
  int kc_bound = 0;   // sum over stages of the largest stage centre count: an upper bound of every |C|
  hipEvent_t pending_ev = nullptr;   // the last report may still be in flight when the stage loop ends
  int poff_done = 0;                 // set when the sort has already cut the clusters into reduction parts
  if (p->k_init_mode == 1) {
    // warm start: one pseudo-stage over all tokens with the previous centres, count fixed
    RET_IF(launch_kstate_warm(st, w.kstate, D.H, D.N, D.cap, k_count, full_flag));
    if (k_stage_of) RET_IF(launch_fill_i32(st, k_stage_of, (size_t)D.H * D.N, 0));
    RET_IF(launch_init_centroids(st, p->dtype, D.d, D.H, D.N, 1, 0, D.cap, w.kstate, nullptr, 0, 1, D.cap, D.cap, K,
                                 k_centroids, w.cent_lp, k_assign, w.bias));
    const int Pw = parts_for(D.N, D.cap);
    for (int it = 0; it < p->k_iters; ++it) {
      RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, D.N, 1, 0, D.cap, w.kstate, nullptr, K, w.cent_lp, w.bias,
                           k_labels, nullptr));
      if (it < p->k_iters - 1 && direct_update_fits(p->dtype, D.N, D.cap)) {
        RET_IF(launch_update_direct(st, D.d, D.H, D.N, D.cap, D.cap, D.cap, w.kstate, k_labels, nullptr, K, k_centroids,
                                    w.cent_lp, k_assign, w.bias));
      } else if (it < p->k_iters - 1) {
        RET_IF(launch_sort(st, D.H, D.N, D.N, D.cap, k_labels, nullptr, nullptr, 0, &w.kstate->m_t, sizeof(KState) / 4,
                           nullptr, 0, w.perm_tmp, w.offs_tmp, D.capmax + 1, w.sort, w.poff, reduce_part_rows(), &poff_done));
        RET_IF(launch_seg_reduce(st, p->dtype, D.d, D.H, D.N, 1, 0, D.cap, Pw, w.kstate, 0, 0, K, w.perm_tmp,
                                 w.offs_tmp, D.capmax + 1, w.poff, w.pcl, w.psum, w.pnorm, w.pmin, w.pmax, poff_done));
        RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 1, 0, D.cap, Pw, D.cap, D.cap, w.kstate, 0, 1, 0, w.offs_tmp,
                               D.capmax + 1, w.poff, w.psum, w.pnorm, w.pmin, w.pmax, k_centroids, w.cent_lp,
                               k_assign, w.bias, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
      }
    }
    RET_IF(launch_kstate_commit(st, w.kstate, D.H));
    if (kc_bound_out) *kc_bound_out = D.cap;
    RET_IF(launch_kstate_export(st, w.kstate, D.H, k_count, full_flag, k_stage_offs));
  } else {
  const int u_min = (int)floor((double)p->min_unassigned_frac * (double)p->N);
  const bool seeded = p->dtype == ADACLUSTER_BF16;
  RET_IF(launch_kstate_init(st, w.kstate, D.H, D.N));
  if (k_stage_of) RET_IF(launch_fill_i32(st, k_stage_of, (size_t)D.H * D.N, -1));
  if (p->tau_abs > 0.f) RET_IF(launch_tau(st, D.H, D.N, nullptr, nullptr, 0.f, p->tau_abs, w.tau));
  // The stage loop has a data-dependent trip count, and grids are sized by what the stage head
  // reports: {active heads, max |U|, max m_t}.  Reading that back before enqueuing the stage
  // would drain the queue once per stage, so the host stays one stage behind: stage t is
  // enqueued with the report of stage t-1 (|U| and m_t never grow, so the older figures are
  // valid bounds; every kernel takes the true counts from the device state), and a stage whose
  // heads all turn out finished runs as empty kernels, once, at the end.
  StageReadback* rb = stage_readback();
  if (!rb) return fail(ADACLUSTER_E_INTERNAL, "stage read-back set-up failed: %s", hipGetErrorString(hipGetLastError()));
  int n_bound = D.N, m_bound = p->k_m0 < D.N ? p->k_m0 : D.N;
  for (int t = 0; t <= p->k_max_stages; ++t) {
    pending_ev = rb->ev[t & 1];
    // the stage head writes its report straight into the pinned slot (no copy in between)
    RET_IF(launch_kstage_begin(st, w.kstate, D.H, D.N, p->k_max_clusters, p->k_m0, p->k_m_min, p->k_max_stages,
                               u_min, rb->dev + 4 * t));
    if (hipEventRecord(rb->ev[t & 1], st) != hipSuccess)
      return fail(ADACLUSTER_E_INTERNAL, "stage read-back failed: %s", hipGetErrorString(hipGetLastError()));
    if (t > 0) {
      if (hipEventSynchronize(rb->ev[(t - 1) & 1]) != hipSuccess)
        return fail(ADACLUSTER_E_INTERNAL, "stage read-back failed: %s", hipGetErrorString(hipGetLastError()));
      const int32_t* summ = rb->host + 4 * (t - 1);
      if (summ[0] == 0) break;                 // stage t-1 had no active head: the loop ended there
      n_bound = summ[1]; m_bound = summ[2];
      kc_bound += m_bound;
    }
    if (t == p->k_max_stages) break;           // the stage head has just closed every head
    if (t == 1 && !(p->dtype == ADACLUSTER_BF16 && (n_bound + 255) / 256 <= STAGE_SUM_BLOCKS &&
                    m_bound <= assign_block_sum_centres())) {
      // Stage 0 removes most points, so its figures (all N points, m_0 centres) are poor bounds for
      // stage 1: unless they still allow the short update (block sums), they would send a few thousand
      // points through the launch chain sized for all of them (two radix passes, segmented
      // reduction).  Then, once per call, the host waits for the report of the stage it is about to
      // enqueue; the other stream keeps the device busy meanwhile.
      if (hipEventSynchronize(rb->ev[1]) != hipSuccess)
        return fail(ADACLUSTER_E_INTERNAL, "stage read-back failed: %s", hipGetErrorString(hipGetLastError()));
      const int32_t* cur = rb->host + 4;
      if (cur[0] == 0) break;                  // no head needs a second stage
      n_bound = cur[1]; m_bound = cur[2];
    }
    if (t > 0 && p->dtype == ADACLUSTER_BF16 && n_bound <= small_stage_points() && m_bound <= small_stage_centres()) {
      // few points and few centres left in every head: one launch runs this and every later stage
      // (|U| and m_t never grow, so the bounds hold for all of them)
      RET_IF(launch_kstages_small(st, D.d, D.H, D.N, D.cap, p->k_max_clusters, p->k_m0, p->k_m_min, p->k_max_stages,
                                  u_min, p->k_iters, w.kstate, w.tau, w.ulist[0], w.ulist[1], K, w.cent_lp, k_assign,
                                  w.bias, k_stage_of));
      kc_bound += m_bound * (p->k_max_stages - t);
      break;
    }
    const int32_t* ul = (t == 0) ? nullptr : w.ulist[t & 1];
    int32_t* ul_next = w.ulist[(t + 1) & 1];
    RET_IF(launch_init_centroids(st, p->dtype, D.d, D.H, D.N, 1, 0, m_bound, w.kstate, ul, 0, 0, D.cap, p->k_m0, K,
                                 w.master, w.cent_lp, k_assign, w.bias));
    const int P = parts_for(n_bound, m_bound);
    // A small stage (few blocks of points, few centres) updates its centres from sums that the
    // assignment kernel leaves per block: no label sort and no segmented reduction in between.
    const int nblk = (n_bound + 255) / 256;
    const bool block_sums = p->dtype == ADACLUSTER_BF16 && nblk <= STAGE_SUM_BLOCKS &&
                            m_bound <= assign_block_sum_centres() && (long long)m_bound * nblk <= D.brow;
    const int Pb = m_bound * nblk;     // rows of the part-sum table the block sums take per head
    for (int it = 0; it < p->k_iters; ++it) {
      const bool update = it < p->k_iters - 1;
      if (block_sums && update) {
        RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, n_bound, 1, 0, D.cap, w.kstate, ul, K, w.cent_lp, w.bias,
                             w.labels_tmp, nullptr, w.bsum, w.bcnt, Pb));        // (distances: last pass only)
        RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 1, 0, m_bound, Pb, D.cap, p->k_m0, w.kstate, 0, 1, 0,
                               nullptr, 0, nullptr, w.bsum, w.pnorm, w.pmin, w.pmax, w.master, w.cent_lp,
                               k_assign, w.bias, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.bcnt, nblk));
        continue;
      }
      // (the last pass of stage 0 runs over all points against the first-stage centres as they will stay:
      // it keeps a copy of its labels and best scores, which the final pass starts from)
      const bool keep = seeded && t == 0 && !update;
      RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, n_bound, 1, 0, D.cap, w.kstate, ul, K, w.cent_lp, w.bias,
                           w.labels_tmp, update ? nullptr : w.dist2, nullptr, nullptr, 0, keep ? w.lab0 : nullptr,
                           keep ? w.score0 : nullptr));
      if (update && direct_update_fits(p->dtype, n_bound, m_bound)) {
        // few points (fp32): every centre gathers its members from the label list itself, one launch
        RET_IF(launch_update_direct(st, D.d, D.H, D.N, m_bound, D.cap, p->k_m0, w.kstate, w.labels_tmp, ul, K, w.master,
                                    w.cent_lp, k_assign, w.bias));
      } else if (update) {
        RET_IF(launch_sort(st, D.H, D.N, n_bound, m_bound, w.labels_tmp, ul, &w.kstate->ucount,
                           sizeof(KState) / 4, &w.kstate->m_t, sizeof(KState) / 4, &w.kstate->active,
                           sizeof(KState) / 4, w.perm_tmp, w.offs_tmp, D.capmax + 1, w.sort, w.poff, reduce_part_rows(), &poff_done));
        RET_IF(launch_seg_reduce(st, p->dtype, D.d, D.H, D.N, 1, 0, m_bound, P, w.kstate, 0, 0, K, w.perm_tmp,
                                 w.offs_tmp, D.capmax + 1, w.poff, w.pcl, w.psum, w.pnorm, w.pmin, w.pmax, poff_done));
        RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 1, 0, m_bound, P, D.cap, p->k_m0, w.kstate, 0, 1, 0,
                               w.offs_tmp, D.capmax + 1, w.poff, w.psum, w.pnorm, w.pmin, w.pmax, w.master, w.cent_lp,
                               k_assign, w.bias, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
      }
    }
    if (t == 0 && !(p->tau_abs > 0.f))
      RET_IF(launch_tau(st, D.H, D.N, w.dist2, w.tau_part, p->tau_factor, 0.f, w.tau));
    RET_IF(launch_filter(st, w.kstate, D.H, D.N, n_bound, w.dist2, w.tau, w.blockcnt, w.u_prev, ul, ul_next,
                         k_stage_of, t));
  }
  if (kc_bound_out) *kc_bound_out = kc_bound < D.cap ? kc_bound : D.cap;
  RET_IF(launch_kstate_export(st, w.kstate, D.H, k_count, full_flag, k_stage_offs, w.tau, tau_used));
  // last step of Algorithm 1: nearest centre among all stage centres, then member statistics.  bf16: the
  // nearest first-stage centre of every point is known from stage 0, so only the later stages' centres are visited.
  if (seeded)
    RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, D.N, 3, 0, D.cap, w.kstate, nullptr, K, w.cent_lp, w.bias,
                         k_labels, nullptr, nullptr, nullptr, 0, nullptr, nullptr, w.lab0, w.score0))
  else
    RET_IF(launch_assign(st, p->dtype, D.d, D.H, D.N, D.N, 2, 0, D.cap, w.kstate, nullptr, K, w.cent_lp, w.bias,
                         k_labels, nullptr));
  }
  RET_IF(launch_sort(st, D.H, D.N, D.N, D.cap, k_labels, nullptr, nullptr, 0, &w.kstate->ccount, sizeof(KState) / 4,
                     nullptr, 0, w.perm_k, w.offs_k, D.cap + 1, w.sort, w.poff, reduce_part_rows(), &poff_done));
  // the key permutation is final here: work that needs nothing else of the clustering may start
  if (sorted_ev && hipEventRecord(sorted_ev, st) != hipSuccess) return fail(ADACLUSTER_E_INTERNAL, "stream fork failed");
  const int want_box = (k_bmin && k_bmax) ? 1 : 0;
  const int P = parts_for(D.N, D.cap);
  if (!poff_done) {       // the cut into reduction parts belongs to the sort's side of the profile mark
    RET_IF(launch_part_scan(st, D.H, D.N, 2, 0, D.cap, P, w.kstate, w.offs_k, D.cap + 1, w.poff, w.pcl));
    poff_done = 2;
  }
  prof_mark(EV_KSORT, st);
  RET_IF(launch_seg_reduce(st, p->dtype, D.d, D.H, D.N, 2, 0, D.cap, P, w.kstate, 0, want_box, K, w.perm_k, w.offs_k,
                           D.cap + 1, w.poff, w.pcl, w.psum, w.pnorm, w.pmin, w.pmax, poff_done));
  prof_mark(EV_KREDUCE, st, EV_KSORT);
  RET_IF(launch_finalize(st, p->dtype, D.d, D.H, 2, 0, D.cap, P, D.cap, D.cap, w.kstate, 0, 0, want_box, w.offs_k,
                         D.cap + 1, w.poff, w.psum, w.pnorm, w.pmin, w.pmax, nullptr, nullptr, nullptr, nullptr, k_centroids,
                         k_assign, k_sizes, nullptr, k_bmin, k_bmax));
  // the pinned report slots are reused by the next call of this thread: let the last report land
  // (its kernel was queued ahead of everything above, so this does not drain the stream)
  if (pending_ev && hipEventSynchronize(pending_ev) != hipSuccess)
    return fail(ADACLUSTER_E_INTERNAL, "stage read-back failed: %s", hipGetErrorString(hipGetLastError()));
  return 0;
}

// ---- attention over selected clusters, given both sorts ---------------------------------------
// K and V rows into cluster order (needs only the key label sort)
int run_permute(const adacluster_params* p, const WS& w, hipStream_t st, const void* K, const void* V, int prof_from) {
  const Dims D = dims_of(p);
  RET_IF(launch_permute_kv(st, D.H, D.N, D.d * (int)esize(p), K, V, w.perm_k, w.Kp, w.Vp));
  prof_mark(EV_PERMUTE, st, prof_from);
  return 0;
}

// range lists, row offsets and query tiles from the selection, then the attention kernel
int run_plan_attention(const adacluster_params* p, const WS& w, hipStream_t st, const void* Q, void* O,
                       const int32_t* k_count, const int32_t* sel_idx, const int32_t* sel_cnt, int prof_from,
                       hipEvent_t permute_done, const void* K = nullptr, const void* V = nullptr) {
  const Dims D = dims_of(p);
  const bool inplace = K && V && rows_in_place(p);
  const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)D.d);
  RET_IF(launch_plan_sparse(st, p->dtype, D.H, D.Cq, D.cap, D.maxr, D.maxtiles, D.BM, w.offs_q, D.Cq + 1, w.offs_k,
                            D.cap + 1, k_count, sel_idx, sel_cnt, w.rng_start, w.rng_pre, w.rng_cnt, w.tiles, w.ntiles,
                            w.merge, w.nmerge, D.d * (int)esize(p), p->dtype == ADACLUSTER_BF16 ? w.krow : nullptr,
                            attn_krow_stride(D.N), inplace ? w.perm_k : nullptr, D.N));
  prof_mark(EV_PLAN, st, prof_from);
  if (permute_done && hipStreamWaitEvent(st, permute_done, 0) != hipSuccess)
    return fail(ADACLUSTER_E_INTERNAL, "stream join failed");
  if (permute_done) prof_mark(EV_JOIN2, st);
  RET_IF(launch_attention(st, p->dtype, D.d, D.H, D.N, D.Cq, D.maxtiles, D.maxr, scale, Q, inplace ? K : w.Kp, inplace ? V : w.Vp, O, w.perm_q,
                          w.tiles, w.ntiles, w.rng_start, w.rng_pre, w.rng_cnt, w.part_o, w.part_ml, w.merge, w.nmerge,
                          w.krow, attn_krow_stride(D.N)));
  prof_mark(EV_ATTN, st, permute_done ? EV_JOIN2 : -1);
  return 0;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

int adacluster_centroid_capacity(const adacluster_params* p) {
  int rc = check_params(p);
  if (rc) return rc;
  return capacity(p);
}

int adacluster_workspace_bytes(const adacluster_params* p, size_t* bytes) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!bytes) return fail(ADACLUSTER_E_BADARG, "bytes is NULL");
  *bytes = layout(p, nullptr, nullptr);
  return 0;
}

int adacluster_last_error(char* buf, size_t buf_bytes) {
  if (!buf || buf_bytes == 0) return ADACLUSTER_E_BADARG;
  strncpy(buf, g_err, buf_bytes - 1);
  buf[buf_bytes - 1] = 0;
  return 0;
}

int adacluster_qcluster(const adacluster_params* p, const void* Q, int32_t* q_labels, float* q_centroids,
                        float* q_assign_centroids, int32_t* q_sizes, float* q_mean_norm, void* ws,
                        size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!Q || !q_labels || !q_centroids || !q_assign_centroids || !q_sizes || !q_mean_norm)
    return fail(ADACLUSTER_E_BADARG, "qcluster: NULL tensor pointer");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  prof_begin((hipStream_t)stream);
  rc = run_qcluster(p, w, (hipStream_t)stream, Q, q_labels, q_centroids, q_assign_centroids, q_sizes, q_mean_norm);
  prof_mark(EV_QCLUSTER, (hipStream_t)stream, EV_START);
  return rc;
}

int adacluster_kcluster(const adacluster_params* p, const void* K, int32_t* k_labels, float* k_centroids,
                        float* k_assign_centroids, float* k_box_min, float* k_box_max, int32_t* k_sizes,
                        int32_t* k_count, int32_t* full_flag, int32_t* k_stage_offs, int32_t* k_stage_of,
                        float* tau_used, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!K || !k_labels || !k_centroids || !k_assign_centroids || !k_sizes || !k_count || !full_flag || !tau_used)
    return fail(ADACLUSTER_E_BADARG, "kcluster: NULL tensor pointer");
  if ((k_box_min == nullptr) != (k_box_max == nullptr))
    return fail(ADACLUSTER_E_BADARG, "kcluster: pass both boxes or neither");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  prof_begin((hipStream_t)stream);
  rc = run_kcluster(p, w, (hipStream_t)stream, K, k_labels, k_centroids, k_assign_centroids, k_box_min, k_box_max,
                    k_sizes, k_count, full_flag, k_stage_offs, k_stage_of, tau_used, nullptr);
  prof_mark(EV_KCLUSTER, (hipStream_t)stream, EV_START);
  return rc;
}

int adacluster_compactness(const adacluster_params* p, const void* K, const int32_t* k_labels,
                           const float* k_centroids, float* k_mse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!K || !k_labels || !k_centroids || !k_mse) return fail(ADACLUSTER_E_BADARG, "compactness: NULL pointer");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  RET_IF(launch_mse((hipStream_t)stream, p->dtype, p->d, p->H, p->N, capacity(p), K, k_labels, k_centroids, w.tau_part,
                    k_mse));
  return 0;
}

int adacluster_compactness_noalloc(const adacluster_params* p, const void* K, const int32_t* k_labels,
                                   const float* k_centroids, float* k_mse, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!K || !k_labels || !k_centroids || !k_mse) return fail(ADACLUSTER_E_BADARG, "compactness_noalloc: NULL pointer");
  const size_t need = (size_t)p->H * (size_t)((p->N + 1023) / 1024);   // one partial sum per head and 1024 rows
  if (need > STATIC_SCRATCH_DOUBLES)
    return fail(ADACLUSTER_E_UNSUPPORTED, "compactness_noalloc: H * ceil(N/1024) = %zu exceeds the %zu partial sums of the "
                "library's scratch array; use adacluster_compactness with a workspace", need, STATIC_SCRATCH_DOUBLES);
  double* part = static_scratch();
  if (!part) return fail(ADACLUSTER_E_INTERNAL, "compactness_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(hipGetLastError()));
  // every partial sum the second kernel reads is written by the first: nothing has to start at zero
  RET_IF(launch_mse((hipStream_t)stream, p->dtype, p->d, p->H, p->N, capacity(p), K, k_labels, k_centroids, part, k_mse));
  return 0;
}

int adacluster_quest_scores(int32_t H, int32_t Lq, int32_t Lk, int32_t d, int32_t dtype, int32_t form, int32_t clamp,
                            const void* Q, const void* R_pos, const void* R_neg, float* S, void* stream) {
  if (H < 1 || Lq < 1 || Lk < 1) return fail(ADACLUSTER_E_BADSHAPE, "quest_scores: H, Lq and Lk must be >= 1");
  if (H > 65535) return fail(ADACLUSTER_E_BADSHAPE, "quest_scores: H must be <= 65535");
  if (d != 64 && d != 128) return fail(ADACLUSTER_E_BADSHAPE, "quest_scores: d must be 64 or 128 (d=%d)", d);
  if (dtype != ADACLUSTER_F32 && dtype != ADACLUSTER_BF16) return fail(ADACLUSTER_E_BADDTYPE, "quest_scores: unknown dtype %d", dtype);
  if (form != ADACLUSTER_QUEST_ALU && form != ADACLUSTER_QUEST_MFMA) return fail(ADACLUSTER_E_BADARG, "quest_scores: unknown form %d", form);
  if (form == ADACLUSTER_QUEST_MFMA && dtype != ADACLUSTER_BF16)
    return fail(ADACLUSTER_E_UNSUPPORTED, "quest_scores: the matrix-core form takes bf16 inputs");
  if ((long long)Lq * Lk >= (1ll << 40) || (long long)Lq * d >= (1ll << 40) || (long long)Lk * d >= (1ll << 40))
    return fail(ADACLUSTER_E_BADSHAPE, "quest_scores: problem too large");
  if ((Lq + 63) / 64 > 2147483647 / 2 || (Lk + 63) / 64 > 65535) return fail(ADACLUSTER_E_BADSHAPE, "quest_scores: Lk must be <= 4194240");
  if (!Q || !R_pos || !R_neg || !S) return fail(ADACLUSTER_E_BADARG, "quest_scores: NULL pointer");
  RET_IF(launch_quest_scores((hipStream_t)stream, dtype, form, clamp ? 1 : 0, H, Lq, Lk, d, Q, R_pos, R_neg, S));
  return 0;
}

int adacluster_select(const adacluster_params* p, const float* q_centroids, const float* q_mean_norm,
                      const float* k_centroids, const float* k_box_min, const float* k_box_max,
                      const int32_t* k_sizes, const int32_t* k_count, const int32_t* full_flag,
                      int32_t* sel_idx, int32_t* sel_cnt, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!q_centroids || !q_mean_norm || !k_centroids || !k_sizes || !k_count || !full_flag || !sel_idx || !sel_cnt)
    return fail(ADACLUSTER_E_BADARG, "select: NULL tensor pointer");
  if (p->score_mode == ADACLUSTER_SCORE_BOX && (!k_box_min || !k_box_max))
    return fail(ADACLUSTER_E_BADARG, "select: BOX scores need k_box_min and k_box_max");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
  RET_IF(launch_select((hipStream_t)stream, p->H, p->q_clusters, capacity(p), p->d, p->score_mode, p->select_mode,
                       p->topk, p->top_p, scale, q_centroids, q_mean_norm, k_centroids, k_box_min, k_box_max, k_sizes,
                       k_count, full_flag, sel_idx, sel_cnt, capacity(p), w.scores));
  return 0;
}

int adacluster_sparse_attn(const adacluster_params* p, const void* Q, const void* K, const void* V,
                           const int32_t* q_labels, const int32_t* k_labels, const int32_t* k_count,
                           const int32_t* sel_idx, const int32_t* sel_cnt, void* O, void* ws, size_t ws_bytes,
                           void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!Q || !K || !V || !q_labels || !k_labels || !k_count || !sel_idx || !sel_cnt || !O)
    return fail(ADACLUSTER_E_BADARG, "sparse_attn: NULL tensor pointer");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  const Dims D = dims_of(p);
  hipStream_t st = (hipStream_t)stream;
  prof_begin(st);
  RET_IF(launch_sort(st, D.H, D.N, D.N, D.Cq, q_labels, nullptr, nullptr, 0, nullptr, 0, nullptr, 0, w.perm_q, w.offs_q,
                     D.Cq + 1, w.sort));
  RET_IF(launch_sort(st, D.H, D.N, D.N, D.cap, k_labels, nullptr, nullptr, 0, k_count, 1, nullptr, 0, w.perm_k, w.offs_k,
                     D.cap + 1, w.sort));
  prof_mark(EV_SELECT, st);   // (time of the two label sorts when called stand-alone)
  if (!rows_in_place(p) && (rc = run_permute(p, w, st, K, V, -1))) return rc;
  return run_plan_attention(p, w, st, Q, O, k_count, sel_idx, sel_cnt, -1, nullptr, K, V);
}

int adacluster_attn(const adacluster_params* p, const void* Q, const void* K, const void* V, void* O,
                    const adacluster_outputs* outs, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!Q || !K || !V || !O) return fail(ADACLUSTER_E_BADARG, "attn: NULL tensor pointer");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  adacluster_outputs o;
  memset(&o, 0, sizeof(o));
  if (outs) o = *outs;
  if ((o.k_box_min == nullptr) != (o.k_box_max == nullptr))
    return fail(ADACLUSTER_E_BADARG, "attn: pass both boxes or neither");
  const bool need_box = p->score_mode == ADACLUSTER_SCORE_BOX;
#define PICK(f, home) auto f = o.f ? o.f : home
  PICK(q_labels, w.q_labels); PICK(q_centroids, w.q_centroids); PICK(q_assign_centroids, w.q_assign);
  PICK(q_sizes, w.q_sizes); PICK(q_mean_norm, w.q_mean_norm);
  PICK(k_labels, w.k_labels); PICK(k_centroids, w.k_centroids); PICK(k_assign_centroids, w.k_assign);
  PICK(k_sizes, w.k_sizes); PICK(k_count, w.k_count); PICK(full_flag, w.full_flag);
  PICK(sel_idx, w.sel_idx); PICK(sel_cnt, w.sel_cnt);
#undef PICK
  float* k_bmin = o.k_box_min ? o.k_box_min : (need_box ? w.k_bmin : nullptr);
  float* k_bmax = o.k_box_max ? o.k_box_max : (need_box ? w.k_bmax : nullptr);
  float* tau_used = o.tau_used ? o.tau_used : w.tau + 2;
  hipStream_t st = (hipStream_t)stream;
  if (p->q_init_mode == 1 && !o.q_centroids)
    return fail(ADACLUSTER_E_BADARG, "attn: q_init_mode 1 needs outs->q_centroids");
  if (p->k_init_mode == 1 && (!o.k_centroids || !o.k_count || !o.full_flag))
    return fail(ADACLUSTER_E_BADARG, "attn: k_init_mode 1 needs outs->k_centroids, k_count and full_flag");
  // The two clusterings do not depend on each other and both are chains of small kernels: the
  // query clustering goes to a second stream, forked from and joined back to the caller's.
  AuxStream* aux = aux_stream();
  if (!aux) return fail(ADACLUSTER_E_INTERNAL, "could not create the second stream: %s", hipGetErrorString(hipGetLastError()));
  prof_begin(st);
  if (hipEventRecord(aux->fork, st) != hipSuccess || hipStreamWaitEvent(aux->s, aux->fork, 0) != hipSuccess)
    return fail(ADACLUSTER_E_INTERNAL, "stream fork failed: %s", hipGetErrorString(hipGetLastError()));
  // From here on work may sit on the second stream.  No error leaves this function with that work still
  // running: where the event join itself fails (or an error comes after the join of the first fork), the
  // host waits for the second stream before it reports the error.
  auto drained = [&](int code) { (void)hipStreamSynchronize(aux->s); return code; };
  hipStream_t qs = aux->s;      // (measured: run in front of Algorithm 1 on the caller's stream instead, every configuration is 1-6 % slower)
  rc = run_qcluster(p, w, qs, Q, q_labels, q_centroids, q_assign_centroids, q_sizes, q_mean_norm);
  prof_mark(EV_QCLUSTER, qs, EV_START);
  if (hipEventRecord(aux->join, qs) != hipSuccess) return drained(fail(ADACLUSTER_E_INTERNAL, "stream join failed"));
  int kc_bound = capacity(p);
  int rck = rc ? 0 : run_kcluster(p, w, st, K, k_labels, k_centroids, k_assign_centroids, k_bmin, k_bmax, k_sizes,
                                   k_count, full_flag, o.k_stage_offs, o.k_stage_of, tau_used, &kc_bound, aux->fork);
  prof_mark(EV_KCLUSTER, st, EV_START);
  // The K/V permutation needs only the key label sort, which is final before the last centroid
  // update of the key clustering: it goes to the second stream too (behind the query clustering
  // there) and runs beside that update, the selection and the planning.
  const bool fork2 = !rc && !rck && !rows_in_place(p);     // (bf16 has no permutation step)
  int rcp = 0;
  if (fork2) {
    if (hipStreamWaitEvent(aux->s, aux->fork, 0) != hipSuccess)
      return drained(fail(ADACLUSTER_E_INTERNAL, "stream fork failed: %s", hipGetErrorString(hipGetLastError())));
    rcp = run_permute(p, w, aux->s, K, V, EV_KSORT);
    if (hipEventRecord(aux->join2, aux->s) != hipSuccess) return drained(fail(ADACLUSTER_E_INTERNAL, "stream join failed"));
  }
  if (hipStreamWaitEvent(st, aux->join, 0) != hipSuccess) return drained(fail(ADACLUSTER_E_INTERNAL, "stream join failed"));
  if (rc || rck || rcp) {
    // whatever was queued on the second stream is joined before the error is reported
    if (fork2 && hipStreamWaitEvent(st, aux->join2, 0) != hipSuccess) return drained(fail(ADACLUSTER_E_INTERNAL, "stream join failed"));
    return rc ? rc : (rck ? rck : rcp);
  }
  prof_mark(EV_JOIN, st);
  const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
  rc = launch_select(st, p->H, p->q_clusters, capacity(p), p->d, p->score_mode, p->select_mode, p->topk, p->top_p,
                     scale, q_centroids, q_mean_norm, k_centroids, k_bmin, k_bmax, k_sizes, k_count, full_flag,
                     sel_idx, sel_cnt, kc_bound, w.scores);
  if (rc) return drained(rc == ADACLUSTER_E_INTERNAL ? fail(rc, "HIP launch failed: %s", hipGetErrorString(hipGetLastError())) : rc);
  prof_mark(EV_SELECT, st, EV_JOIN);
  // both label sorts were left in the workspace by the clustering steps; the attention step joins the
  // permutation of K and V (second stream) before its first kernel that reads it
  rc = run_plan_attention(p, w, st, Q, O, k_count, sel_idx, sel_cnt, EV_SELECT, fork2 ? aux->join2 : nullptr, K, V);
  return rc ? drained(rc) : 0;
}

int adacluster_dense_attn(const adacluster_params* p, const void* Q, const void* K, const void* V, void* O,
                          void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!Q || !K || !V || !O) return fail(ADACLUSTER_E_BADARG, "dense_attn: NULL tensor pointer");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  const Dims D = dims_of(p);
  hipStream_t st = (hipStream_t)stream;
  const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)D.d);
  prof_begin(st);
  RET_IF(launch_plan_dense(st, D.H, D.N, D.maxtiles, attn_block_rows(p->dtype, D.d, D.N, 1), w.rng_start, w.rng_pre, w.rng_cnt, w.tiles, w.ntiles,
                           D.d * (int)esize(p), p->dtype == ADACLUSTER_BF16 ? w.krow : nullptr, attn_krow_stride(D.N)));
  prof_mark(EV_PLAN, st);
  RET_IF(launch_attention(st, p->dtype, D.d, D.H, D.N, 1, D.maxtiles, 1, scale, Q, K, V, O, nullptr, w.tiles,
                          w.ntiles, w.rng_start, w.rng_pre, w.rng_cnt, nullptr, nullptr, nullptr, nullptr,
                          w.krow, attn_krow_stride(D.N)));
  prof_mark(EV_ATTN, st);
  return 0;
}

int adacluster_stats_fetch(const adacluster_params* p, void* ws, size_t ws_bytes, adacluster_head_stats* host_stats,
                           void* stream) {
  int rc = check_params(p);
  if (rc) return rc;
  if (!host_stats) return fail(ADACLUSTER_E_BADARG, "stats_fetch: host_stats is NULL");
  WS w;
  if ((rc = check_ws(p, ws, ws_bytes, &w))) return rc;
  const Dims D = dims_of(p);
  hipStream_t st = (hipStream_t)stream;
  RET_IF(launch_attn_stats(st, D.H, D.Cq, D.maxr, D.maxtiles, w.kstate, w.tiles, w.ntiles, w.rng_pre, w.rng_cnt, w.stats));
  if (hipMemcpyAsync(host_stats, w.stats, (size_t)D.H * sizeof(adacluster_head_stats), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return fail(ADACLUSTER_E_INTERNAL, "stats_fetch: copy to the host failed: %s", hipGetErrorString(hipGetLastError()));
  return 0;
}

int adacluster_mfma_probe(int32_t iters, float* sink, size_t sink_floats, double* flops, void* stream) {
  if (iters < 1 || !sink || !flops) return fail(ADACLUSTER_E_BADARG, "mfma_probe: iters >= 1, sink and flops must be given");
  RET_IF(launch_mfma_probe((hipStream_t)stream, iters, sink, sink_floats, flops));
  return 0;
}

int adacluster_profile_enable(int on) {
  if (on && !g_prof.enabled) {
    for (int i = 0; i < EV_COUNT; ++i)
      if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return fail(ADACLUSTER_E_INTERNAL, "hipEventCreate failed");
    g_prof.enabled = true;
  } else if (!on && g_prof.enabled) {
    for (int i = 0; i < EV_COUNT; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    g_prof.enabled = false;
  }
  return 0;
}

int adacluster_profile_read(float* ms) {
  if (!ms) return fail(ADACLUSTER_E_BADARG, "ms is NULL");
  if (!g_prof.enabled) return fail(ADACLUSTER_E_UNSUPPORTED, "profiling is not enabled");
  int prev = -1;
  for (int i = 0; i < EV_STAGES; ++i) {
    if (i > 0) ms[i - 1] = -1.f;
    if (!g_prof.recorded[i]) continue;
    if (hipEventSynchronize(g_prof.ev[i]) != hipSuccess) return fail(ADACLUSTER_E_INTERNAL, "event sync failed");
    const int from = g_prof.from[i] >= 0 ? g_prof.from[i] : prev;
    if (from >= 0 && i > 0) {
      if (hipEventSynchronize(g_prof.ev[from]) != hipSuccess) return fail(ADACLUSTER_E_INTERNAL, "event sync failed");
      float t = 0.f;
      if (hipEventElapsedTime(&t, g_prof.ev[from], g_prof.ev[i]) != hipSuccess)
        return fail(ADACLUSTER_E_INTERNAL, "event elapsed failed");
      ms[i - 1] = t;
    }
    prev = i;
  }
  return 0;
}

}  // extern "C"
