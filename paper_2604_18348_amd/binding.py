"""ctypes binding of libadacluster.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/adacluster.h),
takes torch CUDA tensors, allocates the outputs with torch and passes raw device
pointers plus the current torch stream.  No step of the method runs in Python,
and there is no fallback: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, asdict

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ADACLUSTER_LIB") or os.path.join(_HERE, "_lib", "libadacluster.so")
MAX_STAGES = 16

F32, BF16 = 0, 1
SCORE_TQ, SCORE_BOX, SCORE_DOT = 0, 1, 2
SELECT_TOPK, SELECT_TOPP = 0, 1


class CParams(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("q_clusters", ctypes.c_int32),
                ("q_iters", ctypes.c_int32), ("k_iters", ctypes.c_int32),
                ("q_init_mode", ctypes.c_int32), ("k_init_mode", ctypes.c_int32), ("k_m0", ctypes.c_int32),
                ("k_m_min", ctypes.c_int32), ("k_max_clusters", ctypes.c_int32),
                ("k_max_stages", ctypes.c_int32), ("tau_abs", ctypes.c_float),
                ("tau_factor", ctypes.c_float), ("min_unassigned_frac", ctypes.c_float),
                ("score_mode", ctypes.c_int32), ("select_mode", ctypes.c_int32),
                ("topk", ctypes.c_int32), ("top_p", ctypes.c_float),
                ("softmax_scale", ctypes.c_float), ("q_no_norm", ctypes.c_int32)]


class COutputs(ctypes.Structure):
    _names = ["q_labels", "q_centroids", "q_assign_centroids", "q_sizes", "q_mean_norm",
              "k_labels", "k_centroids", "k_assign_centroids", "k_box_min", "k_box_max",
              "k_sizes", "k_count", "full_flag", "k_stage_offs", "k_stage_of", "tau_used",
              "sel_idx", "sel_cnt"]
    _fields_ = [(n, ctypes.c_void_p) for n in _names]


class CHeadStats(ctypes.Structure):
    _fields_ = [("k_count", ctypes.c_int32), ("full_flag", ctypes.c_int32), ("stages", ctypes.c_int32),
                ("q_tiles", ctypes.c_int32), ("unassigned", ctypes.c_int32 * (MAX_STAGES + 1)),
                ("reserved", ctypes.c_int32), ("executed_pairs", ctypes.c_int64), ("issued_pairs", ctypes.c_int64)]


@dataclass
class Params:
    H: int
    N: int
    d: int
    dtype: int = BF16
    q_clusters: int = 65
    q_iters: int = 3
    k_iters: int = 3
    q_init_mode: int = 0
    k_init_mode: int = 0
    k_m0: int = 100
    k_m_min: int = 16
    k_max_clusters: int = 1024
    k_max_stages: int = 10
    tau_abs: float = 0.0
    tau_factor: float = 1.5
    min_unassigned_frac: float = 0.0
    score_mode: int = SCORE_TQ
    select_mode: int = SELECT_TOPK
    topk: int = 64
    top_p: float = 0.9
    softmax_scale: float = 0.0
    q_no_norm: int = 0

    def c(self) -> CParams:
        return CParams(**asdict(self))

    @property
    def cap(self) -> int:
        return self.k_max_clusters + self.k_m0


_lib = None


def load_library():
    """Loads the shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_18348_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(CParams)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.adacluster_centroid_capacity.argtypes = [P]
    lib.adacluster_workspace_bytes.argtypes = [P, ctypes.POINTER(sz)]
    lib.adacluster_last_error.argtypes = [ctypes.c_char_p, sz]
    lib.adacluster_qcluster.argtypes = [P] + [vp] * 6 + [vp, sz, vp]
    lib.adacluster_kcluster.argtypes = [P] + [vp] * 12 + [vp, sz, vp]
    lib.adacluster_select.argtypes = [P] + [vp] * 10 + [vp, sz, vp]
    lib.adacluster_sparse_attn.argtypes = [P] + [vp] * 9 + [vp, sz, vp]
    lib.adacluster_attn.argtypes = [P] + [vp] * 4 + [ctypes.POINTER(COutputs), vp, sz, vp]
    lib.adacluster_dense_attn.argtypes = [P] + [vp] * 4 + [vp, sz, vp]
    lib.adacluster_compactness.argtypes = [P] + [vp] * 4 + [vp, sz, vp]
    lib.adacluster_compactness_noalloc.argtypes = [P] + [vp] * 4 + [vp]
    lib.adacluster_mfma_probe.argtypes = [ctypes.c_int32, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    lib.adacluster_stats_fetch.argtypes = [P, vp, sz, ctypes.POINTER(CHeadStats), vp]
    lib.adacluster_quest_scores.argtypes = [ctypes.c_int32] * 7 + [vp] * 5
    lib.adacluster_profile_enable.argtypes = [ctypes.c_int]
    lib.adacluster_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float)]
    for n in ("profile_enable", "profile_read", "centroid_capacity", "workspace_bytes", "last_error", "qcluster", "kcluster", "select",
              "sparse_attn", "attn", "dense_attn", "compactness", "compactness_noalloc", "quest_scores", "stats_fetch", "mfma_probe"):
        getattr(lib, "adacluster_" + n).restype = ctypes.c_int
    _lib = lib
    return lib


EXPORTED = ["adacluster_centroid_capacity", "adacluster_workspace_bytes", "adacluster_last_error",
            "adacluster_qcluster", "adacluster_kcluster", "adacluster_select",
            "adacluster_sparse_attn", "adacluster_attn", "adacluster_dense_attn", "adacluster_compactness",
            "adacluster_compactness_noalloc", "adacluster_quest_scores", "adacluster_stats_fetch", "adacluster_mfma_probe",
            "adacluster_profile_enable", "adacluster_profile_read"]

STAGES = ["qcluster", "kcluster", "select", "permute", "plan", "attention", "kreduce"]


def adacluster_profile_enable(on: bool):
    _check(load_library().adacluster_profile_enable(1 if on else 0), "profile_enable")


def adacluster_profile_read():
    """Stage times (ms) of the last profiled call as a dict; stages that did not run are absent."""
    arr = (ctypes.c_float * len(STAGES))()
    _check(load_library().adacluster_profile_read(arr), "profile_read")
    return {n: float(arr[i]) for i, n in enumerate(STAGES) if arr[i] >= 0}


class AdaClusterError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        buf = ctypes.create_string_buffer(256)
        load_library().adacluster_last_error(buf, 256)
        raise AdaClusterError(f"{what} failed with code {rc}: {buf.value.decode()}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _tdtype(p: Params):
    return torch.bfloat16 if p.dtype == BF16 else torch.float32


def _check_qkv(p: Params, *ts):
    for t in ts:
        if not (t.is_cuda and t.is_contiguous() and t.dtype == _tdtype(p) and tuple(t.shape) == (p.H, p.N, p.d)):
            raise ValueError("tensor must be a contiguous CUDA tensor [H,N,d] of the params dtype")


def adacluster_workspace_bytes(p: Params) -> int:
    out = ctypes.c_size_t(0)
    cp = p.c()
    _check(load_library().adacluster_workspace_bytes(ctypes.byref(cp), ctypes.byref(out)), "workspace_bytes")
    return out.value


_ws_cache = {}


def workspace(p: Params, device="cuda"):
    """A torch uint8 workspace of the required size (cached per size and device)."""
    n = adacluster_workspace_bytes(p)
    key = (str(device), n)
    if key not in _ws_cache:
        _ws_cache.clear()
        _ws_cache[key] = torch.empty(n + 256, dtype=torch.uint8, device=device)
    t = _ws_cache[key]
    off = (-t.data_ptr()) % 256
    return t[off:off + n]


def adacluster_qcluster(p: Params, Q, q_centroids_init=None, ws=None):
    _check_qkv(p, Q)
    dev = Q.device
    ws = workspace(p, dev) if ws is None else ws
    i32, f32 = torch.int32, torch.float32
    out = dict(
        q_labels=torch.empty((p.H, p.N), dtype=i32, device=dev),
        q_centroids=(q_centroids_init.clone() if q_centroids_init is not None
                     else torch.empty((p.H, p.q_clusters, p.d), dtype=f32, device=dev)),
        q_assign_centroids=torch.empty((p.H, p.q_clusters, p.d), dtype=f32, device=dev),
        q_sizes=torch.empty((p.H, p.q_clusters), dtype=i32, device=dev),
        q_mean_norm=torch.empty((p.H, p.q_clusters), dtype=f32, device=dev))
    cp = p.c()
    _check(load_library().adacluster_qcluster(
        ctypes.byref(cp), _ptr(Q), _ptr(out["q_labels"]), _ptr(out["q_centroids"]),
        _ptr(out["q_assign_centroids"]), _ptr(out["q_sizes"]), _ptr(out["q_mean_norm"]),
        _ptr(ws), ws.numel(), _stream()), "adacluster_qcluster")
    return out


def adacluster_kcluster(p: Params, K, want_box=True, ws=None, prev=None):
    """`prev` (warm start, k_init_mode 1): dict with k_centroids, k_count, full_flag of an earlier call."""
    _check_qkv(p, K)
    dev = K.device
    ws = workspace(p, dev) if ws is None else ws
    i32, f32 = torch.int32, torch.float32
    cap = p.cap
    out = dict(
        k_labels=torch.empty((p.H, p.N), dtype=i32, device=dev),
        k_centroids=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev),
        k_assign_centroids=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev),
        k_box_min=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev) if want_box else None,
        k_box_max=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev) if want_box else None,
        k_sizes=torch.empty((p.H, cap), dtype=i32, device=dev),
        k_count=torch.empty((p.H,), dtype=i32, device=dev),
        full_flag=torch.empty((p.H,), dtype=i32, device=dev),
        k_stage_offs=torch.empty((p.H, MAX_STAGES + 1), dtype=i32, device=dev),
        k_stage_of=torch.empty((p.H, p.N), dtype=i32, device=dev),
        tau_used=torch.zeros((1,), dtype=f32, device=dev))
    if prev is not None:
        out["k_centroids"] = prev["k_centroids"].clone()
        out["k_count"] = prev["k_count"].clone()
        out["full_flag"] = prev["full_flag"].clone()
    cp = p.c()
    _check(load_library().adacluster_kcluster(
        ctypes.byref(cp), _ptr(K), _ptr(out["k_labels"]), _ptr(out["k_centroids"]),
        _ptr(out["k_assign_centroids"]), _ptr(out["k_box_min"]), _ptr(out["k_box_max"]),
        _ptr(out["k_sizes"]), _ptr(out["k_count"]), _ptr(out["full_flag"]), _ptr(out["k_stage_offs"]),
        _ptr(out["k_stage_of"]), _ptr(out["tau_used"]), _ptr(ws), ws.numel(), _stream()),
        "adacluster_kcluster")
    return out


def adacluster_select(p: Params, q_centroids, q_mean_norm, k_centroids, k_box_min, k_box_max, k_sizes,
                      k_count, full_flag, ws=None):
    dev = q_centroids.device
    ws = workspace(p, dev) if ws is None else ws
    sel_idx = torch.empty((p.H, p.q_clusters, p.cap), dtype=torch.int32, device=dev)
    sel_cnt = torch.empty((p.H, p.q_clusters), dtype=torch.int32, device=dev)
    cp = p.c()
    _check(load_library().adacluster_select(
        ctypes.byref(cp), _ptr(q_centroids), _ptr(q_mean_norm), _ptr(k_centroids), _ptr(k_box_min),
        _ptr(k_box_max), _ptr(k_sizes), _ptr(k_count), _ptr(full_flag), _ptr(sel_idx), _ptr(sel_cnt),
        _ptr(ws), ws.numel(), _stream()), "adacluster_select")
    return sel_idx, sel_cnt


def adacluster_sparse_attn(p: Params, Q, K, V, q_labels, k_labels, k_count, sel_idx, sel_cnt, out=None, ws=None):
    _check_qkv(p, Q, K, V)
    ws = workspace(p, Q.device) if ws is None else ws
    O = torch.empty_like(Q) if out is None else out
    cp = p.c()
    _check(load_library().adacluster_sparse_attn(
        ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(q_labels), _ptr(k_labels), _ptr(k_count),
        _ptr(sel_idx), _ptr(sel_cnt), _ptr(O), _ptr(ws), ws.numel(), _stream()), "adacluster_sparse_attn")
    return O


def adacluster_compactness(p: Params, K, k_labels, k_centroids, ws=None):
    """Per-head mean squared reconstruction error of a key clustering (Sec. 3.2.1) -> float32 [H]."""
    ws = workspace(p, K.device) if ws is None else ws
    mse = torch.empty((p.H,), dtype=torch.float32, device=K.device)
    cp = p.c()
    _check(load_library().adacluster_compactness(
        ctypes.byref(cp), _ptr(K), _ptr(k_labels), _ptr(k_centroids), _ptr(mse), _ptr(ws), ws.numel(), _stream()),
        "adacluster_compactness")
    return mse


def adacluster_compactness_noalloc(p: Params, K, k_labels, k_centroids, out=None):
    """adacluster_compactness without a workspace: partial sums in the library's own device array.  `out`
    lets the caller pass the [H] float32 result tensor, so that the call itself allocates nothing."""
    mse = torch.empty((p.H,), dtype=torch.float32, device=K.device) if out is None else out
    cp = p.c()
    _check(load_library().adacluster_compactness_noalloc(
        ctypes.byref(cp), _ptr(K), _ptr(k_labels), _ptr(k_centroids), _ptr(mse), _stream()),
        "adacluster_compactness_noalloc")
    return mse


def adacluster_stats_fetch(p: Params, ws):
    """Per-head figures of the last adacluster_attn call on `ws` -> list of dicts (waits for the stream)."""
    arr = (CHeadStats * p.H)()
    cp = p.c()
    _check(load_library().adacluster_stats_fetch(ctypes.byref(cp), _ptr(ws), ws.numel(), arr, _stream()),
           "adacluster_stats_fetch")
    return [dict(k_count=r.k_count, full_flag=r.full_flag, stages=r.stages, q_tiles=r.q_tiles,
                 unassigned=list(r.unassigned), executed_pairs=r.executed_pairs, issued_pairs=r.issued_pairs)
            for r in arr]


def adacluster_mfma_probe(iters: int, sink):
    """Enqueues the register-only MFMA loop on the current stream; returns the flops of the launch."""
    fl = ctypes.c_double(0.0)
    _check(load_library().adacluster_mfma_probe(int(iters), _ptr(sink), sink.numel(), ctypes.byref(fl), _stream()),
           "adacluster_mfma_probe")
    return fl.value


QUEST_ALU, QUEST_MFMA = 0, 1


def adacluster_quest_scores(Q, R_pos, R_neg, form, clamp=False, out=None):
    """Quest scores (Eq. 1 / Eq. 2) of query rows Q [H,Lq,d] against pages with maxima R_pos and minima
    R_neg [H,Lk,d] -> float32 [H,Lq,Lk]."""
    H, Lq, d = Q.shape
    Lk = R_pos.shape[1]
    assert R_pos.shape == (H, Lk, d) and R_neg.shape == (H, Lk, d)
    assert Q.dtype == R_pos.dtype == R_neg.dtype and Q.dtype in (torch.float32, torch.bfloat16)
    assert Q.is_contiguous() and R_pos.is_contiguous() and R_neg.is_contiguous()
    S = torch.empty((H, Lq, Lk), dtype=torch.float32, device=Q.device) if out is None else out
    _check(load_library().adacluster_quest_scores(
        H, Lq, Lk, d, BF16 if Q.dtype == torch.bfloat16 else F32, int(form), 1 if clamp else 0,
        _ptr(Q), _ptr(R_pos), _ptr(R_neg), _ptr(S), _stream()), "adacluster_quest_scores")
    return S


def alloc_outputs(p: Params, dev, want_box=False, want_stage=True):
    """Device tensors for every intermediate of the fused call."""
    i32, f32 = torch.int32, torch.float32
    cap = p.cap
    o = dict(
        q_labels=torch.empty((p.H, p.N), dtype=i32, device=dev),
        q_centroids=torch.empty((p.H, p.q_clusters, p.d), dtype=f32, device=dev),
        q_assign_centroids=torch.empty((p.H, p.q_clusters, p.d), dtype=f32, device=dev),
        q_sizes=torch.empty((p.H, p.q_clusters), dtype=i32, device=dev),
        q_mean_norm=torch.empty((p.H, p.q_clusters), dtype=f32, device=dev),
        k_labels=torch.empty((p.H, p.N), dtype=i32, device=dev),
        k_centroids=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev),
        k_assign_centroids=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev),
        k_box_min=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev) if want_box else None,
        k_box_max=torch.zeros((p.H, cap, p.d), dtype=f32, device=dev) if want_box else None,
        k_sizes=torch.empty((p.H, cap), dtype=i32, device=dev),
        k_count=torch.empty((p.H,), dtype=i32, device=dev),
        full_flag=torch.empty((p.H,), dtype=i32, device=dev),
        k_stage_offs=torch.empty((p.H, MAX_STAGES + 1), dtype=i32, device=dev) if want_stage else None,
        k_stage_of=torch.empty((p.H, p.N), dtype=i32, device=dev) if want_stage else None,
        tau_used=torch.empty((1,), dtype=f32, device=dev),
        sel_idx=torch.empty((p.H, p.q_clusters, cap), dtype=i32, device=dev),
        sel_cnt=torch.empty((p.H, p.q_clusters), dtype=i32, device=dev))
    return o


def adacluster_attn(p: Params, Q, K, V, outs=None, out=None, ws=None):
    """Fused call.  `outs`: dict from alloc_outputs (or None to keep intermediates in the workspace)."""
    _check_qkv(p, Q, K, V)
    ws = workspace(p, Q.device) if ws is None else ws
    O = torch.empty_like(Q) if out is None else out
    co = None
    if outs is not None:
        co = COutputs(**{n: (outs[n].data_ptr() if outs.get(n) is not None else None) for n in COutputs._names})
    cp = p.c()
    _check(load_library().adacluster_attn(
        ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), ctypes.byref(co) if co is not None else None,
        _ptr(ws), ws.numel(), _stream()), "adacluster_attn")
    return O


def adacluster_dense_attn(p: Params, Q, K, V, out=None, ws=None):
    _check_qkv(p, Q, K, V)
    ws = workspace(p, Q.device) if ws is None else ws
    O = torch.empty_like(Q) if out is None else out
    cp = p.c()
    _check(load_library().adacluster_dense_attn(
        ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(ws), ws.numel(), _stream()),
        "adacluster_dense_attn")
    return O
