"""ctypes binding of libbaklava: argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels; nothing here
computes.  PyTorch tensors are used as device memory (`.data_ptr()`) and for
the current stream.  Importing this module does not load the library; the
first call does, and fails loudly if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbaklava.so")

OK, EINVAL, EINFEASIBLE, ECAPACITY, EHIP, ESTATE, ENOMEM = range(7)
BF16, F32 = 0, 1
POLICY_SCORE, POLICY_STREAMING = 0, 1
OPT_CHUNK_TOKENS, OPT_KERNEL, OPT_TIME_KERNEL, OPT_CHUNK_TOKENS_WHOLE, OPT_TARGET_ITEMS, OPT_TARGET_ITEMS_WHOLE = 1, 2, 3, 4, 5, 6
OPT_TRACK_SCORES, OPT_TILED_SELECT_ROWS = 7, 8
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA = 0, 1, 2

EXPORTS = [
    "baklava_strerror", "baklava_last_hip_error", "baklava_alloc_proportional",
    "baklava_alloc_threshold", "baklava_layout", "baklava_plan_schedule", "baklava_workspace_bytes",
    "baklava_create",
    "baklava_destroy", "baklava_set_option", "baklava_reset", "baklava_set_lengths",
    "baklava_append", "baklava_decode_attn", "baklava_append_decode_attn", "baklava_compact", "baklava_lengths", "baklava_profile_read",
    "baklava_stream_probe", "baklava_profile_workspace_bytes", "baklava_profile_similarity", "baklava_kv_importance", "baklava_prefill_scores", "baklava_layer_workspace_bytes", "baklava_layer_similarity",
    "baklava_alloc_two_level", "baklava_layer_similarity_static", "baklava_append_decode_attn_replay",
    "baklava_sync_lengths", "baklava_flush_scores",
]


class BaklavaError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({strerror(status)})")


class Desc(C.Structure):
    _fields_ = [
        ("L", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("batch", C.c_int32),
        ("dtype", C.c_int32), ("sink", C.c_int32), ("recent", C.c_int32), ("policy", C.c_int32),
        ("track_scores", C.c_int32),
        ("k", C.c_void_p), ("v", C.c_void_p), ("score", C.c_void_p), ("pos", C.c_void_p),
        ("off", C.c_void_p), ("cap", C.c_void_p), ("len", C.c_void_p), ("budget", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class WorkItem(C.Structure):
    _fields_ = [("cache", C.c_int32), ("start", C.c_int32), ("count", C.c_int32), ("slot", C.c_int32),
                ("nsplit", C.c_int32), ("reserved", C.c_int32), ("row0", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2502_13176_amd.build). "
            "There is no fallback path.")
    L = C.CDLL(LIB_PATH)
    i32p, i64p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_double)
    L.baklava_strerror.restype = C.c_char_p
    L.baklava_strerror.argtypes = [C.c_int]
    L.baklava_last_hip_error.restype = C.c_int
    L.baklava_alloc_proportional.argtypes = [f64p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, i32p]
    L.baklava_alloc_threshold.argtypes = [f64p, C.c_int32, i32p, C.c_double, C.c_double, i32p]
    L.baklava_layout.argtypes = [i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, i64p, i32p, i64p]
    L.baklava_plan_schedule.argtypes = [i64p, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_int64, C.POINTER(WorkItem), i64p]
    L.baklava_workspace_bytes.restype = C.c_size_t
    L.baklava_workspace_bytes.argtypes = [C.POINTER(Desc), i32p, i32p]
    L.baklava_create.argtypes = [C.POINTER(Desc), i64p, i32p, i32p, i32p, C.POINTER(C.c_void_p)]
    L.baklava_destroy.argtypes = [C.c_void_p]
    L.baklava_set_option.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
    L.baklava_reset.argtypes = [C.c_void_p, C.c_void_p]
    L.baklava_set_lengths.argtypes = [C.c_void_p, i32p, C.c_void_p]
    L.baklava_append.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
    L.baklava_append_decode_attn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
    L.baklava_append_decode_attn_replay.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                    C.c_void_p, C.c_void_p, C.c_void_p]
    L.baklava_sync_lengths.argtypes = [C.c_void_p, C.c_void_p]
    L.baklava_flush_scores.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    L.baklava_decode_attn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.baklava_compact.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.baklava_lengths.argtypes = [C.c_void_p, i32p]
    L.baklava_profile_read.argtypes = [C.c_void_p, f64p, i64p]
    L.baklava_stream_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    L.baklava_profile_workspace_bytes.restype = C.c_size_t
    L.baklava_profile_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    L.baklava_profile_similarity.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_size_t, C.c_void_p]
    L.baklava_layer_workspace_bytes.restype = C.c_size_t
    L.baklava_layer_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    L.baklava_layer_similarity.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.baklava_layer_similarity_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                                  C.c_void_p, C.c_void_p, C.c_void_p]
    L.baklava_alloc_two_level.argtypes = [f64p, f64p, C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int32,
                                          C.c_double, C.c_double, i32p]
    L.baklava_prefill_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.baklava_kv_importance.argtypes = [f64p, C.c_int32, C.c_int32, C.c_int32, f64p]
    for name in EXPORTS:
        if name not in ("baklava_strerror", "baklava_workspace_bytes", "baklava_profile_workspace_bytes",
                        "baklava_layer_workspace_bytes"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().baklava_strerror(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != OK:
        raise BaklavaError(status, what)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


# ---------------------------------------------------------------------------
# host-only calls
# ---------------------------------------------------------------------------

def alloc_proportional(importance: Sequence[float], global_budget: int, lo: int, hi: int) -> List[int]:
    imp = np.ascontiguousarray(importance, dtype=np.float64)
    out = np.zeros(len(imp), dtype=np.int32)
    _check(lib().baklava_alloc_proportional(_p(imp, C.c_double), len(imp), int(global_budget), int(lo),
                                            int(hi), _p(out, C.c_int32)), "baklava_alloc_proportional")
    return out.tolist()


def alloc_threshold(importance: Sequence[float], size_in: Sequence[int], t: float, r: float) -> List[int]:
    imp = np.ascontiguousarray(importance, dtype=np.float64)
    size = _i32(size_in)
    out = np.zeros(len(imp), dtype=np.int32)
    _check(lib().baklava_alloc_threshold(_p(imp, C.c_double), len(imp), _p(size, C.c_int32), float(t),
                                         float(r), _p(out, C.c_int32)), "baklava_alloc_threshold")
    return out.tolist()


def layout(budget: Sequence[int], L: int, Hkv: int, batch: int, slack: int):
    b = _i32(budget)
    n = L * Hkv * batch
    off = np.zeros(n, dtype=np.int64)
    cap = np.zeros(n, dtype=np.int32)
    total = C.c_int64(0)
    _check(lib().baklava_layout(_p(b, C.c_int32), L, Hkv, batch, slack, _p(off, C.c_int64),
                                _p(cap, C.c_int32), C.byref(total)), "baklava_layout")
    return off, cap, int(total.value)


def plan_schedule(off, cap, L: int, caches_per_layer: int, chunk: int, whole_model: bool, max_items=None,
                  target_items: int = 0):
    """baklava_plan_schedule: list of (cache, start, count, slot, nsplit, row0) in launch order."""
    off = np.ascontiguousarray(off, dtype=np.int64)
    cap = _i32(cap)
    n = C.c_int64(0)
    args = (_p(off, C.c_int64), _p(cap, C.c_int32), L, caches_per_layer, chunk, int(target_items),
            int(bool(whole_model)))
    _check(lib().baklava_plan_schedule(*args, 0, None, C.byref(n)), "baklava_plan_schedule")
    cap_items = int(n.value) if max_items is None else int(max_items)
    items = (WorkItem * max(1, cap_items))()
    _check(lib().baklava_plan_schedule(*args, cap_items, items, C.byref(n)), "baklava_plan_schedule")
    return [(it.cache, it.start, it.count, it.slot, it.nsplit, it.row0) for it in items[: int(n.value)]]


# ---------------------------------------------------------------------------
# device context
# ---------------------------------------------------------------------------

def _stream_ptr(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class Arena:
    """Device memory of a ragged KV arena plus a libbaklava context over it.

    Holds torch tensors only to keep the memory alive; all work goes through
    the C-ABI calls.
    """

    def __init__(self, L: int, Hq: int, Hkv: int, D: int, batch: int, dtype: str, budget: Sequence[int],
                 slack: int, sink: int, recent: int, policy: int = POLICY_SCORE, track_scores: bool = False,
                 device: str = "cuda:0", workspace_fill: int = 0):
        import torch
        self.torch = torch
        self.L, self.Hq, self.Hkv, self.D, self.batch = L, Hq, Hkv, D, batch
        self.G = Hq // Hkv
        self.dtype = dtype
        self.device = torch.device(device)
        self.budget_host = _i32(budget)
        self.off_host, self.cap_host, self.total_tokens = layout(budget, L, Hkv, batch, slack)
        self.n_caches = L * batch * Hkv
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        dev = self.device
        self.k = torch.zeros((self.total_tokens, D), dtype=tdt, device=dev)
        self.v = torch.zeros((self.total_tokens, D), dtype=tdt, device=dev)
        self.score = torch.zeros((self.total_tokens,), dtype=torch.float32, device=dev)
        self.pos = torch.zeros((self.total_tokens,), dtype=torch.int32, device=dev)
        self.off = torch.from_numpy(self.off_host).to(dev)
        self.cap = torch.from_numpy(self.cap_host).to(dev)
        self.len = torch.zeros((self.n_caches,), dtype=torch.int32, device=dev)
        self.budget = torch.from_numpy(self.budget_host).to(dev)

        d = Desc()
        d.L, d.Hq, d.Hkv, d.D, d.batch = L, Hq, Hkv, D, batch
        d.dtype = BF16 if dtype == "bf16" else F32
        d.sink, d.recent, d.policy, d.track_scores = sink, recent, policy, int(bool(track_scores))
        ws_bytes = lib().baklava_workspace_bytes(C.byref(d), _p(self.cap_host, C.c_int32),
                                                 _p(self.budget_host, C.c_int32))
        if ws_bytes == 0:
            raise BaklavaError(EINVAL, "baklava_workspace_bytes")
        # the library does not rely on the workspace's initial contents; tests fill it with 0xFF bytes
        self.workspace = torch.full((ws_bytes,), int(workspace_fill), dtype=torch.uint8, device=dev)
        d.k, d.v = self.k.data_ptr(), self.v.data_ptr()
        d.score, d.pos = self.score.data_ptr(), self.pos.data_ptr()
        d.off, d.cap, d.len, d.budget = (self.off.data_ptr(), self.cap.data_ptr(), self.len.data_ptr(),
                                         self.budget.data_ptr())
        d.workspace, d.workspace_bytes = self.workspace.data_ptr(), ws_bytes
        self.desc = d
        torch.cuda.synchronize(dev)
        ctx = C.c_void_p()
        _check(lib().baklava_create(C.byref(d), _p(self.off_host, C.c_int64), _p(self.cap_host, C.c_int32),
                                    None, _p(self.budget_host, C.c_int32), C.byref(ctx)), "baklava_create")
        self.ctx = ctx

    def close(self) -> None:
        if getattr(self, "ctx", None):
            lib().baklava_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- thin wrappers with the C names ------------------------------------------------
    def set_option(self, option: int, value: int) -> None:
        _check(lib().baklava_set_option(self.ctx, option, int(value)), "baklava_set_option")

    def reset(self, stream=None) -> None:
        _check(lib().baklava_reset(self.ctx, _stream_ptr(stream)), "baklava_reset")

    def set_lengths(self, len_host: Sequence[int], stream=None) -> None:
        a = _i32(len_host)
        _check(lib().baklava_set_lengths(self.ctx, _p(a, C.c_int32), _stream_ptr(stream)), "baklava_set_lengths")

    def append(self, layer_begin: int, layer_count: int, k_new, v_new, token_pos: int, stream=None) -> None:
        _check(lib().baklava_append(self.ctx, layer_begin, layer_count, k_new.data_ptr(), v_new.data_ptr(),
                                    int(token_pos), _stream_ptr(stream)), "baklava_append")

    def append_decode_attn(self, layer_begin: int, layer_count: int, k_new, v_new, token_pos: int, q, out,
                           stream=None) -> None:
        _check(lib().baklava_append_decode_attn(self.ctx, layer_begin, layer_count, k_new.data_ptr(),
                                                v_new.data_ptr(), int(token_pos), q.data_ptr(), out.data_ptr(),
                                                _stream_ptr(stream)), "baklava_append_decode_attn")

    def append_decode_attn_replay(self, layer_begin: int, layer_count: int, k_new, v_new, token_pos_dev, q, out,
                                  stream=None) -> None:
        _check(lib().baklava_append_decode_attn_replay(self.ctx, layer_begin, layer_count, k_new.data_ptr(),
                                                       v_new.data_ptr(), token_pos_dev.data_ptr(), q.data_ptr(),
                                                       out.data_ptr(), _stream_ptr(stream)),
               "baklava_append_decode_attn_replay")

    def sync_lengths(self, stream=None) -> None:
        _check(lib().baklava_sync_lengths(self.ctx, _stream_ptr(stream)), "baklava_sync_lengths")

    def flush_scores(self, layer_begin: int, layer_count: int, stream=None) -> None:
        _check(lib().baklava_flush_scores(self.ctx, layer_begin, layer_count, _stream_ptr(stream)),
               "baklava_flush_scores")

    def decode_attn(self, layer_begin: int, layer_count: int, q, out, stream=None) -> None:
        _check(lib().baklava_decode_attn(self.ctx, layer_begin, layer_count, q.data_ptr(), out.data_ptr(),
                                         _stream_ptr(stream)), "baklava_decode_attn")

    def compact(self, layer_begin: int, layer_count: int, kept_idx_out=None, stream=None) -> None:
        ptr = kept_idx_out.data_ptr() if kept_idx_out is not None else None
        _check(lib().baklava_compact(self.ctx, layer_begin, layer_count, ptr, _stream_ptr(stream)),
               "baklava_compact")

    def profile_read(self):
        ms, n = C.c_double(0.0), C.c_int64(0)
        _check(lib().baklava_profile_read(self.ctx, C.byref(ms), C.byref(n)), "baklava_profile_read")
        return float(ms.value), int(n.value)

    def lengths(self) -> np.ndarray:
        out = np.zeros(self.n_caches, dtype=np.int32)
        _check(lib().baklava_lengths(self.ctx, _p(out, C.c_int32)), "baklava_lengths")
        return out


def stream_probe(dst, src, nbytes: int, mode: int, stream=None) -> None:
    """baklava_stream_probe on two torch device tensors (mode 0: copy, 1: read only, 2: read only with non-temporal loads, 3: mode 2 on 64 workgroups)."""
    _check(lib().baklava_stream_probe(dst.data_ptr(), src.data_ptr(), int(nbytes), int(mode),
                                      _stream_ptr(stream)), "baklava_stream_probe")


def _hold_until_stream_passes(tensors, stream) -> None:
    """Tensors allocated here on torch's current stream but used by kernels enqueued on another one:
    the caching allocator must not hand their memory out again before that stream has passed the call
    (the workspace is dropped as soon as the wrapper returns)."""
    if stream is None:
        return
    for t in tensors:
        if t is not None:
            t.record_stream(stream)


def kv_importance(similarity, L: int, Hq: int, Hkv: int) -> np.ndarray:
    """baklava_kv_importance: [L, Hq] head similarities -> [L, Hkv] KV-cache importances (host only)."""
    sim = np.ascontiguousarray(similarity, dtype=np.float64).reshape(-1)
    if sim.size != L * Hq:
        raise ValueError("similarity must hold L * Hq values")
    out = np.zeros(L * Hkv, dtype=np.float64)
    _check(lib().baklava_kv_importance(_p(sim, C.c_double), L, Hq, Hkv, _p(out, C.c_double)), "baklava_kv_importance")
    return out.reshape(L, Hkv)


def profile_workspace_bytes(batch: int, Hq: int, T: int) -> int:
    return int(lib().baklava_profile_workspace_bytes(batch, Hq, T))


def profile_similarity(q, k, v, want_cos: bool = True, want_lse: bool = False, stream=None):
    """baklava_profile_similarity on torch device tensors q [batch, Hq, T, D], k / v [batch, Hkv, T, D]
    (bf16).  Returns (sim [batch, Hq], cos [batch, Hq, T] or None) as torch fp32 device tensors, and
    the per-token log2-sum-exp [batch, Hq, T] as a third value when want_lse is set."""
    import torch
    batch, Hq, T, D = q.shape
    Hkv = k.shape[1]
    if k.shape != (batch, Hkv, T, D) or v.shape != k.shape:
        raise ValueError("k and v must be [batch, Hkv, T, D]")
    if q.dtype != torch.bfloat16 or k.dtype != torch.bfloat16 or v.dtype != torch.bfloat16:
        raise ValueError("bf16 tensors expected")
    if not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
        raise ValueError("contiguous tensors expected")
    sim = torch.empty((batch, Hq), dtype=torch.float32, device=q.device)
    cos = torch.empty((batch, Hq, T), dtype=torch.float32, device=q.device) if want_cos else None
    lse = torch.empty((batch, Hq, T), dtype=torch.float32, device=q.device) if want_lse else None
    nbytes = profile_workspace_bytes(batch, Hq, T)
    ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=q.device)
    _check(lib().baklava_profile_similarity(q.data_ptr(), k.data_ptr(), v.data_ptr(), batch, Hq, Hkv, T, D, BF16,
                                            cos.data_ptr() if want_cos else None, sim.data_ptr(),
                                            lse.data_ptr() if want_lse else None, ws.data_ptr(),
                                            nbytes, _stream_ptr(stream)), "baklava_profile_similarity")
    _hold_until_stream_passes((ws, sim, cos, lse), stream)
    return (sim, cos, lse) if want_lse else (sim, cos)


def prefill_scores(q, k_plane, lse, score_plane, batch: int, Hq: int, Hkv: int, T: int, row_off=None, stream=None):
    """baklava_prefill_scores: q [batch, Hq, T, 128] bf16, lse [batch, Hq, T] fp32, k_plane a bf16 tensor of
    rows of 128 elements, score_plane fp32 rows, row_off an int64 device tensor [batch * Hkv] or None (dense)."""
    _check(lib().baklava_prefill_scores(q.data_ptr(), k_plane.data_ptr(), lse.data_ptr(),
                                        row_off.data_ptr() if row_off is not None else None, batch, Hq, Hkv, T, 128,
                                        BF16, score_plane.data_ptr(), _stream_ptr(stream)), "baklava_prefill_scores")


def alloc_two_level(layer_importance, head_importance, global_budget: int, lo: int, hi: int, t: float, r: float):
    """baklava_alloc_two_level: head_importance [L, Hkv] -> list of L * Hkv budgets (host only)."""
    himp = np.ascontiguousarray(head_importance, dtype=np.float64)
    L, Hkv = himp.shape
    limp = np.ascontiguousarray(layer_importance, dtype=np.float64)
    if limp.size != L:
        raise ValueError("one importance per layer expected")
    out = np.zeros(L * Hkv, dtype=np.int32)
    _check(lib().baklava_alloc_two_level(_p(limp, C.c_double), _p(himp.reshape(-1), C.c_double), L, Hkv,
                                         int(global_budget), lo, hi, float(t), float(r), _p(out, C.c_int32)),
           "baklava_alloc_two_level")
    return out.tolist()


def layer_similarity(x_in, x_out, want_cos: bool = True, stream=None):
    """baklava_layer_similarity on torch device tensors [n_seq, T, hidden] (bf16).
    Returns (sim [n_seq], cos [n_seq, T] or None) as torch fp32 device tensors."""
    import torch
    n_seq, T, hidden = x_in.shape
    if x_out.shape != x_in.shape or x_in.dtype != torch.bfloat16 or x_out.dtype != torch.bfloat16:
        raise ValueError("two bf16 tensors of equal shape expected")
    if not (x_in.is_contiguous() and x_out.is_contiguous()):
        raise ValueError("contiguous tensors expected")
    sim = torch.empty((n_seq,), dtype=torch.float32, device=x_in.device)
    cos = torch.empty((n_seq, T), dtype=torch.float32, device=x_in.device) if want_cos else None
    nbytes = int(lib().baklava_layer_workspace_bytes(n_seq, T))
    ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=x_in.device)
    _check(lib().baklava_layer_similarity(x_in.data_ptr(), x_out.data_ptr(), n_seq, T, hidden, BF16,
                                          cos.data_ptr() if want_cos else None, sim.data_ptr(), ws.data_ptr(), nbytes,
                                          _stream_ptr(stream)), "baklava_layer_similarity")
    _hold_until_stream_passes((ws, sim, cos), stream)
    return sim, cos



LAYER_STATIC_MAX_TILES = 65536


def layer_similarity_static(x_in, x_out, sim, cos=None, stream=None) -> None:
    """baklava_layer_similarity_static: as layer_similarity, but the caller passes the outputs (sim [n_seq],
    cos [n_seq, T] or None, fp32 device tensors) and nothing is allocated, here or in the library."""
    n_seq, T, hidden = x_in.shape
    _check(lib().baklava_layer_similarity_static(x_in.data_ptr(), x_out.data_ptr(), n_seq, T, hidden, BF16,
                                                 cos.data_ptr() if cos is not None else None, sim.data_ptr(),
                                                 _stream_ptr(stream)), "baklava_layer_similarity_static")
