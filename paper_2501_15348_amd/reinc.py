"""ctypes binding over libreinc_hip.so -- argument marshalling only.

Method names are the C entry points of include/reinc.h without the `reinc_` prefix.  torch is used
for device memory and streams; every computation runs in the library's HIP kernels.  There is no
CPU fallback: if the library is missing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libreinc_hip.so")

OK, E_ARG, E_STATE, E_NOMEM, E_HIP, E_UNSUPPORTED = 0, -1, -2, -3, -4, -5
AGG = {"sum": 0, "mean": 1, "sym": 2}
RNN = {"gru": 0, "lstm": 1}
DTYPE = {"fp32": 0, "bf16": 1}
MAX_GCN_LAYERS = 3
KERNEL_KINDS = ("agg_full", "agg_inc", "gemm_rows", "rnn", "reduce", "elem", "diff", "agg_minmax")
OPS = {"max": 0, "min": 1}


class Config(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("device", ctypes.c_int32),
        ("num_nodes", ctypes.c_int64),
        ("num_snapshots", ctypes.c_int32),
        ("num_gcn_layers", ctypes.c_int32),
        ("dims", ctypes.c_int32 * (MAX_GCN_LAYERS + 1)),
        ("rnn_kind", ctypes.c_int32),
        ("rnn_hidden", ctypes.c_int32),
        ("agg_kind", ctypes.c_int32),
        ("self_loop", ctypes.c_int32),
        ("feat_dtype", ctypes.c_int32),
        ("fallback_ratio", ctypes.c_float),
        ("arena", ctypes.c_void_p),
        ("arena_bytes", ctypes.c_uint64),
    ]


class DeltaInfo(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in (
        "num_edges_prev", "num_edges_cur", "n_ins", "n_del", "n_changed", "n_fchg_entries", "n_rows", "n_entries")]


class Stats(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in (
        "arena_used", "arena_peak", "global_hits", "global_misses", "steps_incremental", "steps_full",
        "steps_fallback", "delta_entries_processed", "local_bytes", "global_admitted", "global_refused",
        "global_evicted", "global_expired", "global_bytes", "global_peak_bytes")]


POLICIES = ("keep_all", "score", "lru", "lfu")  # REINC_POLICY_*
POLICY_COUNTERS = ("hits", "misses", "admitted", "refused", "evicted", "expired", "used", "peak_used")


class ReincError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"reinc error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libreinc_hip.so; raises if it has not been built (python -m paper_2501_15348_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_15348_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    p, i32, i64, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int
    sig = {
        "reinc_create": [ctypes.POINTER(p), ctypes.POINTER(Config)],
        "reinc_destroy": [p],
        "reinc_arena_free_bytes": [p, ctypes.POINTER(ctypes.c_uint64)],
        "reinc_load_edges": [p, i32, p, p, i64, ci],
        "reinc_load_features_full": [p, i32, p, ci],
        "reinc_load_features_delta": [p, i32, p, i64, p],
        "reinc_build_deltas": [p, i32, p],
        "reinc_get_delta_info": [p, i32, ctypes.POINTER(DeltaInfo)],
        "reinc_get_delta_csr": [p, i32, ci, p, p, ctypes.POINTER(i64)],
        "reinc_get_merged_delta": [p, i32, p, p, p, p],
        "reinc_get_snapshot_csr": [p, i32, ci, p, p, ctypes.POINTER(i64)],
        "reinc_aggregate_full": [p, i32, ci, p, ci, i32, ci, p, p],
        "reinc_aggregate_incremental": [p, i32, p, p, p, p],
        "reinc_aggregate_full_minmax": [p, i32, ci, p, ci, i32, p, p, p],
        "reinc_aggregate_incremental_minmax": [p, i32, ci, p, p, p, p, p, p],
        "reinc_aggregate_incremental_minmax_static": [p, i32, ci, p, p, p, p, p, p],
        "reinc_gcn_transform": [p, p, ci, i64, i32, i32, p, p, p, ci, p, p],
        "reinc_rnn_step": [p, ci, p, i64, i32, i32, p, p, p, p, p, p, p, p, p, p],
        "reinc_forward_window": [p, i32, i32, p, p, p, p, p],
        "reinc_backward_window": [p, i32, i32, p, p, p, p],
        "reinc_forward_window_integrated": [p, i32, i32, p, p, p, p, p],
        "reinc_backward_window_integrated": [p, i32, i32, p, p, p, p],
        "reinc_sgd_step": [p, p, p, i64, ctypes.c_float, p],
        "reinc_reset_derived": [p],
        "reinc_profile_begin": [p, ctypes.c_uint32],
        "reinc_profile_end": [p, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)],
        "reinc_cache_clear": [p],
        "reinc_cache_peek": [p, i32, ctypes.POINTER(p)],
        "reinc_cache_configure": [p, i32, i64, i32, i32],
        "reinc_batch_plan": [p, p, i64, i32, p, p],
        "reinc_batch_node_list": [p, p],
        "reinc_batch_load": [p, p],
        "reinc_set_loss_rows": [p, i64],
        "reinc_policy_create": [ctypes.POINTER(p), i32, i64],
        "reinc_policy_destroy": [p],
        "reinc_policy_access": [p, i64, ctypes.POINTER(i32)],
        "reinc_policy_offer": [p, i64, i64, i64, i64, ctypes.POINTER(i32), ctypes.POINTER(i64), i32, ctypes.POINTER(i32)],
        "reinc_policy_rescore": [p, i64, i64, i64],
        "reinc_policy_contains": [p, i64, ctypes.POINTER(i32)],
        "reinc_policy_counters": [p, ctypes.POINTER(i64)],
        "reinc_get_stats": [p, ctypes.POINTER(Stats)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    lib.reinc_last_error.argtypes = [p]
    lib.reinc_last_error.restype = ctypes.c_char_p
    lib.reinc_version.argtypes = []
    lib.reinc_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """One reinc_ctx plus the torch tensor that backs its arena."""

    def __init__(self, num_nodes: int, num_snapshots: int, dims, rnn: str, hidden: int, agg: str, self_loop: bool,
                 feat_dtype: str = "fp32", fallback_ratio: float = 0.5, arena_bytes: int = 1 << 30, device: int = 0):
        import torch

        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: libreinc_hip has no CPU path")
        self.device = torch.device("cuda", device)
        self.arena = torch.empty(int(arena_bytes) + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) & ~255
        cfg = Config()
        cfg.struct_size = ctypes.sizeof(Config)
        cfg.device = device
        cfg.num_nodes = num_nodes
        cfg.num_snapshots = num_snapshots
        cfg.num_gcn_layers = len(dims) - 1
        for i, d in enumerate(dims):
            cfg.dims[i] = d
        cfg.rnn_kind = RNN[rnn]
        cfg.rnn_hidden = hidden
        cfg.agg_kind = AGG[agg]
        cfg.self_loop = int(self_loop)
        cfg.feat_dtype = DTYPE[feat_dtype]
        cfg.fallback_ratio = fallback_ratio
        cfg.arena = base
        cfg.arena_bytes = int(arena_bytes)
        self.cfg = cfg
        self.n, self.T, self.dims, self.hidden = num_nodes, num_snapshots, tuple(dims), hidden
        self.rnn, self.feat_dtype = rnn, feat_dtype
        self.handle = ctypes.c_void_p()
        rc = self.lib.reinc_create(ctypes.byref(self.handle), ctypes.byref(cfg))
        if rc != OK:
            msg = self.lib.reinc_last_error(self.handle).decode() if self.handle else "bad config"
            if self.handle:
                self.lib.reinc_destroy(self.handle)
                self.handle = None
            raise ReincError(rc, msg)

    @classmethod
    def for_workload(cls, wl, arena_bytes: int, fallback_ratio: float = 0.5, device: int = 0) -> "Context":
        return cls(wl.num_nodes, wl.num_snapshots, wl.dims, wl.rnn, wl.hidden, wl.agg, wl.self_loop, wl.feat_dtype,
                   fallback_ratio, arena_bytes, device)

    def close(self):
        if getattr(self, "handle", None):
            self.lib.reinc_destroy(self.handle)
            self.handle = None
        self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc: int):
        if rc != OK:
            raise ReincError(rc, self.lib.reinc_last_error(self.handle).decode())

    # ---- loading
    def load_edges(self, t: int, src, dst):
        """src, dst: int32 endpoint arrays, numpy (host) or torch tensors on this context's device."""
        import torch

        if isinstance(src, torch.Tensor) or isinstance(dst, torch.Tensor):
            if not (isinstance(src, torch.Tensor) and isinstance(dst, torch.Tensor)) or src.dtype != torch.int32 or dst.dtype != torch.int32:
                raise ValueError("device edge lists are two int32 tensors")
            if src.shape != dst.shape or src.dim() != 1:
                raise ValueError("src and dst differ in length")
            self._ck(self.lib.reinc_load_edges(self.handle, t, _dev_ptr(src), _dev_ptr(dst), src.numel(), 1))
            return
        src = np.ascontiguousarray(src, dtype=np.int32)
        dst = np.ascontiguousarray(dst, dtype=np.int32)
        if src.shape != dst.shape:
            raise ValueError("src and dst differ in length")
        self._ck(self.lib.reinc_load_edges(self.handle, t, _np_ptr(src), _np_ptr(dst), src.size, 0))

    def _host_feats(self, x: np.ndarray) -> np.ndarray:
        if self.feat_dtype == "bf16":
            if x.dtype != np.uint16:
                raise ValueError("bf16 features are passed as uint16 bit patterns")
            return np.ascontiguousarray(x)
        return np.ascontiguousarray(x, dtype=np.float32)

    def load_features_full(self, t: int, x):
        import torch

        if isinstance(x, torch.Tensor):
            self._ck(self.lib.reinc_load_features_full(self.handle, t, _dev_ptr(x), 1))
        else:
            x = self._host_feats(x)
            if x.shape != (self.n, self.dims[0]):
                raise ValueError("feature matrix must be [N, dims[0]]")
            self._ck(self.lib.reinc_load_features_full(self.handle, t, _np_ptr(x), 0))

    def load_features_delta(self, t: int, rows: np.ndarray, vals: np.ndarray):
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        vals = self._host_feats(vals)
        if vals.shape != (rows.size, self.dims[0]):
            raise ValueError("values must be [len(rows), dims[0]]")
        self._ck(self.lib.reinc_load_features_delta(self.handle, t, _np_ptr(rows), rows.size, _np_ptr(vals)))

    # ---- deltas
    def build_deltas(self, t: int = -1):
        self._ck(self.lib.reinc_build_deltas(self.handle, t, _stream()))

    def get_delta_info(self, t: int) -> dict:
        info = DeltaInfo()
        self._ck(self.lib.reinc_get_delta_info(self.handle, t, ctypes.byref(info)))
        return {k: getattr(info, k) for k, _ in DeltaInfo._fields_}

    def get_delta_csr(self, t: int, kind: int) -> Tuple[np.ndarray, np.ndarray]:
        nnz = ctypes.c_int64()
        self._ck(self.lib.reinc_get_delta_csr(self.handle, t, kind, None, None, ctypes.byref(nnz)))
        rp = np.empty(self.n + 1, dtype=np.int64)
        col = np.empty(nnz.value, dtype=np.int32)
        self._ck(self.lib.reinc_get_delta_csr(self.handle, t, kind, _np_ptr(rp), _np_ptr(col), None))
        return rp, col

    def get_merged_delta(self, t: int):
        info = self.get_delta_info(t)
        ptr = np.empty(self.n + 1, dtype=np.int64)
        ent = np.empty(info["n_entries"], dtype=np.uint32)
        rows = np.empty(info["n_rows"], dtype=np.int32)
        changed = np.empty(info["n_changed"], dtype=np.int32)
        self._ck(self.lib.reinc_get_merged_delta(self.handle, t, _np_ptr(ptr), _np_ptr(ent), _np_ptr(rows), _np_ptr(changed)))
        return ptr, ent, rows, changed

    def get_snapshot_csr(self, t: int, transpose: bool = False):
        nnz = ctypes.c_int64()
        self._ck(self.lib.reinc_get_snapshot_csr(self.handle, t, int(transpose), None, None, ctypes.byref(nnz)))
        ptr = np.empty(self.n + 1, dtype=np.int64)
        idx = np.empty(nnz.value, dtype=np.int32)
        self._ck(self.lib.reinc_get_snapshot_csr(self.handle, t, int(transpose), _np_ptr(ptr), _np_ptr(idx), None))
        return ptr, idx

    # ---- aggregation
    def aggregate_full(self, t: int, x=None, transpose: bool = False, apply_q: bool = False, out=None):
        import torch

        if x is None:
            d, dt = self.dims[0], DTYPE[self.feat_dtype]
        else:
            d = x.shape[1]
            dt = 1 if x.dtype == torch.bfloat16 else 0
            if x.dtype not in (torch.float32, torch.bfloat16) or x.shape[0] != self.n:
                raise ValueError("x must be fp32 or bf16 [N, d]")
        if out is None:
            out = torch.empty((self.n, d), dtype=torch.float32, device=self.device)
        self._ck(self.lib.reinc_aggregate_full(self.handle, t, int(transpose), _dev_ptr(x), dt, d, int(apply_q),
                                               _dev_ptr(out), _stream()))
        return out

    def aggregate_incremental(self, t: int, s_prev, s_out=None, agg_out=None):
        import torch

        if s_prev.dtype != torch.float32 or tuple(s_prev.shape) != (self.n, self.dims[0]):
            raise ValueError("S_prev must be fp32 [N, dims[0]]")
        if s_out is None:
            s_out = torch.empty_like(s_prev)
        self._ck(self.lib.reinc_aggregate_incremental(self.handle, t, _dev_ptr(s_prev), _dev_ptr(s_out),
                                                      _dev_ptr(agg_out), _stream()))
        return s_out

    def aggregate_full_minmax(self, t: int, op: str, x=None, out=None, contrib=None):
        """Max / min over the in-neighbourhood with the contributing source ids (paper Section 3.2)."""
        import torch

        if x is None:
            d, dt = self.dims[0], DTYPE[self.feat_dtype]
        else:
            d = x.shape[1]
            dt = 1 if x.dtype == torch.bfloat16 else 0
            if x.dtype not in (torch.float32, torch.bfloat16) or x.shape[0] != self.n:
                raise ValueError("x must be fp32 or bf16 [N, d]")
        if out is None:
            out = torch.empty((self.n, d), dtype=torch.float32, device=self.device)
        if contrib is None:
            contrib = torch.empty((self.n, d), dtype=torch.int32, device=self.device)
        self._ck(self.lib.reinc_aggregate_full_minmax(self.handle, t, OPS[op], _dev_ptr(x), dt, d, _dev_ptr(out),
                                                      _dev_ptr(contrib), _stream()))
        return out, contrib

    def aggregate_incremental_minmax(self, t: int, op: str, m_prev, c_prev, m_out=None, c_out=None, work=None):
        """(M_t, C_t) from (M_{t-1}, C_{t-1}); returns (M, C, work) with work[0] = rows aggregated from scratch."""
        import torch

        shape = (self.n, self.dims[0])
        if m_prev.dtype != torch.float32 or tuple(m_prev.shape) != shape or c_prev.dtype != torch.int32 or tuple(c_prev.shape) != shape:
            raise ValueError("M_prev must be fp32 and C_prev int32, both [N, dims[0]]")
        if m_out is None:
            m_out, c_out = torch.empty_like(m_prev), torch.empty_like(c_prev)
        if work is None:
            work = torch.empty(2 * self.n + 4, dtype=torch.int32, device=self.device)
        self._ck(self.lib.reinc_aggregate_incremental_minmax(self.handle, t, OPS[op], _dev_ptr(m_prev), _dev_ptr(c_prev),
                                                             _dev_ptr(m_out), _dev_ptr(c_out), _dev_ptr(work), _stream()))
        return m_out, c_out, work

    def aggregate_incremental_minmax_static(self, t: int, op: str, m_prev, c_prev, m_out, c_out, n_redone=None):
        """The same step with the library's static work area: no allocation here or in the library (the caller
        passes every buffer); n_redone: int32 device scalar or None."""
        self._ck(self.lib.reinc_aggregate_incremental_minmax_static(self.handle, t, OPS[op], _dev_ptr(m_prev),
                                                                    _dev_ptr(c_prev), _dev_ptr(m_out), _dev_ptr(c_out),
                                                                    _dev_ptr(n_redone), _stream()))

    # ---- dense steps
    def gcn_transform(self, a, w, b=None, row_scale=None, relu: bool = True, out=None):
        import torch

        n, d_in = a.shape
        d_out = w.shape[1]
        if out is None:
            out = torch.empty((n, d_out), dtype=torch.float32, device=self.device)
        self._ck(self.lib.reinc_gcn_transform(self.handle, _dev_ptr(a), 1 if a.dtype == torch.bfloat16 else 0, n, d_in,
                                              d_out, _dev_ptr(row_scale), _dev_ptr(w), _dev_ptr(b), int(relu),
                                              _dev_ptr(out), _stream()))
        return out

    def rnn_step(self, kind: str, x, h_prev, c_prev, w_i, w_h, b_i, b_h, saved=None):
        import torch

        n, d_in = x.shape
        hd = w_h.shape[0]
        h_out = torch.empty((n, hd), dtype=torch.float32, device=self.device)
        c_out = torch.empty((n, hd), dtype=torch.float32, device=self.device) if kind == "lstm" else None
        self._ck(self.lib.reinc_rnn_step(self.handle, RNN[kind], _dev_ptr(x), n, d_in, hd, _dev_ptr(h_prev),
                                         _dev_ptr(c_prev), _dev_ptr(w_i), _dev_ptr(w_h), _dev_ptr(b_i), _dev_ptr(b_h),
                                         _dev_ptr(h_out), _dev_ptr(c_out), _dev_ptr(saved), _stream()))
        return h_out, c_out

    # ---- window driver
    def forward_window(self, t0: int, length: int, params, target=None, loss_out=None, h_last=None):
        self._ck(self.lib.reinc_forward_window(self.handle, t0, length, _dev_ptr(params), _dev_ptr(target),
                                               _dev_ptr(loss_out), _dev_ptr(h_last), _stream()))

    def backward_window(self, t0: int, length: int, params, target, grads):
        self._ck(self.lib.reinc_backward_window(self.handle, t0, length, _dev_ptr(params), _dev_ptr(target),
                                                _dev_ptr(grads), _stream()))

    def forward_window_integrated(self, t0: int, length: int, params, target=None, loss_out=None, h_last=None):
        """Integrated model (graph operations inside the gates); params = W_i [dims[0], K*H], W_h, b_i, b_h."""
        self._ck(self.lib.reinc_forward_window_integrated(self.handle, t0, length, _dev_ptr(params), _dev_ptr(target),
                                                          _dev_ptr(loss_out), _dev_ptr(h_last), _stream()))

    def backward_window_integrated(self, t0: int, length: int, params, target, grads):
        self._ck(self.lib.reinc_backward_window_integrated(self.handle, t0, length, _dev_ptr(params), _dev_ptr(target),
                                                           _dev_ptr(grads), _stream()))

    def sgd_step(self, params, grads, lr: float):
        self._ck(self.lib.reinc_sgd_step(self.handle, _dev_ptr(params), _dev_ptr(grads), params.numel(), lr, _stream()))

    def reset_derived(self):
        self._ck(self.lib.reinc_reset_derived(self.handle))

    def profile_begin(self, kinds=("agg_full",)):
        mask = 0
        for k in kinds:
            mask |= 1 << KERNEL_KINDS.index(k)
        self._ck(self.lib.reinc_profile_begin(self.handle, mask))

    def profile_end(self) -> dict:
        n = len(KERNEL_KINDS)
        launches = (ctypes.c_int64 * n)()
        total = (ctypes.c_double * n)()
        self._ck(self.lib.reinc_profile_end(self.handle, launches, total))
        return {k: (launches[i], total[i]) for i, k in enumerate(KERNEL_KINDS)}

    def cache_clear(self):
        self._ck(self.lib.reinc_cache_clear(self.handle))

    def cache_configure(self, policy: str, budget_bytes: int = 0, window: int = 1, stride: int = 1):
        """Limits what the layer-1 cache retains between windows; policy is one of POLICIES."""
        self._ck(self.lib.reinc_cache_configure(self.handle, POLICIES.index(policy), int(budget_bytes), window, stride))

    # ---- node mini-batches
    def set_loss_rows(self, rows: int):
        self._ck(self.lib.reinc_set_loss_rows(self.handle, int(rows)))

    def batch_plan(self, nodes, hops: int = 0):
        """Plans the sub-sequence of a node batch; returns (nodes of the sub-sequence, inner nodes)."""
        import numpy as np

        nodes = np.ascontiguousarray(nodes, dtype=np.int32)
        total, inner = ctypes.c_int64(), ctypes.c_int64()
        self._ck(self.lib.reinc_batch_plan(self.handle, nodes.ctypes.data_as(ctypes.c_void_p), nodes.size, hops,
                                           ctypes.byref(total), ctypes.byref(inner)))
        return total.value, inner.value

    def batch_node_list(self, total: int):
        import numpy as np

        out = np.empty(total, dtype=np.int32)
        self._ck(self.lib.reinc_batch_node_list(self.handle, out.ctypes.data_as(ctypes.c_void_p)))
        return out

    def batch_context(self, nodes, arena_bytes: int, hops: int = 0, planned_total: Optional[int] = None, **kw) -> "Context":
        """A new context holding the sub-sequence of `nodes` (same model configuration; keyword arguments override
        constructor arguments such as fallback_ratio).  planned_total: the node count batch_plan returned for these
        nodes and hops, if the caller has just planned them (say, to size the arena); the plan is then not repeated."""
        total = planned_total if planned_total is not None else self.batch_plan(nodes, hops)[0]
        args = dict(fallback_ratio=self.cfg.fallback_ratio, device=self.cfg.device)
        args.update(kw)
        agg = [k for k, v in AGG.items() if v == self.cfg.agg_kind][0]
        child = Context(total, self.T, self.dims, self.rnn, self.hidden, agg, bool(self.cfg.self_loop), self.feat_dtype,
                        arena_bytes=arena_bytes, **args)
        try:
            self._ck(self.lib.reinc_batch_load(self.handle, child.handle))
        except Exception:
            child.close()
            raise
        return child

    def aggregate_bytes(self) -> int:
        """Size of one cached layer-1 aggregate (the unit a budget is counted in)."""
        return (self.n * self.dims[0] * 4 + 255) & ~255

    def cache_peek(self, t: int):
        """The cached layer-1 sums of snapshot t as a tensor view into the arena, or None."""
        import torch

        ptr = ctypes.c_void_p()
        self._ck(self.lib.reinc_cache_peek(self.handle, t, ctypes.byref(ptr)))
        if not ptr.value:
            return None
        off = ptr.value - self.arena.data_ptr()
        nbytes = self.n * self.dims[0] * 4
        return self.arena[off:off + nbytes].view(torch.float32).view(self.n, self.dims[0])

    def get_stats(self) -> dict:
        st = Stats()
        self._ck(self.lib.reinc_get_stats(self.handle, ctypes.byref(st)))
        return {k: getattr(st, k) for k, _ in Stats._fields_}

    def arena_free_bytes(self) -> int:
        out = ctypes.c_uint64()
        self._ck(self.lib.reinc_arena_free_bytes(self.handle, ctypes.byref(out)))
        return out.value

    # ---- convenience (marshalling only): load a whole generated sequence
    def load_sequence(self, seq, delta_features: bool = True, progress=None):
        from . import synth

        conv = (lambda a: synth.bf16_bits(a)) if self.feat_dtype == "bf16" else (lambda a: a)
        for t, (s, d) in enumerate(seq.edges):
            self.load_edges(t, s, d)
            if progress is not None:
                progress("load", t, seq.num_snapshots)
        self.load_features_full(0, conv(seq.x0))
        x = seq.x0
        for t in range(1, seq.num_snapshots):
            if delta_features:
                self.load_features_delta(t, seq.feat_rows[t], conv(seq.feat_vals[t]))
            else:
                x = x.copy()
                x[seq.feat_rows[t]] = seq.feat_vals[t]
                self.load_features_full(t, conv(x))


class PolicyStore:
    """The cache policies as a stand-alone host-side store of (key, size, F, I) records (no GPU needed)."""

    def __init__(self, policy: str, budget: int):
        self.lib = load_library()
        self.handle = ctypes.c_void_p()
        code = self.lib.reinc_policy_create(ctypes.byref(self.handle), POLICIES.index(policy), int(budget))
        if code != 0:
            raise ReincError(code, "reinc_policy_create failed")

    def close(self):
        if self.handle:
            self.lib.reinc_policy_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        self.close()

    def _ck(self, code: int):
        if code != 0:
            raise ReincError(code, "policy store call failed")

    def access(self, key: int) -> bool:
        hit = ctypes.c_int32()
        self._ck(self.lib.reinc_policy_access(self.handle, key, ctypes.byref(hit)))
        return bool(hit.value)

    def offer(self, key: int, size: int, future: int, imminence: int, cap: int = 64):
        admitted, n_out = ctypes.c_int32(), ctypes.c_int32()
        buf = (ctypes.c_int64 * cap)()
        self._ck(self.lib.reinc_policy_offer(self.handle, key, size, future, imminence, ctypes.byref(admitted), buf, cap,
                                             ctypes.byref(n_out)))
        if n_out.value > cap:
            raise ReincError(-1, f"{n_out.value} keys were evicted, room for {cap}")
        return bool(admitted.value), list(buf[:n_out.value])

    def rescore(self, key: int, future: int, imminence: int):
        self._ck(self.lib.reinc_policy_rescore(self.handle, key, future, imminence))

    def __contains__(self, key: int) -> bool:
        present = ctypes.c_int32()
        self._ck(self.lib.reinc_policy_contains(self.handle, key, ctypes.byref(present)))
        return bool(present.value)

    def counters(self) -> dict:
        out = (ctypes.c_int64 * len(POLICY_COUNTERS))()
        self._ck(self.lib.reinc_policy_counters(self.handle, out))
        return dict(zip(POLICY_COUNTERS, out))
