"""ctypes binding with the same names as the C ABI declared in include/mgwfbp.h.

Argument marshalling only.  Device buffers are passed as integer addresses (e.g. torch's
`tensor.data_ptr()`), streams as integer handles (e.g. `torch.cuda.current_stream().cuda_stream`)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

F32 = 0
BF16 = 1
F16 = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

_STATUS = {0: "MGWFBP_OK", -1: "MGWFBP_EINVAL", -2: "MGWFBP_ENOMEM", -3: "MGWFBP_EHIP", -4: "MGWFBP_ECAPACITY"}


class MgwfbpError(RuntimeError):
    def __init__(self, fn: str, status: int, hip_error: int = 0):
        self.status = status
        self.hip_error = hip_error
        extra = f" (hipError_t {hip_error})" if status == -3 else ""
        super().__init__(f"{fn} failed: {_STATUS.get(status, status)}{extra}")


def library_path() -> str:
    return os.environ.get("MGWFBP_LIBRARY", os.path.join(_HERE, "libmgwfbp.so"))


_u64p = C.POINTER(C.c_uint64)
_i32p = C.POINTER(C.c_int32)
_u32p = C.POINTER(C.c_uint32)
_u8p = C.POINTER(C.c_uint8)
_f64p = C.POINTER(C.c_double)
_vp = C.c_void_p

_SIGNATURES = {
    "mgwfbp_plan": (C.c_int, [_u64p, _f64p, C.c_int32, C.c_double, C.c_double, _u8p, _i32p, _i32p]),
    "mgwfbp_plan_opt": (C.c_int, [_u64p, _f64p, C.c_int32, C.c_double, C.c_double, _u8p, _i32p, _i32p, _f64p]),
    "mgwfbp_eval": (C.c_int, [_u8p, _u64p, _f64p, C.c_int32, C.c_double, C.c_double, _f64p]),
    "mgwfbp_group_ready_times": (C.c_int, [_u8p, _f64p, C.c_int32, _f64p, _i32p]),
    "mgwfbp_allreduce_ab": (C.c_int, [C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_double, _f64p, _f64p]),
    "mgwfbp_fit_ab": (C.c_int, [_u64p, _f64p, C.c_int32, _f64p, _f64p]),
    "mgwfbp_simulate": (C.c_int, [_u64p, _f64p, C.c_int32, C.c_double, C.c_int32, C.c_double, C.c_double, C.c_double,
                                  _i32p, C.c_int32, _f64p, _f64p, _f64p, _i32p]),
    "mgwfbp_ctx_create": (C.c_int, [C.POINTER(_vp), _u64p, C.c_int32, _u8p, C.c_int32, C.c_int32]),
    "mgwfbp_ctx_create_host": (C.c_int, [C.POINTER(_vp), _u64p, C.c_int32, _u8p, C.c_int32, C.c_int32]),
    "mgwfbp_ctx_destroy": (None, [_vp]),
    "mgwfbp_ctx_dims": (C.c_int, [_vp, _i32p, _i32p, _i32p, _i32p, _u64p, _i32p, _i32p]),
    "mgwfbp_ctx_layout": (C.c_int, [_vp, _u64p, _i32p, _u64p, _u64p]),
    "mgwfbp_ctx_tables": (C.c_int, [_vp, _i32p, _vp, _u64p, _u32p, _i32p, _i32p]),
    "mgwfbp_ctx_set_launch": (C.c_int, [_vp, C.c_int32, C.c_int32, C.c_int32]),
    "mgwfbp_ctx_set_pacing": (C.c_int, [_vp, C.c_int32, C.c_int32]),
    "mgwfbp_ctx_set_small_launch": (C.c_int, [_vp, C.c_int32]),
    "mgwfbp_ctx_set_resident_bytes": (C.c_int, [_vp, C.c_uint64]),
    "mgwfbp_pack": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp]),
    "mgwfbp_pack_tensors": (C.c_int, [_vp, C.c_int32, C.c_int32, _vp, _vp, _vp]),
    "mgwfbp_reduce": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp]),
    "mgwfbp_unpack_update": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_reduce_update": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_group_pipeline": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_direct_update": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_group_pipeline_span": (C.c_int, [_vp, C.c_int32, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_group_pipeline_static": (C.c_int, [_vp, C.c_int32, _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, _vp]),
    "mgwfbp_handler_replay": (C.c_int, [_vp, _f64p, C.c_double, C.c_int32, C.POINTER(_vp), C.c_int32, _vp, _vp, _vp, _vp, _vp,
                                        C.c_float, C.c_float, _f64p]),
    "mgwfbp_last_hip_error": (C.c_int, []),
    "mgwfbp_version": (C.c_char_p, []),
}


def lib() -> C.CDLL:
    """The loaded library.  Raises if it is missing: there is no fallback path."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise MgwfbpError(f"load {path} (not built; run `python -m paper_1912_09268_amd.build`)", -1)
        handle = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = handle
    return _LIB


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise MgwfbpError(fn, status, lib().mgwfbp_last_hip_error())


def _arr(x, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=dtype))


def _ptr(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(ctype)


# --------------------------------------------------------------------------------------------
# host: planning
# --------------------------------------------------------------------------------------------

def plan(size_bytes: Sequence[int], t_backward_s: Sequence[float], a_s: float, b_s_per_byte: float
         ) -> Tuple[np.ndarray, np.ndarray]:
    """mgwfbp_plan.  Returns (merged[L] uint8, group_first[G] int32)."""
    sz = _arr(size_bytes, np.uint64)
    tb = _arr(t_backward_s, np.float64)
    L = int(sz.shape[0])
    if tb.shape[0] != L:
        raise ValueError("size_bytes and t_backward_s differ in length")
    merged = np.zeros(L, np.uint8)
    first = np.zeros(L + 1, np.int32)
    G = C.c_int32(0)
    _check("mgwfbp_plan", lib().mgwfbp_plan(_ptr(sz, _u64p), _ptr(tb, _f64p), L, float(a_s), float(b_s_per_byte),
                                            _ptr(merged, _u8p), _ptr(first, _i32p), C.byref(G)))
    return merged, first[:G.value].copy()


def plan_opt(size_bytes: Sequence[int], t_backward_s: Sequence[float], a_s: float, b_s_per_byte: float
             ) -> Tuple[np.ndarray, np.ndarray, float]:
    """mgwfbp_plan_opt.  Returns (merged[L] uint8, group_first[G] int32, optimal t_iter - t_f)."""
    sz = _arr(size_bytes, np.uint64)
    tb = _arr(t_backward_s, np.float64)
    L = int(sz.shape[0])
    if tb.shape[0] != L:
        raise ValueError("size_bytes and t_backward_s differ in length")
    merged = np.zeros(L, np.uint8)
    first = np.zeros(L + 1, np.int32)
    G = C.c_int32(0)
    t = C.c_double(0.0)
    _check("mgwfbp_plan_opt", lib().mgwfbp_plan_opt(_ptr(sz, _u64p), _ptr(tb, _f64p), L, float(a_s),
                                                    float(b_s_per_byte), _ptr(merged, _u8p), _ptr(first, _i32p),
                                                    C.byref(G), C.byref(t)))
    return merged, first[:G.value].copy(), t.value


def eval_plan(merged: Sequence[int], size_bytes: Sequence[int], t_backward_s: Sequence[float],
              a_s: float, b_s_per_byte: float) -> float:
    """mgwfbp_eval: t_iter - t_f of a plan."""
    m = _arr(merged, np.uint8)
    sz = _arr(size_bytes, np.uint64)
    tb = _arr(t_backward_s, np.float64)
    out = C.c_double(0.0)
    _check("mgwfbp_eval", lib().mgwfbp_eval(_ptr(m, _u8p), _ptr(sz, _u64p), _ptr(tb, _f64p), int(sz.shape[0]),
                                            float(a_s), float(b_s_per_byte), C.byref(out)))
    return out.value


def group_ready_times(merged: Sequence[int], t_backward_s: Sequence[float]) -> np.ndarray:
    """mgwfbp_group_ready_times -> ready[G], seconds from the start of the backward pass."""
    m = _arr(merged, np.uint8)
    tb = _arr(t_backward_s, np.float64)
    if m.shape[0] != tb.shape[0]:
        raise ValueError("merged and t_backward_s differ in length")
    L = int(m.shape[0])
    out = np.zeros(max(L, 1), np.float64)
    G = C.c_int32(0)
    _check("mgwfbp_group_ready_times", lib().mgwfbp_group_ready_times(_ptr(m, _u8p), _ptr(tb, _f64p), L,
                                                                      _ptr(out, _f64p), C.byref(G)))
    return out[:G.value].copy()


AR_BINARY_TREE, AR_RECURSIVE_DOUBLING, AR_HALVING_DOUBLING, AR_DOUBLE_BINARY_TREES, AR_RING = range(5)


def allreduce_ab(algorithm: int, n_workers: int, alpha_s: float, beta_s_per_byte: float, gamma_s_per_byte: float
                 ) -> Tuple[float, float]:
    """mgwfbp_allreduce_ab -> (a, b)."""
    a, b = C.c_double(), C.c_double()
    _check("mgwfbp_allreduce_ab", lib().mgwfbp_allreduce_ab(int(algorithm), int(n_workers), float(alpha_s),
                                                            float(beta_s_per_byte), float(gamma_s_per_byte),
                                                            C.byref(a), C.byref(b)))
    return a.value, b.value


def fit_ab(message_bytes: Sequence[int], seconds: Sequence[float]) -> Tuple[float, float]:
    """mgwfbp_fit_ab -> (a, b)."""
    m = _arr(message_bytes, np.uint64)
    t = _arr(seconds, np.float64)
    if m.shape[0] != t.shape[0]:
        raise ValueError("message_bytes and seconds differ in length")
    a, b = C.c_double(), C.c_double()
    _check("mgwfbp_fit_ab", lib().mgwfbp_fit_ab(_ptr(m, _u64p), _ptr(t, _f64p), int(m.shape[0]), C.byref(a), C.byref(b)))
    return a.value, b.value


def simulate(size_bytes: Sequence[int], t_backward_s: Sequence[float], t_forward_s: float, algorithm: int,
             alpha_s: float, beta_s_per_byte: float, gamma_s_per_byte: float, worker_counts: Sequence[int]):
    """mgwfbp_simulate -> (t_wfbp[n], t_single[n], t_mgwfbp[n], groups[n])."""
    sz = _arr(size_bytes, np.uint64)
    tb = _arr(t_backward_s, np.float64)
    wc = _arr(worker_counts, np.int32)
    n = int(wc.shape[0])
    tw, ts, tm = np.zeros(n), np.zeros(n), np.zeros(n)
    g = np.zeros(n, np.int32)
    _check("mgwfbp_simulate", lib().mgwfbp_simulate(
        _ptr(sz, _u64p), _ptr(tb, _f64p), int(sz.shape[0]), float(t_forward_s), int(algorithm), float(alpha_s),
        float(beta_s_per_byte), float(gamma_s_per_byte), _ptr(wc, _i32p), n, _ptr(tw, _f64p), _ptr(ts, _f64p),
        _ptr(tm, _f64p), _ptr(g, _i32p)))
    return tw, ts, tm, g


# --------------------------------------------------------------------------------------------
# context + device calls
# --------------------------------------------------------------------------------------------

TILE_HDR_DTYPE = np.dtype([("first_start", np.int64), ("first_end", np.int32), ("seg0", np.int32),
                           ("nseg", np.int32), ("valid", np.int32), ("layer0", np.int32),
                           ("flags", np.int32)])


class Context:
    """Owns one mgwfbp_ctx.  `host_only=True` builds the tables without touching a GPU (device calls
    on such a context are rejected by the library)."""

    def __init__(self, n_elems: Sequence[int], merged: Sequence[int], P: int, grad_dtype: int = F32,
                 host_only: bool = False):
        self._h = _vp(None)
        ne = _arr(n_elems, np.uint64)
        m = _arr(merged, np.uint8)
        if ne.shape[0] != m.shape[0]:
            raise ValueError("n_elems and merged differ in length")
        fn = "mgwfbp_ctx_create_host" if host_only else "mgwfbp_ctx_create"
        _check(fn, getattr(lib(), fn)(C.byref(self._h), _ptr(ne, _u64p), int(ne.shape[0]), _ptr(m, _u8p),
                                      int(P), int(grad_dtype)))
        L, G, Pq, dt, tile, nt = (C.c_int32() for _ in range(6))
        arena = C.c_uint64()
        _check("mgwfbp_ctx_dims", lib().mgwfbp_ctx_dims(self._h, C.byref(L), C.byref(G), C.byref(Pq), C.byref(dt),
                                                        C.byref(arena), C.byref(tile), C.byref(nt)))
        self.L, self.n_groups, self.P, self.grad_dtype = L.value, G.value, Pq.value, dt.value
        self.arena_elems, self.tile_elems, self.n_tiles = arena.value, tile.value, nt.value

    def close(self) -> None:
        if self._h:
            lib().mgwfbp_ctx_destroy(self._h)
            self._h = _vp(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- inspection -------------------------------------------------------------------
    def layout(self):
        """mgwfbp_ctx_layout -> (tensor_off[L], tensor_group[L], group_base[G], group_elems[G])."""
        off = np.zeros(self.L, np.uint64)
        grp = np.zeros(self.L, np.int32)
        base = np.zeros(self.n_groups, np.uint64)
        ge = np.zeros(self.n_groups, np.uint64)
        _check("mgwfbp_ctx_layout", lib().mgwfbp_ctx_layout(self._h, _ptr(off, _u64p), _ptr(grp, _i32p),
                                                            _ptr(base, _u64p), _ptr(ge, _u64p)))
        return off, grp, base, ge

    def tables(self):
        """mgwfbp_ctx_tables -> dict of the tile / segment tables that drive the kernels."""
        S = C.c_int32()
        _check("mgwfbp_ctx_tables", lib().mgwfbp_ctx_tables(self._h, C.byref(S), None, None, None, None, None))
        tiles = np.zeros(self.n_tiles, TILE_HDR_DTYPE)
        seg_off = np.zeros(S.value + 1, np.uint64)
        seg_n = np.zeros(S.value, np.uint32)
        seg_layer = np.zeros(S.value, np.int32)
        group_tile = np.zeros(self.n_groups + 1, np.int32)
        _check("mgwfbp_ctx_tables", lib().mgwfbp_ctx_tables(
            self._h, C.byref(S), tiles.ctypes.data_as(_vp), _ptr(seg_off, _u64p), _ptr(seg_n, _u32p),
            _ptr(seg_layer, _i32p), _ptr(group_tile, _i32p)))
        return {"tiles": tiles, "seg_off": seg_off, "seg_n": seg_n, "seg_layer": seg_layer,
                "group_tile": group_tile}

    def set_launch(self, blocks_per_cu: int = 0, xcd_contiguous: bool = False, tiles_per_workgroup: int = 0) -> None:
        _check("mgwfbp_ctx_set_launch", lib().mgwfbp_ctx_set_launch(self._h, int(blocks_per_cu), int(bool(xcd_contiguous)),
                                                                    int(tiles_per_workgroup)))

    def set_pacing(self, workgroups_per_cu: int = 0, vectors_per_step: int = 0) -> None:
        _check("mgwfbp_ctx_set_pacing", lib().mgwfbp_ctx_set_pacing(self._h, int(workgroups_per_cu), int(vectors_per_step)))

    def set_small_launch(self, max_tiles: int = -1) -> None:
        _check("mgwfbp_ctx_set_small_launch", lib().mgwfbp_ctx_set_small_launch(self._h, int(max_tiles)))

    def set_resident_bytes(self, nbytes: int) -> None:
        _check("mgwfbp_ctx_set_resident_bytes", lib().mgwfbp_ctx_set_resident_bytes(self._h, int(nbytes)))

    # ---- device calls: addresses are plain integers ---------------------------------------
    def pack(self, group: int, d_grad_ptrs: int, d_merge_bufs: int, stream: int = 0) -> None:
        _check("mgwfbp_pack", lib().mgwfbp_pack(self._h, int(group), _vp(d_grad_ptrs), _vp(d_merge_bufs), _vp(stream)))

    def pack_tensors(self, first_tensor: int, last_tensor: int, d_grad_ptrs: int, d_merge_bufs: int,
                     stream: int = 0) -> None:
        _check("mgwfbp_pack_tensors", lib().mgwfbp_pack_tensors(self._h, int(first_tensor), int(last_tensor),
                                                                _vp(d_grad_ptrs), _vp(d_merge_bufs), _vp(stream)))

    def reduce(self, group: int, d_merge_bufs: int, d_reduced: int, stream: int = 0) -> None:
        _check("mgwfbp_reduce", lib().mgwfbp_reduce(self._h, int(group), _vp(d_merge_bufs), _vp(d_reduced), _vp(stream)))

    def unpack_update(self, group: int, d_reduced: int, d_w_ptrs: int, d_v_ptrs: int, lr: float, momentum: float,
                      stream: int = 0) -> None:
        _check("mgwfbp_unpack_update", lib().mgwfbp_unpack_update(
            self._h, int(group), _vp(d_reduced), _vp(d_w_ptrs), _vp(d_v_ptrs), float(lr), float(momentum), _vp(stream)))

    def reduce_update(self, group: int, d_merge_bufs: int, d_w_ptrs: int, d_v_ptrs: int, lr: float, momentum: float,
                      stream: int = 0) -> None:
        _check("mgwfbp_reduce_update", lib().mgwfbp_reduce_update(
            self._h, int(group), _vp(d_merge_bufs), _vp(d_w_ptrs), _vp(d_v_ptrs), float(lr), float(momentum), _vp(stream)))

    def group_pipeline(self, group: int, d_grad_ptrs: int, d_merge_bufs: int, d_reduced: int, d_w_ptrs: int,
                       d_v_ptrs: int, lr: float, momentum: float, stream: int = 0) -> None:
        _check("mgwfbp_group_pipeline", lib().mgwfbp_group_pipeline(
            self._h, int(group), _vp(d_grad_ptrs), _vp(d_merge_bufs), _vp(d_reduced or None), _vp(d_w_ptrs),
            _vp(d_v_ptrs), float(lr), float(momentum), _vp(stream)))

    def direct_update(self, group: int, d_grad_ptrs: int, d_reduced: int, d_w_ptrs: int, d_v_ptrs: int,
                      lr: float, momentum: float, stream: int = 0) -> None:
        _check("mgwfbp_direct_update", lib().mgwfbp_direct_update(
            self._h, int(group), _vp(d_grad_ptrs), _vp(d_reduced or None), _vp(d_w_ptrs), _vp(d_v_ptrs),
            float(lr), float(momentum), _vp(stream)))

    def group_pipeline_span(self, group_first: int, group_count: int, d_grad_ptrs: int, d_merge_bufs: int,
                            d_reduced: int, d_w_ptrs: int, d_v_ptrs: int, lr: float, momentum: float,
                            stream: int = 0) -> None:
        _check("mgwfbp_group_pipeline_span", lib().mgwfbp_group_pipeline_span(
            self._h, int(group_first), int(group_count), _vp(d_grad_ptrs), _vp(d_merge_bufs), _vp(d_reduced or None),
            _vp(d_w_ptrs), _vp(d_v_ptrs), float(lr), float(momentum), _vp(stream)))

    def group_pipeline_static(self, group: int, d_grad_ptrs: int, d_merge_bufs: int, d_reduced: int, d_w_ptrs: int,
                              d_v_ptrs: int, lr: float, momentum: float, stream: int = 0) -> None:
        _check("mgwfbp_group_pipeline_static", lib().mgwfbp_group_pipeline_static(
            self._h, int(group), _vp(d_grad_ptrs), _vp(d_merge_bufs), _vp(d_reduced or None), _vp(d_w_ptrs),
            _vp(d_v_ptrs), float(lr), float(momentum), _vp(stream)))

    def handler_replay(self, group_ready_s: Sequence[float], time_scale: float, max_groups_per_launch: int,
                       streams: Sequence[int], d_grad_ptrs: int, d_merge_bufs: int, d_reduced: int, d_w_ptrs: int, d_v_ptrs: int,
                       lr: float, momentum: float):
        """mgwfbp_handler_replay (blocks until the work is done) -> (launches, last_ready_s, done_s, exposed_s)."""
        ready = _arr(group_ready_s, np.float64)
        if ready.shape[0] != self.n_groups:
            raise ValueError("group_ready_s must have one entry per group")
        table = (_vp * max(len(streams), 1))(*[int(x) for x in streams])
        stats = np.zeros(4, np.float64)
        _check("mgwfbp_handler_replay", lib().mgwfbp_handler_replay(
            self._h, _ptr(ready, _f64p), float(time_scale), int(max_groups_per_launch), table, len(streams), _vp(d_grad_ptrs), _vp(d_merge_bufs),
            _vp(d_reduced or None), _vp(d_w_ptrs), _vp(d_v_ptrs), float(lr), float(momentum), _ptr(stats, _f64p)))
        return int(stats[0]), float(stats[1]), float(stats[2]), float(stats[3])
