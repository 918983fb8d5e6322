"""Thin ctypes binding of libautosage.so (argument marshalling only).

Every function mirrors the C entry point of the same name in include/autosage.h.
Device arrays are torch tensors (used for memory and streams only); every step of
the computation runs in the library's HIP kernels.  There is no CPU fallback:
if the library cannot be loaded, importing this module raises.
"""
from __future__ import annotations

import ctypes
import json
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libautosage.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_HIP, ERR_IO, ERR_REPLAY_MISS = range(7)
F32, BF16, F16 = 0, 1, 2
OP_SPMM, OP_SDDMM, OP_SOFTMAX, OP_ATTENTION = 0, 1, 2, 3
MAP_PLAIN, MAP_WAVE_ROW, MAP_MULTI_ROW, MAP_FUSED = 0, 1, 2, 3


class Schedule(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("mapping", "f_tile", "waves_per_wg", "vec_bytes", "unroll", "hub_t", "hub_chunk", "xcd_remap", "group_lanes")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}

    def __repr__(self):
        return "Schedule(%s)" % ", ".join("%s=%d" % kv for kv in self.as_dict().items())


class AutosageError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libautosage.so is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "or `python paper_2511_17594_amd/build.py`")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i64, i32, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_size_t
    sp = c.POINTER(Schedule)
    sigs = {
        "autosage_create": [c.POINTER(vp), c.c_int],
        "autosage_destroy": [vp],
        "autosage_set_param": [vp, c.c_char_p, c.c_double],
        "autosage_get_param": [vp, c.c_char_p, c.POINTER(c.c_double)],
        "autosage_spmm": [vp, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, i32, c.c_int, sp, vp, sz, vp],
        "autosage_spmm_static": [vp, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, i32, c.c_int, sp, vp],
        "autosage_sddmm": [vp, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, i32, c.c_int, vp, sp, vp, sz, vp],
        "autosage_csr_row_softmax": [vp, i64, i64, vp, vp, vp, i32, i32, i32, vp, sz, vp],
        "autosage_csr_attention": [vp, i64, i64, vp, vp, vp, vp, vp, vp, vp, i32, i32, c.c_float, c.c_int, sp, vp, sz, vp],
        "autosage_workspace_bytes": [vp, c.c_int, i64, i64, i32, i32, sp, c.POINTER(sz)],
        "autosage_hub_partition": [vp, i64, vp, i32, i32, c.POINTER(i32), vp, vp, c.POINTER(i32), vp, vp, sz, vp],
        "autosage_graph_features": [vp, i64, i64, vp, c.POINTER(i64), c.POINTER(i64), c.POINTER(i64),
                                    c.POINTER(c.c_uint64), vp],
        "autosage_validate_csr": [vp, i64, i64, i64, vp, vp, vp],
        "autosage_narrow_indices": [vp, i64, vp, vp, i64, vp],
        "autosage_shortlist": [vp, c.c_int, i64, i64, i64, c.POINTER(i64), i64, i32, c.c_int, i32, sp,
                               c.POINTER(c.c_double), i32, c.POINTER(i32)],
        "autosage_decide_from_times": [i32, c.POINTER(c.c_double), c.c_double, c.c_double, c.POINTER(i32)],
        "autosage_decide": [vp, c.c_int, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, vp, i64, i32, c.c_int, vp, sz, vp, sp],
        "autosage_last_decision": [vp, c.c_char_p, sz],
        "autosage_cache_load": [vp, c.c_char_p],
        "autosage_cache_save": [vp, c.c_char_p],
        "autosage_cache_clear": [vp],
        "autosage_forget_graph": [vp, vp],
        "autosage_cache_lookup": [vp, c.c_uint64, i32, i32, c.c_int, c.c_int, sp, c.POINTER(i32)],
        "autosage_cache_insert": [vp, c.c_uint64, i32, i32, c.c_int, c.c_int, sp],
        "autosage_decide_attention": [vp, i64, i64, vp, vp, vp, vp, vp, vp, i32, i32, c.c_float, c.c_int, vp, sz, vp, sp],
        "autosage_baseline_schedule": [sp],
        "autosage_csr_row_softmax_backward": [vp, i64, i64, vp, vp, vp, vp, i32, i32, i32, vp, sz, vp],
        "autosage_csr_transpose_workspace_bytes": [vp, i64, i64, i64, c.POINTER(sz)],
        "autosage_csr_transpose": [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        "autosage_gather_values": [vp, i64, i32, vp, vp, vp, vp],
        "autosage_csr_attention_backward_workspace_bytes": [vp, i64, i64, i32, i32, i32, i32, c.POINTER(sz)],
        "autosage_csr_attention_backward": [vp, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32,
                                            c.c_float, c.c_int, i32, i32, vp, sz, vp],
        "autosage_stream_probe": [vp, c.c_int, vp, vp, sz, vp],
        "autosage_stream_probe_dst_bytes": [vp, c.POINTER(sz)],
        "autosage_gather_probe": [vp, vp, i64, i32, vp, i64, vp, vp],
        "autosage_profile_begin": [vp],
        "autosage_profile_read": [vp, c.c_char_p, sz],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)          # raises AttributeError if the library lacks a declared symbol
        fn.argtypes = args
        fn.restype = c.c_int
    lib.autosage_status_string.argtypes = [c.c_int]
    lib.autosage_status_string.restype = c.c_char_p
    return lib, sorted(list(sigs) + ["autosage_status_string"])


_lib, EXPORTED = _load()


STREAM_READ, STREAM_COPY, STREAM_INPLACE = 0, 1, 2
STATIC_SCRATCH_BYTES = 32 << 20


def status_string(status: int) -> str:
    return _lib.autosage_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise AutosageError(status, where)


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    return ctypes.c_void_p(t.data_ptr())


def _sched(s: Optional[Schedule]):
    return None if s is None else ctypes.byref(s)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(getattr(stream, "cuda_stream", stream))


def baseline_schedule() -> Schedule:
    s = Schedule()
    _check(_lib.autosage_baseline_schedule(ctypes.byref(s)), "autosage_baseline_schedule")
    return s


def decide_from_times(t_cand, t_baseline: float, alpha: float) -> int:
    n = len(t_cand)
    arr = (ctypes.c_double * max(n, 1))(*[float(x) for x in t_cand])
    choice = ctypes.c_int32(0)
    _check(_lib.autosage_decide_from_times(n, arr, float(t_baseline), float(alpha), ctypes.byref(choice)),
           "autosage_decide_from_times")
    return int(choice.value)


class Handle:
    """Owner of an autosage_handle_t.  device < 0 gives a host-only handle (selector, cache, estimate)."""

    def __init__(self, device: int = 0):
        self._h = ctypes.c_void_p()
        _check(_lib.autosage_create(ctypes.byref(self._h), int(device)), "autosage_create")
        self.device = device

    def close(self):
        if self._h:
            _lib.autosage_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- parameters --------------------------------------------------------------------
    def set_param(self, name: str, value: float):
        _check(_lib.autosage_set_param(self._h, name.encode(), float(value)), "autosage_set_param(%s)" % name)

    def get_param(self, name: str) -> float:
        v = ctypes.c_double()
        _check(_lib.autosage_get_param(self._h, name.encode(), ctypes.byref(v)), "autosage_get_param(%s)" % name)
        return float(v.value)

    # -- hot path ----------------------------------------------------------------------
    def workspace_bytes(self, op: int, n_rows: int, nnz: int, F: int, H: int = 1, sched: Optional[Schedule] = None) -> int:
        out = ctypes.c_size_t()
        _check(_lib.autosage_workspace_bytes(self._h, op, n_rows, nnz, F, H, _sched(sched), ctypes.byref(out)),
               "autosage_workspace_bytes")
        return int(out.value)

    def spmm(self, n_rows, n_cols, rowptr, colind, val, B, C, F, dt=F32, sched=None, workspace=None, stream=None,
             ldb=None, ldc=None, nnz=None):
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_spmm(self._h, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(val), _ptr(B),
                                  F if ldb is None else ldb, _ptr(C), F if ldc is None else ldc, F, dt, _sched(sched),
                                  _ptr(workspace), ws_bytes, _stream(stream)), "autosage_spmm")

    def spmm_static(self, n_rows, n_cols, rowptr, colind, val, B, C, F, sched, dt=F32, stream=None, ldb=None, ldc=None,
                    nnz=None):
        """autosage_spmm_static: explicit schedule, scratch in the library's fixed array, nothing allocated."""
        nnz = int(colind.numel()) if nnz is None else nnz
        _check(_lib.autosage_spmm_static(self._h, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(val), _ptr(B),
                                         F if ldb is None else ldb, _ptr(C), F if ldc is None else ldc, F, dt, _sched(sched),
                                         _stream(stream)), "autosage_spmm_static")

    def sddmm(self, n_rows, n_cols, rowptr, colind, X, Y, out, F, dt=F32, sched=None, workspace=None, stream=None,
              ldx=None, ldy=None, nnz=None, val=None):
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_sddmm(self._h, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(val), _ptr(X),
                                   F if ldx is None else ldx, _ptr(Y), F if ldy is None else ldy, F, dt, _ptr(out),
                                   _sched(sched), _ptr(workspace), ws_bytes, _stream(stream)), "autosage_sddmm")

    def csr_row_softmax(self, n_rows, nnz, rowptr, s_in, s_out, H=1, hub_t=0, hub_chunk=0, workspace=None, stream=None):
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_csr_row_softmax(self._h, n_rows, nnz, _ptr(rowptr), _ptr(s_in), _ptr(s_out), H, hub_t,
                                             hub_chunk, _ptr(workspace), ws_bytes, _stream(stream)),
               "autosage_csr_row_softmax")

    def csr_attention(self, N, rowptr, colind, Q, K, V, O, H, d, scale, in_dt=BF16, sched=None, workspace=None,
                      stream=None, nnz=None):
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_csr_attention(self._h, N, nnz, _ptr(rowptr), _ptr(colind), None, _ptr(Q), _ptr(K), _ptr(V),
                                           _ptr(O), H, d, float(scale), in_dt, _sched(sched), _ptr(workspace), ws_bytes,
                                           _stream(stream)), "autosage_csr_attention")

    # -- adjoint helpers --------------------------------------------------------------
    def csr_row_softmax_backward(self, n_rows, nnz, rowptr, P, dP, dS, H=1, hub_t=0, hub_chunk=0, workspace=None,
                                 stream=None):
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_csr_row_softmax_backward(self._h, n_rows, nnz, _ptr(rowptr), _ptr(P), _ptr(dP), _ptr(dS), H,
                                                      hub_t, hub_chunk, _ptr(workspace), ws_bytes, _stream(stream)),
               "autosage_csr_row_softmax_backward")

    def csr_transpose_workspace_bytes(self, n_rows, n_cols, nnz) -> int:
        out = ctypes.c_size_t()
        _check(_lib.autosage_csr_transpose_workspace_bytes(self._h, n_rows, n_cols, nnz, ctypes.byref(out)),
               "autosage_csr_transpose_workspace_bytes")
        return int(out.value)

    def csr_transpose(self, n_rows, n_cols, nnz, rowptr, colind, val, t_rowptr, t_colind, t_val, perm, workspace,
                      stream=None):
        ws_bytes = workspace.numel() * workspace.element_size()
        _check(_lib.autosage_csr_transpose(self._h, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(val),
                                           _ptr(t_rowptr), _ptr(t_colind), _ptr(t_val), _ptr(perm), _ptr(workspace),
                                           ws_bytes, _stream(stream)), "autosage_csr_transpose")

    def gather_values(self, n, width, perm, src, dst, stream=None):
        _check(_lib.autosage_gather_values(self._h, n, width, _ptr(perm), _ptr(src), _ptr(dst), _stream(stream)),
               "autosage_gather_values")

    # -- metadata ----------------------------------------------------------------------
    def csr_attention_backward_workspace_bytes(self, N, nnz, H, d, hub_t=0, hub_chunk=0) -> int:
        out = ctypes.c_size_t()
        _check(_lib.autosage_csr_attention_backward_workspace_bytes(self._h, N, nnz, H, d, hub_t, hub_chunk, ctypes.byref(out)),
               "autosage_csr_attention_backward_workspace_bytes")
        return int(out.value)

    def csr_attention_backward(self, N, rowptr, colind, t_rowptr, t_colind, perm, Q, K, V, dO, dQ, dK, dV, H, d, scale,
                               in_dt=BF16, hub_t=0, hub_chunk=0, workspace=None, stream=None, nnz=None):
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        _check(_lib.autosage_csr_attention_backward(self._h, N, nnz, _ptr(rowptr), _ptr(colind), _ptr(t_rowptr), _ptr(t_colind),
                                                    _ptr(perm), _ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(dQ), _ptr(dK),
                                                    _ptr(dV), H, d, scale, in_dt, hub_t, hub_chunk, _ptr(workspace), ws_bytes,
                                                    _stream(stream)), "autosage_csr_attention_backward")

    def hub_partition(self, n_rows, rowptr, hub_t, hub_chunk, hub_rows, chunk_ptr, light_rows, workspace, stream=None):
        """Fills the device tensors hub_rows / chunk_ptr / light_rows; returns (n_hub, n_light)."""
        nh, nl = ctypes.c_int32(), ctypes.c_int32()
        ws_bytes = workspace.numel() * workspace.element_size()
        _check(_lib.autosage_hub_partition(self._h, n_rows, _ptr(rowptr), hub_t, hub_chunk, ctypes.byref(nh),
                                           _ptr(hub_rows), _ptr(chunk_ptr), ctypes.byref(nl), _ptr(light_rows),
                                           _ptr(workspace), ws_bytes, _stream(stream)), "autosage_hub_partition")
        return int(nh.value), int(nl.value)

    def graph_features(self, n_rows, n_cols, rowptr, stream=None):
        """Returns (hist[33] list, max_deg, nnz, signature)."""
        hist = (ctypes.c_int64 * 33)()
        mx, nnz, sig = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_uint64()
        _check(_lib.autosage_graph_features(self._h, n_rows, n_cols, _ptr(rowptr), hist, ctypes.byref(mx),
                                            ctypes.byref(nnz), ctypes.byref(sig), _stream(stream)),
               "autosage_graph_features")
        return [int(x) for x in hist], int(mx.value), int(nnz.value), int(sig.value)

    def validate_csr(self, n_rows, n_cols, nnz, rowptr, colind, stream=None) -> bool:
        st = _lib.autosage_validate_csr(self._h, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _stream(stream))
        if st == OK:
            return True
        if st == ERR_INVALID_ARG:
            return False
        raise AutosageError(st, "autosage_validate_csr")

    # -- selector ----------------------------------------------------------------------
    def narrow_indices(self, src, dst, limit: int, stream=None):
        """dst (int32) = src (int64) on the device; raises when a value lies outside [0, limit]."""
        n = int(src.numel())
        _check(_lib.autosage_narrow_indices(self._h, n, _ptr(src), _ptr(dst), int(limit), _stream(stream)),
               "autosage_narrow_indices")

    def shortlist(self, op, n_rows, n_cols, nnz, hist33, max_deg, F, dt=F32, align_bytes=16, max_out=64):
        """Host only.  Returns [(Schedule, estimated seconds), ...] in ascending estimated time."""
        hist = (ctypes.c_int64 * 33)(*[int(x) for x in hist33])
        out = (Schedule * max_out)()
        est = (ctypes.c_double * max_out)()
        n = ctypes.c_int32()
        _check(_lib.autosage_shortlist(self._h, op, n_rows, n_cols, nnz, hist, max_deg, F, dt, align_bytes, out, est,
                                       max_out, ctypes.byref(n)), "autosage_shortlist")
        res = []
        for i in range(n.value):
            s = Schedule()
            ctypes.memmove(ctypes.byref(s), ctypes.byref(out[i]), ctypes.sizeof(Schedule))
            res.append((s, float(est[i])))
        return res

    def decide(self, op, n_rows, n_cols, rowptr, colind, val, dense0, dense1, out, F, dt=F32, workspace=None,
               stream=None, ld0=None, ld1=None, ld_out=None, nnz=None) -> Schedule:
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        chosen = Schedule()
        if ld_out is None:
            ld_out = F if op == OP_SPMM else 1
        _check(_lib.autosage_decide(self._h, op, n_rows, n_cols, nnz, _ptr(rowptr), _ptr(colind), _ptr(val), _ptr(dense0),
                                    F if ld0 is None else ld0, _ptr(dense1), F if ld1 is None else ld1, _ptr(out), ld_out,
                                    F, dt, _ptr(workspace), ws_bytes, _stream(stream), ctypes.byref(chosen)),
               "autosage_decide")
        return chosen

    def decide_attention(self, N, rowptr, colind, Q, K, V, O, H, d, scale, dt=BF16, workspace=None, stream=None,
                         nnz=None) -> Schedule:
        nnz = int(colind.numel()) if nnz is None else nnz
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        chosen = Schedule()
        _check(_lib.autosage_decide_attention(self._h, N, nnz, _ptr(rowptr), _ptr(colind), _ptr(Q), _ptr(K), _ptr(V),
                                              _ptr(O), H, d, float(scale), dt, _ptr(workspace), ws_bytes,
                                              _stream(stream), ctypes.byref(chosen)), "autosage_decide_attention")
        return chosen

    def last_decision(self) -> dict:
        buf = ctypes.create_string_buffer(1 << 16)
        _check(_lib.autosage_last_decision(self._h, buf, len(buf)), "autosage_last_decision")
        return json.loads(buf.value.decode())

    def stream_probe_dst_bytes(self) -> int:
        out = ctypes.c_size_t()
        _check(_lib.autosage_stream_probe_dst_bytes(self._h, ctypes.byref(out)), "autosage_stream_probe_dst_bytes")
        return int(out.value)

    def stream_probe(self, mode: int, src, dst, n_bytes: int, stream=None):
        """One launch of the plain streaming kernel `mode` (STREAM_READ / STREAM_COPY / STREAM_INPLACE) over n_bytes."""
        _check(_lib.autosage_stream_probe(self._h, mode, _ptr(src), _ptr(dst), n_bytes, _stream(stream)), "autosage_stream_probe")

    def gather_probe(self, table, n_table_rows: int, row_bytes: int, idx, dst, n_idx=None, stream=None):
        """One launch of the random-row gather kernel: rows idx[0..n_idx) of `row_bytes` bytes out of `table`."""
        n_idx = int(idx.numel()) if n_idx is None else n_idx
        _check(_lib.autosage_gather_probe(self._h, _ptr(table), n_table_rows, row_bytes, _ptr(idx), n_idx, _ptr(dst),
                                          _stream(stream)), "autosage_gather_probe")

    def profile_begin(self):
        _check(_lib.autosage_profile_begin(self._h), "autosage_profile_begin")

    def profile_read(self) -> dict:
        buf = ctypes.create_string_buffer(1 << 14)
        _check(_lib.autosage_profile_read(self._h, buf, len(buf)), "autosage_profile_read")
        return json.loads(buf.value.decode())

    def cache_load(self, path: str):
        _check(_lib.autosage_cache_load(self._h, path.encode()), "autosage_cache_load")

    def cache_save(self, path: str):
        _check(_lib.autosage_cache_save(self._h, path.encode()), "autosage_cache_save")

    def cache_clear(self):
        _check(_lib.autosage_cache_clear(self._h), "autosage_cache_clear")

    def forget_graph(self, rowptr_address: int):
        """Drops the remembered degree features of the graph whose rowptr started at this device address."""
        _check(_lib.autosage_forget_graph(self._h, ctypes.c_void_p(int(rowptr_address))), "autosage_forget_graph")

    def cache_lookup(self, graph_sig: int, F: int, op: int, dt: int = F32, H: int = 1) -> Optional[Schedule]:
        s, found = Schedule(), ctypes.c_int32()
        _check(_lib.autosage_cache_lookup(self._h, graph_sig, F, H, op, dt, ctypes.byref(s), ctypes.byref(found)),
               "autosage_cache_lookup")
        return s if found.value else None

    def cache_insert(self, graph_sig: int, F: int, op: int, dt: int, sched: Schedule, H: int = 1):
        _check(_lib.autosage_cache_insert(self._h, graph_sig, F, H, op, dt, ctypes.byref(sched)), "autosage_cache_insert")
