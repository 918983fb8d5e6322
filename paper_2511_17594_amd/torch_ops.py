"""PyTorch operators over the C-ABI library (the paper's Implementation section exposes
`autosage::spmm_csr`, `autosage::spmm_csr_split` and `autosage::sddmm_csr`, and its CSR-attention
subsection adds `sddmm_csr_auto` and `csr_attention_forward`).

Importing this module registers, in the `autosage` namespace of `torch.ops`:

    spmm_csr(rowptr, colind, val, B) -> C                    selector-chosen schedule
    spmm_csr_split(rowptr, colind, val, B, hub_t) -> C       wavefront-per-row + hub split at hub_t
    sddmm_csr(rowptr, colind, X, Y) -> out                   selector-chosen schedule ("sddmm_csr_auto")
    csr_row_softmax(rowptr, s) -> P                          s is [nnz] or [nnz, H]
    csr_attention_forward(rowptr, colind, Q, K, V, scale) -> O

Every arithmetic step runs in the library's HIP kernels; this file only allocates outputs and
workspaces with torch, passes pointers, and wires the adjoints (themselves library calls: SpMM on
the transposed pattern, SDDMM, the row-softmax backward) into autograd.  Index tensors are int32 on
the GPU; dense tensors are float32 (bfloat16 is accepted as an input dtype of the forward kernels).
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import torch

from . import binding as ab

_handles: Dict[int, ab.Handle] = {}
_transposes: Dict[Tuple, Tuple] = {}
# rowptr address -> (its storage, kept alive; the tensor version seen).  The library remembers the degree features of
# a graph per rowptr address; an entry here pins the storage, so that the address cannot be handed to another graph
# while the library still remembers it, and records the version, so that an in-place overwrite is noticed.
_patterns: Dict[int, Tuple] = {}
_MAX_PATTERNS = 16


def handle(device: Optional[torch.device] = None) -> ab.Handle:
    """The per-device library handle used by the operators (created on first use)."""
    idx = torch.cuda.current_device() if device is None or device.index is None else device.index
    if idx not in _handles:
        _handles[idx] = ab.Handle(idx)
    return _handles[idx]


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ab.F32
    if t.dtype == torch.bfloat16:
        return ab.BF16
    if t.dtype == torch.float16:
        return ab.F16
    raise TypeError("dense operands must be float32, bfloat16 or float16, got %s" % t.dtype)


def _check_csr(rowptr, colind):
    if rowptr.dtype != torch.int32 or colind.dtype != torch.int32 or not rowptr.is_cuda or not colind.is_cuda:
        raise TypeError("rowptr and colind must be int32 CUDA tensors")
    _note_pattern(rowptr)


def _note_pattern(rowptr: torch.Tensor):
    """Keeps the library's per-address memory of degree features in step with the tensors: a rowptr that was
    overwritten in place is forgotten, and so is the oldest one when more than 16 are pinned."""
    ptr = rowptr.data_ptr()
    seen = _patterns.pop(ptr, None)
    if seen is not None and seen[1] != rowptr._version:
        handle(rowptr.device).forget_graph(ptr)
    _patterns[ptr] = (rowptr.untyped_storage(), rowptr._version, rowptr.device)
    while len(_patterns) > _MAX_PATTERNS:
        old_ptr = next(iter(_patterns))
        _, _, dev = _patterns.pop(old_ptr)
        handle(dev).forget_graph(old_ptr)


def csr_indices_int32(rowptr: torch.Tensor, colind: torch.Tensor, n_cols: int):
    """int32 copies of int64 CSR index tensors (what `torch.sparse_csr_tensor` holds by default), made on the
    device by the library; raises when an index does not fit the 32-bit kernels.  int32 inputs pass through."""
    if rowptr.dtype == torch.int32 and colind.dtype == torch.int32:
        return rowptr, colind
    if rowptr.dtype != torch.int64 or colind.dtype != torch.int64 or not rowptr.is_cuda or not colind.is_cuda:
        raise TypeError("rowptr and colind must both be int32 or both be int64 CUDA tensors")
    h = handle(rowptr.device)
    rp = torch.empty(rowptr.numel(), dtype=torch.int32, device=rowptr.device)
    ci = torch.empty(colind.numel(), dtype=torch.int32, device=colind.device)
    h.narrow_indices(rowptr.contiguous(), rp, colind.numel())
    h.narrow_indices(colind.contiguous(), ci, max(n_cols - 1, 0))
    return rp, ci


def _spmm(rowptr, colind, val, B, sched, n_rows=None, ldb=None, out=None, ldc=None, F=None):
    _check_csr(rowptr, colind)
    h = handle(B.device)
    n_rows = rowptr.numel() - 1 if n_rows is None else n_rows
    n_cols = B.shape[0]
    F = B.shape[1] if F is None else F
    nnz = colind.numel()
    C = torch.empty((n_rows, F), dtype=torch.float32, device=B.device) if out is None else out
    ws = _ws(h.workspace_bytes(ab.OP_SPMM, n_rows, nnz, F, 1, sched), B.device)
    h.spmm(n_rows, n_cols, rowptr, colind, val, B, C, F, dt=_dt(B), sched=sched, workspace=ws, nnz=nnz, ldb=ldb, ldc=ldc)
    return C


def _sddmm(rowptr, colind, X, Y, sched=None, ldx=None, ldy=None, F=None, out=None):
    _check_csr(rowptr, colind)
    h = handle(X.device)
    n_rows, n_cols = rowptr.numel() - 1, Y.shape[0]
    F = X.shape[1] if F is None else F
    nnz = colind.numel()
    out = torch.empty(nnz, dtype=torch.float32, device=X.device) if out is None else out
    ws = _ws(h.workspace_bytes(ab.OP_SDDMM, n_rows, nnz, F, 1, sched), X.device)
    h.sddmm(n_rows, n_cols, rowptr, colind, X, Y, out, F, dt=_dt(X), sched=sched, workspace=ws, nnz=nnz, ldx=ldx, ldy=ldy)
    return out


def transpose(rowptr: torch.Tensor, colind: torch.Tensor, n_cols: int):
    """(t_rowptr, t_colind, perm) of the pattern, cached per (address, version) of the index tensors.  An entry
    holds the index tensors themselves: while it lives their memory cannot be freed and handed to another pattern
    of the same size, so an equal key always means the same pattern."""
    key = (rowptr.data_ptr(), colind.data_ptr(), rowptr._version, colind._version, colind.numel(), n_cols)
    hit = _transposes.get(key)
    if hit is not None:
        return hit[:3]
    h = handle(rowptr.device)
    n_rows, nnz = rowptr.numel() - 1, colind.numel()
    t_rowptr = torch.empty(n_cols + 1, dtype=torch.int32, device=rowptr.device)
    t_colind = torch.empty(max(nnz, 1), dtype=torch.int32, device=rowptr.device)
    perm = torch.empty(max(nnz, 1), dtype=torch.int32, device=rowptr.device)
    ws = _ws(h.csr_transpose_workspace_bytes(n_rows, n_cols, nnz), rowptr.device)
    h.csr_transpose(n_rows, n_cols, nnz, rowptr, colind, None, t_rowptr, t_colind, None, perm, ws)
    if len(_transposes) >= 8:
        _transposes.pop(next(iter(_transposes)))
    _transposes[key] = (t_rowptr, t_colind[:nnz], perm[:nnz], rowptr, colind)
    return _transposes[key][:3]


def _gather(perm, values):
    """values[perm] through the library (values is [nnz] or [nnz, w] float32)."""
    out = torch.empty_like(values)
    w = 1 if values.dim() == 1 else values.shape[1]
    handle(values.device).gather_values(perm.numel(), w, perm, values.contiguous(), out)
    return out


# ----------------------------------------------------------------------------- SpMM ---
@torch.library.custom_op("autosage::spmm_csr", mutates_args=())
def spmm_csr(rowptr: torch.Tensor, colind: torch.Tensor, val: torch.Tensor, B: torch.Tensor) -> torch.Tensor:
    return _spmm(rowptr, colind, val, B.contiguous(), None)


@torch.library.custom_op("autosage::spmm_csr_split", mutates_args=())
def spmm_csr_split(rowptr: torch.Tensor, colind: torch.Tensor, val: torch.Tensor, B: torch.Tensor, hub_t: int) -> torch.Tensor:
    sched = ab.Schedule(mapping=ab.MAP_WAVE_ROW, hub_t=hub_t, hub_chunk=hub_t)
    return _spmm(rowptr, colind, val, B.contiguous(), sched)


def _spmm_fake(rowptr, colind, val, B, *_):
    return B.new_empty((rowptr.shape[0] - 1, B.shape[1]), dtype=torch.float32)


spmm_csr.register_fake(_spmm_fake)
spmm_csr_split.register_fake(_spmm_fake)


def _spmm_setup(ctx, inputs, output):
    rowptr, colind, val, B = inputs[:4]
    ctx.save_for_backward(rowptr, colind, val, B)


def _spmm_backward(ctx, dC):
    rowptr, colind, val, B = ctx.saved_tensors
    dC = dC.contiguous()
    dval = dB = None
    if ctx.needs_input_grad[3]:
        t_rowptr, t_colind, perm = transpose(rowptr, colind, B.shape[0])
        dB = _spmm(t_rowptr, t_colind, _gather(perm, val), dC, None, n_rows=B.shape[0]).to(B.dtype)
    if ctx.needs_input_grad[2]:
        dval = _sddmm(rowptr, colind, dC, B.float().contiguous())
    return (None, None, dval, dB) + (None,) * (len(ctx.needs_input_grad) - 4)


spmm_csr.register_autograd(_spmm_backward, setup_context=_spmm_setup)
spmm_csr_split.register_autograd(_spmm_backward, setup_context=_spmm_setup)


# ---------------------------------------------------------------------------- SDDMM ---
@torch.library.custom_op("autosage::sddmm_csr", mutates_args=())
def sddmm_csr(rowptr: torch.Tensor, colind: torch.Tensor, X: torch.Tensor, Y: torch.Tensor) -> torch.Tensor:
    return _sddmm(rowptr, colind, X.contiguous(), Y.contiguous())


@sddmm_csr.register_fake
def _(rowptr, colind, X, Y):
    return X.new_empty((colind.shape[0],), dtype=torch.float32)


def _sddmm_setup(ctx, inputs, output):
    ctx.save_for_backward(*inputs)


def _sddmm_backward(ctx, dout):
    rowptr, colind, X, Y = ctx.saved_tensors
    dout = dout.contiguous()
    dX = dY = None
    if ctx.needs_input_grad[2]:       # dX_i = sum_p dout[p] Y_j
        dX = _spmm(rowptr, colind, dout, Y.contiguous(), None).to(X.dtype)
    if ctx.needs_input_grad[3]:       # dY_j = sum_{p: col = j} dout[p] X_i
        t_rowptr, t_colind, perm = transpose(rowptr, colind, Y.shape[0])
        dY = _spmm(t_rowptr, t_colind, _gather(perm, dout), X.contiguous(), None, n_rows=Y.shape[0]).to(Y.dtype)
    return None, None, dX, dY


sddmm_csr.register_autograd(_sddmm_backward, setup_context=_sddmm_setup)


# -------------------------------------------------------------------------- softmax ---
def _softmax_hub(rowptr):
    return 1024          # rows this long are split; shorter graphs never reach it


@torch.library.custom_op("autosage::csr_row_softmax", mutates_args=())
def csr_row_softmax(rowptr: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    h = handle(s.device)
    s = s.contiguous()
    n_rows, nnz = rowptr.numel() - 1, s.shape[0]
    H = 1 if s.dim() == 1 else s.shape[1]
    out = torch.zeros_like(s)            # entries of empty rows do not exist; zeros keep the result defined
    hub = _softmax_hub(rowptr)
    ws = _ws(h.workspace_bytes(ab.OP_SOFTMAX, n_rows, nnz, 1, H, ab.Schedule(hub_t=hub)), s.device)
    h.csr_row_softmax(n_rows, nnz, rowptr, s, out, H=H, hub_t=hub, workspace=ws)
    return out


@csr_row_softmax.register_fake
def _(rowptr, s):
    return torch.empty_like(s)


def _softmax_setup(ctx, inputs, output):
    ctx.save_for_backward(inputs[0], output)


def _softmax_backward(ctx, dP):
    rowptr, P = ctx.saved_tensors
    h = handle(P.device)
    dP = dP.contiguous()
    n_rows, nnz = rowptr.numel() - 1, P.shape[0]
    H = 1 if P.dim() == 1 else P.shape[1]
    dS = torch.empty_like(P)
    hub = _softmax_hub(rowptr)
    ws = _ws(h.workspace_bytes(ab.OP_SOFTMAX, n_rows, nnz, 1, H, ab.Schedule(hub_t=hub)), P.device)
    h.csr_row_softmax_backward(n_rows, nnz, rowptr, P, dP, dS, H=H, hub_t=hub, workspace=ws)
    return None, dS


csr_row_softmax.register_autograd(_softmax_backward, setup_context=_softmax_setup)


# ------------------------------------------------------------------------ attention ---
@torch.library.custom_op("autosage::csr_attention_forward", mutates_args=())
def csr_attention_forward(rowptr: torch.Tensor, colind: torch.Tensor, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                          scale: float) -> torch.Tensor:
    _check_csr(rowptr, colind)
    h = handle(Q.device)
    Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
    N, H, d = Q.shape
    nnz = colind.numel()
    O = torch.empty((N, H, d), dtype=torch.float32, device=Q.device)
    ws = _ws(h.workspace_bytes(ab.OP_ATTENTION, N, nnz, d, H), Q.device)
    h.csr_attention(N, rowptr, colind, Q, K, V, O, H, d, scale, in_dt=_dt(Q), workspace=ws, nnz=nnz)
    return O


@csr_attention_forward.register_fake
def _(rowptr, colind, Q, K, V, scale):
    return Q.new_empty(Q.shape, dtype=torch.float32)


def _attention_setup(ctx, inputs, output):
    rowptr, colind, Q, K, V, scale = inputs
    ctx.save_for_backward(rowptr, colind, Q, K, V)
    ctx.scale = scale


def _attention_backward(ctx, dO):
    """One library call (autosage_csr_attention_backward): probabilities recomputed from Q and K, then
    dV = P^T dO, dP = <dO, V>, dS = scale * softmax'(P, dP), dQ = dS K, dK = dS^T Q, all heads at once."""
    rowptr, colind, Q, K, V = ctx.saved_tensors
    h = handle(Q.device)
    N, H, d = Q.shape
    nnz = colind.numel()
    Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
    dO = dO.float().contiguous()
    t_rowptr, t_colind, perm = transpose(rowptr, colind, N)
    dQ, dK, dV = (torch.empty((N, H, d), dtype=torch.float32, device=Q.device) for _ in range(3))
    hub = 512            # rows of the pattern, and of its transpose, this long are split over workgroups
    ws = _ws(h.csr_attention_backward_workspace_bytes(N, nnz, H, d, hub), Q.device)
    h.csr_attention_backward(N, rowptr, colind, t_rowptr, t_colind, perm, Q, K, V, dO, dQ, dK, dV, H, d, ctx.scale,
                             in_dt=_dt(Q), hub_t=hub, workspace=ws, nnz=nnz)
    return None, None, dQ.to(Q.dtype), dK.to(K.dtype), dV.to(V.dtype), None


def _softmax_backward_raw(rowptr, P, dP):
    h = handle(P.device)
    n_rows, nnz = rowptr.numel() - 1, P.shape[0]
    dS = torch.empty_like(P)
    hub = _softmax_hub(rowptr)
    ws = _ws(h.workspace_bytes(ab.OP_SOFTMAX, n_rows, nnz, 1, 1, ab.Schedule(hub_t=hub)), P.device)
    h.csr_row_softmax_backward(n_rows, nnz, rowptr, P, dP, dS, H=1, hub_t=hub, workspace=ws)
    return dS


csr_attention_forward.register_autograd(_attention_backward, setup_context=_attention_setup)

# the paper's name for the scheduler-routed SDDMM
sddmm_csr_auto = sddmm_csr
