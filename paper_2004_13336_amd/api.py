"""Thin Python binding of the C-ABI library: argument marshalling and size checks only.

Function names and argument order follow include/shardupdate.h.  Tensors are torch CUDA
tensors (torch provides device memory and streams, nothing else); every step of the path runs
in the library's HIP kernels.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, Optional, Sequence, Tuple

import torch

from ._lib import AdafactorHP, AdamHP, LambHP, LarsHP, MomentumHP, ShardError, lib

SHARD_F32, SHARD_BF16 = 0, 1
SHARD_VAR_NO_DECAY, SHARD_VAR_NO_ADAPT = 1, 2
KERNEL_IDS = {"format": 0, "unshard": 1, "adam": 2, "momentum": 3, "lamb_p1": 4, "norm_reduce": 5,
              "lamb_p2": 6, "ptr_table": 7, "lars_p1": 8, "lars_p2": 9, "rowcol_p1": 10, "rowcol_p2": 11,
              "adafactor_state": 12, "adafactor_usq": 13, "adafactor_apply": 14, "plain_copy": 15, "item_total": 16, "adam_shape": 17}

_DTYPES = {torch.float32: SHARD_F32, torch.bfloat16: SHARD_BF16}


def _check(status: int, where: str) -> None:
    if status != 0:
        raise ShardError(status, where)


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev(t: Optional[torch.Tensor], numel: int, dtype, what: str) -> C.c_void_p:
    """Device pointer of a contiguous CUDA tensor with at least `numel` elements of `dtype`."""
    if t is None:
        return C.c_void_p(None)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous CUDA tensor" % what)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s, got %s" % (what, dtype, t.dtype))
    if t.numel() < numel:
        raise ValueError("%s holds %d elements, needs %d" % (what, t.numel(), numel))
    return C.c_void_p(t.data_ptr())


class Plan:
    """Owner of a shard_plan_t handle (and of the workspace tensor, if it allocated one)."""

    def __init__(self, numel: Sequence[int], N: int, align_elems: int = 8,
                 var_flags: Optional[Sequence[int]] = None, chunk_elems: int = 0, cols: Optional[Sequence[int]] = None):
        """Flat plan over numel[i] elements, or, with cols, a row plan over numel[i] x cols[i] matrices."""
        V = len(numel)
        arr = (C.c_int64 * max(V, 1))(*[int(n) for n in numel])
        flags = None
        if var_flags is not None:
            if len(var_flags) != V:
                raise ValueError("var_flags must have one entry per variable")
            flags = (C.c_uint32 * max(V, 1))(*[int(f) for f in var_flags])
        handle = C.c_void_p()
        if cols is None:
            _check(lib().shard_plan(V, arr, int(N), int(align_elems), flags, int(chunk_elems), C.byref(handle)),
                   "shard_plan")
            self.numel = tuple(int(n) for n in numel)
        else:
            if len(cols) != V:
                raise ValueError("cols must have one entry per variable")
            carr = (C.c_int64 * max(V, 1))(*[int(c) for c in cols])
            _check(lib().shard_plan_rows(V, arr, carr, int(N), int(align_elems), flags, int(chunk_elems),
                                         C.byref(handle)), "shard_plan_rows")
            self.numel = tuple(int(n) * int(c) for n, c in zip(numel, cols))
        self.handle = handle
        self.V, self.N, self.align = V, int(N), int(align_elems)
        S, total, nch, chunk, wsb = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int(), C.c_size_t()
        _check(lib().shard_plan_info(handle, C.byref(S), C.byref(total), C.byref(nch), C.byref(chunk), C.byref(wsb)),
               "shard_plan_info")
        self.S, self.total, self.n_chunks, self.workspace_bytes = S.value, total.value, nch.value, wsb.value
        self.chunk_elems = chunk.value
        self.workspace: Optional[torch.Tensor] = None

    def segments(self) -> Tuple[Tuple[int, ...], Tuple[int, ...]]:
        off = (C.c_int64 * max(self.V, 1))()
        length = (C.c_int64 * max(self.V, 1))()
        _check(lib().shard_plan_segments(self.handle, off, length), "shard_plan_segments")
        return tuple(off[: self.V]), tuple(length[: self.V])

    def real_count(self, r: int) -> Tuple[int, ...]:
        real = (C.c_int64 * max(self.V, 1))()
        _check(lib().shard_plan_real_count(self.handle, int(r), real), "shard_plan_real_count")
        return tuple(real[: self.V])

    def free(self) -> None:
        if self.handle is not None and self.handle.value:
            lib().shard_plan_free(self.handle)
        self.handle = None
        self.workspace = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def shard_plan(numel, N, align_elems=8, var_flags=None, chunk_elems=0) -> Plan:
    return Plan(numel, N, align_elems, var_flags, chunk_elems)


def shard_plan_rows(rows, cols, N, align_elems=8, var_flags=None, chunk_elems=0) -> Plan:
    return Plan(rows, N, align_elems, var_flags, chunk_elems, cols=cols)


def shard_plan_bind(plan: Plan, workspace: Optional[torch.Tensor] = None, stream=None, device="cuda") -> Plan:
    """Binds caller memory; with workspace=None a uint8 tensor of the needed size is allocated here."""
    if workspace is None:
        workspace = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=device)
    _check(lib().shard_plan_bind(plan.handle, _dev(workspace, 0, torch.uint8, "workspace"),
                                 workspace.numel(), _stream(stream)), "shard_plan_bind")
    plan.workspace = workspace
    return plan


class FullTensors:
    """A list of full tensors checked and marshalled once, for callers that pass the same tensors every
    step (the per-call checks walk all V tensors in Python).  Keeps the tensors alive."""

    def __init__(self, plan: Plan, tensors: Sequence[torch.Tensor], what: str = "full_tensors"):
        self.tensors = list(tensors)
        self.V = plan.V
        self.arr, self.dtype = _full_ptrs(plan, self.tensors, what)


def _full_ptrs(plan: Plan, tensors, what: str):
    if isinstance(tensors, FullTensors):
        if tensors.V != plan.V:
            raise ValueError("%s was built for another plan" % what)
        return tensors.arr, tensors.dtype
    if len(tensors) != plan.V:
        raise ValueError("%s: expected %d tensors, got %d" % (what, plan.V, len(tensors)))
    dtype = None
    arr = (C.c_void_p * max(plan.V, 1))()
    for i, t in enumerate(tensors):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("%s[%d] must be a contiguous CUDA tensor" % (what, i))
        if t.numel() != plan.numel[i]:
            raise ValueError("%s[%d] has %d elements, the plan says %d" % (what, i, t.numel(), plan.numel[i]))
        if t.dtype not in _DTYPES:
            raise ValueError("%s[%d]: unsupported dtype %s" % (what, i, t.dtype))
        if dtype is None:
            dtype = t.dtype
        elif t.dtype != dtype:
            raise ValueError("%s: mixed dtypes" % what)
        arr[i] = t.data_ptr() if t.numel() > 0 else None
    return arr, (dtype or torch.float32)


def shard_format(plan: Plan, r: int, full_tensors: Sequence[torch.Tensor], shard_out: torch.Tensor, stream=None):
    arr, src = _full_ptrs(plan, full_tensors, "full_tensors")
    if shard_out.dtype not in _DTYPES:
        raise ValueError("unsupported shard dtype")
    _check(lib().shard_format(plan.handle, int(r), arr, _DTYPES[src], _dev(shard_out, plan.S, None, "shard_out"),
                              _DTYPES[shard_out.dtype], _stream(stream)), "shard_format")
    return shard_out


def _rows(plan: Plan, t: torch.Tensor, what: str):
    """(pointer, row stride) of an [N, S] tensor with unit stride along S, or of a flat N*S tensor."""
    if t.dtype not in _DTYPES or not t.is_cuda:
        raise ValueError("%s must be a float32 or bfloat16 CUDA tensor" % what)
    if t.dim() == 2:
        if t.shape != (plan.N, plan.S) or (plan.S > 0 and t.stride(1) != 1):
            raise ValueError("%s must have shape [N, S] with unit stride along S" % what)
        stride = t.stride(0) if plan.N > 1 else plan.S
        if stride < plan.S:
            raise ValueError("%s rows overlap" % what)
        return C.c_void_p(t.data_ptr()), stride
    return _dev(t, plan.N * plan.S, None, what), plan.S


def shard_format_all(plan: Plan, full_tensors, out: torch.Tensor, stream=None):
    """out: [N, S] (rows may be strided, e.g. from gathered_empty) or flat N*S; row r receives shard_r."""
    arr, src = _full_ptrs(plan, full_tensors, "full_tensors")
    ptr, stride = _rows(plan, out, "out")
    _check(lib().shard_format_all(plan.handle, arr, _DTYPES[src], ptr, int(stride), _DTYPES[out.dtype],
                                  _stream(stream)), "shard_format_all")
    return out


def gathered_empty(plan: Plan, dtype=torch.float32, device="cuda") -> torch.Tensor:
    """An uninitialised [N, S] view whose rows start on 128-byte boundaries (the layout unshard_format likes)."""
    per_line = 128 // torch.empty((), dtype=dtype).element_size()
    stride = -(-plan.S // per_line) * per_line
    return torch.empty((plan.N, stride), dtype=dtype, device=device)[:, : plan.S]


def unshard_format(plan: Plan, gathered: torch.Tensor, full_tensors: Sequence[torch.Tensor], stream=None):
    """gathered: [N, S] (rows may be strided, e.g. from gathered_empty) or a flat tensor of N*S elements."""
    arr, dst = _full_ptrs(plan, full_tensors, "full_tensors")
    ptr, stride = _rows(plan, gathered, "gathered")
    _check(lib().unshard_format(plan.handle, ptr, int(stride), _DTYPES[gathered.dtype], arr, _DTYPES[dst],
                                _stream(stream)), "unshard_format")
    return full_tensors


def shard_plan_release_captured_tables(plan: Plan) -> None:
    """Lets other lists of tensors reuse the pointer tables that captured calls reserved (once their graphs are gone)."""
    _check(lib().shard_plan_release_captured_tables(plan.handle), "shard_plan_release_captured_tables")


COPY_WALKS = {"auto": 0, "by_replica": 1, "by_variable": 2}
COPIES = {"unshard_format": 0, "shard_format_all": 1}


def shard_plan_set_copy_walk(plan: Plan, walk: str) -> None:
    """Order of the work items of shard_format_all and unshard_format: "auto" (small pieces by variable, large ones by
    replica unless shard_plan_tune_copy_walk found otherwise), "by_replica" or "by_variable"."""
    if walk not in COPY_WALKS:
        raise ValueError("walk must be one of %s" % sorted(COPY_WALKS))
    _check(lib().shard_plan_set_copy_walk(plan.handle, COPY_WALKS[walk]), "shard_plan_set_copy_walk")


def shard_plan_copy_walk(plan: Plan, copy: str, full_tensors=None, with_times: bool = False):
    """The order the next `copy` ("unshard_format" or "shard_format_all") with these full tensors takes.
    with_times: also what shard_plan_tune_copy_walk measured for them (ms per launch by replica, by variable;
    zeros if it has not been called)."""
    if copy not in COPIES:
        raise ValueError("copy must be one of %s" % sorted(COPIES))
    arr = None if full_tensors is None else _full_ptrs(plan, full_tensors, "full_tensors")[0]
    out = C.c_int(-1)
    best = (C.c_float * 2)()
    _check(lib().shard_plan_copy_walk(plan.handle, COPIES[copy], arr, C.byref(out), best), "shard_plan_copy_walk")
    walk = {v: k for k, v in COPY_WALKS.items()}[out.value]
    return (walk, (best[0], best[1])) if with_times else walk


def shard_plan_tune_copy_walk(plan: Plan, copy: str, gathered: torch.Tensor, full_tensors, stream=None):
    """Measures both orders of `copy` on these buffers (the copy really runs, 8 times, and is waited for) and fixes
    the order for later calls with the same tensors.  Returns (order, (ms by replica, ms by variable))."""
    if copy not in COPIES:
        raise ValueError("copy must be one of %s" % sorted(COPIES))
    arr, full_dtype = _full_ptrs(plan, full_tensors, "full_tensors")
    ptr, stride = _rows(plan, gathered, "gathered")
    out = C.c_int(-1)
    best = (C.c_float * 2)()
    _check(lib().shard_plan_tune_copy_walk(plan.handle, COPIES[copy], ptr, int(stride), _DTYPES[gathered.dtype], arr,
                                           _DTYPES[full_dtype], _stream(stream), C.byref(out), best),
           "shard_plan_tune_copy_walk")
    return {v: k for k, v in COPY_WALKS.items()}[out.value], (best[0], best[1])


def _hp(cls, hp: Dict[str, float]):
    """The C struct of an optimizer's hyper-parameters.  Every field must be given except weight_decay
    (0 if absent); a key the struct does not have is an error, so that a misspelt name cannot silently
    become a zero."""
    fields = [name for name, _ in cls._fields_]
    unknown = sorted(set(hp) - set(fields))
    if unknown:
        raise ValueError("%s: unknown hyper-parameter(s) %s (expected %s)" % (cls.__name__, unknown, fields))
    missing = [name for name in fields if name not in hp and name != "weight_decay"]
    if missing:
        raise ValueError("%s: missing hyper-parameter(s) %s" % (cls.__name__, missing))
    return cls(**{name: float(hp.get(name, 0.0)) for name in fields})


def shard_update_adam(plan: Plan, r: int, w, g, m, v, hp: Dict[str, float], step: int, w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_adam(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                   _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                   _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                   C.byref(_hp(AdamHP, hp)), int(step), _stream(stream)), "shard_update_adam")


def shard_update_momentum(plan: Plan, r: int, w, g, m, hp: Dict[str, float], w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_momentum(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                       _dev(m, plan.S, f, "m"),
                                       _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                       C.byref(_hp(MomentumHP, hp)), _stream(stream)), "shard_update_momentum")


def shard_update_lamb_partials(plan: Plan, r: int, w, g, m, v, hp, step: int, local_sumsq_out, stream=None):
    f = torch.float32
    _check(lib().shard_update_lamb_partials(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                            _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                            C.byref(_hp(LambHP, hp)), int(step),
                                            _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                            _stream(stream)), "shard_update_lamb_partials")


def shard_update_lamb_apply(plan: Plan, r: int, w, m, v, hp, step: int, global_sumsq, w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_lamb_apply(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(m, plan.S, f, "m"),
                                         _dev(v, plan.S, f, "v"),
                                         _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                         C.byref(_hp(LambHP, hp)), int(step),
                                         _dev(global_sumsq, 2 * plan.V, f, "global_sumsq"),
                                         _stream(stream)), "shard_update_lamb_apply")


def shard_update_lamb(plan: Plan, r: int, w, g, m, v, hp, step: int, other_replicas_sumsq=None,
                      local_sumsq_out=None, w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_lamb(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                   _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                   _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                   C.byref(_hp(LambHP, hp)), int(step),
                                   _dev(other_replicas_sumsq, 2 * plan.V, f, "other_replicas_sumsq"),
                                   _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                   _stream(stream)), "shard_update_lamb")


def shard_update_lamb_noalloc(plan: Plan, r: int, w, g, m, v, hp, step: int, other_replicas_sumsq=None,
                              local_sumsq_out=None, w_bf16_out=None, stream=None):
    """shard_update_lamb with the intermediate sums in the library's own static device array (no allocation)."""
    f = torch.float32
    _check(lib().shard_update_lamb_noalloc(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                           _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                           _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                           C.byref(_hp(LambHP, hp)), int(step),
                                           _dev(other_replicas_sumsq, 2 * plan.V, f, "other_replicas_sumsq"),
                                           _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                           _stream(stream)), "shard_update_lamb_noalloc")


def shard_update_lamb_partials_full_grads(plan: Plan, r: int, w, full_grads, m, v, hp, step: int, local_sumsq_out,
                                          stream=None):
    """Phase 1 with the gradient read in place from the full tensors (list or FullTensors)."""
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_lamb_partials_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                                       _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                                       C.byref(_hp(LambHP, hp)), int(step),
                                                       _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                                       _stream(stream)), "shard_update_lamb_partials_full_grads")


def shard_update_lamb_full_grads(plan: Plan, r: int, w, full_grads, m, v, hp, step: int, other_replicas_sumsq=None,
                                 local_sumsq_out=None, w_bf16_out=None, stream=None):
    """shard_update_lamb with the gradient read in place from the full tensors (list or FullTensors)."""
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_lamb_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                              _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                              _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                              C.byref(_hp(LambHP, hp)), int(step),
                                              _dev(other_replicas_sumsq, 2 * plan.V, f, "other_replicas_sumsq"),
                                              _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                              _stream(stream)), "shard_update_lamb_full_grads")


def shard_update_lars_partials(plan: Plan, r: int, w, g, local_sumsq_out, stream=None):
    f = torch.float32
    _check(lib().shard_update_lars_partials(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                            _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                            _stream(stream)), "shard_update_lars_partials")


def shard_update_lars_apply(plan: Plan, r: int, w, g, m, hp, global_sumsq, w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_lars_apply(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                         _dev(m, plan.S, f, "m"),
                                         _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                         C.byref(_hp(LarsHP, hp)),
                                         _dev(global_sumsq, 2 * plan.V, f, "global_sumsq"),
                                         _stream(stream)), "shard_update_lars_apply")


def shard_update_lars(plan: Plan, r: int, w, g, m, hp, other_replicas_sumsq=None, local_sumsq_out=None,
                      w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_lars(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                   _dev(m, plan.S, f, "m"),
                                   _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                   C.byref(_hp(LarsHP, hp)),
                                   _dev(other_replicas_sumsq, 2 * plan.V, f, "other_replicas_sumsq"),
                                   _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                   _stream(stream)), "shard_update_lars")


# ---- the same updates with the gradient read in place from the full tensors (list or FullTensors) ----

def shard_update_adam_full_grads(plan: Plan, r: int, w, full_grads, m, v, hp, step: int, w_bf16_out=None, stream=None):
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_adam_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                              _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"),
                                              _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                              C.byref(_hp(AdamHP, hp)), int(step), _stream(stream)),
           "shard_update_adam_full_grads")


def shard_update_momentum_full_grads(plan: Plan, r: int, w, full_grads, m, hp, w_bf16_out=None, stream=None):
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_momentum_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                                  _dev(m, plan.S, f, "m"),
                                                  _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                                  C.byref(_hp(MomentumHP, hp)), _stream(stream)),
           "shard_update_momentum_full_grads")


def shard_update_lars_partials_full_grads(plan: Plan, r: int, w, full_grads, local_sumsq_out, stream=None):
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_lars_partials_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                                       _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                                       _stream(stream)), "shard_update_lars_partials_full_grads")


def shard_update_lars_apply_full_grads(plan: Plan, r: int, w, full_grads, m, hp, global_sumsq, w_bf16_out=None,
                                       stream=None):
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_lars_apply_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                                    _dev(m, plan.S, f, "m"),
                                                    _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                                    C.byref(_hp(LarsHP, hp)),
                                                    _dev(global_sumsq, 2 * plan.V, f, "global_sumsq"),
                                                    _stream(stream)), "shard_update_lars_apply_full_grads")


def shard_update_lars_full_grads(plan: Plan, r: int, w, full_grads, m, hp, other_replicas_sumsq=None,
                                 local_sumsq_out=None, w_bf16_out=None, stream=None):
    f = torch.float32
    arr, src = _full_ptrs(plan, full_grads, "full_grads")
    _check(lib().shard_update_lars_full_grads(plan.handle, int(r), _dev(w, plan.S, f, "w"), arr, _DTYPES[src],
                                              _dev(m, plan.S, f, "m"),
                                              _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                              C.byref(_hp(LarsHP, hp)),
                                              _dev(other_replicas_sumsq, 2 * plan.V, f, "other_replicas_sumsq"),
                                              _dev(local_sumsq_out, 2 * plan.V, f, "local_sumsq_out"),
                                              _stream(stream)), "shard_update_lars_full_grads")


def shard_plan_rowcol_layout(plan: Plan):
    """(row_off[V], col_off[V], total_rows, total_cols) of a row plan's row-sum and column-sum outputs."""
    cached = getattr(plan, "_rowcol_layout", None)          # a plan never changes: asked of the library once
    if cached is None:
        ro = (C.c_int64 * max(plan.V, 1))(); co = (C.c_int64 * max(plan.V, 1))()
        tr, tc = C.c_int64(), C.c_int64()
        _check(lib().shard_plan_rowcol_layout(plan.handle, ro, co, C.byref(tr), C.byref(tc)), "shard_plan_rowcol_layout")
        cached = plan._rowcol_layout = (tuple(ro[: plan.V]), tuple(co[: plan.V]), tr.value, tc.value)
    return cached


def shard_reduce_sq_rows_cols(plan: Plan, r: int, x, row_out, col_out, stream=None):
    f = torch.float32
    _, _, total_rows, total_cols = shard_plan_rowcol_layout(plan)
    _check(lib().shard_reduce_sq_rows_cols(plan.handle, int(r), _dev(x, plan.S, f, "x"),
                                           _dev(row_out, total_rows, f, "row_out"),
                                           _dev(col_out, total_cols, f, "col_out"), _stream(stream)),
           "shard_reduce_sq_rows_cols")


ADAFACTOR_DEFAULTS = {"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2}


def _adafactor_hp(hp: Dict[str, float]):
    """Every field has the published default (ADAFACTOR_DEFAULTS); unknown keys are an error."""
    unknown = sorted(set(hp) - set(ADAFACTOR_DEFAULTS))
    if unknown:
        raise ValueError("AdafactorHP: unknown hyper-parameter(s) %s (expected %s)" % (unknown, sorted(ADAFACTOR_DEFAULTS)))
    return AdafactorHP(**{name: float(hp.get(name, ADAFACTOR_DEFAULTS[name])) for name, _ in AdafactorHP._fields_})


def shard_update_adafactor_partials(plan: Plan, r: int, w, g, R, row_sq_out, col_sq_out, table_out, stream=None):
    f = torch.float32
    _, _, total_rows, total_cols = shard_plan_rowcol_layout(plan)
    _check(lib().shard_update_adafactor_partials(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                                 _dev(R, total_rows, f, "R"), _dev(row_sq_out, total_rows, f, "row_sq_out"),
                                                 _dev(col_sq_out, total_cols, f, "col_sq_out"),
                                                 _dev(table_out, 2 * plan.V, f, "table_out"), _stream(stream)),
           "shard_update_adafactor_partials")


def shard_update_adafactor_moments(plan: Plan, r: int, g, R, Cst, row_sq, col_sq_global, table_global, hp, step: int,
                                   u_sumsq_out, stream=None):
    f = torch.float32
    _, _, total_rows, total_cols = shard_plan_rowcol_layout(plan)
    _check(lib().shard_update_adafactor_moments(plan.handle, int(r), _dev(g, plan.S, f, "g"), _dev(R, total_rows, f, "R"),
                                                _dev(Cst, total_cols, f, "C"), _dev(row_sq, total_rows, f, "row_sq"),
                                                _dev(col_sq_global, total_cols, f, "col_sq_global"),
                                                _dev(table_global, 2 * plan.V, f, "table_global"),
                                                C.byref(_adafactor_hp(hp)), int(step),
                                                _dev(u_sumsq_out, plan.V, f, "u_sumsq_out"), _stream(stream)),
           "shard_update_adafactor_moments")


def shard_update_adafactor_apply(plan: Plan, r: int, w, g, table_global, u_sumsq_global, hp, step: int,
                                 w_bf16_out=None, stream=None):
    f = torch.float32
    _check(lib().shard_update_adafactor_apply(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                              _dev(table_global, 2 * plan.V, f, "table_global"),
                                              _dev(u_sumsq_global, plan.V, f, "u_sumsq_global"),
                                              _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                              C.byref(_adafactor_hp(hp)), int(step), _stream(stream)),
           "shard_update_adafactor_apply")


def shard_update_adafactor(plan: Plan, r: int, w, g, R, Cst, hp, step: int, other_col_sq=None, other_table=None,
                           other_u_sumsq=None, w_bf16_out=None, stream=None):
    f = torch.float32
    _, _, total_rows, total_cols = shard_plan_rowcol_layout(plan)
    _check(lib().shard_update_adafactor(plan.handle, int(r), _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                        _dev(R, total_rows, f, "R"), _dev(Cst, total_cols, f, "C"),
                                        _dev(w_bf16_out, plan.S, torch.bfloat16, "w_bf16_out"),
                                        C.byref(_adafactor_hp(hp)), int(step),
                                        _dev(other_col_sq, total_cols, f, "other_col_sq"),
                                        _dev(other_table, 2 * plan.V, f, "other_table"),
                                        _dev(other_u_sumsq, plan.V, f, "other_u_sumsq"), _stream(stream)),
           "shard_update_adafactor")


def shard_profile_enable(plan: Plan, on: bool) -> None:
    _check(lib().shard_profile_enable(plan.handle, 1 if on else 0), "shard_profile_enable")


def shard_profile_read(plan: Plan, kernel: str) -> Tuple[int, float]:
    """(launches, total milliseconds) of one kernel since the last reset; waits for recorded events."""
    n, ms = C.c_int64(), C.c_double()
    _check(lib().shard_profile_read(plan.handle, KERNEL_IDS[kernel], C.byref(n), C.byref(ms)), "shard_profile_read")
    return n.value, ms.value


def shard_profile_reset(plan: Plan) -> None:
    _check(lib().shard_profile_reset(plan.handle), "shard_profile_reset")


def shard_profile_plain_copy(plan: Plan, dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """The plainest device copy (measurement aid): dst and src contiguous CUDA tensors of the same byte size."""
    nbytes = src.numel() * src.element_size()
    if not (dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()) or \
            dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must be contiguous CUDA tensors of equal size")
    _check(lib().shard_profile_plain_copy(plan.handle, C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes,
                                          _stream(stream)), "shard_profile_plain_copy")


def shard_profile_adam_shape(plan: Plan, w, g, m, v, hp, step: int, block_threads: int, workgroups_per_cu: int,
                             stream=None) -> None:
    """shard_update_adam in a named launch shape (measurement aid): 128 or 256 threads, 0 or 3..16 workgroups per CU."""
    f = torch.float32
    _check(lib().shard_profile_adam_shape(plan.handle, _dev(w, plan.S, f, "w"), _dev(g, plan.S, f, "g"),
                                          _dev(m, plan.S, f, "m"), _dev(v, plan.S, f, "v"), C.byref(_hp(AdamHP, hp)),
                                          int(step), int(block_threads), int(workgroups_per_cu), _stream(stream)),
           "shard_profile_adam_shape")


# ---- replica arrays (host only) ---------------------------------------------------------------------

def shard_partial_sharding(rows: int, cols: int, replica: int):
    """(group, shard_id, shard_group[cols], reduce_group[rows]) of a replica in a rows x cols array."""
    group, sid = C.c_int(), C.c_int()
    sg, rg = (C.c_int * max(int(cols), 1))(), (C.c_int * max(int(rows), 1))()
    _check(lib().shard_partial_sharding(int(rows), int(cols), int(replica), C.byref(group), C.byref(sid), sg, rg),
           "shard_partial_sharding")
    return group.value, sid.value, list(sg[: cols]), list(rg[: rows])


def shard_two_phase_shard_id(rows: int, cols: int, replica: int) -> int:
    sid = C.c_int()
    _check(lib().shard_two_phase_shard_id(int(rows), int(cols), int(replica), C.byref(sid)), "shard_two_phase_shard_id")
    return sid.value


def shard_concat_partition(total: int, parts: int, part: int) -> Tuple[int, int]:
    start, length = C.c_int64(), C.c_int64()
    _check(lib().shard_concat_partition(int(total), int(parts), int(part), C.byref(start), C.byref(length)),
           "shard_concat_partition")
    return start.value, length.value


def shard_peak_memory(W: float, V: float, P: float, N: int) -> Tuple[float, float]:
    rep, sh = C.c_double(), C.c_double()
    _check(lib().shard_peak_memory(float(W), float(V), float(P), int(N), C.byref(rep), C.byref(sh)), "shard_peak_memory")
    return rep.value, sh.value


def shard_plan_peak_bytes(plan: Plan, weight_bytes: int, aux_bytes: int, P: int) -> Tuple[int, int]:
    rep, sh = C.c_int64(), C.c_int64()
    _check(lib().shard_plan_peak_bytes(plan.handle, int(weight_bytes), int(aux_bytes), int(P), C.byref(rep),
                                       C.byref(sh)), "shard_plan_peak_bytes")
    return rep.value, sh.value
