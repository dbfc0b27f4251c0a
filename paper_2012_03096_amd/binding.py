"""Thin ctypes binding of libpbkd.so (include/pbkd.h): argument marshalling only.

Every step of the distillation path runs inside the library's HIP kernels.  PyTorch appears only as
the owner of device memory (the workspace, inputs, targets are torch tensors whose data_ptr() is
handed over) and of HIP streams.  Loading fails loudly if the library has not been built; there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpbkd.so")

OK, EINVAL, ESHAPE, ENOMEM, EHIP, ESTATE, EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
CONV3X3, DWSEP3X3 = 0, 1
STUDENT_PARAM, STUDENT_GRAD, STUDENT_MOMENTUM, TEACHER_PARAM, STUDENT_ACT, TEACHER_ACT, STUDENT_BN_RUNNING, TEACHER_BN_RUNNING = range(8)

EXPORTS = [
    "pbkd_arch_validate", "pbkd_block_workspace_bytes", "pbkd_block_create", "pbkd_block_destroy",
    "pbkd_teacher_forward", "pbkd_student_step", "pbkd_distill_step", "pbkd_block_set_aux_stream", "pbkd_block_set_graph_mode", "pbkd_student_forward", "pbkd_block_last_loss",
    "pbkd_schedule_blocks", "pbkd_distill_step_all", "pbkd_run_tasks_work_stealing", "pbkd_network_forward", "pbkd_feature_mse", "pbkd_feature_mse_noalloc", "pbkd_select_blocks", "pbkd_block_flops", "pbkd_arch_flops",
    "pbkd_block_get_tensor", "pbkd_block_set_tensor", "pbkd_last_error",
    "pbkd_kernel_kinds", "pbkd_kernel_kind_name", "pbkd_block_profile_enable", "pbkd_block_profile_read",
]


class LayerDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("cin", ctypes.c_int), ("cout", ctypes.c_int), ("stride", ctypes.c_int),
                ("trainable", ctypes.c_int)]


class ArchDesc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int), ("c", ctypes.c_int), ("h", ctypes.c_int), ("w", ctypes.c_int),
                ("n_layers", ctypes.c_int), ("layers", ctypes.POINTER(LayerDesc)), ("shortcut", ctypes.c_int),
                ("shortcut_stride", ctypes.c_int), ("pool", ctypes.c_int), ("bn_eps", ctypes.c_float)]


class TrainDesc(ctypes.Structure):
    _fields_ = [("momentum", ctypes.c_float), ("loss_reduction", ctypes.c_int), ("bn_decay", ctypes.c_float)]


class PbkdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pbkd status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Loads libpbkd.so once; raises if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # PyTorch ships its own copy of the HIP runtime (same soname).  Import it first so that the
        # dynamic loader binds libpbkd.so to that one instance: two HIP runtimes in one process cannot
        # share device memory or streams.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, fp, ip = ctypes.c_void_p, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)
        ullp = ctypes.POINTER(ctypes.c_ulonglong)
        ap = ctypes.POINTER(ArchDesc)
        L.pbkd_arch_validate.argtypes = [ap, ap]
        L.pbkd_arch_validate.restype = ctypes.c_int
        L.pbkd_block_workspace_bytes.argtypes = [ap, ap]
        L.pbkd_block_workspace_bytes.restype = ctypes.c_size_t
        L.pbkd_block_create.argtypes = [ap, ctypes.POINTER(fp), ap, ctypes.POINTER(fp), ctypes.POINTER(TrainDesc), vp,
                                        ctypes.c_size_t, vp, ctypes.POINTER(vp)]
        L.pbkd_block_create.restype = ctypes.c_int
        L.pbkd_block_destroy.argtypes = [vp]
        L.pbkd_block_destroy.restype = ctypes.c_int
        L.pbkd_teacher_forward.argtypes = [vp, vp, vp, vp]
        L.pbkd_teacher_forward.restype = ctypes.c_int
        L.pbkd_student_step.argtypes = [vp, vp, vp, ctypes.c_float, fp, vp]
        L.pbkd_student_step.restype = ctypes.c_int
        L.pbkd_distill_step.argtypes = [vp, vp, vp, ctypes.c_float, fp, vp, vp]
        L.pbkd_distill_step.restype = ctypes.c_int
        L.pbkd_run_tasks_work_stealing.argtypes = [ctypes.c_int, vp, vp, vp, ctypes.c_float, ctypes.POINTER(ctypes.c_int), ctypes.c_int,
                                                   vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                                   ctypes.POINTER(ctypes.c_int)]
        L.pbkd_run_tasks_work_stealing.restype = ctypes.c_int
        L.pbkd_network_forward.argtypes = [ctypes.c_int, vp, ctypes.POINTER(ctypes.c_int), ctypes.c_int, vp, vp, vp]
        L.pbkd_network_forward.restype = ctypes.c_int
        L.pbkd_select_blocks.argtypes = [ctypes.c_int, vp, ctypes.c_int, vp, vp, vp, ctypes.c_double, ctypes.POINTER(ctypes.c_int),
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp]
        L.pbkd_select_blocks.restype = ctypes.c_int
        L.pbkd_feature_mse.argtypes = [vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), vp]
        L.pbkd_feature_mse.restype = ctypes.c_int
        L.pbkd_feature_mse_noalloc.argtypes = [vp, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), vp]
        L.pbkd_feature_mse_noalloc.restype = ctypes.c_int
        L.pbkd_block_set_graph_mode.argtypes = [vp, ctypes.c_int]
        L.pbkd_block_set_graph_mode.restype = ctypes.c_int
        L.pbkd_block_set_aux_stream.argtypes = [vp, vp]
        L.pbkd_block_set_aux_stream.restype = ctypes.c_int
        L.pbkd_student_forward.argtypes = [vp, vp, vp, vp]
        L.pbkd_student_forward.restype = ctypes.c_int
        L.pbkd_block_last_loss.argtypes = [vp, fp]
        L.pbkd_block_last_loss.restype = ctypes.c_int
        L.pbkd_schedule_blocks.argtypes = [ctypes.c_int, ullp, ctypes.POINTER(vp), ctypes.c_int, ctypes.c_int, ip, ip, ullp]
        L.pbkd_schedule_blocks.restype = ctypes.c_int
        L.pbkd_distill_step_all.argtypes = [ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                            ctypes.c_float, ctypes.c_int, ctypes.POINTER(vp), ip, ip, ctypes.c_int, vp]
        L.pbkd_distill_step_all.restype = ctypes.c_int
        L.pbkd_block_flops.argtypes = [vp, ctypes.c_int]
        L.pbkd_block_flops.restype = ctypes.c_ulonglong
        L.pbkd_arch_flops.argtypes = [ap, ctypes.c_int]
        L.pbkd_arch_flops.restype = ctypes.c_ulonglong
        L.pbkd_block_get_tensor.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, ctypes.c_size_t]
        L.pbkd_block_get_tensor.restype = ctypes.c_int
        L.pbkd_block_set_tensor.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, ctypes.c_size_t]
        L.pbkd_block_set_tensor.restype = ctypes.c_int
        L.pbkd_last_error.argtypes = []
        L.pbkd_last_error.restype = ctypes.c_char_p
        L.pbkd_kernel_kinds.argtypes = []
        L.pbkd_kernel_kinds.restype = ctypes.c_int
        L.pbkd_kernel_kind_name.argtypes = [ctypes.c_int]
        L.pbkd_kernel_kind_name.restype = ctypes.c_char_p
        L.pbkd_block_profile_enable.argtypes = [vp, ctypes.c_uint, ctypes.c_int]
        L.pbkd_block_profile_enable.restype = ctypes.c_int
        L.pbkd_block_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ip]
        L.pbkd_block_profile_read.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int):
    if status != OK:
        raise PbkdError(status, lib().pbkd_last_error().decode())


def make_arch(arch) -> ArchDesc:
    """Converts a workloads.Arch (or anything with the same attributes) into the C descriptor.
    The returned struct keeps its layer array alive."""
    layers = (LayerDesc * len(arch.layers))(*[LayerDesc(L.kind, L.cin, L.cout, L.stride, L.trainable) for L in arch.layers])
    d = ArchDesc(arch.n, arch.c, arch.h, arch.w, len(arch.layers), layers, arch.shortcut, arch.shortcut_stride, arch.pool,
                 arch.bn_eps)
    d._keep = layers
    return d


def arch_validate(teacher, student) -> int:
    return lib().pbkd_arch_validate(ctypes.byref(make_arch(teacher)), ctypes.byref(make_arch(student)))


def last_error() -> str:
    return lib().pbkd_last_error().decode()


def workspace_bytes(teacher, student) -> int:
    return lib().pbkd_block_workspace_bytes(ctypes.byref(make_arch(teacher)), ctypes.byref(make_arch(student)))


def arch_flops(arch, training_step: bool) -> int:
    return lib().pbkd_arch_flops(ctypes.byref(make_arch(arch)), int(training_step))


def schedule_blocks(weights: Optional[Sequence[int]], n_streams: int, policy: int = 0, blocks: Optional[Sequence["Block"]] = None):
    """Returns (stream_of_block, order, stream_load)."""
    n = len(weights) if weights is not None else len(blocks)
    w = (ctypes.c_ulonglong * n)(*weights) if weights is not None else None
    hb = (ctypes.c_void_p * n)(*[b.handle for b in blocks]) if blocks is not None else None
    sob = (ctypes.c_int * max(n, 1))()
    order = (ctypes.c_int * max(n, 1))()
    load = (ctypes.c_ulonglong * max(n_streams, 1))()
    _check(lib().pbkd_schedule_blocks(n, w, hb, n_streams, policy, sob, order, load))
    return list(sob)[:n], list(order)[:n], list(load)[:n_streams]


def kernel_kind_names() -> List[str]:
    L = lib()
    return [L.pbkd_kernel_kind_name(i).decode() for i in range(L.pbkd_kernel_kinds())]


def _params_array(params: Sequence[Sequence[np.ndarray]]):
    flat = []
    for lp in params:
        for q in lp:
            a = np.ascontiguousarray(q, dtype=np.float32)
            flat.append(a)
    arr = (ctypes.POINTER(ctypes.c_float) * len(flat))(*[a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) for a in flat])
    return arr, flat


class Block:
    """One distillation task on the GPU.  Owns a torch uint8 workspace tensor and the library handle."""

    def __init__(self, teacher, teacher_params, student, student_params, momentum: float = 0.9, loss_reduction: int = 0,
                 device: str = "cuda:0", stream=None, bn_decay: float = 0.99):
        import torch
        self.teacher, self.student = teacher, student
        self._ta, self._sa = make_arch(teacher), make_arch(student)
        st = lib().pbkd_arch_validate(ctypes.byref(self._ta), ctypes.byref(self._sa))
        _check(st)
        nbytes = lib().pbkd_block_workspace_bytes(ctypes.byref(self._ta), ctypes.byref(self._sa))
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        base = self.workspace.data_ptr()
        aligned = (base + 255) & ~255
        tp, keep_t = _params_array(teacher_params)
        sp, keep_s = _params_array(student_params)
        train = TrainDesc(momentum, loss_reduction, bn_decay)
        handle = ctypes.c_void_p()
        sptr = stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream
        _check(lib().pbkd_block_create(ctypes.byref(self._ta), tp, ctypes.byref(self._sa), sp, ctypes.byref(train),
                                       ctypes.c_void_p(aligned), nbytes, ctypes.c_void_p(sptr), ctypes.byref(handle)))
        self.handle = handle
        self.workspace_bytes = nbytes

    def close(self):
        if getattr(self, "handle", None):
            lib().pbkd_block_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _sptr(stream):
        import torch
        return ctypes.c_void_p(stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream)

    def teacher_forward(self, x, target, stream=None):
        _check(lib().pbkd_teacher_forward(self.handle, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(target.data_ptr()),
                                          self._sptr(stream)))

    def student_forward(self, x, out, stream=None):
        _check(lib().pbkd_student_forward(self.handle, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                          self._sptr(stream)))

    def set_aux_stream(self, stream) -> None:
        """Second stream for the weight-gradient branch of the backward pass (None: off)."""
        self._aux = stream     # keep it alive
        _check(lib().pbkd_block_set_aux_stream(self.handle, ctypes.c_void_p(stream.cuda_stream if stream is not None else 0)))

    def set_graph_mode(self, on: bool) -> None:
        """Capture each step's launches into a HIP graph once and replay it (pbkd_block_set_graph_mode)."""
        _check(lib().pbkd_block_set_graph_mode(self.handle, int(bool(on))))

    def distill_step(self, x, target, lr: float, want_loss: bool = True, student_stream=None,
                     teacher_stream=None) -> Optional[float]:
        """Teacher forward into `target` on teacher_stream and the student step on student_stream, overlapped."""
        loss = ctypes.c_float()
        _check(lib().pbkd_distill_step(self.handle, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(target.data_ptr()), lr,
                                       ctypes.byref(loss) if want_loss else None, self._sptr(student_stream),
                                       self._sptr(teacher_stream)))
        return loss.value if want_loss else None

    def student_step(self, x, target, lr: float, want_loss: bool = True, stream=None) -> Optional[float]:
        loss = ctypes.c_float()
        _check(lib().pbkd_student_step(self.handle, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(target.data_ptr()), lr,
                                       ctypes.byref(loss) if want_loss else None, self._sptr(stream)))
        return loss.value if want_loss else None

    def last_loss(self) -> float:
        loss = ctypes.c_float()
        _check(lib().pbkd_block_last_loss(self.handle, ctypes.byref(loss)))
        return loss.value

    def flops(self, which: int) -> int:
        return lib().pbkd_block_flops(self.handle, which)

    def get_tensor(self, which: int, layer: int, slot: int, shape) -> np.ndarray:
        out = np.empty(shape, dtype=np.float32)
        _check(lib().pbkd_block_get_tensor(self.handle, which, layer, slot, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                           out.size))
        return out

    def set_tensor(self, which: int, layer: int, slot: int, value: np.ndarray):
        a = np.ascontiguousarray(value, dtype=np.float32)
        _check(lib().pbkd_block_set_tensor(self.handle, which, layer, slot, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                           a.size))

    def profile_enable(self, kinds: Optional[Sequence[str]], capacity: int):
        """kinds: kernel-kind names to time (None = all); capacity 0 switches timing off."""
        names = kernel_kind_names()
        mask = 0
        for i, nm in enumerate(names):
            if kinds is None or nm in kinds:
                mask |= 1 << i
        _check(lib().pbkd_block_profile_enable(self.handle, mask, capacity))

    def profile_read(self):
        """{kind name: (summed ms, launches)} of the timed launches since the last read."""
        n = lib().pbkd_kernel_kinds()
        ms = (ctypes.c_double * n)()
        cnt = (ctypes.c_int * n)()
        _check(lib().pbkd_block_profile_read(self.handle, n, ms, cnt))
        return {nm: (ms[i], cnt[i]) for i, nm in enumerate(kernel_kind_names()) if cnt[i]}

    def student_params(self) -> List[List[np.ndarray]]:
        from .workloads import param_shapes
        return [[self.get_tensor(STUDENT_PARAM, l, k, shp) for k, shp in enumerate(lp)]
                for l, lp in enumerate(param_shapes(self.student))]

    def student_grads(self) -> List[List[np.ndarray]]:
        from .workloads import param_shapes
        return [[self.get_tensor(STUDENT_GRAD, l, k, shp) for k, shp in enumerate(lp)]
                for l, lp in enumerate(param_shapes(self.student))]


def distill_step_all(blocks: Sequence[Block], xs, targets, lr: float, streams, stream_of_block, order, chain: bool,
                     teacher_stream=None):
    """One concurrent distillation step of all blocks (pbkd_distill_step_all).  xs / targets: torch tensors;
    streams: torch.cuda.Stream objects."""
    n = len(blocks)
    hb = (ctypes.c_void_p * n)(*[b.handle for b in blocks])
    xp = (ctypes.c_void_p * n)(*[x.data_ptr() for x in xs])
    tp = (ctypes.c_void_p * n)(*[t.data_ptr() for t in targets])
    sp = (ctypes.c_void_p * len(streams))(*[s.cuda_stream for s in streams])
    sob = (ctypes.c_int * n)(*stream_of_block)
    od = (ctypes.c_int * n)(*order)
    ts = ctypes.c_void_p(teacher_stream.cuda_stream) if teacher_stream is not None else ctypes.c_void_p(0)
    _check(lib().pbkd_distill_step_all(n, hb, xp, tp, lr, len(streams), sp, sob, od, int(chain), ts))


def run_tasks_work_stealing(blocks: Sequence[Block], xs, targets, lr: float, steps: Sequence[int], streams,
                            queue_of_task: Sequence[int]):
    """pbkd_run_tasks_work_stealing: whole training tasks over streams with dynamic load balancing.
    Returns (ran_on, n_steals).  Blocks until every task has finished."""
    n = len(blocks)
    hb = (ctypes.c_void_p * n)(*[b.handle for b in blocks])
    xp = (ctypes.c_void_p * n)(*[x.data_ptr() for x in xs])
    tp = (ctypes.c_void_p * n)(*[t.data_ptr() for t in targets])
    sp = (ctypes.c_void_p * len(streams))(*[s.cuda_stream for s in streams])
    st = (ctypes.c_int * n)(*steps)
    qt = (ctypes.c_int * n)(*queue_of_task)
    ran = (ctypes.c_int * n)()
    ns = ctypes.c_int()
    _check(lib().pbkd_run_tasks_work_stealing(n, hb, xp, tp, lr, st, len(streams), sp, qt, ran, ctypes.byref(ns)))
    return list(ran), ns.value


def network_forward(blocks: Sequence[Block], use_student: Sequence[int], x, outs, stream=None, bn_mode: int = 0) -> None:
    """pbkd_network_forward: the chain of blocks on x, block k by its student where use_student[k] is non-zero;
    bn_mode 0 = BatchNorm with batch statistics, 1 = with the running statistics (inference mode)."""
    n = len(blocks)
    hb = (ctypes.c_void_p * n)(*[b.handle for b in blocks])
    us = (ctypes.c_int * n)(*[int(u) for u in use_student])
    op = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    _check(lib().pbkd_network_forward(n, hb, us, int(bn_mode), ctypes.c_void_p(x.data_ptr()), op, Block._sptr(stream)))


def select_blocks(blocks: Sequence[Block], x, teacher_outs, scratch_outs, threshold: float, stream=None, bn_mode: int = 0):
    """pbkd_select_blocks: returns (use_student, per-block feature error, error of the reassembled network)."""
    n = len(blocks)
    hb = (ctypes.c_void_p * n)(*[b.handle for b in blocks])
    tp = (ctypes.c_void_p * n)(*[o.data_ptr() for o in teacher_outs])
    sp = (ctypes.c_void_p * n)(*[o.data_ptr() for o in scratch_outs])
    use = (ctypes.c_int * n)()
    errs = (ctypes.c_double * n)()
    final = ctypes.c_double()
    _check(lib().pbkd_select_blocks(n, hb, int(bn_mode), ctypes.c_void_p(x.data_ptr()), tp, sp, ctypes.c_double(threshold),
                                    use, errs, ctypes.byref(final), Block._sptr(stream)))
    return list(use), list(errs), final.value


def feature_mse(block: Block, a, b, stream=None) -> float:
    """pbkd_feature_mse: mean squared difference of two device tensors (fp64 accumulation)."""
    out = ctypes.c_double()
    _check(lib().pbkd_feature_mse(block.handle, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()), a.numel(),
                                  ctypes.byref(out), Block._sptr(stream)))
    return out.value


def feature_mse_noalloc(a, b, stream=None, n: Optional[int] = None) -> float:
    """pbkd_feature_mse_noalloc: the same figure with the library's static scratch array (no block, no allocation)."""
    out = ctypes.c_double()
    _check(lib().pbkd_feature_mse_noalloc(ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()),
                                          a.numel() if n is None else n, ctypes.byref(out), Block._sptr(stream)))
    return out.value
