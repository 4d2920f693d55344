"""ctypes binding of libng.so: the C ABI of include/ng.h under the same names.

Argument marshalling only -- every step of the optimizer runs inside the
library's HIP kernels.  PyTorch appears here solely as the owner of device
memory and of the stream.  Importing this module raises if the library has not
been built (``python -m paper_2410_16029_amd.build``); there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libng.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libng.so is missing: build it with `python -m paper_2410_16029_amd.build` "
        "(the HIP library is the only implementation; there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

NG_F32, NG_BF16 = 0, 1
NG_SIDE_LEFT, NG_SIDE_RIGHT = 0, 1
NG_NORM_S, NG_NORM_COUNT = 0, 1
NG_ADAM_STANDARD, NG_ADAM_PRINTED = 0, 1
NG_OK = 0
NG_ERR_INVALID_ARG, NG_ERR_SHAPE, NG_ERR_DTYPE, NG_ERR_HPARAM = -1, -2, -3, -4
NG_ERR_NO_PROJECTOR, NG_ERR_HIP, NG_ERR_NUMERIC, NG_ERR_WORKSPACE, NG_ERR_NOT_CONVERGED = -5, -6, -7, -8, -9
NG_BUF_P, NG_BUF_M, NG_BUF_V, NG_BUF_H, NG_BUF_K, NG_BUF_N, NG_BUF_AUX, NG_NBUF = range(8)
NG_INIT_DEFAULT, NG_INIT_NO_CLEAR, NG_INIT_HOST_ONLY = 0, 1, 2
NG_NPHASE = 5
PHASE_NAMES = ("project", "gram", "solve", "adam", "update")


class ng_matrix_desc(C.Structure):
    _fields_ = [("m", C.c_int32), ("n", C.c_int32), ("r", C.c_int32), ("side", C.c_int32),
                ("ld_w", C.c_int64), ("ld_g", C.c_int64)]


class ng_hparams(C.Structure):
    _fields_ = [("s", C.c_int32), ("lambda_", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("scale", C.c_float), ("weight_decay", C.c_float),
                ("grad_dtype", C.c_int32), ("adam_mode", C.c_int32),
                ("refresh_power_iters", C.c_int32), ("refresh_oversample", C.c_int32),
                ("refresh_sweeps", C.c_int32), ("hist_dtype", C.c_int32), ("fisher_norm", C.c_int32),
                ("carry_history", C.c_int32), ("proj_dtype", C.c_int32), ("seed", C.c_uint64)]


class ng_matrix_buffers(C.Structure):
    _fields_ = [("buf", C.c_void_p * NG_NBUF)]


class ng_matrix_layout(C.Structure):
    _fields_ = [("ldn", C.c_int32), ("l", C.c_int32), ("slot_elems", C.c_int64),
                ("panel_cols", C.c_int32), ("reserved0", C.c_int32),
                ("k_gram_off", C.c_int64), ("k_w64_off", C.c_int64), ("k_w32_off", C.c_int64),
                ("aux_pb_off", C.c_int64), ("aux_pbt_off", C.c_int64)]


_P = C.POINTER
_lib.ng_default_hparams.argtypes = [_P(ng_hparams)]
_lib.ng_query_sizes.argtypes = [_P(ng_matrix_desc), C.c_int, _P(ng_hparams), _P(C.c_size_t), _P(C.c_size_t)]
_lib.ng_init_state.argtypes = [_P(ng_matrix_desc), _P(ng_matrix_buffers), C.c_int, _P(ng_hparams), C.c_void_p,
                               C.c_size_t, C.c_uint32, C.c_void_p, _P(C.c_void_p)]
_lib.ng_refresh_projector.argtypes = [C.c_void_p, _P(C.c_void_p), C.c_void_p]
_lib.ng_commit_projector.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
_lib.ng_step.argtypes = [C.c_void_p, _P(C.c_void_p), _P(C.c_void_p), C.c_float, C.c_void_p]
_lib.ng_step_static.argtypes = [C.c_void_p, _P(C.c_void_p), _P(C.c_void_p), C.c_float, C.c_void_p]
_lib.ng_get_counters.argtypes = [C.c_void_p, C.c_int, _P(C.c_int64), _P(C.c_int32), _P(C.c_int32), _P(C.c_int64)]
_lib.ng_set_counters.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_int32, C.c_int64]
_lib.ng_get_layout.argtypes = [C.c_void_p, C.c_int, _P(ng_matrix_layout)]
_lib.ng_get_status.argtypes = [C.c_void_p, C.c_void_p]
_lib.ng_set_profiling.argtypes = [C.c_void_p, C.c_int]
_lib.ng_get_phase_ms.argtypes = [C.c_void_p, _P(C.c_double), _P(C.c_int64), C.c_int]
_lib.ng_microbench.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, _P(C.c_double),
                               _P(C.c_double)]
_lib.ng_microbench.restype = C.c_int
_lib.ng_struct_size.argtypes = [C.c_int]
_lib.ng_struct_size.restype = C.c_size_t
for _which, _cls in enumerate((ng_matrix_desc, ng_hparams, ng_matrix_buffers, ng_matrix_layout)):
    if _lib.ng_struct_size(_which) != C.sizeof(_cls):
        raise ImportError("binding.py and libng.so disagree on sizeof(%s): rebuild the library" % _cls.__name__)
_lib.ng_strerror.argtypes = [C.c_int]
_lib.ng_strerror.restype = C.c_char_p
_lib.ng_destroy.argtypes = [C.c_void_p]
_lib.ng_destroy.restype = None
for _name in ("ng_default_hparams", "ng_query_sizes", "ng_init_state", "ng_refresh_projector", "ng_commit_projector",
              "ng_step", "ng_step_static", "ng_get_counters", "ng_set_counters", "ng_get_layout", "ng_get_status", "ng_set_profiling",
              "ng_get_phase_ms"):
    getattr(_lib, _name).restype = C.c_int


class NgError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, ng_strerror(code), code))


def ng_strerror(code: int) -> str:
    return _lib.ng_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != NG_OK:
        raise NgError(code, where)


def ng_default_hparams() -> ng_hparams:
    hp = ng_hparams()
    _check(_lib.ng_default_hparams(C.byref(hp)), "ng_default_hparams")
    return hp


def make_descs(shapes: Sequence, r, ld_w=None, ld_g=None, sides=None):
    """sides: None (all left), "auto" (right where m > n), or one NG_SIDE_* per matrix."""
    n = len(shapes)
    arr = (ng_matrix_desc * n)()
    for i, (m, nn) in enumerate(shapes):
        ri = r[i] if isinstance(r, (list, tuple)) else r
        if sides is None:
            side = NG_SIDE_LEFT
        elif isinstance(sides, str):
            side = NG_SIDE_RIGHT if (sides == "auto" and m > nn) or sides == "right" else NG_SIDE_LEFT
        else:
            side = sides[i]
        arr[i] = ng_matrix_desc(m, nn, ri, side, (ld_w[i] if ld_w else nn), (ld_g[i] if ld_g else nn))
    return arr


def ng_query_sizes(descs, hp: ng_hparams):
    """Returns (bytes[n_mats][NG_NBUF], workspace_bytes).  Host only."""
    n = len(descs)
    sizes = (C.c_size_t * (n * NG_NBUF))()
    ws = C.c_size_t()
    _check(_lib.ng_query_sizes(descs, n, C.byref(hp), sizes, C.byref(ws)), "ng_query_sizes")
    return [[sizes[i * NG_NBUF + b] for b in range(NG_NBUF)] for i in range(n)], ws.value


def ng_init_state(descs, bufs, hp: ng_hparams, workspace_ptr: int, workspace_bytes: int, flags: int, stream: int):
    st = C.c_void_p()
    _check(_lib.ng_init_state(descs, bufs, len(descs), C.byref(hp), C.c_void_p(workspace_ptr), workspace_bytes,
                              flags, C.c_void_p(stream), C.byref(st)), "ng_init_state")
    return st


def _ptr_array(ptrs: Sequence[int]):
    arr = (C.c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


def ng_refresh_projector(st, grad_ptrs: Sequence[int], stream: int) -> None:
    _check(_lib.ng_refresh_projector(st, _ptr_array(grad_ptrs), C.c_void_p(stream)), "ng_refresh_projector")


def ng_commit_projector(st, clear_history: bool, stream: int) -> None:
    _check(_lib.ng_commit_projector(st, int(clear_history), C.c_void_p(stream)), "ng_commit_projector")


def ng_step(st, grad_ptrs, weight_ptrs, lr: float, stream: int) -> None:
    _check(_lib.ng_step(st, grad_ptrs if not isinstance(grad_ptrs, (list, tuple)) else _ptr_array(grad_ptrs),
                        weight_ptrs if not isinstance(weight_ptrs, (list, tuple)) else _ptr_array(weight_ptrs),
                        lr, C.c_void_p(stream)), "ng_step")


def ng_step_static(st, grad_ptrs, weight_ptrs, lr: float, stream: int) -> None:
    _check(_lib.ng_step_static(st, grad_ptrs if not isinstance(grad_ptrs, (list, tuple)) else _ptr_array(grad_ptrs),
                               weight_ptrs if not isinstance(weight_ptrs, (list, tuple)) else _ptr_array(weight_ptrs),
                               lr, C.c_void_p(stream)), "ng_step_static")


def ng_get_counters(st, mat: int):
    t, head, count, nref = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int64()
    _check(_lib.ng_get_counters(st, mat, C.byref(t), C.byref(head), C.byref(count), C.byref(nref)), "ng_get_counters")
    return t.value, head.value, count.value, nref.value


def ng_set_counters(st, mat: int, t: int, head: int, count: int, n_refresh: int) -> None:
    _check(_lib.ng_set_counters(st, mat, t, head, count, n_refresh), "ng_set_counters")


def ng_get_layout(st, mat: int) -> ng_matrix_layout:
    lay = ng_matrix_layout()
    _check(_lib.ng_get_layout(st, mat, C.byref(lay)), "ng_get_layout")
    return lay


def ng_get_status(st, stream: int) -> int:
    return _lib.ng_get_status(st, C.c_void_p(stream))


def ng_set_profiling(st, enabled: bool) -> None:
    _check(_lib.ng_set_profiling(st, int(enabled)), "ng_set_profiling")


def ng_get_phase_ms(st, reset: bool = True):
    ms = (C.c_double * NG_NPHASE)()
    steps = C.c_int64()
    _check(_lib.ng_get_phase_ms(st, ms, C.byref(steps), int(reset)), "ng_get_phase_ms")
    return [ms[i] for i in range(NG_NPHASE)], steps.value


NG_MB_COPY, NG_MB_READ, NG_MB_MFMA_BF16, NG_MB_MFMA_BF16_RANDOM = 0, 1, 2, 3


def ng_microbench(which: int, a_ptr: int, b_ptr: int, nbytes: int, reps: int, stream: int):
    """Returns (mean ms per launch, bytes or flops per launch)."""
    ms, work = C.c_double(), C.c_double()
    _check(_lib.ng_microbench(which, C.c_void_p(a_ptr), C.c_void_p(b_ptr), nbytes, reps, C.c_void_p(stream),
                              C.byref(ms), C.byref(work)), "ng_microbench")
    return ms.value, work.value


def ng_destroy(st) -> None:
    _lib.ng_destroy(st)


# --------------------------------------------------------------------------
# Convenience owner of the device memory (torch tensors) behind one handle.
# --------------------------------------------------------------------------
class LayerSet:
    """Allocates the caller-owned buffers as torch tensors and forwards to the C ABI."""

    def __init__(self, shapes: Sequence, r, *, s=4, lam=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                 weight_decay=0.0, dtype="f32", adam_mode="standard", power_iters=None, oversample=None,
                 sweeps=None, seed=0, device="cuda:0", ld_w=None, ld_g=None, no_clear=False, hist_dtype=None,
                 sides=None, fisher_norm="s", carry_history=False, host_only=False, proj_dtype=None):
        self.device = torch.device(device)
        self.shapes = [tuple(x) for x in shapes]
        self.r = r
        hp = ng_default_hparams()
        hp.s, hp.lambda_, hp.beta1, hp.beta2, hp.eps = s, lam, beta1, beta2, eps
        hp.scale, hp.weight_decay = scale, weight_decay
        hp.grad_dtype = {"f32": NG_F32, "bf16": NG_BF16}[dtype]
        hp.adam_mode = {"standard": NG_ADAM_STANDARD, "printed": NG_ADAM_PRINTED}[adam_mode]
        if power_iters is not None:
            hp.refresh_power_iters = power_iters
        if oversample is not None:
            hp.refresh_oversample = oversample
        if sweeps is not None:
            hp.refresh_sweeps = sweeps
        hp.seed = seed
        if hist_dtype is not None:
            hp.hist_dtype = {"f32": NG_F32, "bf16": NG_BF16}[hist_dtype]
        self.hist_dtype = hist_dtype if hist_dtype is not None else "f32"
        hp.fisher_norm = {"s": NG_NORM_S, "count": NG_NORM_COUNT}[fisher_norm]
        hp.carry_history = 1 if carry_history else 0
        if proj_dtype is not None:
            hp.proj_dtype = {"f32": NG_F32, "bf16": NG_BF16}[proj_dtype]
        self.proj_dtype = proj_dtype if proj_dtype is not None else "f32"
        self.hp = hp
        self.dtype = dtype
        self.descs = make_descs(self.shapes, r, ld_w, ld_g, sides)
        self.sizes, self.workspace_bytes = ng_query_sizes(self.descs, hp)
        n = len(self.shapes)
        self.buffers: List[List[torch.Tensor]] = []
        self._bufs = (ng_matrix_buffers * n)()
        for i in range(n):
            row = []
            for b in range(NG_NBUF):
                nbytes = self.sizes[i][b]
                if no_clear or host_only:
                    t = torch.zeros(max(nbytes, 16), dtype=torch.uint8, device=self.device)
                else:
                    t = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=self.device)
                row.append(t)
                self._bufs[i].buf[b] = t.data_ptr()
            self.buffers.append(row)
        self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self.st = ng_init_state(self.descs, self._bufs, hp, ws_ptr, self.workspace_bytes,
                                (NG_INIT_NO_CLEAR if no_clear else NG_INIT_DEFAULT)
                                | (NG_INIT_HOST_ONLY if host_only else 0), self.stream())
        self.layouts = [ng_get_layout(self.st, i) for i in range(n)]

    def stream(self) -> int:
        if self.device.type == "cuda":
            return torch.cuda.current_stream(self.device).cuda_stream
        return 0

    @staticmethod
    def _ptrs(tensors) -> List[int]:
        return [t.data_ptr() for t in tensors]

    def refresh(self, grads) -> None:
        ng_refresh_projector(self.st, self._ptrs(grads), self.stream())

    def commit_projector(self, clear_history: bool = True) -> None:
        ng_commit_projector(self.st, clear_history, self.stream())

    def step(self, grads, weights, lr: float) -> None:
        ng_step(self.st, self._ptrs(grads), self._ptrs(weights), lr, self.stream())

    def step_static(self, grads, weights, lr: float) -> None:
        ng_step_static(self.st, self._ptrs(grads), self._ptrs(weights), lr, self.stream())

    def status(self) -> int:
        return ng_get_status(self.st, self.stream())

    def counters(self, mat: int = 0):
        return ng_get_counters(self.st, mat)

    # ---- typed views of the state buffers (no copies, except M, V, H of panelled states)
    def _view(self, i, b, dtype, count, offset=0):
        t = self.buffers[i][b]
        esz = torch.empty((), dtype=dtype).element_size()
        return t[offset:offset + count * esz].view(dtype)

    def side(self, i) -> int:
        return self.descs[i].side

    def eff_shape(self, i):
        """(m, n) of the problem the library works on: the weight's shape, swapped on the right side."""
        m, n = self.shapes[i]
        return (n, m) if self.descs[i].side == NG_SIDE_RIGHT else (m, n)

    def P(self, i):
        """The projector as a float32 [m][r] tensor: a view of NG_BUF_P, or, for the low-memory
        projector (proj_dtype bf16: there is no float P), the decoded bf16 copy."""
        if self.proj_dtype == "bf16":
            return self.Pb(i)
        m, _ = self.eff_shape(i)
        r = self.descs[i].r
        return self._view(i, NG_BUF_P, torch.float32, m * r).view(m, r)

    def _state_elems(self, i):
        """Elements of M, V or one history slot as stored (the last panel of a panelled state is padded)."""
        r, ldn, pw = self.descs[i].r, self.layouts[i].ldn, self.layouts[i].panel_cols
        return r * (-(-ldn // pw) * pw)

    def _unpanel(self, i, flat):
        """[..., stored elements] in the library's column-panel order -> [..., r, ldn] row-major
        (a view when the array has one panel, else a copy)."""
        r, ldn, pw = self.descs[i].r, self.layouts[i].ldn, self.layouts[i].panel_cols
        lead = flat.shape[:-1]
        if pw >= ldn:
            return flat.view(*lead, r, ldn)
        npan = -(-ldn // pw)
        x = flat.view(*lead, npan, r, pw)
        x = x.movedim(-3, -2).reshape(*lead, r, npan * pw)
        return x[..., :ldn]

    def M(self, i):
        return self._unpanel(i, self._view(i, NG_BUF_M, torch.float32, self._state_elems(i)))

    def V(self, i):
        return self._unpanel(i, self._view(i, NG_BUF_V, torch.float32, self._state_elems(i)))

    def H(self, i):
        s = max(self.hp.s, 1)
        ht = torch.bfloat16 if self.hist_dtype == "bf16" else torch.float32
        n = self._state_elems(i)
        return self._unpanel(i, self._view(i, NG_BUF_H, ht, s * n).view(s, n))

    def K(self, i):
        s = self.hp.s
        return self._view(i, NG_BUF_K, torch.float64, s * s, self.layouts[i].k_gram_off).view(s, s)

    def w(self, i):
        return self._view(i, NG_BUF_K, torch.float64, self.hp.s, self.layouts[i].k_w64_off)

    def N(self, i):
        """Update direction as a float32 [r][n] tensor (decodes the octet layout for bf16)."""
        r, ldn = self.descs[i].r, self.layouts[i].ldn
        n = self.eff_shape(i)[1]
        if self.dtype == "f32":
            return self._view(i, NG_BUF_N, torch.float32, r * ldn).view(r, ldn)[:, :n]
        roct = (r + 7) // 8
        raw = self._view(i, NG_BUF_N, torch.bfloat16, roct * ldn * 8).view(roct, ldn, 8)
        return raw.permute(0, 2, 1).reshape(roct * 8, ldn)[:r, :n].float()

    def Pb(self, i):
        """The bf16 copy of P that the update GEMM multiplies with, decoded from its blocked layout
        to a float32 [m][r] tensor (bf16 layer sets only)."""
        m, _ = self.eff_shape(i)
        r = self.descs[i].r
        nblk = (r + 31) // 32
        raw = self._view(i, NG_BUF_AUX, torch.bfloat16, nblk * m * 32, self.layouts[i].aux_pb_off).view(nblk, m, 32)
        return raw.permute(1, 0, 2).reshape(m, nblk * 32)[:, :r].float()

    def PbT(self, i):
        """The bf16 copy of P that the projection GEMM multiplies with (stored transposed and
        blocked), decoded to a float32 [m][r] tensor (bf16 layer sets only)."""
        m, _ = self.eff_shape(i)
        r = self.descs[i].r
        nblk = (m + 31) // 32
        raw = self._view(i, NG_BUF_AUX, torch.bfloat16, nblk * r * 32, self.layouts[i].aux_pbt_off).view(nblk, r, 32)
        return raw.permute(0, 2, 1).reshape(nblk * 32, r)[:m].float()

    def close(self) -> None:
        if getattr(self, "st", None) is not None:
            ng_destroy(self.st)
            self.st = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
