"""ctypes binding of the C boundary (include/lopt.h). Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("LOPT_LIB_PATH") or os.path.join(_HERE, "liblopt.so")   # override: A/B builds

LOPT_SMALL_FC = 0
LOPT_VELO = 1
APPLY_KERNELS = {"auto": 0, "valu": 1, "mfma_f32": 2, "mfma_f16s": 3}   # lopt_apply_kernel
STATE_PASSES = {"auto": 0, "stats": 1, "apply": 2}                        # lopt_state_pass
N_PASSES = 7
_STATUS = {0: "LOPT_OK", 1: "LOPT_EINVAL", 2: "LOPT_ESHAPE", 3: "LOPT_ESTATE", 4: "LOPT_ENOMEM", 5: "LOPT_EHIP",
           6: "LOPT_ELIMIT"}
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ["lopt_default_config", "lopt_weights_count", "lopt_create", "lopt_destroy", "lopt_state_bytes",
           "lopt_init_state", "lopt_step", "lopt_step_static", "lopt_set_loss", "lopt_stats_offsets",
           "lopt_last_error",
           "lopt_profile_enable", "lopt_profile_read", "lopt_pass_name"]


class LoptError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class lopt_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("kind", C.c_uint32), ("hidden", C.c_uint32),
                ("mom_decay", C.c_float * 3), ("rms_decay", C.c_float), ("fac_decay", C.c_float * 3),
                ("eps_acc", C.c_float), ("eps_norm", C.c_float), ("exp_mult", C.c_float),
                ("step_mult", C.c_float), ("lstm_hidden", C.c_uint32), ("n_bank", C.c_uint32),
                ("apply_kernel", C.c_uint32), ("groups", C.c_uint32), ("state_pass", C.c_uint32)]


class lopt_tensor_desc(C.Structure):
    _fields_ = [("ndim", C.c_uint32), ("rows", C.c_int64), ("cols", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """Load liblopt.so (built in-tree by `python -m paper_2506_10315_amd.build`). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2506_10315_amd.build` "
                          "(there is no CPU fallback)")
    # PyTorch ships its own HIP runtime (same soname as the system one). It has to be in the
    # process before liblopt.so so that both share one runtime, one device context and one set of streams.
    import torch  # noqa: F401
    L = C.CDLL(_LIB_PATH)
    vp, sz, fp = C.c_void_p, C.c_size_t, C.POINTER(C.c_float)
    L.lopt_default_config.argtypes = [C.c_uint32, C.POINTER(lopt_config)]
    L.lopt_default_config.restype = C.c_int
    L.lopt_weights_count.argtypes = [C.POINTER(lopt_config)]
    L.lopt_weights_count.restype = sz
    L.lopt_create.argtypes = [C.POINTER(lopt_config), fp, sz, C.POINTER(vp)]
    L.lopt_create.restype = C.c_int
    L.lopt_destroy.argtypes = [vp]
    L.lopt_destroy.restype = None
    L.lopt_state_bytes.argtypes = [vp, sz, C.POINTER(lopt_tensor_desc), C.POINTER(sz), C.POINTER(sz)]
    L.lopt_state_bytes.restype = C.c_int
    L.lopt_init_state.argtypes = [vp, sz, C.POINTER(lopt_tensor_desc), C.POINTER(vp), vp, vp]
    L.lopt_init_state.restype = C.c_int
    L.lopt_step.argtypes = [vp, sz, C.POINTER(lopt_tensor_desc), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                            vp, C.c_int64, C.c_float, C.c_float, vp]
    L.lopt_step.restype = C.c_int
    L.lopt_step_static.argtypes = [vp, sz, C.POINTER(lopt_tensor_desc), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                   C.c_int64, C.c_float, C.c_float, vp]
    L.lopt_step_static.restype = C.c_int
    L.lopt_set_loss.argtypes = [vp, C.c_float]
    L.lopt_set_loss.restype = C.c_int
    L.lopt_stats_offsets.argtypes = [vp, sz, C.POINTER(lopt_tensor_desc), C.POINTER(sz)]
    L.lopt_stats_offsets.restype = C.c_int
    L.lopt_profile_enable.argtypes = [vp, C.c_int]
    L.lopt_profile_enable.restype = C.c_int
    L.lopt_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    L.lopt_profile_read.restype = C.c_int
    L.lopt_pass_name.argtypes = [C.c_int]
    L.lopt_pass_name.restype = C.c_char_p
    L.lopt_last_error.argtypes = [vp]
    L.lopt_last_error.restype = C.c_char_p
    _lib = L
    return L


def _check(status: int, ctx=None):
    if status != 0:
        msg = lib().lopt_last_error(ctx)
        raise LoptError(status, msg.decode() if msg else "")


def default_config(kind: int) -> lopt_config:
    cfg = lopt_config()
    _check(lib().lopt_default_config(kind, C.byref(cfg)))
    return cfg


def weights_count(cfg: lopt_config) -> int:
    return int(lib().lopt_weights_count(C.byref(cfg)))


class LearnedOptimizer:
    """Owns a lopt_ctx plus the torch tensors used as state blobs and workspace.

    params/grads are lists of contiguous fp32 CUDA tensors; shapes are flattened to
    (rows, cols) as include/lopt.h prescribes. All arithmetic happens in lopt_step.
    """

    def __init__(self, cfg: lopt_config, weights, shapes: Sequence[Sequence[int]], device="cuda:0"):
        import numpy as np
        import torch
        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        w = np.ascontiguousarray(weights, dtype=np.float32).ravel()
        self._ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().lopt_create(C.byref(cfg), w.ctypes.data_as(C.POINTER(C.c_float)), w.size,
                                     C.byref(self._ctx)))
        self.n = len(shapes)
        self._descs = (lopt_tensor_desc * max(self.n, 1))()
        for i, shp in enumerate(shapes):
            nd, rows, cols = flatten_shape(shp)
            self._descs[i].ndim, self._descs[i].rows, self._descs[i].cols = nd, rows, cols
        per = (C.c_size_t * max(self.n, 1))()
        wsb = C.c_size_t()
        _check(lib().lopt_state_bytes(self._ctx, self.n, self._descs, per, C.byref(wsb)), self._ctx)
        self.state_bytes = [int(per[i]) for i in range(self.n)]
        self.workspace_bytes = int(wsb.value)
        self.state = [torch.empty(b // 4, dtype=torch.float32, device=self.device) for b in self.state_bytes]
        self.workspace = torch.empty(max(self.workspace_bytes // 4, 64), dtype=torch.float32, device=self.device)
        self._state_ptrs = (C.c_void_p * max(self.n, 1))(*[t.data_ptr() for t in self.state])
        self.step_count = 0
        self.init_state()

    def _stream(self):
        return C.c_void_p(self._torch.cuda.current_stream(self.device).cuda_stream)

    def init_state(self):
        with self._torch.cuda.device(self.device):
            _check(lib().lopt_init_state(self._ctx, self.n, self._descs, self._state_ptrs,
                                         C.c_void_p(self.workspace.data_ptr()), self._stream()), self._ctx)
        self.step_count = 0

    def set_loss(self, loss: float):
        """The loss value that goes with the gradients of the following steps (VeLO's loss features)."""
        _check(lib().lopt_set_loss(self._ctx, float(loss)), self._ctx)

    def step(self, params: List, grads: List, lr: float = 1.0, weight_decay: float = 0.0,
             step: Optional[int] = None, static: bool = False, loss: Optional[float] = None,
             indices: Optional[Sequence[int]] = None):
        """lopt_step, or lopt_step_static (library-owned fixed scratch, no allocation) with static=True.
        `loss`, if given, is handed to lopt_set_loss first. `indices` steps only those tensors of the list this
        object was built for (params/grads then hold just them, in that order); the others keep their state."""
        if indices is None:
            n, descs, sp = self.n, self._descs, self._state_ptrs
        else:
            n = len(indices)
            descs = (lopt_tensor_desc * max(n, 1))(*[self._descs[i] for i in indices])
            sp = (C.c_void_p * max(n, 1))(*[self.state[i].data_ptr() for i in indices])
        assert len(params) == n and len(grads) == n
        if loss is not None:
            self.set_loss(loss)
        pp = (C.c_void_p * max(n, 1))(*[p.data_ptr() for p in params])
        gp = (C.c_void_p * max(n, 1))(*[g.data_ptr() for g in grads])
        t = self.step_count if step is None else step
        with self._torch.cuda.device(self.device):
            if static:
                _check(lib().lopt_step_static(self._ctx, n, descs, pp, gp, sp, t, lr,
                                              weight_decay, self._stream()), self._ctx)
            else:
                _check(lib().lopt_step(self._ctx, n, descs, pp, gp, sp,
                                       C.c_void_p(self.workspace.data_ptr()), t, lr, weight_decay,
                                       self._stream()), self._ctx)
        self.step_count = t + 1

    def profile_enable(self, on: bool = True):
        _check(lib().lopt_profile_enable(self._ctx, 1 if on else 0), self._ctx)

    def profile_read(self):
        """({pass name: total ms since the last read}, number of steps)."""
        ms = (C.c_double * N_PASSES)()
        k = C.c_uint64()
        _check(lib().lopt_profile_read(self._ctx, ms, C.byref(k)), self._ctx)
        return {lib().lopt_pass_name(i).decode(): float(ms[i]) for i in range(N_PASSES)}, int(k.value)

    def stats(self):
        """Per-tensor feature statistics left in the workspace by the last step (list of 1-D tensors)."""
        off = (C.c_size_t * max(self.n, 1))()
        _check(lib().lopt_stats_offsets(self._ctx, self.n, self._descs, off), self._ctx)
        d = 28 if self.cfg.kind == LOPT_SMALL_FC else 29
        base = (-self.workspace.data_ptr()) % 256 // 4     # the library rounds the base up to 256 bytes
        return [self.workspace[base + off[i] // 4: base + off[i] // 4 + d] for i in range(self.n)]

    def state_views(self, i: int):
        """Views of tensor i's state blob: dict with M[3,m,n], V[m,n], r[3,m], c[3,n] (+ h, cl)."""
        d = self._descs[i]
        m, n = int(d.rows), int(d.cols)
        N = m * n
        p4 = lambda x: (x + 3) & ~3
        s = self.state[i]
        o = 0
        out = {}
        out["M"] = [s[o + k * p4(N): o + k * p4(N) + N].view(m, n) for k in range(3)]
        o += 3 * p4(N)
        out["V"] = s[o:o + N].view(m, n)
        o += p4(N)
        out["r"] = [s[o + k * p4(m): o + k * p4(m) + m] for k in range(3)]
        o += 3 * p4(m)
        out["c"] = [s[o + k * p4(n): o + k * p4(n) + n] for k in range(3)]
        o += 3 * p4(n)
        if self.cfg.kind == LOPT_VELO:
            HL = int(self.cfg.lstm_hidden)
            out["h"] = s[o:o + HL]
            out["cl"] = s[o + p4(HL): o + p4(HL) + HL]
        return out

    def close(self):
        if getattr(self, "_ctx", None) and self._ctx.value:
            self._torch.cuda.synchronize(self.device)
            lib().lopt_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def flatten_shape(shape: Sequence[int]):
    """(ndim, rows, cols) per include/lopt.h: squeeze leading 1s, 1-D -> 1 x n, ndim > 2 -> (dim0, rest)."""
    shp = [int(s) for s in shape]
    while len(shp) > 1 and shp[0] == 1:
        shp = shp[1:]
    if len(shp) == 1:
        return 1, 1, shp[0]
    rest = 1
    for s in shp[1:]:
        rest *= s
    return len(shp), shp[0], rest
