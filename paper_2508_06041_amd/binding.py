"""ctypes binding with the same names as include/dpllm.h.  Argument marshalling only.

Tensors are torch tensors used purely as device memory: the binding passes data_ptr() and the
current HIP stream to the C functions.  Functions raise DpllmError on a negative return code.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdpllm.so")

DPLLM_OK, DPLLM_EINVAL, DPLLM_ESHAPE, DPLLM_ERANGE, DPLLM_ESTATE, DPLLM_EHIP = 0, -1, -2, -3, -4, -5
DPLLM_SEL_NONE, DPLLM_SEL_PROJ, DPLLM_SEL_LINREG = 0, 1, 2
DPLLM_MAX_BATCH = 8
DPLLM_MAX_PAIRS = 8
DPLLM_MAX_TARGETS = 8
DPLLM_STEP_SELECT, DPLLM_STEP_GEMV = 1, 2

SYMBOLS = ["dpllm_model_create", "dpllm_model_destroy", "dpllm_last_error", "dpllm_linear_device_bytes",
           "dpllm_workspace_bytes", "dpllm_set_workspace",
           "dpllm_load_linear", "dpllm_set_selector", "dpllm_set_threshold", "dpllm_set_active_pair",
           "dpllm_set_target_entry", "dpllm_set_target", "dpllm_set_selector_input",
           "dpllm_estimate", "dpllm_estimate_noalloc", "dpllm_gemv", "dpllm_decode_step", "dpllm_decode_step_parts", "dpllm_debug_unpack", "dpllm_debug_locate",
           "dpllm_debug_copy", "dpllm_debug_read"]


class DpllmError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("dpllm error %d: %s" % (code, msg))
        self.code = code


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libdpllm.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    L = C.CDLL(_LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int, C.c_float, C.c_size_t
    L.dpllm_model_create.argtypes = [C.POINTER(vp), i32]
    L.dpllm_model_destroy.argtypes = [vp]
    L.dpllm_model_destroy.restype = None
    L.dpllm_last_error.argtypes = [vp]
    L.dpllm_last_error.restype = C.c_char_p
    L.dpllm_linear_device_bytes.argtypes = [i32, i32, i32, i32, C.POINTER(sz)]
    L.dpllm_debug_locate.argtypes = [i32, i32, i32, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(i32)]
    L.dpllm_load_linear.argtypes = [vp, i32, i32, i32, i32, i32, vp, C.POINTER(vp), i32, vp, sz, vp]
    L.dpllm_set_selector.argtypes = [vp, i32, i32, i32, i32, vp, i32, f32, f32, f32]
    L.dpllm_set_threshold.argtypes = [vp, i32, i32, i32, f32]
    L.dpllm_set_active_pair.argtypes = [vp, i32, i32, i32]
    L.dpllm_set_selector_input.argtypes = [vp, i32, vp]
    L.dpllm_workspace_bytes.argtypes = [vp, C.POINTER(sz)]
    L.dpllm_set_workspace.argtypes = [vp, vp, sz, vp]
    L.dpllm_set_target_entry.argtypes = [vp, i32, i32, i32, i32, f32]
    L.dpllm_set_target.argtypes = [vp, i32, vp]
    L.dpllm_estimate.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
    L.dpllm_estimate_noalloc.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp]
    L.dpllm_gemv.argtypes = [vp, i32, i32, vp, vp, vp, i32, vp]
    L.dpllm_decode_step.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, vp, vp]
    L.dpllm_decode_step_parts.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp, vp, i32, vp]
    L.dpllm_debug_unpack.argtypes = [vp, i32, i32, vp, vp]
    L.dpllm_debug_copy.argtypes = [vp, vp, sz, vp]
    L.dpllm_debug_read.argtypes = [vp, sz, vp, vp]
    return L


lib = _load()


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def _check(model, rc):
    if rc != 0:
        msg = lib.dpllm_last_error(model).decode() if model else ""
        raise DpllmError(rc, msg)


def dpllm_linear_device_bytes(out, in_, p, kmin):
    n = C.c_size_t(0)
    rc = lib.dpllm_linear_device_bytes(out, in_, p, kmin, C.byref(n))
    if rc != 0:
        raise DpllmError(rc, "dpllm_linear_device_bytes(%d,%d,%d,%d)" % (out, in_, p, kmin))
    return n.value


def dpllm_debug_copy(dst, src):
    nbytes = src.numel() * src.element_size()
    rc = lib.dpllm_debug_copy(_ptr(dst), _ptr(src), nbytes, _stream())
    if rc != 0:
        raise DpllmError(rc, "dpllm_debug_copy")


def dpllm_debug_read(src, sink):
    nbytes = src.numel() * src.element_size()
    rc = lib.dpllm_debug_read(_ptr(src), nbytes, _ptr(sink), _stream())
    if rc != 0:
        raise DpllmError(rc, "dpllm_debug_read")


class Model:
    """Owns the C handle and the torch tensors used as device memory (arenas, workspace)."""

    def __init__(self, n_linears):
        h = C.c_void_p()
        rc = lib.dpllm_model_create(C.byref(h), n_linears)
        if rc != 0:
            raise DpllmError(rc, "dpllm_model_create")
        self.h = h
        self.n = n_linears
        self.arenas = {}
        self.keep = {}
        self.shapes = {}
        self._sel_inputs = {}
        self.workspace = None
        self._ws_stale = True      # the model changed in a way that may ask for a larger workspace

    def dpllm_workspace_bytes(self):
        n = C.c_size_t(0)
        _check(self.h, lib.dpllm_workspace_bytes(self.h, C.byref(n)))
        return n.value

    def dpllm_set_workspace(self, tensor=None):
        """Hands the model a workspace: `tensor` (device, uint8) or a fresh allocation of the size the model asks
        for.  The calls that need one allocate it on first use; call this yourself to choose the moment."""
        need = self.dpllm_workspace_bytes()
        if tensor is None:
            tensor = torch.empty(need, dtype=torch.uint8, device="cuda")
        _check(self.h, lib.dpllm_set_workspace(self.h, _ptr(tensor), tensor.numel() * tensor.element_size(), _stream()))
        old, self.workspace = self.workspace, tensor
        self._ws_stale = False
        return old   # the caller decides when the previous one may go (work enqueued earlier may still use it)

    def _need_workspace(self):
        if self._ws_stale and (self.workspace is None or self.workspace.numel() < self.dpllm_workspace_bytes()):
            old = self.dpllm_set_workspace()
            if old is not None:
                torch.cuda.current_stream().synchronize()
        self._ws_stale = False

    def close(self):
        if self.h:
            lib.dpllm_model_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def dpllm_load_linear(self, id, planes, luts, kmin):
        """planes: int32/uint32 [p][out][in/32] (numpy or torch, host or device);
        luts: dict or list of fp16/uint16 [out][2^k] for k = kmin..p."""
        import numpy as np
        if isinstance(planes, np.ndarray):
            planes = torch.from_numpy(planes.view(np.int32))
        p, out, nw = planes.shape
        if isinstance(luts, dict):
            luts = [luts[k] for k in range(kmin, p + 1)]
        luts = [torch.from_numpy(t.view(np.int16)) if isinstance(t, np.ndarray) else t for t in luts]
        on_dev = planes.is_cuda
        luts = [(t.cuda() if on_dev else t.cpu()).contiguous() for t in luts]
        planes = planes.contiguous()
        nbytes = dpllm_linear_device_bytes(out, nw * 32, p, kmin)
        arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        arr = (C.c_void_p * len(luts))(*[t.data_ptr() for t in luts])
        rc = lib.dpllm_load_linear(self.h, id, out, nw * 32, p, kmin, _ptr(planes), arr, 1 if on_dev else 0,
                                   _ptr(arena), nbytes, _stream())
        _check(self.h, rc)
        self.arenas[id] = arena
        self.shapes[id] = (out, nw * 32, p, kmin)
        self._ws_stale = True

    def dpllm_set_selector(self, id, l, h, kind, G=None, alpha=0.0, beta=0.0, T=float("inf")):
        r = 0
        if G is not None:
            G = G.contiguous()
            assert G.is_cuda and G.dtype == torch.float16
            r = G.shape[0]
            self.keep[(id, l, h)] = G
        _check(self.h, lib.dpllm_set_selector(self.h, id, l, h, kind, _ptr(G), r, alpha, beta, T))
        self._ws_stale = True

    def dpllm_set_threshold(self, id, l, h, T):
        _check(self.h, lib.dpllm_set_threshold(self.h, id, l, h, T))

    def dpllm_set_active_pair(self, id, l, h):
        _check(self.h, lib.dpllm_set_active_pair(self.h, id, l, h))

    def dpllm_set_target_entry(self, target, id, l, h, T):
        _check(self.h, lib.dpllm_set_target_entry(self.h, target, id, l, h, T))

    def dpllm_set_target(self, target):
        self._need_workspace()
        _check(self.h, lib.dpllm_set_target(self.h, target, _stream()))

    def dpllm_set_selector_input(self, id, x_sel):
        """x_sel: device fp16 [in] the selector of linear id reads in the step calls (None: its immediate input).
        The model keeps a reference to the tensor."""
        self._sel_inputs[id] = x_sel
        _check(self.h, lib.dpllm_set_selector_input(self.h, id, _ptr(x_sel)))

    def dpllm_estimate(self, id, l, h, x, e_out=None, k_out=None):
        e_out = torch.empty(1, dtype=torch.float32, device="cuda") if e_out is None else e_out
        k_out = torch.empty(1, dtype=torch.int32, device="cuda") if k_out is None else k_out
        self._need_workspace()
        _check(self.h, lib.dpllm_estimate(self.h, id, l, h, _ptr(x), _ptr(e_out), _ptr(k_out), _stream()))
        return e_out, k_out

    def dpllm_estimate_noalloc(self, id, l, h, x, e_out, k_out):
        """The variant that allocates nothing: the caller passes every buffer, no workspace is touched."""
        _check(self.h, lib.dpllm_estimate_noalloc(self.h, id, l, h, _ptr(x), _ptr(e_out), _ptr(k_out), _stream()))
        return e_out, k_out

    def dpllm_gemv(self, id, k, x, y=None, k_dev=None):
        """k >= 0: fixed bitwidth.  k < 0: read the bitwidth from k_dev on the device."""
        out = self.shapes.get(id, (1,))[0]   # an unknown id is reported by the library
        B = 1 if x.dim() == 1 else x.shape[0]
        if y is None:
            y = torch.empty((out,) if x.dim() == 1 else (B, out), dtype=torch.float16, device="cuda")
        self._need_workspace()
        _check(self.h, lib.dpllm_gemv(self.h, id, k, _ptr(k_dev), _ptr(x), _ptr(y), B, _stream()))
        return y

    def pointers(self, tensors):
        """The host array of n_linears device pointers the step calls take; build it once for tensors that stay
        where they are and pass it instead of the list (the caller keeps the tensors alive)."""
        if isinstance(tensors, C.Array):
            return tensors
        assert len(tensors) == self.n
        return (C.c_void_p * self.n)(*[t.data_ptr() for t in tensors])

    def dpllm_decode_step(self, xs, ys, k_out, e_out):
        self._need_workspace()
        _check(self.h, lib.dpllm_decode_step(self.h, self.pointers(xs), self.pointers(ys), _ptr(k_out), _ptr(e_out),
                                             _stream()))

    def dpllm_decode_step_parts(self, xs, ys, k_out, e_out, parts):
        self._need_workspace()
        _check(self.h, lib.dpllm_decode_step_parts(self.h, self.pointers(xs), self.pointers(ys), _ptr(k_out),
                                                   _ptr(e_out), parts, _stream()))

    def dpllm_debug_unpack(self, id, k):
        out, in_, _, _ = self.shapes.get(id, (1, 32, 0, 0))
        idx = torch.empty((out, in_), dtype=torch.uint8, device="cuda")
        _check(self.h, lib.dpllm_debug_unpack(self.h, id, k, _ptr(idx), _stream()))
        return idx
