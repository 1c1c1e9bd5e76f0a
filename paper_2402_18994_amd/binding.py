"""ctypes binding of the C ABI in include/snn.h.  Argument marshalling only.

PyTorch appears here for two things: device memory (the workspace, the input
raster, the labels) and the HIP stream handle.  There is no fallback: if the
built library is missing or no HIP device is usable, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

SURROGATES = {"superspike": 0, "arctan": 1, "sigmoid": 2, "triangular": 3, "boxcar": 4, "ste": 5}
PRECISIONS = {"fp32": 0, "bf16": 1}
LOSSES = {"max": 0, "integral": 1}
TENSORS = {"weight": 0, "rweight": 1, "grad_w": 2, "grad_r": 3, "current": 4, "membrane": 5,
           "spikes": 6, "d_spikes": 7, "d_current": 8, "readout_current": 9, "readout_trace": 10,
           "logits": 11, "argmax_t": 12, "d_logits": 13, "d_readout_current": 14, "loss": 15,
           "loss_per_sample": 16, "beta": 17, "grad_beta": 18, "adaptation": 19}
STEPS = {"current_gemm": 0, "lif_forward": 1, "readout_forward": 2, "readout_reverse": 3,
         "lif_reverse": 4, "weight_grad": 5, "input_grad": 6}
KERNELS = {"none": -1, "current_gemm": 0, "lif_forward": 1, "rlif_forward": 2, "readout_forward": 3,
           "readout_reverse": 4, "lif_reverse": 5, "rlif_reverse": 6, "weight_grad": 7,
           "input_grad": 8, "sgd": 9, "calibrate": 10, "grad_reduce": 11, "event_pair": 12}
OPTIONS = {"layer_forward": 0, "layer_pair": 1, "layer_reverse": 2, "top_scans": 3, "defer_reduce": 4,
           "layer_min_batch": 5, "layer_neurons": 6, "layer_max_neurons": 7, "stream_min_mb": 8,
           "stream_gemm": 9, "tile_rows": 10, "layer_time_split": 11, "wgrad_tr": 12, "rlif_persist": 13, "wait_limit_log2": 14,
           "wait_fault": 15}
CALIBRATE_US = 10.0
STATIC_SCRATCH_BYTES = 16 << 20
STATUS = {0: "SNN_OK", 1: "SNN_ERR_NULL", 2: "SNN_ERR_ARG", 3: "SNN_ERR_SHAPE", 4: "SNN_ERR_WORKSPACE",
          5: "SNN_ERR_STATE", 6: "SNN_ERR_HIP", 7: "SNN_ERR_UNSUPPORTED"}


class SnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS.get(status, status)}: {text}")
        self.status = status


class snn_config(C.Structure):
    _fields_ = [("T", C.c_int32), ("B", C.c_int32), ("n_layers", C.c_int32),
                ("sizes", C.POINTER(C.c_int32)), ("recurrent", C.POINTER(C.c_uint8)),
                ("beta", C.POINTER(C.c_float)), ("threshold", C.c_float), ("surrogate", C.c_int32),
                ("slope", C.c_float), ("precision", C.c_int32), ("loss", C.c_int32), ("learn_beta", C.c_int32),
                ("adapt_decay", C.POINTER(C.c_float)), ("adapt_step", C.POINTER(C.c_float))]


def library_path() -> str:
    return os.path.join(HERE, "libsnn_hip.so")


_lib = None


def load_library():
    """dlopen the built library and declare the entry points' signatures."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built: run `python -m paper_2402_18994_amd.build`")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.snn_workspace_bytes.argtypes = [C.POINTER(snn_config), C.POINTER(sz)]
    lib.snn_init.argtypes = [C.POINTER(snn_config), vp, sz, C.POINTER(vp), C.POINTER(vp), vp, C.POINTER(vp)]
    lib.snn_forward.argtypes = [vp, vp, vp, C.POINTER(C.c_float)]
    lib.snn_forward_packed.argtypes = [vp, vp, vp, C.POINTER(C.c_float)]
    lib.snn_backward.argtypes = [vp]
    lib.snn_sgd_step.argtypes = [vp, C.c_float]
    lib.snn_get_tensor.argtypes = [vp, i32, i32, vp, sz]
    lib.snn_set_tensor.argtypes = [vp, i32, i32, vp, sz]
    lib.snn_run_step.argtypes = [vp, i32, i32, vp, vp]
    lib.snn_set_option.argtypes = [vp, i32, i32]
    lib.snn_get_option.argtypes = [vp, i32, C.POINTER(i32)]
    lib.snn_weight_grad_static.argtypes = [vp, vp, vp, C.c_int64, i32, i32, vp]
    lib.snn_profile_select.argtypes = [vp, i32, i32]
    lib.snn_profile_every.argtypes = [vp, i32]
    lib.snn_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.snn_destroy.argtypes = [vp]
    lib.snn_last_error.argtypes = [vp]
    lib.snn_last_error.restype = C.c_char_p
    for name in ("snn_workspace_bytes", "snn_init", "snn_forward", "snn_forward_packed", "snn_backward", "snn_sgd_step",
                 "snn_get_tensor", "snn_set_tensor", "snn_run_step", "snn_set_option", "snn_get_option",
                 "snn_weight_grad_static", "snn_profile_select", "snn_profile_every", "snn_profile_read", "snn_destroy"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


class _Cfg:
    """Keeps the arrays a snn_config points to alive."""

    def __init__(self, T, B, sizes, recurrent, beta, theta, surrogate, slope, precision, loss="max",
                 learn_beta=False, adapt_decay=None, adapt_step=None):
        L = len(sizes) - 1
        self.adapt_decay = self.adapt_step = None
        if adapt_step is not None:
            self.adapt_decay = (C.c_float * max(1, L - 1))(*[float(x) for x in adapt_decay])
            self.adapt_step = (C.c_float * max(1, L - 1))(*[float(x) for x in adapt_step])
        self.sizes = (C.c_int32 * (L + 1))(*[int(s) for s in sizes])
        rec = list(recurrent) if recurrent is not None else [0] * (L - 1)
        self.rec = (C.c_uint8 * max(1, L - 1))(*[int(bool(r)) for r in rec])
        self.beta = (C.c_float * L)(*[float(b) for b in beta])
        self.c = snn_config(int(T), int(B), L, self.sizes, self.rec, self.beta, float(theta),
                            SURROGATES[surrogate] if isinstance(surrogate, str) else int(surrogate),
                            float(slope),
                            PRECISIONS[precision] if isinstance(precision, str) else int(precision),
                            LOSSES[loss] if isinstance(loss, str) else int(loss), int(bool(learn_beta)),
                            self.adapt_decay, self.adapt_step)


def workspace_bytes(T, B, sizes, recurrent, beta, theta, surrogate, slope, precision, loss="max",
                    adapt_decay=None, adapt_step=None) -> int:
    lib = load_library()
    cfg = _Cfg(T, B, sizes, recurrent, beta, theta, surrogate, slope, precision, loss,
               adapt_decay=adapt_decay, adapt_step=adapt_step)
    n = C.c_size_t(0)
    rc = lib.snn_workspace_bytes(C.byref(cfg.c), C.byref(n))
    if rc:
        raise SnnError(rc, lib.snn_last_error(None).decode())
    return n.value


class SNN:
    """One network on one GPU.  Methods mirror the C entry points one to one."""

    def __init__(self, T, B, sizes, recurrent, beta, theta, surrogate, slope, precision,
                 W: Sequence[np.ndarray], R: Optional[Sequence[Optional[np.ndarray]]] = None,
                 device: str = "cuda:0", loss: str = "max", learn_beta: bool = False, options=None,
                 adapt_decay=None, adapt_step=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no HIP device: this library has no CPU path")
        self.lib = load_library()
        self.torch = torch
        self.device = torch.device(device)
        self.T, self.B, self.sizes = int(T), int(B), [int(s) for s in sizes]
        self.L = len(self.sizes) - 1
        self.recurrent = [bool(r) for r in (recurrent if recurrent is not None else [0] * (self.L - 1))]
        self.precision = precision
        self._cfg = _Cfg(T, B, sizes, self.recurrent, beta, theta, surrogate, slope, precision, loss, learn_beta,
                         adapt_decay, adapt_step)
        n = C.c_size_t(0)
        self._chk(self.lib.snn_workspace_bytes(C.byref(self._cfg.c), C.byref(n)), None)
        self.workspace = torch.empty(n.value, dtype=torch.uint8, device=self.device)
        Wc = [np.ascontiguousarray(w, dtype=np.float32) for w in W]
        for l, w in enumerate(Wc):
            assert w.shape == (self.sizes[l], self.sizes[l + 1]), (l, w.shape)
        Wp = (C.c_void_p * self.L)(*[w.ctypes.data for w in Wc])
        Rc = [None if (R is None or R[l] is None) else np.ascontiguousarray(R[l], dtype=np.float32)
              for l in range(self.L - 1)]
        Rp = (C.c_void_p * max(1, self.L - 1))(*[None if r is None else r.ctypes.data for r in Rc])
        self.stream = torch.cuda.current_stream(self.device)
        ctx = C.c_void_p(None)
        with torch.cuda.device(self.device):
            rc = self.lib.snn_init(C.byref(self._cfg.c), self.workspace.data_ptr(), n.value, Wp, Rp,
                                   C.c_void_p(self.stream.cuda_stream), C.byref(ctx))
        self._chk(rc, None)
        self.ctx = ctx
        self._x = None
        self._labels = None
        for name, value in (options or {}).items():
            self.set_option(name, value)

    # ------------------------------------------------------------------ helpers
    def _chk(self, rc, ctx):
        if rc:
            raise SnnError(rc, self.lib.snn_last_error(ctx).decode())

    def _dev_u8(self, x):
        t = self.torch
        if isinstance(x, np.ndarray):
            x = t.from_numpy(np.ascontiguousarray(x, dtype=np.uint8)).to(self.device)
        assert x.dtype == t.uint8 and x.is_contiguous() and x.device.type == "cuda"
        return x

    def _dev_i32(self, y):
        t = self.torch
        if isinstance(y, np.ndarray):
            y = t.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(self.device)
        assert y.dtype == t.int32 and y.is_contiguous() and y.device.type == "cuda"
        return y

    def _shape(self, name, layer):
        T, B, s, L = self.T, self.B, self.sizes, self.L
        if name in ("weight", "grad_w"):
            return (s[layer - 1], s[layer]), np.float32
        if name in ("rweight", "grad_r"):
            return (s[layer], s[layer]), np.float32
        if name in ("current", "membrane", "d_spikes", "d_current", "adaptation"):
            return (T, B, s[layer]), np.float32
        if name == "spikes":
            return (T, B, s[layer]), np.uint8
        if name in ("readout_current", "readout_trace", "d_readout_current"):
            return (T, B, s[L]), np.float32
        if name in ("logits", "d_logits"):
            return (B, s[L]), np.float32
        if name == "argmax_t":
            return (B, s[L]), np.int32
        if name in ("beta", "grad_beta"):
            return (s[layer],), np.float32
        if name == "loss":
            return (1,), np.float32
        if name == "loss_per_sample":
            return (B,), np.float32
        raise KeyError(name)

    # ------------------------------------------------------------------ the entry points
    def forward(self, x, labels, want_loss: bool = True):
        """snn_forward.  x: uint8 [T,B,N0] (numpy or cuda tensor), labels: int32 [B]."""
        self._x, self._labels = self._dev_u8(x), self._dev_i32(labels)
        assert tuple(self._x.shape) == (self.T, self.B, self.sizes[0]), tuple(self._x.shape)
        assert tuple(self._labels.shape) == (self.B,)
        loss = C.c_float(0.0)
        rc = self.lib.snn_forward(self.ctx, self._x.data_ptr(), self._labels.data_ptr(),
                                  C.byref(loss) if want_loss else None)
        self._chk(rc, self.ctx)
        return loss.value if want_loss else None

    def forward_packed(self, x_packed, labels, want_loss: bool = True):
        """snn_forward_packed.  x_packed: uint8 [ceil(T/8),B,N0] = numpy.packbits(x, axis=0)."""
        self._x, self._labels = self._dev_u8(x_packed), self._dev_i32(labels)
        assert tuple(self._x.shape) == ((self.T + 7) // 8, self.B, self.sizes[0]), tuple(self._x.shape)
        assert tuple(self._labels.shape) == (self.B,)
        loss = C.c_float(0.0)
        rc = self.lib.snn_forward_packed(self.ctx, self._x.data_ptr(), self._labels.data_ptr(),
                                         C.byref(loss) if want_loss else None)
        self._chk(rc, self.ctx)
        return loss.value if want_loss else None

    def backward(self):
        self._chk(self.lib.snn_backward(self.ctx), self.ctx)

    def sgd_step(self, lr: float):
        self._chk(self.lib.snn_sgd_step(self.ctx, float(lr)), self.ctx)

    def get_tensor(self, name: str, layer: int = 0) -> np.ndarray:
        shape, dt = self._shape(name, layer)
        out = np.empty(shape, dtype=dt)
        self._chk(self.lib.snn_get_tensor(self.ctx, TENSORS[name], layer, out.ctypes.data, out.nbytes), self.ctx)
        return out

    def set_tensor(self, name: str, layer: int, value: np.ndarray):
        shape, dt = self._shape(name, layer)
        v = np.ascontiguousarray(value, dtype=dt)
        assert v.shape == tuple(shape), (v.shape, shape)
        self._chk(self.lib.snn_set_tensor(self.ctx, TENSORS[name], layer, v.ctypes.data, v.nbytes), self.ctx)

    def run_step(self, step: str, layer: int, x=None, labels=None):
        if x is not None:
            self._x = self._dev_u8(x)
        if labels is not None:
            self._labels = self._dev_i32(labels)
        xp = self._x.data_ptr() if self._x is not None else None
        lp = self._labels.data_ptr() if self._labels is not None else None
        self._chk(self.lib.snn_run_step(self.ctx, STEPS[step], layer, xp, lp), self.ctx)

    def set_option(self, name: str, value: int):
        self._chk(self.lib.snn_set_option(self.ctx, OPTIONS[name], int(value)), self.ctx)

    def get_option(self, name: str) -> int:
        v = C.c_int32(0)
        self._chk(self.lib.snn_get_option(self.ctx, OPTIONS[name], C.byref(v)), None)
        return v.value

    def profile_select(self, kernel: str, layer: int = 0):
        self._chk(self.lib.snn_profile_select(self.ctx, KERNELS[kernel], layer), self.ctx)

    def profile_every(self, n: int):
        self._chk(self.lib.snn_profile_every(self.ctx, n), self.ctx)

    def profile_read(self):
        ms, n = C.c_double(0), C.c_int64(0)
        self._chk(self.lib.snn_profile_read(self.ctx, C.byref(ms), C.byref(n)), self.ctx)
        return ms.value, n.value

    def synchronize(self):
        self.stream.synchronize()

    def destroy(self):
        if getattr(self, "ctx", None) is not None and self.ctx.value is not None:
            self.lib.snn_destroy(self.ctx)
            self.ctx = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def weight_grad_static(S, G, dW, stream=None):
    """snn_weight_grad_static: dW [K,N] = S^T G for S uint8 [M,K] and G float32 [M,N], all cuda
    tensors the caller owns; nothing is allocated."""
    import torch
    lib = load_library()
    assert S.dtype == torch.uint8 and G.dtype == torch.float32 and dW.dtype == torch.float32
    assert S.is_contiguous() and G.is_contiguous() and dW.is_contiguous()
    M, K = S.shape
    N = G.shape[1]
    assert G.shape[0] == M and tuple(dW.shape) == (K, N)
    st = stream if stream is not None else torch.cuda.current_stream(S.device)
    with torch.cuda.device(S.device):
        rc = lib.snn_weight_grad_static(S.data_ptr(), G.data_ptr(), dW.data_ptr(), M, K, N, C.c_void_p(st.cuda_stream))
    if rc:
        raise SnnError(rc, lib.snn_last_error(None).decode())


def from_workload(wl, inputs, device: str = "cuda:0", learn_beta: bool = False, options=None) -> SNN:
    """Build an SNN for a workloads.Workload and the weights of a workloads.Inputs."""
    return SNN(wl.T, wl.B, wl.sizes, wl.recurrent, wl.beta, wl.theta, wl.surrogate, wl.slope,
               wl.precision, inputs.W, inputs.R, device=device, loss=getattr(wl, "loss", "max"),
               learn_beta=learn_beta, options=options, adapt_decay=getattr(wl, "adapt_decay", None),
               adapt_step=getattr(wl, "adapt_step", None))
