"""ctypes binding of include/moonwalk.h. Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
TILE_AUTO, TILE_128, TILE_64, TILE_32K4, TILE_32K8, TILE_64K2, TILE_128W8, TILE_64X128 = 0, 1, 2, 3, 4, 5, 6, 7
PLAN_MOONWALK, PLAN_BACKPROP = 1, 2
FETCH_MASK, FETCH_FRAG, FETCH_FRAG_OFFSETS, FETCH_FRAG_BASE, FETCH_H0, FETCH_P, FETCH_CHECKPOINT = range(1, 8)
FETCH_Z, FETCH_H, FETCH_H_FORWARD = 8, 9, 10

EXPORTED_SYMBOLS = [
    "moonwalk_setup", "moonwalk_refresh", "moonwalk_refresh_incremental", "moonwalk_sgd_step", "moonwalk_grad", "backprop_grad", "moonwalk_grad_layout",
    "moonwalk_memory_stats", "moonwalk_debug_fetch", "moonwalk_destroy", "moonwalk_strerror",
    "moonwalk_profile_filter", "moonwalk_profile_launches",
    "mw_gemm_f32", "mw_bias_act_mask", "mw_rev_scale", "mw_frag_offsets", "mw_frag_offsets_work_words", "mw_frag_compact",
    "mw_vijp_epilogue", "mw_colsum", "mw_colsum_wide", "mw_colsum_work_floats", "mw_colsum_wide_noalloc", "mw_colsum_noalloc_max_floats", "mw_loss_grad", "mw_loss_scratch_doubles", "mw_copy_f32",
    "mw_probe_operand_stream",
    "moonwalk_conv_setup", "moonwalk_conv_refresh", "moonwalk_conv_grad", "backprop_conv_grad",
    "moonwalk_conv_grad_layout", "moonwalk_conv_memory_stats", "moonwalk_conv_fetch", "moonwalk_conv_destroy",
    "moonwalk_conv_sgd_step", "mw_conv_im2col", "mw_conv_col2im", "mw_conv_forward", "mw_conv_input_cotangent", "mw_conv_weight_grad_work_floats",
    "mw_conv_weight_grad",
]


class MoonwalkError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libmoonwalk error {code}: {text}")
        self.code = code


ERR_INVALID_ARG, ERR_NOT_SUBMERSIVE, ERR_OOM, ERR_FRAG_OVERFLOW, ERR_HIP, ERR_SIGN_MISMATCH, ERR_NOT_PLANNED, ERR_TOO_LARGE, \
    ERR_NONFINITE = -1, -2, -3, -4, -5, -6, -7, -8, -9


class _Layer(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("W", C.c_void_p), ("b", C.c_void_p),
                ("alpha", C.c_float)]


_ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
_FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class _Config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("reseed_interval", C.c_int32), ("loss_scale", C.c_float),
                ("plan", C.c_int32), ("fuse", C.c_int32), ("frag_capacity_factor", C.c_double),
                ("dev_alloc", _ALLOC_FN), ("dev_free", _FREE_FN), ("alloc_ctx", C.c_void_p),
                ("segment_length", C.c_int32), ("debug_keep", C.c_int32),
                ("phase3_parallel_segments", C.c_int32), ("phase3_overlap", C.c_int32),
                ("refresh_precision", C.c_int32)]


class _ConvLayer(C.Structure):
    _fields_ = [("channels_in", C.c_int32), ("channels_out", C.c_int32), ("k", C.c_int32), ("stride", C.c_int32),
                ("pad", C.c_int32), ("w", C.c_void_p), ("b", C.c_void_p), ("alpha", C.c_float),
                ("kind", C.c_int32), ("block", C.c_int32)]


class _ConvShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "height", "width", "channels_in", "channels_out", "kh", "kw", "stride",
                                         "pad_h", "pad_w")]


class _ConvConfig(C.Structure):
    _fields_ = [("batch", C.c_int32), ("height", C.c_int32), ("width", C.c_int32), ("reseed_interval", C.c_int32),
                ("loss_scale", C.c_float), ("plan", C.c_int32), ("kernels", C.c_int32), ("input_cotangent", C.c_int32),
                ("max_images_per_launch", C.c_int32), ("patch_bytes", C.c_size_t),
                ("dev_alloc", _ALLOC_FN), ("dev_free", _FREE_FN), ("alloc_ctx", C.c_void_p)]


class _ConvMemStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "bytes_masks", "bytes_tap_inverses", "bytes_packed_weights", "bytes_fragments", "bytes_checkpoints", "bytes_input_cotangent",
        "bytes_scratch", "bytes_patches", "bytes_bp_activations", "bytes_bp_scratch", "bytes_live", "bytes_peak", "sign_mismatches",
        "nonfinite_loss")]


class _MemStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "bytes_P", "bytes_masks", "bytes_fragments", "bytes_frag_index", "bytes_checkpoints",
        "bytes_mw_scratch", "bytes_bp_activations", "bytes_bp_scratch", "bytes_live", "bytes_peak",
        "bytes_setup_peak", "frag_used", "sign_mismatches")] + [("frag_overflow", C.c_int32),
                                                                 ("phase3_group_width", C.c_int32),
                                                                 ("bytes_debug", C.c_uint64),
                                                                 ("nonfinite_loss", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoonwalk.so")


def load_library() -> C.CDLL:
    """Load libmoonwalk.so (built in-tree by __graft_entry__.build()). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: run `python __graft_entry__.py` to build the HIP library")
    lib = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    lib.moonwalk_setup.argtypes = [C.POINTER(vp), C.POINTER(_Layer), i32, C.POINTER(_Config), vp]
    lib.moonwalk_refresh.argtypes = [vp, vp]
    lib.moonwalk_refresh_incremental.argtypes = [vp, i32, vp, vp]
    lib.moonwalk_sgd_step.argtypes = [vp, vp, vp, f32, i32, vp, vp, vp]
    lib.moonwalk_grad.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.backprop_grad.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.moonwalk_grad_layout.argtypes = [vp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    lib.moonwalk_memory_stats.argtypes = [vp, C.POINTER(_MemStats)]
    lib.moonwalk_debug_fetch.argtypes = [vp, i32, i32, vp, sz, C.POINTER(sz)]
    lib.moonwalk_profile_filter.argtypes = [vp, i32]
    lib.moonwalk_profile_launches.argtypes = [vp, i32, C.POINTER(C.c_uint64)]
    lib.moonwalk_destroy.argtypes = [vp]
    lib.moonwalk_destroy.restype = None
    lib.moonwalk_strerror.argtypes = [C.c_int]
    lib.moonwalk_strerror.restype = C.c_char_p
    lib.mw_gemm_f32.argtypes = [i32, i32, i32, i32, i32, f32, vp, i32, vp, i32, f32, vp, i32, vp]
    lib.mw_bias_act_mask.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp]
    lib.mw_rev_scale.argtypes = [vp, vp, i64, f32, vp, vp]
    lib.mw_frag_offsets.argtypes = [vp, i64, vp, vp, vp]
    lib.mw_frag_offsets_work_words.argtypes = [i64]
    lib.mw_frag_offsets_work_words.restype = sz
    lib.mw_frag_compact.argtypes = [vp, vp, vp, i64, vp, C.c_uint64, vp, vp]
    lib.mw_vijp_epilogue.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp, vp, vp, vp]
    lib.mw_colsum.argtypes = [vp, i64, i32, f32, vp, vp]
    lib.mw_colsum_wide.argtypes = [vp, i64, i32, f32, vp, vp, vp]
    lib.mw_colsum_work_floats.argtypes = [i32]
    lib.mw_colsum_work_floats.restype = C.c_size_t
    lib.mw_colsum_wide_noalloc.argtypes = [vp, i64, i32, f32, vp, vp]
    lib.mw_colsum_noalloc_max_floats.argtypes = []
    lib.mw_colsum_noalloc_max_floats.restype = sz
    lib.mw_loss_grad.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp, vp]
    lib.mw_loss_scratch_doubles.argtypes = []
    lib.mw_loss_scratch_doubles.restype = sz
    lib.mw_copy_f32.argtypes = [vp, vp, i64, vp]
    lib.mw_probe_operand_stream.argtypes = [i32, i32, i32, i32, vp, vp, vp, i32, vp]
    lib.moonwalk_conv_setup.argtypes = [C.POINTER(vp), C.POINTER(_ConvLayer), i32, C.POINTER(_ConvConfig), vp]
    lib.moonwalk_conv_refresh.argtypes = [vp, vp]
    lib.moonwalk_conv_grad.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.moonwalk_conv_sgd_step.argtypes = [vp, vp, vp, C.c_float, vp, vp]
    lib.backprop_conv_grad.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.moonwalk_conv_grad_layout.argtypes = [vp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    lib.moonwalk_conv_memory_stats.argtypes = [vp, C.POINTER(_ConvMemStats)]
    lib.moonwalk_conv_fetch.argtypes = [vp, i32, i32, vp, sz, C.POINTER(sz)]
    lib.moonwalk_conv_destroy.argtypes = [vp]
    lib.moonwalk_conv_destroy.restype = None
    lib.mw_conv_im2col.argtypes = [vp, i32, i32, i32, i32, i32, i32, i64, i64, vp, vp]
    lib.mw_conv_forward.argtypes = [C.POINTER(_ConvShape), vp, vp, vp, C.c_float, vp, vp, vp]
    lib.mw_conv_input_cotangent.argtypes = [C.POINTER(_ConvShape), vp, vp, vp, vp, vp]
    lib.mw_conv_weight_grad_work_floats.argtypes = [C.POINTER(_ConvShape)]
    lib.mw_conv_weight_grad_work_floats.restype = C.c_size_t
    lib.mw_conv_weight_grad.argtypes = [C.POINTER(_ConvShape), vp, vp, C.c_float, vp, vp, vp, vp]
    lib.mw_conv_col2im.argtypes = [vp, i32, i32, i32, i32, i32, i32, i64, i64, vp, vp]
    _lib = lib
    return lib


def _check(code: int):
    if code != 0:
        raise MoonwalkError(code, load_library().moonwalk_strerror(code).decode())


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("libmoonwalk needs a GPU: there is no CPU path")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return t.data_ptr()


def _f32(t: torch.Tensor) -> torch.Tensor:
    if t.dtype != torch.float32:
        raise ValueError("expected float32")
    return t


@dataclass
class GradResult:
    flat: torch.Tensor                # the grads_out buffer
    dW: List[torch.Tensor]            # views into flat, [d_out][d_in]
    db: List[torch.Tensor]            # views into flat, [d_out]
    loss: torch.Tensor                # 1-element device tensor


class MoonwalkNet:
    """A fixed dense network and batch size bound to a libmoonwalk handle."""

    def __init__(self, Ws: Sequence[torch.Tensor], bs: Sequence[Optional[torch.Tensor]], alphas: Sequence[float],
                 batch: int, reseed_interval: int = 0, loss_scale: float = 1.0,
                 plan: int = PLAN_MOONWALK | PLAN_BACKPROP, fuse: bool = True,
                 frag_capacity_factor: float = 1.0, segment_length: int = 0, debug_keep: bool = False,
                 phase3_parallel_segments: int = 0, phase3_overlap: bool = False, refresh_bf16: bool = False):
        """refresh_bf16: refresh_incremental / sgd_step form the residual I - P W^T in fp32 and round the operands of
        the correction product that is added to P to bfloat16 (mw_config_t.refresh_precision = 1)."""
        _require_gpu()
        self._lib = load_library()
        self._handle = C.c_void_p()
        self.Ws = [_f32(w) for w in Ws]
        self.bs = list(bs)
        self.alphas = [float(a) for a in alphas]
        self.batch = int(batch)
        self.device = self.Ws[0].device
        self.x = None
        self.t = None
        self._held = {}          # device buffers handed to the library, keyed by address
        self.alloc_peak = 0
        self._alloc_live = 0

        def _alloc(nbytes, _ctx):
            try:
                buf = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            except Exception:
                return None
            self._held[buf.data_ptr()] = buf
            self._alloc_live += int(nbytes)
            self.alloc_peak = max(self.alloc_peak, self._alloc_live)
            return buf.data_ptr()

        def _free(ptr, _ctx):
            buf = self._held.pop(ptr, None)
            if buf is not None:
                self._alloc_live -= buf.numel()

        self._alloc_cb, self._free_cb = _ALLOC_FN(_alloc), _FREE_FN(_free)
        n = len(self.Ws)
        layers = (_Layer * n)()
        for i, (w, b, a) in enumerate(zip(self.Ws, self.bs, self.alphas)):
            if w.dim() != 2:
                raise ValueError("W must be [d_out][d_in]")
            layers[i] = _Layer(w.shape[1], w.shape[0], _ptr(w), _ptr(_f32(b)) if b is not None else None, a)
        cfg = _Config(self.batch, int(reseed_interval), float(loss_scale), int(plan), 1 if fuse else 0,
                      float(frag_capacity_factor), self._alloc_cb, self._free_cb, None, int(segment_length), 1 if debug_keep else 0,
                      int(phase3_parallel_segments), 1 if phase3_overlap else 0, 1 if refresh_bf16 else 0)
        with torch.cuda.device(self.device):
            _check(self._lib.moonwalk_setup(C.byref(self._handle), layers, n, C.byref(cfg), _stream()))
        total = C.c_size_t()
        dW_off, db_off = (C.c_size_t * n)(), (C.c_size_t * n)()
        _check(self._lib.moonwalk_grad_layout(self._handle, C.byref(total), dW_off, db_off))
        self.total_floats = int(total.value)
        self.dW_off, self.db_off = list(dW_off), list(db_off)

    @classmethod
    def from_workload(cls, wl, device="cuda:0", **kw) -> "MoonwalkNet":
        dev = torch.device(device)

        def put(a):
            if isinstance(a, torch.Tensor):
                return a.to(device=dev, dtype=torch.float32).contiguous()
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)

        Ws = [put(w) for w in wl.W]
        bs = [put(b) for b in wl.b]
        kw.setdefault("reseed_interval", wl.reseed_interval)
        kw.setdefault("loss_scale", wl.loss_scale)
        net = cls(Ws, bs, wl.alphas, wl.batch, **kw)
        net.x = put(wl.x)
        net.t = put(wl.t)
        return net

    # ------------------------------------------------------------------ gradient steps
    def new_grads(self) -> torch.Tensor:
        return torch.empty(self.total_floats, dtype=torch.float32, device=self.device)

    def _views(self, flat: torch.Tensor, loss: torch.Tensor) -> GradResult:
        dW, db = [], []
        for i, w in enumerate(self.Ws):
            d_out, d_in = w.shape
            dW.append(flat[self.dW_off[i]: self.dW_off[i] + d_out * d_in].view(d_out, d_in))
            db.append(flat[self.db_off[i]: self.db_off[i] + d_out])
        return GradResult(flat, dW, db, loss)

    def _grad(self, fn, x, target, grads_out, loss_out) -> GradResult:
        if self._handle is None:
            raise RuntimeError("handle is closed")
        d0, dL = self.Ws[0].shape[1], self.Ws[-1].shape[0]
        if tuple(x.shape) != (self.batch, d0) or tuple(target.shape) != (self.batch, dL):
            raise ValueError("x must be [B][d_0] and target [B][d_L]")
        flat = grads_out if grads_out is not None else self.new_grads()
        if flat.numel() != self.total_floats:
            raise ValueError("grads_out has the wrong size")
        loss = loss_out if loss_out is not None else torch.empty(1, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(fn(self._handle, _ptr(_f32(x)), _ptr(_f32(target)), _ptr(_f32(flat)), _ptr(loss), _stream()))
        return self._views(flat, loss)

    def moonwalk_grad(self, x, target, grads_out=None, loss_out=None) -> GradResult:
        return self._grad(self._lib.moonwalk_grad, x, target, grads_out, loss_out)

    def backprop_grad(self, x, target, grads_out=None, loss_out=None) -> GradResult:
        return self._grad(self._lib.backprop_grad, x, target, grads_out, loss_out)

    def refresh(self):
        with torch.cuda.device(self.device):
            _check(self._lib.moonwalk_refresh(self._handle, _stream()))

    def refresh_incremental(self, iters: int = 2, residual: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Newton-Schulz refresh of every P_i after a small in-place change of the weights.
        Returns the device float holding the residual measured before the last iteration."""
        with torch.cuda.device(self.device):
            if residual is None:
                residual = torch.empty(1, dtype=torch.float32, device=self.device)
            _check(self._lib.moonwalk_refresh_incremental(self._handle, int(iters), _ptr(residual), _stream()))
        return residual

    def sgd_step(self, x: torch.Tensor, target: torch.Tensor, lr: float, refresh_iters: int = 2,
                 loss_out: Optional[torch.Tensor] = None, residual: Optional[torch.Tensor] = None):
        """One in-place training step: the W and b tensors given at construction are updated by
        this call (W -= lr dW, b -= lr db), then P is refreshed. Returns (loss, residual) device floats."""
        with torch.cuda.device(self.device):
            if loss_out is None:
                loss_out = torch.empty(1, dtype=torch.float32, device=self.device)
            if residual is None:
                residual = torch.empty(1, dtype=torch.float32, device=self.device)
            _check(self._lib.moonwalk_sgd_step(self._handle, _ptr(_f32(x)), _ptr(_f32(target)), float(lr),
                                               int(refresh_iters), _ptr(loss_out), _ptr(residual), _stream()))
        return loss_out, residual

    # ------------------------------------------------------------------ introspection
    def memory_stats(self, check: bool = True) -> dict:
        st = _MemStats()
        code = self._lib.moonwalk_memory_stats(self._handle, C.byref(st))
        out = {name: int(getattr(st, name)) for name, _ in _MemStats._fields_ if name != "reserved"}
        out["status"] = code
        if check:
            _check(code)
        return out

    KCLASSES = ("fwd", "rev", "vijp", "dw", "ew", "phase3")

    def profile_filter(self, kclass: Optional[str]):
        """Run only the launches of one kernel class ("fwd", "rev", "vijp", "dw", "ew", "phase3"); None = all."""
        k = -1 if kclass is None else self.KCLASSES.index(kclass)
        _check(self._lib.moonwalk_profile_filter(self._handle, k))

    def profile_launches(self) -> dict:
        out = {}
        for k, name in enumerate(self.KCLASSES):
            n = C.c_uint64()
            _check(self._lib.moonwalk_profile_launches(self._handle, k, C.byref(n)))
            out[name] = int(n.value)
        return out

    def _fetch(self, layer: int, what: int, dtype) -> np.ndarray:
        n = C.c_size_t()
        _check(self._lib.moonwalk_debug_fetch(self._handle, layer, what, None, 0, C.byref(n)))
        out = np.empty(n.value // np.dtype(dtype).itemsize, dtype=dtype)
        if n.value:
            _check(self._lib.moonwalk_debug_fetch(self._handle, layer, what, out.ctypes.data_as(C.c_void_p),
                                                  out.nbytes, C.byref(n)))
        return out

    def fetch_mask(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_MASK, np.uint64)

    def fetch_fragments(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_FRAG, np.float32)

    def fetch_frag_offsets(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_FRAG_OFFSETS, np.uint32)

    def fetch_frag_base(self, layer: int) -> int:
        return int(self._fetch(layer, FETCH_FRAG_BASE, np.uint64)[0])

    def fetch_h0(self) -> np.ndarray:
        return self._fetch(0, FETCH_H0, np.float32).reshape(self.batch, -1)

    def fetch_P(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_P, np.float32).reshape(self.Ws[layer].shape)

    def fetch_checkpoint(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_CHECKPOINT, np.float32).reshape(self.batch, -1)

    def fetch_z(self, layer: int) -> np.ndarray:
        """Phase-I pre-activations of a layer (needs debug_keep)."""
        return self._fetch(layer, FETCH_Z, np.float32).reshape(self.batch, -1)

    def fetch_h(self, layer: int) -> np.ndarray:
        """Phase-II cotangent at the output of a layer, scaled by loss_scale (needs debug_keep)."""
        return self._fetch(layer, FETCH_H, np.float32).reshape(self.batch, -1)

    def fetch_h_forward(self, layer: int) -> np.ndarray:
        """Phase-III cotangent at the output of a layer, scaled by loss_scale (needs debug_keep)."""
        return self._fetch(layer, FETCH_H_FORWARD, np.float32).reshape(self.batch, -1)

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            self._lib.moonwalk_destroy(self._handle)
        self._handle = None
        self._held.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


CONV_KERNELS_AUTO, CONV_KERNELS_PATCH_MATRIX = 0, 1
CONV_H0_FULL, CONV_H0_AS_READ = 0, 1
CONV_SUBMERSIVE, CONV_FRAGMENTAL_1D = 0, 1


class ConvMoonwalkNet:
    """A chain of submersive 2-D convolutional layers (channels-last) behind moonwalk_conv_*.

    ws: kernels [k][k][C_in][C_out]; bs: biases or None; one stride and padding for all layers.
    kernels: CONV_KERNELS_AUTO (patch matrix gathered inside the products where the channel counts
    allow it) or CONV_KERNELS_PATCH_MATRIX (always through the patch buffer).
    input_cotangent: CONV_H0_FULL (h_0 for every input element) or CONV_H0_AS_READ (only the entries
    the first layer's vijp reads; the first layer's reverse product is skipped).
    max_images_per_launch: the gathered kernels take the batch in launches of at most this many images
    (0 = bounded by the 2 GiB operand limit only).
    kind = CONV_FRAGMENTAL_1D: length-preserving 1-D layers with fragmental checkpointing; ws are
    [k][C_in][C_out], height must be 1, stride 1, pad (k - 1) / 2, block = positions per block."""

    def __init__(self, ws: Sequence[torch.Tensor], bs: Sequence[Optional[torch.Tensor]], alphas: Sequence[float],
                 batch: int, height: int, width: int, stride: int, pad: int, reseed_interval: int = 0,
                 loss_scale: float = 1.0, plan: int = PLAN_MOONWALK | PLAN_BACKPROP, patch_bytes: int = 0,
                 kernels: int = 0, input_cotangent: int = 0, kind: int = 0, block: int = 0,
                 max_images_per_launch: int = 0):
        _require_gpu()
        self._lib = load_library()
        self._handle = C.c_void_p()
        self.ws = [_f32(w) for w in ws]
        self.bs = list(bs)
        self.alphas = [float(a) for a in alphas]
        self.batch, self.height, self.width = int(batch), int(height), int(width)
        self.stride, self.pad = int(stride), int(pad)
        self.device = self.ws[0].device
        self.x = None
        self.t = None
        self._held = {}
        self.alloc_peak = 0
        self._alloc_live = 0

        def _alloc(nbytes, _ctx):
            try:
                buf = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            except Exception:
                return None
            self._held[buf.data_ptr()] = buf
            self._alloc_live += int(nbytes)
            self.alloc_peak = max(self.alloc_peak, self._alloc_live)
            return buf.data_ptr()

        def _free(ptr, _ctx):
            buf = self._held.pop(ptr, None)
            if buf is not None:
                self._alloc_live -= buf.numel()

        self._alloc_cb, self._free_cb = _ALLOC_FN(_alloc), _FREE_FN(_free)
        n = len(self.ws)
        layers = (_ConvLayer * n)()
        for i, (w, b, a) in enumerate(zip(self.ws, self.bs, self.alphas)):
            if kind == CONV_FRAGMENTAL_1D:
                if w.dim() != 3:
                    raise ValueError("kernels of 1-D layers must be [k][C_in][C_out]")
                layers[i] = _ConvLayer(w.shape[1], w.shape[2], w.shape[0], self.stride, self.pad, _ptr(w),
                                       _ptr(_f32(b)) if b is not None else None, a, int(kind), int(block))
                continue
            if w.dim() != 4 or w.shape[0] != w.shape[1]:
                raise ValueError("kernels must be [k][k][C_in][C_out]")
            layers[i] = _ConvLayer(w.shape[2], w.shape[3], w.shape[0], self.stride, self.pad, _ptr(w),
                                   _ptr(_f32(b)) if b is not None else None, a, int(kind), int(block))
        cfg = _ConvConfig(self.batch, self.height, self.width, int(reseed_interval), float(loss_scale), int(plan),
                          int(kernels), int(input_cotangent), int(max_images_per_launch), int(patch_bytes), self._alloc_cb,
                          self._free_cb, None)
        with torch.cuda.device(self.device):
            _check(self._lib.moonwalk_conv_setup(C.byref(self._handle), layers, n, C.byref(cfg), _stream()))
        total = C.c_size_t()
        dW_off, db_off = (C.c_size_t * n)(), (C.c_size_t * n)()
        _check(self._lib.moonwalk_conv_grad_layout(self._handle, C.byref(total), dW_off, db_off))
        self.total_floats = int(total.value)
        self.dW_off, self.db_off = list(dW_off), list(db_off)

    @classmethod
    def from_workload(cls, wl, device="cuda:0", **kw) -> "ConvMoonwalkNet":
        dev = torch.device(device)

        def put(a):
            if isinstance(a, torch.Tensor):
                return a.to(device=dev, dtype=torch.float32).contiguous()
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)

        if hasattr(wl, "block"):   # a 1-D network with fragmental checkpointing: [S][N][C] is a one-row image
            net = cls([put(w) for w in wl.w], [put(b) for b in wl.b], wl.alphas, wl.batch, 1, wl.length, 1, (wl.k - 1) // 2,
                      kind=CONV_FRAGMENTAL_1D, block=wl.block, **kw)
        else:
            net = cls([put(w) for w in wl.w], [put(b) for b in wl.b], wl.alphas, wl.batch, wl.side, wl.side, wl.s, wl.p, **kw)
        net.x = put(wl.x)
        net.t = put(wl.t)
        return net

    def new_grads(self) -> torch.Tensor:
        return torch.empty(self.total_floats, dtype=torch.float32, device=self.device)

    def _grad(self, fn, x, target, grads_out, loss_out) -> GradResult:
        flat = grads_out if grads_out is not None else self.new_grads()
        loss = loss_out if loss_out is not None else torch.empty(1, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(fn(self._handle, _ptr(_f32(x)), _ptr(_f32(target)), _ptr(_f32(flat)), _ptr(loss), _stream()))
        dW, db = [], []
        for i, w in enumerate(self.ws):
            dW.append(flat[self.dW_off[i]: self.dW_off[i] + w.numel()].view(w.shape))
            db.append(flat[self.db_off[i]: self.db_off[i] + w.shape[-1]])
        return GradResult(flat, dW, db, loss)

    def moonwalk_grad(self, x, target, grads_out=None, loss_out=None) -> GradResult:
        return self._grad(self._lib.moonwalk_conv_grad, x, target, grads_out, loss_out)

    def backprop_grad(self, x, target, grads_out=None, loss_out=None) -> GradResult:
        return self._grad(self._lib.backprop_conv_grad, x, target, grads_out, loss_out)

    def refresh(self):
        with torch.cuda.device(self.device):
            _check(self._lib.moonwalk_conv_refresh(self._handle, _stream()))

    def sgd_step(self, x, target, lr: float, loss_out=None) -> torch.Tensor:
        """One training step in place: self.ws / self.bs are updated; returns the loss before the update."""
        loss = loss_out if loss_out is not None else torch.empty(1, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self._lib.moonwalk_conv_sgd_step(self._handle, _ptr(_f32(x)), _ptr(_f32(target)), float(lr), _ptr(loss),
                                                    _stream()))
        return loss

    def memory_stats(self, check: bool = True) -> dict:
        st = _ConvMemStats()
        code = self._lib.moonwalk_conv_memory_stats(self._handle, C.byref(st))
        out = {name: int(getattr(st, name)) for name, _ in _ConvMemStats._fields_}
        out["status"] = code
        if check:
            _check(code)
        return out

    def _fetch(self, layer: int, what: int, dtype) -> np.ndarray:
        n = C.c_size_t()
        _check(self._lib.moonwalk_conv_fetch(self._handle, layer, what, None, 0, C.byref(n)))
        out = np.empty(n.value // np.dtype(dtype).itemsize, dtype=dtype)
        if n.value:
            _check(self._lib.moonwalk_conv_fetch(self._handle, layer, what, out.ctypes.data_as(C.c_void_p), out.nbytes,
                                                 C.byref(n)))
        return out

    def fetch_mask(self, layer: int) -> np.ndarray:
        return self._fetch(layer, FETCH_MASK, np.uint64)

    def fetch_h0(self) -> np.ndarray:
        return self._fetch(0, FETCH_H0, np.float32)

    def fetch_checkpoint(self, layer: int) -> np.ndarray:
        """The cotangent kept at the output of `layer`, as layer + 1 reads it: [B][H'][W'][C_out] of layer + 1."""
        return self._fetch(layer, FETCH_CHECKPOINT, np.float32)

    def fetch_fragments(self, layer: int) -> np.ndarray:
        """Fragmental layers: the stored positions of ct_z, [B N / block][k - 1][C_out] flattened."""
        return self._fetch(layer, FETCH_FRAG, np.float32)

    def fetch_tap_inverse(self, layer: int) -> np.ndarray:
        c = self.ws[layer].shape[-1]
        return self._fetch(layer, FETCH_P, np.float32).reshape(c, c)

    def close(self):
        if getattr(self, "_handle", None) is not None and self._handle.value:
            self._lib.moonwalk_conv_destroy(self._handle)
        self._handle = None
        self._held.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def conv_im2col(x: torch.Tensor, k: int, stride: int, pad: int, row0: int = 0, n_rows: Optional[int] = None) -> torch.Tensor:
    """Patch matrix rows [row0, row0 + n_rows) of the channels-last tensor x [B][H][W][C]."""
    _require_gpu()
    B, H, W, Cc = x.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    if n_rows is None:
        n_rows = B * Ho * Wo - row0
    out = torch.empty(n_rows, k * k * Cc, dtype=torch.float32, device=x.device)
    _check(load_library().mw_conv_im2col(_ptr(_f32(x)), H, W, Cc, k, stride, pad, row0, n_rows, _ptr(out), _stream()))
    return out


def conv_col2im(dpatches: torch.Tensor, shape, k: int, stride: int, pad: int) -> torch.Tensor:
    """Transpose of conv_im2col for all images of a tensor of the given [B][H][W][C] shape."""
    _require_gpu()
    B, H, W, Cc = shape
    out = torch.empty(B, H, W, Cc, dtype=torch.float32, device=dpatches.device)
    _check(load_library().mw_conv_col2im(_ptr(_f32(dpatches)), H, W, Cc, k, stride, pad, 0, B, _ptr(out), _stream()))
    return out


def _conv_shape(x_shape, w: torch.Tensor, stride: int, pad_h: int, pad_w: int) -> "_ConvShape":
    B, H, W, Ci = x_shape
    kh, kw, ci, co = w.shape
    if ci != Ci:
        raise ValueError("kernel and input channel counts differ")
    return _ConvShape(B, H, W, Ci, co, kh, kw, int(stride), int(pad_h), int(pad_w))


def conv_forward(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], stride: int, pad_h: int, pad_w: int,
                 alpha: float = 1.0, want_mask: bool = False):
    """act(conv(x, w) + b) by the product that gathers the patch matrix; x [B][H][W][C_in], w [kh][kw][C_in][C_out].
    Returns xout, or (xout, mask words) with want_mask."""
    _require_gpu()
    sh = _conv_shape(x.shape, w, stride, pad_h, pad_w)
    Ho, Wo = (sh.height + 2 * sh.pad_h - sh.kh) // sh.stride + 1, (sh.width + 2 * sh.pad_w - sh.kw) // sh.stride + 1
    out = torch.empty(sh.batch, Ho, Wo, sh.channels_out, dtype=torch.float32, device=x.device)
    mask = torch.zeros((out.numel() + 63) // 64, dtype=torch.int64, device=x.device) if want_mask else None
    _check(load_library().mw_conv_forward(C.byref(sh), _ptr(_f32(x)), _ptr(_f32(w)), _ptr(_f32(b)) if b is not None else None,
                                          float(alpha), _ptr(out), _ptr(mask) if want_mask else None, _stream()))
    return (out, mask) if want_mask else out


def conv_input_cotangent(ctz: torch.Tensor, w: torch.Tensor, in_hw, stride: int, pad_h: int, pad_w: int) -> torch.Tensor:
    """vjp of the convolution w.r.t. its input, applied to ctz [B][H'][W'][C_out]; returns h [B][H][W][C_in]."""
    _require_gpu()
    B = ctz.shape[0]
    sh = _conv_shape((B, in_hw[0], in_hw[1], w.shape[2]), w, stride, pad_h, pad_w)
    h = torch.empty(B, in_hw[0], in_hw[1], w.shape[2], dtype=torch.float32, device=ctz.device)
    work = torch.empty(w.numel(), dtype=torch.float32, device=ctz.device)
    _check(load_library().mw_conv_input_cotangent(C.byref(sh), _ptr(_f32(ctz)), _ptr(_f32(w)), _ptr(h), _ptr(work), _stream()))
    return h


def conv_weight_grad(x: torch.Tensor, ctz: torch.Tensor, kh: int, kw: int, stride: int, pad_h: int, pad_w: int, scale: float = 1.0):
    """(dw [kh][kw][C_in][C_out], db [C_out]) = scale * the parameter vjp of the convolution."""
    _require_gpu()
    B, H, W, Ci = x.shape
    Co = ctz.shape[3]
    sh = _ConvShape(B, H, W, Ci, Co, int(kh), int(kw), int(stride), int(pad_h), int(pad_w))
    lib = load_library()
    n_work = int(lib.mw_conv_weight_grad_work_floats(C.byref(sh)))
    if n_work == 0:
        raise MoonwalkError(-1, "shape not supported by the gathered weight-gradient kernel")
    work = torch.empty(n_work, dtype=torch.float32, device=x.device)
    dw = torch.empty(kh, kw, Ci, Co, dtype=torch.float32, device=x.device)
    db = torch.empty(Co, dtype=torch.float32, device=x.device)
    _check(lib.mw_conv_weight_grad(C.byref(sh), _ptr(_f32(x)), _ptr(_f32(ctz)), float(scale), _ptr(dw), _ptr(db), _ptr(work), _stream()))
    return dw, db


# ---------------------------------------------------------------------- kernel-level entries

def gemm_f32(op: int, A: torch.Tensor, B: torch.Tensor, C_out: Optional[torch.Tensor] = None,
             alpha: float = 1.0, beta: float = 0.0, tile: int = TILE_AUTO) -> torch.Tensor:
    """op NT: A[M][K], B[N][K]; NN: A[M][K], B[K][N]; TN: A[K][M], B[K][N]. Returns C[M][N]."""
    _require_gpu()
    lib = load_library()
    if op == GEMM_NT:
        (M, K), (N, K2) = A.shape, B.shape
    elif op == GEMM_NN:
        (M, K), (K2, N) = A.shape, B.shape
    elif op == GEMM_TN:
        (K, M), (K2, N) = A.shape, B.shape
    else:
        raise ValueError("bad op")
    if K != K2:
        raise ValueError("inner dimensions differ")
    if C_out is None:
        C_out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    if tuple(C_out.shape) != (M, N):
        raise ValueError("C has the wrong shape")
    for t in (A, B, C_out):          # row-strided views are allowed: the row stride becomes the leading dimension
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("expected 2-D float32 CUDA tensors with unit column stride")
    _check(lib.mw_gemm_f32(op, tile, M, N, K, alpha, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), beta,
                           C_out.data_ptr(), C_out.stride(0), _stream()))
    return C_out


def _n_words(n: int) -> int:
    return (n + 63) // 64


def bias_act_mask(z: torch.Tensor, bias: Optional[torch.Tensor], alpha: float):
    _require_gpu()
    rows, d = z.shape
    x = torch.empty_like(z)
    mask = torch.zeros(max(_n_words(rows * d), 1), dtype=torch.int64, device=z.device)
    _check(load_library().mw_bias_act_mask(_ptr(_f32(z)), _ptr(bias), rows, d, alpha, _ptr(x), _ptr(mask), _stream()))
    return x, mask


def rev_scale(h: torch.Tensor, mask: torch.Tensor, alpha: float) -> torch.Tensor:
    _require_gpu()
    out = torch.empty_like(h)
    _check(load_library().mw_rev_scale(_ptr(_f32(h)), _ptr(mask), h.numel(), alpha, _ptr(out), _stream()))
    return out


def frag_offsets(mask: torch.Tensor, n: int) -> torch.Tensor:
    _require_gpu()
    lib = load_library()
    off = torch.empty(_n_words(n) + 1, dtype=torch.int32, device=mask.device)
    work = torch.empty(int(lib.mw_frag_offsets_work_words(n)), dtype=torch.int32, device=mask.device)
    _check(lib.mw_frag_offsets(_ptr(mask), n, _ptr(off), _ptr(work), _stream()))
    return off


def frag_compact(h: torch.Tensor, mask: torch.Tensor, offsets: torch.Tensor, capacity: Optional[int] = None):
    _require_gpu()
    n = h.numel()
    cap = n if capacity is None else int(capacity)
    frag = torch.zeros(max(cap, 1), dtype=torch.float32, device=h.device)
    flag = torch.zeros(1, dtype=torch.int32, device=h.device)
    _check(load_library().mw_frag_compact(_ptr(_f32(h)), _ptr(mask), _ptr(offsets), n, _ptr(frag), cap, _ptr(flag),
                                          _stream()))
    return frag, flag


def vijp_epilogue(z: torch.Tensor, ct_z: torch.Tensor, alpha: float, mask=None, offsets=None, frag=None):
    """Returns (x, h_y); ct_z is modified in place for alpha == 0."""
    _require_gpu()
    rows, d = z.shape
    x, h_y = torch.empty_like(z), torch.empty_like(z)
    _check(load_library().mw_vijp_epilogue(_ptr(_f32(z)), _ptr(_f32(ct_z)), rows, d, alpha, _ptr(mask), _ptr(offsets),
                                           _ptr(frag), _ptr(x), _ptr(h_y), _stream()))
    return x, h_y


def colsum(a: torch.Tensor, scale: float = 1.0) -> torch.Tensor:
    _require_gpu()
    rows, d = a.shape
    out = torch.empty(d, dtype=torch.float32, device=a.device)
    _check(load_library().mw_colsum(_ptr(_f32(a)), rows, d, scale, _ptr(out), _stream()))
    return out


def colsum_wide(a: torch.Tensor, scale: float = 1.0) -> torch.Tensor:
    """Column sums of a tall matrix, the rows cut into ranges summed side by side (mw_colsum_wide)."""
    _require_gpu()
    lib = load_library()
    rows, d = a.shape
    out = torch.empty(d, dtype=torch.float32, device=a.device)
    work = torch.empty(int(lib.mw_colsum_work_floats(d)), dtype=torch.float32, device=a.device)
    _check(lib.mw_colsum_wide(_ptr(_f32(a)), rows, d, scale, _ptr(out), _ptr(work), _stream()))
    return out


def colsum_wide_noalloc(a: torch.Tensor, out: torch.Tensor, scale: float = 1.0) -> torch.Tensor:
    """mw_colsum_wide_noalloc: the same sums into the caller's `out`, the partial sums in the library's own
    fixed array; neither the library nor this wrapper allocates. Raises MoonwalkError (ERR_TOO_LARGE) when
    the partial sums would not fit."""
    _require_gpu()
    rows, d = a.shape
    if out.numel() != d:
        raise ValueError("out must have one element per column")
    _check(load_library().mw_colsum_wide_noalloc(_ptr(_f32(a)), rows, d, scale, _ptr(_f32(out)), _stream()))
    return out


def loss_grad(xL: torch.Tensor, t: torch.Tensor, scale: float = 1.0):
    _require_gpu()
    lib = load_library()
    rows, d = xL.shape
    hL = torch.empty_like(xL)
    loss = torch.empty(1, dtype=torch.float32, device=xL.device)
    scratch = torch.empty(int(lib.mw_loss_scratch_doubles()), dtype=torch.float64, device=xL.device)
    _check(lib.mw_loss_grad(_ptr(_f32(xL)), _ptr(_f32(t)), rows, d, scale, _ptr(hL), _ptr(loss), _ptr(scratch), _stream()))
    return hL, loss


def probe_operand_stream(A: torch.Tensor, B: torch.Tensor, tile: int, sink: Optional[torch.Tensor] = None,
                         repeats: int = 1):
    """Load-only model of the tiled product A[M][K] B[N][K]^T (see mw_probe_operand_stream)."""
    _require_gpu()
    M, K = A.shape
    N = B.shape[0]
    if sink is None:
        sink = torch.empty((M // tile) * (N // tile) * 256, dtype=torch.float32, device=A.device)
    _check(load_library().mw_probe_operand_stream(M, N, K, tile, _ptr(_f32(A)), _ptr(_f32(B)), _ptr(sink), repeats,
                                                  _stream()))
    return sink


def copy_f32(src: torch.Tensor, dst: torch.Tensor):
    _require_gpu()
    _check(load_library().mw_copy_f32(_ptr(_f32(src)), _ptr(_f32(dst)), src.numel(), _stream()))
    return dst
