"""Thin ctypes binding of libalexnet_hip.so (include/alexnet.h).

Argument marshalling only: every step of the training path runs inside the
HIP library.  PyTorch is used to own device memory and streams.  Importing
this module fails loudly when the library has not been built
(python -m paper_1412_2302_amd.build); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libalexnet_hip.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1412_2302_amd.build`")
_lib = C.CDLL(LIB_PATH)

OK, EINVAL, ESHAPE, EALIGN, ELABEL, EHIP, ENOTIMPL, ENOMEM = 0, -1, -2, -3, -4, -5, -6, -7

T_INPUT, T_CONV_ACT, T_LRN, T_POOL, T_ARGMAX, T_FC_ACT, T_CROP_X, T_CROP_Y, T_FLIP, T_DLOGITS, T_CONV_DACT = range(11)
_INT_KINDS = {T_ARGMAX, T_CROP_X, T_CROP_Y, T_FLIP}


class ConvCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("cout", "k", "stride", "pad", "groups", "lrn", "pool")]


class Config(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("in_c", C.c_int32), ("crop_h", C.c_int32), ("crop_w", C.c_int32),
        ("raw_h", C.c_int32), ("raw_w", C.c_int32),
        ("conv", ConvCfg * 5), ("fc", C.c_int32 * 3),
        ("lrn_n", C.c_int32), ("lrn_k", C.c_float), ("lrn_alpha", C.c_float), ("lrn_beta", C.c_float),
        ("dropout_p", C.c_float), ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float),
        ("precision", C.c_int32), ("flags", C.c_int32), ("seed", C.c_uint64),
    ]


_vp, _i32, _u64, _sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t
_SIGS = {
    "alexnet_query": [C.POINTER(Config), C.POINTER(_sz), C.POINTER(_sz)],
    "alexnet_create": [C.POINTER(Config), _vp, _vp, _vp, _sz, _vp, C.POINTER(_vp)],
    "alexnet_preprocess": [_vp, _vp, _vp, _u64, _i32, _vp],
    "alexnet_set_input": [_vp, _vp, _i32, _vp],
    "alexnet_train_step": [_vp, _i32, _vp, _u64, _vp, _vp],
    "alexnet_forward_backward": [_vp, _i32, _vp, _u64, _vp, _vp],
    "alexnet_apply_update": [_vp, _vp],
    "alexnet_forward": [_vp, _vp, _vp, _vp],
    "alexnet_average_replicas": [_vp, _vp, _vp],
    "alexnet_average_gradients_update": [_vp, _vp, _vp],
    "alexnet_preprocess_center": [_vp, _vp, _vp, _i32, _vp],
    "alexnet_loader_create": [_vp, _vp, _vp, _vp, C.c_int64, _i32, _vp, _vp, _vp, _vp, _vp, C.POINTER(_vp)],
    "alexnet_loader_stage": [_vp, _u64, _vp, _vp, _vp, C.POINTER(_vp)],
    "alexnet_loader_done": [_vp, _u64, _vp],
    "alexnet_loader_destroy": [_vp],
    "alexnet_validate": [_vp, _i32, _vp, C.POINTER(_i32), _i32, _vp, _vp],
    "alexnet_set_params": [_vp, _vp, _vp],
    "alexnet_get_params": [_vp, _vp, _vp],
    "alexnet_set_momentum": [_vp, _vp, _vp],
    "alexnet_get_momentum": [_vp, _vp, _vp],
    "alexnet_get_grads": [_vp, _vp, _vp],
    "alexnet_tensor_elems": [_vp, _i32, _i32, C.POINTER(_sz)],
    "alexnet_get_tensor": [_vp, _i32, _i32, _vp, _vp],
    "alexnet_check": [_vp, _vp],
    "alexnet_conv_forward": [_vp, _i32, _vp, _vp, _vp, _i32, _vp, _vp],
    "alexnet_conv_backward_data": [_vp, _i32, _vp, _vp, _vp, _vp],
    "alexnet_conv_backward_weight": [_vp, _i32, _vp, _vp, _vp, _vp, _vp],
    "alexnet_nchw_to_nhwc": [_vp, _vp, _i32, _i32, _i32, _i32, _vp],
    "alexnet_nhwc_to_nchw": [_vp, _vp, _i32, _i32, _i32, _i32, _vp],
    "alexnet_pack_conv_weight": [_vp, _i32, _vp, _vp, _vp, _vp],
    "alexnet_unpack_conv_weight": [_vp, _i32, _vp, _vp, _vp],
    "alexnet_conv_forward_nhwc": [_vp, _i32, _vp, _vp, _vp, _i32, _vp, _vp],
    "alexnet_conv_backward_data_nhwc": [_vp, _i32, _vp, _vp, _vp, _vp, _vp],
    "alexnet_conv_backward_weight_nhwc": [_vp, _i32, _vp, _vp, _vp, _vp, _vp],
}


class ProfEntry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("calls", C.c_int32), ("total_ms", C.c_float),
                ("flops", C.c_double), ("bytes", C.c_double)]


_SIGS.update({
    "alexnet_lrn_forward": [_vp, _i32, _vp, _vp, _vp],
    "alexnet_lrn_backward": [_vp, _i32, _vp, _vp, _i32, _vp, _vp],
    "alexnet_pool_forward": [_vp, _i32, _vp, _vp, _vp, _vp],
    "alexnet_pool_backward": [_vp, _i32, _vp, _vp, _i32, _vp, _vp],
    "alexnet_lrn_pool_forward": [_vp, _i32, _vp, _vp, _vp, _vp],
    "alexnet_pool_lrn_backward": [_vp, _i32, _vp, _vp, _i32, _vp, _vp, _vp],
    "alexnet_fc_forward": [_vp, _i32, _vp, _vp, _vp, _i32, _vp, _vp],
    "alexnet_fc_backward": [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "alexnet_softmax_xent": [_vp, _vp, _vp, _vp, _vp, _vp],
    "alexnet_softmax_xent_static": [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp],
})
_SIGS["alexnet_profile_begin"] = []
_SIGS["alexnet_profile_end"] = [C.POINTER(ProfEntry), _i32, C.POINTER(_i32)]
for _name, _args in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = C.c_int
_lib.alexnet_destroy.argtypes = [_vp]
_lib.alexnet_destroy.restype = None
_lib.alexnet_last_error.restype = C.c_char_p
_lib.alexnet_version.restype = C.c_char_p
EXPORTS = sorted(list(_SIGS) + ["alexnet_destroy", "alexnet_last_error", "alexnet_version"])


class AlexNetError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libalexnet_hip error {code}: {msg}")
        self.code = code


def last_error() -> str:
    return (_lib.alexnet_last_error() or b"").decode()


def version() -> str:
    return _lib.alexnet_version().decode()


def profile_begin():
    _check(_lib.alexnet_profile_begin())


def profile_end(cap: int = 256):
    """Returns [{name, calls, total_ms, flops, bytes}] for the kernels launched since profile_begin."""
    buf = (ProfEntry * cap)()
    n = _i32()
    _check(_lib.alexnet_profile_end(buf, cap, C.byref(n)))
    return [dict(name=buf[i].name.decode(), calls=buf[i].calls, total_ms=buf[i].total_ms, flops=buf[i].flops,
                 bytes=buf[i].bytes) for i in range(min(n.value, cap))]


def _check(rc: int):
    if rc != OK:
        raise AlexNetError(rc, last_error())


FLAG_DIRECT_CONV = 1


def make_config(workload: dict, batch: int, seed: int = 0, precision: int = 0, flags: int = 0) -> Config:
    cfg = Config()
    cfg.batch = batch
    cfg.in_c = workload["in_c"]
    cfg.crop_h = cfg.crop_w = workload["crop"]
    cfg.raw_h = cfg.raw_w = workload["raw"]
    for i, (co, k, st, pd, g, l, p) in enumerate(workload["conv"]):
        cfg.conv[i] = ConvCfg(co, k, st, pd, g, l, p)
    for j, f in enumerate(workload["fc"]):
        cfg.fc[j] = f
    n, k, a, b = workload["lrn"]
    cfg.lrn_n, cfg.lrn_k, cfg.lrn_alpha, cfg.lrn_beta = n, k, a, b
    cfg.dropout_p, cfg.lr = workload["dropout_p"], workload["lr"]
    cfg.momentum, cfg.weight_decay = workload["momentum"], workload["weight_decay"]
    cfg.precision, cfg.flags, cfg.seed = precision, flags, seed
    return cfg


def query(cfg: Config) -> Tuple[int, int]:
    n, w = _sz(), _sz()
    _check(_lib.alexnet_query(C.byref(cfg), C.byref(n), C.byref(w)))
    return n.value, w.value


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else _vp(t.data_ptr())


def _need(t, dtype, numel: int, what: str) -> torch.Tensor:
    """The library takes bare device pointers: a tensor of the wrong kind, place or size would be read past its
    end on the GPU, so it is refused here."""
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{what}: expected a torch.Tensor, got {type(t).__name__}")
    if not t.is_cuda:
        raise ValueError(f"{what}: expected a device tensor, got one on {t.device}")
    if t.dtype != dtype:
        raise ValueError(f"{what}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: expected a contiguous tensor")
    if t.numel() < numel:
        raise ValueError(f"{what}: expected at least {numel} elements, got {t.numel()}")
    return t


def _stream(stream: Optional[torch.cuda.Stream]):
    s = stream if stream is not None else torch.cuda.current_stream()
    return _vp(s.cuda_stream)


def _dev(a, dtype=None) -> torch.Tensor:
    if isinstance(a, torch.Tensor):
        t = a.to("cuda")
    else:
        t = torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
    if dtype is not None:
        t = t.to(dtype)
    return t.contiguous()


class AlexNet:
    """One replica: owns parameter, momentum and workspace tensors on cuda:0."""

    def __init__(self, workload: dict, batch: int, seed: int = 0, precision: int = 0, flags: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libalexnet_hip needs a GPU; there is no CPU path")
        self.workload, self.batch = workload, batch
        self.cfg = make_config(workload, batch, seed, precision, flags)
        self.n_params, self.ws_bytes = query(self.cfg)
        dev = torch.device("cuda", 0)
        self.params = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.momentum = torch.zeros(self.n_params, dtype=torch.float32, device=dev)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        h = _vp()
        _check(_lib.alexnet_create(C.byref(self.cfg), _ptr(self.params), _ptr(self.momentum), _ptr(self.workspace),
                                   self.ws_bytes, _stream(None), C.byref(h)))
        self._h = h
        self.shapes = self._param_shapes()

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:  # _lib is gone at interpreter shutdown
            _lib.alexnet_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # ---- bookkeeping of the canonical flat vector (marshalling only) ----
    def _param_shapes(self) -> Dict[str, Tuple[int, ...]]:
        wl = self.workload
        c, h = wl["in_c"], wl["crop"]
        ws, bs = {}, {}
        for i, (co, k, st, pd, g, l, p) in enumerate(wl["conv"]):
            ws[f"conv{i+1}.w"] = (co, c // g, k, k)
            bs[f"conv{i+1}.b"] = (co,)
            h = (h + 2 * pd - k) // st + 1
            if p:
                h = (h - 3) // 2 + 1
            c = co
        fin = c * h * h
        for j, fo in enumerate(wl["fc"]):
            ws[f"fc{6+j}.w"] = (fo, fin)
            bs[f"fc{6+j}.b"] = (fo,)
            fin = fo
        ws.update(bs)
        total = sum(int(np.prod(s)) for s in ws.values())
        assert total == self.n_params, (total, self.n_params)
        return ws

    def flatten(self, d: Dict[str, np.ndarray]) -> np.ndarray:
        return np.concatenate([np.asarray(d[k], np.float32).ravel() for k in self.shapes])

    def unflatten(self, flat: np.ndarray) -> Dict[str, np.ndarray]:
        out, o = {}, 0
        for k, s in self.shapes.items():
            n = int(np.prod(s))
            out[k] = flat[o:o + n].reshape(s)
            o += n
        return out

    # ---- parameters ----
    def _set(self, fn, d):
        flat = _dev(self.flatten(d) if isinstance(d, dict) else d, torch.float32)
        assert flat.numel() == self.n_params
        _check(fn(self._h, _ptr(flat), _stream(None)))
        torch.cuda.current_stream().synchronize()

    def _get(self, fn) -> Dict[str, np.ndarray]:
        flat = torch.empty(self.n_params, dtype=torch.float32, device="cuda")
        _check(fn(self._h, _ptr(flat), _stream(None)))
        return self.unflatten(flat.cpu().numpy())

    def set_params(self, d): self._set(_lib.alexnet_set_params, d)
    def set_momentum(self, d): self._set(_lib.alexnet_set_momentum, d)
    def get_params(self): return self._get(_lib.alexnet_get_params)
    def get_momentum(self): return self._get(_lib.alexnet_get_momentum)
    def get_grads(self): return self._get(_lib.alexnet_get_grads)

    # ---- the hot path ----
    def _raw_elems(self) -> int:
        return self.workload["in_c"] * self.workload["raw"] * self.workload["raw"]

    def _input_elems(self) -> int:
        return self.batch * self.workload["in_c"] * self.workload["crop"] * self.workload["crop"]

    def preprocess(self, raw_u8: torch.Tensor, mean: torch.Tensor, step: int, slot: int, stream=None):
        _need(raw_u8, torch.uint8, self.batch * self._raw_elems(), "preprocess: stored pictures")
        _need(mean, torch.float32, self._raw_elems(), "preprocess: mean image")
        _check(_lib.alexnet_preprocess(self._h, _ptr(raw_u8), _ptr(mean), step, slot, _stream(stream)))

    def preprocess_center(self, raw_u8: torch.Tensor, mean: torch.Tensor, slot: int, stream=None):
        _need(raw_u8, torch.uint8, self.batch * self._raw_elems(), "preprocess_center: stored pictures")
        _need(mean, torch.float32, self._raw_elems(), "preprocess_center: mean image")
        _check(_lib.alexnet_preprocess_center(self._h, _ptr(raw_u8), _ptr(mean), slot, _stream(stream)))

    def validate(self, labels: torch.Tensor, ks, counts: torch.Tensor, slot: int = 0, stream=None):
        """counts (int32, device, one per k) += pictures of input slot `slot` whose label is in the top k."""
        _need(labels, torch.int32, self.batch, "validate: labels")
        _need(counts, torch.int32, len(ks), "validate: counts")
        arr = (_i32 * len(ks))(*ks)
        _check(_lib.alexnet_validate(self._h, slot, _ptr(labels), arr, len(ks), _ptr(counts), _stream(stream)))

    def set_input(self, x_nchw: torch.Tensor, slot: int = 0, stream=None):
        _need(x_nchw, torch.float32, self._input_elems(), "set_input: input")
        _check(_lib.alexnet_set_input(self._h, _ptr(x_nchw), slot, _stream(stream)))

    def train_step(self, labels: torch.Tensor, step: int, slot: int = 0, stream=None) -> torch.Tensor:
        _need(labels, torch.int32, self.batch, "train_step: labels")
        _check(_lib.alexnet_train_step(self._h, slot, _ptr(labels), step, _ptr(self.loss), _stream(stream)))
        return self.loss

    def forward_backward(self, labels: torch.Tensor, step: int, slot: int = 0, stream=None) -> torch.Tensor:
        _need(labels, torch.int32, self.batch, "forward_backward: labels")
        _check(_lib.alexnet_forward_backward(self._h, slot, _ptr(labels), step, _ptr(self.loss), _stream(stream)))
        return self.loss

    def apply_update(self, stream=None):
        _check(_lib.alexnet_apply_update(self._h, _stream(stream)))

    def forward(self, x_nchw: torch.Tensor, stream=None) -> torch.Tensor:
        _need(x_nchw, torch.float32, self._input_elems(), "forward: input")
        probs = torch.empty(self.batch, self.workload["fc"][-1], dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_forward(self._h, _ptr(x_nchw), _ptr(probs), _stream(stream)))
        return probs

    def check(self, stream=None):
        _check(_lib.alexnet_check(self._h, _stream(stream)))

    def tensor(self, kind: int, layer: int) -> np.ndarray:
        n = _sz()
        _check(_lib.alexnet_tensor_elems(self._h, kind, layer, C.byref(n)))
        out = torch.empty(n.value, dtype=torch.int32 if kind in _INT_KINDS else torch.float32, device="cuda")
        _check(_lib.alexnet_get_tensor(self._h, kind, layer, _ptr(out), _stream(None)))
        return out.cpu().numpy()

    # ---- single operators on canonical tensors ----
    def conv_forward(self, layer, x, w, b, relu=False):
        xs, wt = _dev(x, torch.float32), _dev(w, torch.float32)
        bt = None if b is None else _dev(b, torch.float32)
        n = _sz()
        _check(_lib.alexnet_tensor_elems(self._h, T_CONV_ACT, layer, C.byref(n)))
        y = torch.empty(n.value, dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_conv_forward(self._h, layer, _ptr(xs), _ptr(wt), _ptr(bt), int(relu), _ptr(y), _stream(None)))
        return y

    def conv_backward_data(self, layer, dy, w, x_shape):
        dyt, wt = _dev(dy, torch.float32), _dev(w, torch.float32)
        dx = torch.empty(int(np.prod(x_shape)), dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_conv_backward_data(self._h, layer, _ptr(dyt), _ptr(wt), _ptr(dx), _stream(None)))
        return dx.view(*x_shape)

    def conv_backward_weight(self, layer, x, dy, w_shape):
        xs, dyt = _dev(x, torch.float32), _dev(dy, torch.float32)
        dw = torch.empty(int(np.prod(w_shape)), dtype=torch.float32, device="cuda")
        db = torch.empty(w_shape[0], dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_conv_backward_weight(self._h, layer, _ptr(xs), _ptr(dyt), _ptr(dw), _ptr(db), _stream(None)))
        return dw.view(*w_shape), db

    # channel-last variants: no conversion kernels in the call
    def pack_conv_weight(self, layer, w_oihw: torch.Tensor):
        wf, wb = torch.empty_like(w_oihw).view(-1), torch.empty_like(w_oihw).view(-1)
        _check(_lib.alexnet_pack_conv_weight(self._h, layer, _ptr(w_oihw), _ptr(wf), _ptr(wb), _stream(None)))
        return wf, wb

    def unpack_conv_weight(self, layer, wf: torch.Tensor, w_shape):
        w = torch.empty(int(np.prod(w_shape)), dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_unpack_conv_weight(self._h, layer, _ptr(wf), _ptr(w), _stream(None)))
        return w.view(*w_shape)

    def _conv_elems(self, layer: int) -> Tuple[int, int, int, int]:
        """Elements of a convolution stage's input, output, weights and bias (the geometry rule of the library:
        out = (in + 2 pad - k) / stride + 1, 3x3 stride-2 pooling behind the stages that pool)."""
        if not 1 <= layer <= len(self.workload["conv"]):
            raise ValueError(f"layer must be 1..{len(self.workload['conv'])}")
        c, h = self.workload["in_c"], self.workload["crop"]
        for i, (cout, k, stride, pad, groups, _lrn, pool) in enumerate(self.workload["conv"], start=1):
            ho = (h + 2 * pad - k) // stride + 1
            if i == layer:
                return self.batch * h * h * c, self.batch * ho * ho * cout, cout * (c // groups) * k * k, cout
            c, h = cout, ((ho - 3) // 2 + 1 if pool else ho)
        raise AssertionError

    def conv_forward_nhwc(self, layer, x, wf, b, relu, y, stream=None):
        nx, ny, nw, nb = self._conv_elems(layer)
        _need(x, torch.float32, nx, "conv_forward_nhwc: x")
        _need(wf, torch.float32, nw, "conv_forward_nhwc: wf")
        _need(y, torch.float32, ny, "conv_forward_nhwc: y")
        if b is not None:
            _need(b, torch.float32, nb, "conv_forward_nhwc: bias")
        _check(_lib.alexnet_conv_forward_nhwc(self._h, layer, _ptr(x), _ptr(wf), _ptr(b), int(relu), _ptr(y), _stream(stream)))

    def conv_backward_data_nhwc(self, layer, dy, wb, dx, wf=None, stream=None):
        nx, ny, nw, _ = self._conv_elems(layer)
        _need(dy, torch.float32, ny, "conv_backward_data_nhwc: dy")
        _need(wb, torch.float32, nw, "conv_backward_data_nhwc: wb")
        _need(dx, torch.float32, nx, "conv_backward_data_nhwc: dx")
        if wf is not None:
            _need(wf, torch.float32, nw, "conv_backward_data_nhwc: wf")
        _check(_lib.alexnet_conv_backward_data_nhwc(self._h, layer, _ptr(dy), _ptr(wf), _ptr(wb), _ptr(dx), _stream(stream)))

    def conv_backward_weight_nhwc(self, layer, x, dy, dwf, db, stream=None):
        nx, ny, nw, nb = self._conv_elems(layer)
        _need(x, torch.float32, nx, "conv_backward_weight_nhwc: x")
        _need(dy, torch.float32, ny, "conv_backward_weight_nhwc: dy")
        _need(dwf, torch.float32, nw, "conv_backward_weight_nhwc: dwf")
        if db is not None:
            _need(db, torch.float32, nb, "conv_backward_weight_nhwc: db")
        _check(_lib.alexnet_conv_backward_weight_nhwc(self._h, layer, _ptr(x), _ptr(dy), _ptr(dwf), _ptr(db), _stream(stream)))


    # ---- bandwidth-bound operators and dense layers alone (canonical tensors) ----
    def lrn_forward(self, layer, a):
        at = _dev(a, torch.float32)
        b = torch.empty_like(at)
        _check(_lib.alexnet_lrn_forward(self._h, layer, _ptr(at), _ptr(b), _stream(None)))
        return b

    def lrn_backward(self, layer, a, db, relu_gate=False):
        at, dbt = _dev(a, torch.float32), _dev(db, torch.float32)
        da = torch.empty_like(at)
        _check(_lib.alexnet_lrn_backward(self._h, layer, _ptr(at), _ptr(dbt), int(relu_gate), _ptr(da), _stream(None)))
        return da

    def pool_forward(self, layer, x):
        xt = _dev(x, torch.float32)
        n, c, h, w = xt.shape
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        y = torch.empty(n, c, ho, wo, dtype=torch.float32, device="cuda")
        arg = torch.empty(n, c, ho, wo, dtype=torch.int32, device="cuda")
        _check(_lib.alexnet_pool_forward(self._h, layer, _ptr(xt), _ptr(y), _ptr(arg), _stream(None)))
        return y, arg

    def pool_backward(self, layer, x, dy, relu_gate=False):
        xt, dyt = _dev(x, torch.float32), _dev(dy, torch.float32)
        dx = torch.empty_like(xt)
        _check(_lib.alexnet_pool_backward(self._h, layer, _ptr(xt), _ptr(dyt), int(relu_gate), _ptr(dx), _stream(None)))
        return dx

    def lrn_pool_forward(self, layer, a):
        """The fused normalisation + pool kernel of a training step, alone: pooled values and winning taps."""
        at = _dev(a, torch.float32)
        n, c, h, w = at.shape
        ho, wo = (h - 3) // 2 + 1, (w - 3) // 2 + 1
        y = torch.empty(n, c, ho, wo, dtype=torch.float32, device="cuda")
        arg = torch.empty(n, c, ho, wo, dtype=torch.int32, device="cuda")
        _check(_lib.alexnet_lrn_pool_forward(self._h, layer, _ptr(at), _ptr(y), _ptr(arg), _stream(None)))
        return y, arg

    def pool_lrn_backward(self, layer, a, dy, relu_gate=True):
        """The fused pool adjoint + normalisation adjoint + gate + bias sums kernel, alone: (da, db)."""
        at, dyt = _dev(a, torch.float32), _dev(dy, torch.float32)
        da = torch.empty_like(at)
        db = torch.empty(at.shape[1], dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_pool_lrn_backward(self._h, layer, _ptr(at), _ptr(dyt), int(relu_gate), _ptr(da), _ptr(db),
                                              _stream(None)))
        return da, db

    def fc_forward(self, layer, x, w, b, relu=False):
        xt, wt, bt = _dev(x, torch.float32), _dev(w, torch.float32), _dev(b, torch.float32)
        y = torch.empty(xt.shape[0], wt.shape[0], dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_fc_forward(self._h, layer, _ptr(xt), _ptr(wt), _ptr(bt), int(relu), _ptr(y), _stream(None)))
        return y

    def fc_backward(self, layer, x, w, dy):
        xt, wt, dyt = _dev(x, torch.float32), _dev(w, torch.float32), _dev(dy, torch.float32)
        dx, dw = torch.empty_like(xt), torch.empty_like(wt)
        db = torch.empty(wt.shape[0], dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_fc_backward(self._h, layer, _ptr(xt), _ptr(wt), _ptr(dyt), _ptr(dx), _ptr(dw), _ptr(db),
                                        _stream(None)))
        return dx, dw, db

    def softmax_xent(self, logits, labels):
        zt, lt = _dev(logits, torch.float32), _dev(labels, torch.int32)
        dz = torch.empty_like(zt)
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        _check(_lib.alexnet_softmax_xent(self._h, _ptr(zt), _ptr(lt), _ptr(dz), _ptr(loss), _stream(None)))
        return dz, loss


def average_replicas(a: AlexNet, b: AlexNet, stream=None):
    _check(_lib.alexnet_average_replicas(a._h, b._h, _stream(stream)))


class Loader:
    """Section 2.1's loading thread: `images` (uint8 [count][C][RH][RW]) and `labels` (int32 [count]) are CPU
    tensors standing for the disk; staging memory (pinned host + device) is allocated here with torch."""

    def __init__(self, net: AlexNet, images: torch.Tensor, labels: torch.Tensor, depth: int = 2, copy_stream=None):
        """copy_stream: the stream of the host-to-device copies (best the side stream later given to stage());
        None lets the library create one."""
        want = (net.workload["in_c"], net.workload["raw"], net.workload["raw"])
        if images.dtype != torch.uint8 or images.is_cuda or images.dim() != 4 or tuple(images.shape[1:]) != want:
            raise ValueError(f"Loader: images must be a CPU uint8 tensor [count]{list(want)}, got "
                             f"{images.dtype} {list(images.shape)} on {images.device}")
        if labels.dtype != torch.int32 or labels.is_cuda or labels.numel() != images.shape[0]:
            raise ValueError("Loader: labels must be a CPU int32 tensor with one entry per picture")
        if depth < 1 or images.shape[0] < 1:
            raise ValueError("Loader: need at least one staging set and one picture")
        self.net, self.images, self.labels = net, images.contiguous(), labels.contiguous()
        per = net.batch * int(np.prod(images.shape[1:]))
        self.pinned_raw = torch.empty(depth * per, dtype=torch.uint8, pin_memory=True)
        self.pinned_labels = torch.empty(depth * net.batch, dtype=torch.int32, pin_memory=True)
        self.d_raw = torch.empty(depth * per, dtype=torch.uint8, device="cuda")
        self.d_labels = torch.empty(depth * net.batch, dtype=torch.int32, device="cuda")
        h = _vp()
        _check(_lib.alexnet_loader_create(net._h, C.byref(net.cfg), self.images.data_ptr(), self.labels.data_ptr(),
                                          self.images.shape[0], depth, self.pinned_raw.data_ptr(),
                                          self.pinned_labels.data_ptr(), self.d_raw.data_ptr(),
                                          self.d_labels.data_ptr(),
                                          None if copy_stream is None else _stream(copy_stream), C.byref(h)))
        self._h = h
        self._copy_stream = copy_stream  # keep the torch stream alive as long as the loader

    def stage(self, k: int, mean: torch.Tensor, side_stream, compute_stream) -> torch.Tensor:
        """Returns the labels of minibatch k (a view of the loader's device buffer)."""
        _need(mean, torch.float32, self.net._raw_elems(), "Loader.stage: mean image")
        p = _vp()
        _check(_lib.alexnet_loader_stage(self._h, k, _ptr(mean), _stream(side_stream), _stream(compute_stream),
                                         C.byref(p)))
        off = (p.value - self.d_labels.data_ptr()) // 4
        return self.d_labels[off:off + self.net.batch]

    def done(self, k: int, compute_stream):
        _check(_lib.alexnet_loader_done(self._h, k, _stream(compute_stream)))

    def close(self):
        if self._h is not None and _lib is not None:
            _lib.alexnet_loader_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


def softmax_xent_static(logits: torch.Tensor, labels: torch.Tensor, dz: torch.Tensor, loss: torch.Tensor,
                        bad_label: Optional[torch.Tensor] = None, stream=None):
    """alexnet_softmax_xent_static: no handle, no workspace; every tensor is the caller's."""
    batch, classes = logits.shape
    _need(logits, torch.float32, batch * classes, "softmax_xent_static: logits")
    _need(labels, torch.int32, batch, "softmax_xent_static: labels")
    _need(dz, torch.float32, batch * classes, "softmax_xent_static: dz")
    _need(loss, torch.float32, 1, "softmax_xent_static: loss")
    if bad_label is not None:
        _need(bad_label, torch.int32, 1, "softmax_xent_static: bad_label")
    _check(_lib.alexnet_softmax_xent_static(_ptr(logits), _ptr(labels), batch, classes, _ptr(dz), _ptr(loss),
                                            _ptr(bad_label), _stream(stream)))


def average_gradients_update(a: AlexNet, b: AlexNet, stream=None):
    _check(_lib.alexnet_average_gradients_update(a._h, b._h, _stream(stream)))


def nchw_to_nhwc(x: torch.Tensor) -> torch.Tensor:
    n, c, h, w = x.shape
    y = torch.empty(n, h, w, c, dtype=torch.float32, device="cuda")
    _check(_lib.alexnet_nchw_to_nhwc(_ptr(x.contiguous()), _ptr(y), n, c, h, w, _stream(None)))
    return y


def nhwc_to_nchw(x: torch.Tensor) -> torch.Tensor:
    n, h, w, c = x.shape
    y = torch.empty(n, c, h, w, dtype=torch.float32, device="cuda")
    _check(_lib.alexnet_nhwc_to_nchw(_ptr(x.contiguous()), _ptr(y), n, c, h, w, _stream(None)))
    return y
