"""ctypes binding of libstrait.so: the same names as include/strait.h, argument marshalling only.

PyTorch appears here for plumbing alone: it owns the HIP streams handed to the library and the
device tensors passed to the kernel-level entry points.  There is no CPU fallback: if the
library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libstrait.so")

# PyTorch-ROCm ships its own copy of the HIP runtime.  It has to be in the process before
# libstrait.so is opened, so that the library's dependency on libamdhip64.so.7 resolves to that
# same copy: two HIP runtimes in one process do not share devices, streams or memory.
import torch  # noqa: E402,F401

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(there is no fallback path)")
lib = C.CDLL(LIB_PATH)

OK, E_INVALID, E_HIP, E_FORMAT, E_NOMEM, E_SHAPE, E_BUSY, E_BATCH = 0, -1, -2, -3, -4, -5, -6, -7
PRIO_HIGH, PRIO_LOW = 0, 1
ACT_NONE, ACT_RELU, ACT_RELU6, ACT_GELU = 0, 1, 2, 3
MAX_STREAMS = 8


class StraitError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"strait status {status}: {msg}")
        self.status = status


class CtxDesc(C.Structure):
    _fields_ = [("device", C.c_int32), ("n_hp", C.c_int32), ("n_lp", C.c_int32), ("n_copy", C.c_int32),
                ("hp_streams", C.c_void_p * MAX_STREAMS), ("lp_streams", C.c_void_p * MAX_STREAMS),
                ("copy_streams", C.c_void_p * MAX_STREAMS)]


class ModelDesc(C.Structure):
    _fields_ = [("weights", C.c_void_p), ("weights_bytes", C.c_size_t), ("max_batch", C.c_int32),
                ("n_instances", C.c_int32)]


class Record(C.Structure):
    _fields_ = [("model_id", C.c_int32), ("priority", C.c_int32), ("batch", C.c_int32), ("instance", C.c_int32),
                ("t_enqueue_ns", C.c_int64), ("t_issued_ns", C.c_int64), ("t_done_ns", C.c_int64),
                ("h2d_ms", C.c_float), ("kernel_ms", C.c_float), ("d2h_ms", C.c_float), ("total_ms", C.c_float)]


class LayerInfo(C.Structure):
    _fields_ = [("name", C.c_char * 40), ("kind", C.c_int32), ("macs_per_sample", C.c_int64),
                ("bytes_per_sample", C.c_int64), ("weight_bytes", C.c_int64),
                ("gemm_m_per_sample", C.c_int32), ("gemm_n", C.c_int32), ("gemm_k", C.c_int32)]


_vp, _i32, _i64, _sz, _f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_double
_SIGS = {
    "strait_last_error": (C.c_char_p, []),
    "strait_version": (_i32, []),
    "strait_ctx_create": (_i32, [C.POINTER(CtxDesc), C.POINTER(_vp)]),
    "strait_ctx_destroy": (_i32, [_vp]),
    "strait_ctx_set_wave_priority": (_i32, [_vp, _i32]),
    "strait_ctx_set_graphs": (_i32, [_vp, _i32]),
    "strait_ctx_set_h2d_kernel_limit": (_i32, [_vp, C.c_int64]),
    "strait_ctx_set_branch_streams": (_i32, [_vp, _i32]),
    "strait_ctx_set_lp_yield": (_i32, [_vp, _i32]),
    "strait_ctx_set_pair_fusion": (_i32, [_vp, _i64]),
    "strait_ctx_set_proj_fusion": (_i32, [_vp, _i64]),
    "strait_model_load": (_i32, [_vp, C.POINTER(ModelDesc), C.POINTER(_vp)]),
    "strait_model_free": (_i32, [_vp]),
    "strait_model_io": (_i32, [_vp, _i32, C.POINTER(_sz), C.POINTER(_sz)]),
    "strait_model_info": (_i32, [_vp, C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32 * 8)]),
    "strait_model_staging": (_i32, [_vp, _i32, C.POINTER(_vp), C.POINTER(_sz)]),
    "strait_model_layer": (_i32, [_vp, _i32, C.POINTER(LayerInfo)]),
    "strait_submit": (_i32, [_vp, _i32, _i32, _vp, _vp, _vp, C.POINTER(_vp)]),
    "strait_poll": (_i32, [_vp, C.POINTER(_i32)]),
    "strait_wait": (_i32, [_vp, C.POINTER(Record)]),
    "strait_copy_in": (_i32, [_vp, _i32, _i32, _i32, _vp, _vp]),
    "strait_run": (_i32, [_vp, _i32, _i32, _i32]),
    "strait_copy_out": (_i32, [_vp, _i32, _i32, _i32, _vp]),
    "strait_sync": (_i32, [_vp, _i32, _i32]),
    "strait_run_timed": (_i32, [_vp, _i32, _i32, _i32, _vp]),
    "strait_read_activation": (_i32, [_vp, _i32, _i32, _i32, _vp, _sz, C.POINTER(_sz)]),
    "strait_k_conv2d": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32]),
    "strait_k_gemm": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32]),
    "strait_k_gemm_noalloc": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32]),
    "strait_k_conv1x1_proj": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i32]),
    "strait_k_expand_dw": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i32]),
    "strait_k_stem3x3s2_dw": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _i32]),
    "strait_k_stem3x3s2": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i32]),
    "strait_k_pointwise_pair": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32]),
    "strait_k_pointwise_pair_proj": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32]),
    "strait_k_dwconv3x3": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _i32, _i32, _vp, _i32]),
    "strait_k_maxpool3x3s2": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32]),
    "strait_k_stem_pool": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _i32]),
    "strait_k_maxpool2x2s2": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _vp, _i32]),
    "strait_k_vit_tokens": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32]),
    "strait_k_global_avgpool": (_i32, [_vp, _vp, _i32, _i32, _i32, _vp, _i32]),
    "strait_k_softmax_top1": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp, _i32]),
    "strait_k_layernorm": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, C.c_float, _vp, _i32]),
    "strait_k_attention": (_i32, [_vp, _vp, _vp, _i32, _i32, _i32, _vp, _i32]),
    "strait_k_argmax_f16": (_i32, [_vp, _vp, _i32, _i32, _i64, _vp, _i32]),
    "strait_link_create": (_i32, [C.POINTER(_vp)]),
    "strait_link_destroy": (_i32, [_vp]),
    "strait_link_available": (_i32, [_vp, C.POINTER(_i64)]),
    "strait_link_predict": (_i32, [_vp, _i64, C.POINTER(_i64)]),
    "strait_link_schedule": (_i32, [_vp, _i64, _i64, C.POINTER(C.c_uint64), C.POINTER(_i64)]),
    "strait_link_complete": (_i32, [_vp, C.c_uint64, _i64]),
    "strait_intf_create": (_i32, [_vp, C.POINTER(_vp)]),
    "strait_intf_destroy": (_i32, [_vp]),
    "strait_intf_get_params": (_i32, [_vp, _vp]),
    "strait_intf_demand": (_i32, [_vp, _vp, _i32, _vp]),
    "strait_intf_predict": (_i32, [_vp, _vp, _f64, _f64, _i32, _f64, C.POINTER(_f64), C.POINTER(_f64)]),
    "strait_intf_update": (_i32, [_vp, _vp, _f64, _f64, _i32, _f64, C.POINTER(_f64)]),
    "strait_intf_arrive": (_i32, [_vp, _i64, _vp, C.POINTER(C.c_uint64)]),
    "strait_intf_depart": (_i32, [_vp, C.c_uint64, _i64, _vp]),
    "strait_intf_pressure": (_i32, [_vp, C.c_uint64, _vp]),
    "strait_sched_create": (_i32, [_i32, _vp, C.POINTER(_vp)]),
    "strait_sched_destroy": (_i32, [_vp]),
    "strait_sched_set_profile": (_i32, [_vp, _i32, _i32, _vp, _i32]),
    "strait_sched_tick": (_i32, [_vp, _i64, C.POINTER(_f64)]),
    "strait_sched_decide": (_i32, [_vp, _i32, _i64, _vp, _vp, _i32, _vp]),
    "strait_sched_complete": (_i32, [_vp, _i32, C.c_uint64, _i64, _f64, _i64, _vp]),
    "strait_sched_get_params": (_i32, [_vp, _vp]),
    "strait_model_profile": (_i32, [_vp, _i32, _i32, _i32, _vp]),
    "strait_server_create": (_i32, [_vp, _i32, _i64, _vp, C.POINTER(_vp)]),
    "strait_server_add_model": (_i32, [_vp, _vp]),
    "strait_server_start": (_i32, [_vp]),
    "strait_server_request": (_i32, [_vp, _i32, _vp, _i32, _vp, C.POINTER(C.c_uint64)]),
    "strait_server_wait_idle": (_i32, [_vp, _i64]),
    "strait_server_results": (_i32, [_vp, _vp, _i32, C.POINTER(_i32)]),
    "strait_server_get_stats": (_i32, [_vp, _vp]),
    "strait_server_stop": (_i32, [_vp]),
    "strait_server_destroy": (_i32, [_vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
EXPORTS = tuple(_SIGS.keys())


def last_error() -> str:
    return (lib.strait_last_error() or b"").decode()


def _check(status: int):
    if status != OK:
        raise StraitError(status, last_error())


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_vp)


def _dev(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Context:
    """strait_ctx over streams created through PyTorch (all at the default stream priority)."""

    def __init__(self, device: int = 0, n_hp: int = 1, n_lp: int = 1, n_copy: int = 2):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("strait needs a GPU: no HIP device is visible (there is no CPU path)")
        self.torch = torch
        self.device = device
        torch.cuda.set_device(device)
        mk = lambda n: [torch.cuda.Stream(device=device) for _ in range(n)]
        self.hp_streams, self.lp_streams, self.copy_streams = mk(n_hp), mk(n_lp), mk(n_copy)
        d = CtxDesc()
        d.device, d.n_hp, d.n_lp, d.n_copy = device, n_hp, n_lp, n_copy
        for i, s in enumerate(self.hp_streams):
            d.hp_streams[i] = s.cuda_stream
        for i, s in enumerate(self.lp_streams):
            d.lp_streams[i] = s.cuda_stream
        for i, s in enumerate(self.copy_streams):
            d.copy_streams[i] = s.cuda_stream
        self.handle = _vp()
        _check(lib.strait_ctx_create(C.byref(d), C.byref(self.handle)))

    def load(self, weights: bytes, max_batch: int, n_instances: int = 1) -> "Model":
        return Model(self, weights, max_batch, n_instances)

    def set_graphs(self, enabled: bool):
        _check(lib.strait_ctx_set_graphs(self.handle, 1 if enabled else 0))

    def set_pair_fusion(self, min_pixels: int):
        _check(lib.strait_ctx_set_pair_fusion(self.handle, int(min_pixels)))

    def set_proj_fusion(self, min_pixels: int):
        _check(lib.strait_ctx_set_proj_fusion(self.handle, int(min_pixels)))

    def set_lp_yield(self, layers_per_segment: int):
        _check(lib.strait_ctx_set_lp_yield(self.handle, int(layers_per_segment)))

    def set_branch_streams(self, enabled: bool):
        _check(lib.strait_ctx_set_branch_streams(self.handle, 1 if enabled else 0))

    def set_h2d_kernel_limit(self, max_bytes: int):
        _check(lib.strait_ctx_set_h2d_kernel_limit(self.handle, int(max_bytes)))

    def set_wave_priority(self, enabled: bool):
        _check(lib.strait_ctx_set_wave_priority(self.handle, int(enabled)))

    def close(self):
        if self.handle:
            _check(lib.strait_ctx_destroy(self.handle))
            self.handle = _vp()


class Model:
    def __init__(self, ctx: Context, weights: bytes, max_batch: int, n_instances: int):
        self.ctx = ctx
        buf = (C.c_char * len(weights)).from_buffer_copy(weights)
        d = ModelDesc(C.cast(buf, _vp), len(weights), max_batch, n_instances)
        self.handle = _vp()
        _check(lib.strait_model_load(ctx.handle, C.byref(d), C.byref(self.handle)))
        arch, nl, mb, ni = _i32(), _i32(), _i32(), _i32()
        hyper = (_i32 * 8)()
        _check(lib.strait_model_info(self.handle, C.byref(arch), C.byref(nl), C.byref(mb), C.byref(ni), C.byref(hyper)))
        self.arch, self.n_layers, self.max_batch, self.n_instances = arch.value, nl.value, mb.value, ni.value
        self.hyper = tuple(hyper)
        self._keep = {}

    # ---- queries
    def io_bytes(self, batch: int):
        a, b = _sz(), _sz()
        _check(lib.strait_model_io(self.handle, batch, C.byref(a), C.byref(b)))
        return a.value, b.value

    def layer(self, i: int) -> LayerInfo:
        li = LayerInfo()
        _check(lib.strait_model_layer(self.handle, i, C.byref(li)))
        return li

    def layers(self):
        return [self.layer(i) for i in range(self.n_layers)]

    # ---- output decoding (layout documented in strait.h)
    def new_output(self, batch: int) -> np.ndarray:
        return np.empty(self.io_bytes(batch)[1], dtype=np.uint8)

    def decode(self, out: np.ndarray, batch: int):
        if self.arch == 3:
            _, hidden, _, _, seq = self.hyper[:5]
            n = batch * seq * hidden
            return {"hidden": out[:2 * n].view(np.float16).reshape(batch, seq, hidden),
                    "top1": out[2 * n:2 * n + 4 * batch].view(np.int32)}
        classes = self.hyper[3]
        n = batch * classes
        return {"logits": out[:4 * n].view(np.float32).reshape(batch, classes),
                "probs": out[4 * n:8 * n].view(np.float32).reshape(batch, classes),
                "top1": out[8 * n:8 * n + 4 * batch].view(np.int32)}

    # ---- the served path
    def staging(self, instance: int, batch: int) -> np.ndarray:
        """The instance's pinned input buffer as an fp16 array shaped like a batch of `batch` inputs; submit() given
        this array uses that instance without copying."""
        ptr, cap = _vp(), _sz()
        _check(lib.strait_model_staging(self.handle, instance, C.byref(ptr), C.byref(cap)))
        nbytes = self.io_bytes(batch)[0]
        buf = (C.c_char * nbytes).from_address(ptr.value)
        a = np.frombuffer(buf, dtype=np.float16)
        if self.arch == 3:
            _, hidden, _, _, seq = self.hyper[:5]
            return a.reshape(batch, seq, hidden)
        h, w, c = self.hyper[:3]
        return a.reshape(batch, h, w, c)

    def submit(self, prio: int, x: np.ndarray, valid_len: Optional[np.ndarray], out: np.ndarray) -> int:
        batch = x.shape[0]
        assert x.dtype == np.float16 and x.flags.c_contiguous and out.flags.c_contiguous
        if valid_len is not None:
            valid_len = np.ascontiguousarray(valid_len, dtype=np.int32)
        t = _vp()
        _check(lib.strait_submit(self.handle, prio, batch, _np_ptr(x), _np_ptr(valid_len), _np_ptr(out), C.byref(t)))
        self._keep[t.value] = (x, valid_len, out)
        return t.value

    def try_submit(self, prio, x, valid_len, out):
        """Like submit, but returns None instead of raising when every instance is busy."""
        try:
            return self.submit(prio, x, valid_len, out)
        except StraitError as e:
            if e.status == E_BUSY:
                return None
            raise

    def poll(self, ticket: int) -> bool:
        d = _i32()
        _check(lib.strait_poll(_vp(ticket), C.byref(d)))
        return bool(d.value)

    def wait(self, ticket: int) -> Record:
        r = Record()
        st = lib.strait_wait(_vp(ticket), C.byref(r))
        self._keep.pop(ticket, None)
        _check(st)
        return r

    def infer(self, x: np.ndarray, valid_len=None, prio: int = PRIO_HIGH):
        out = self.new_output(x.shape[0])
        rec = self.wait(self.submit(prio, x, valid_len, out))
        return self.decode(out, x.shape[0]), rec

    # ---- sub-steps
    def copy_in(self, instance, prio, x, valid_len=None):
        if valid_len is not None:
            valid_len = np.ascontiguousarray(valid_len, dtype=np.int32)
        _check(lib.strait_copy_in(self.handle, instance, prio, x.shape[0], _np_ptr(x), _np_ptr(valid_len)))

    def run(self, instance, prio, batch):
        _check(lib.strait_run(self.handle, instance, prio, batch))

    def copy_out(self, instance, prio, batch) -> np.ndarray:
        out = self.new_output(batch)
        _check(lib.strait_copy_out(self.handle, instance, prio, batch, _np_ptr(out)))
        return out

    def sync(self, instance, prio):
        _check(lib.strait_sync(self.handle, instance, prio))

    def run_timed(self, instance, prio, batch) -> np.ndarray:
        ms = np.zeros(self.n_layers, dtype=np.float32)
        _check(lib.strait_run_timed(self.handle, instance, prio, batch, _np_ptr(ms)))
        return ms

    def read_activation(self, instance, layer, batch) -> np.ndarray:
        need = _sz()
        _check(lib.strait_read_activation(self.handle, instance, layer, batch, None, 0, C.byref(need)))
        out = np.empty(need.value // 2, dtype=np.float16)
        _check(lib.strait_read_activation(self.handle, instance, layer, batch, _np_ptr(out), need.value, None))
        return out

    def free(self):
        if self.handle:
            _check(lib.strait_model_free(self.handle))
            self.handle = _vp()


# ---- kernel-level entry points on torch device tensors ---------------------------------------

def _stream(stream=None) -> int:
    import torch
    return (stream or torch.cuda.current_stream()).cuda_stream


def k_conv2d(x, w_krsc, bias, stride, pad, act=ACT_NONE, res=None, out_f32=False, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    k, r, s, c2 = w_krsc.shape
    assert c2 == c
    p, q = (h + 2 * pad - r) // stride + 1, (w + 2 * pad - s) // stride + 1
    y = torch.empty((n, p, q, k), dtype=torch.float32 if out_f32 else torch.float16, device=x.device)
    _check(lib.strait_k_conv2d(_stream(stream), _dev(x), n, h, w, c, _dev(w_krsc), _dev(bias), k, r, s, stride, pad,
                               act, _dev(res), _dev(y), int(out_f32), hp))
    return y


def k_gemm(x, w, bias, act=ACT_NONE, res=None, out_f32=False, hp=0, stream=None):
    import torch
    m, k = x.shape
    n = w.shape[0]
    y = torch.empty((m, n), dtype=torch.float32 if out_f32 else torch.float16, device=x.device)
    _check(lib.strait_k_gemm(_stream(stream), _dev(x), _dev(w), _dev(bias), m, n, k, act, _dev(res), _dev(y), int(out_f32), hp))
    return y


def k_gemm_noalloc(x, w, bias, y, act=ACT_NONE, res=None, out_f32=False, hp=0, stream=None):
    """strait_k_gemm_noalloc into the caller's output tensor `y` (nothing is allocated on the way)."""
    m, k = x.shape
    n = w.shape[0]
    assert tuple(y.shape) == (m, n)
    _check(lib.strait_k_gemm_noalloc(_stream(stream), _dev(x), _dev(w), _dev(bias), m, n, k, act, _dev(res), _dev(y), int(out_f32), hp))
    return y


def k_pointwise_pair(x, w3, b3, res, w1, b1, act1=ACT_RELU, act2=ACT_RELU, hp=0, stream=None):
    import torch
    m, k1 = x.shape
    n1, n2 = w3.shape[0], w1.shape[0]
    y = torch.empty((m, n1), dtype=torch.float16, device=x.device)
    z = torch.empty((m, n2), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_pointwise_pair(_stream(stream), _dev(x), _dev(w3), _dev(b3), _dev(res), _dev(y), _dev(w1), _dev(b1),
                                       _dev(z), m, k1, n1, n2, act1, act2, hp))
    return y, z


def k_conv1x1_proj(x, x2, stride2, w, bias, act=ACT_NONE, hp=0, stream=None):
    import torch
    n, p_, q, c = x.shape
    _, h2, w2, k2 = x2.shape
    cout = w.shape[0]
    y = torch.empty((n, p_, q, cout), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_conv1x1_proj(_stream(stream), _dev(x), n, p_, q, c, _dev(x2), h2, w2, k2, stride2, _dev(w), _dev(bias),
                                     cout, act, _dev(y), hp))
    return y


def k_pointwise_pair_proj(x, x2, w3, b3, w1, b1, act1=ACT_RELU, act2=ACT_RELU, hp=0, stream=None):
    import torch
    m, k1 = x.shape
    k2 = x2.shape[1] if x2 is not None else 0
    n1, n2 = w3.shape[0], w1.shape[0]
    y = torch.empty((m, n1), dtype=torch.float16, device=x.device)
    z = torch.empty((m, n2), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_pointwise_pair_proj(_stream(stream), _dev(x), _dev(x2), _dev(w3), _dev(b3), _dev(y), _dev(w1), _dev(b1),
                                            _dev(z), m, k1, k2, n1, n2, act1, act2, hp))
    return y, z


def k_dwconv3x3(x, w_rsc, bias, stride, act=ACT_NONE, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    p, q = (h - 1) // stride + 1, (w - 1) // stride + 1
    y = torch.empty((n, p, q, c), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_dwconv3x3(_stream(stream), _dev(x), n, h, w, c, _dev(w_rsc), _dev(bias), stride, act, _dev(y), hp))
    return y


def k_maxpool3x3s2(x, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    y = torch.empty((n, (h - 1) // 2 + 1, (w - 1) // 2 + 1, c), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_maxpool3x3s2(_stream(stream), _dev(x), n, h, w, c, _dev(y), hp))
    return y


def k_stem_pool(x, wf, bias, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    assert c == 3
    p, q = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    y = torch.empty((n, (p - 1) // 2 + 1, (q - 1) // 2 + 1, 64), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_stem_pool(_stream(stream), _dev(x), n, h, w, _dev(wf), _dev(bias), _dev(y), hp))
    return y


def k_stem3x3s2_dw(x, wf, bias, wd_rsc, bd, act1=ACT_RELU6, act2=ACT_RELU6, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    assert c == 3
    y = torch.empty((n, (h - 1) // 2 + 1, (w - 1) // 2 + 1, 32), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_stem3x3s2_dw(_stream(stream), _dev(x), n, h, w, _dev(wf), _dev(bias), act1, _dev(wd_rsc), _dev(bd), act2, _dev(y), hp))
    return y


def k_expand_dw(x, w1, b1, wd_rsc, bd, stride, act1=ACT_RELU6, act2=ACT_RELU6, hp=0, stream=None):
    import torch
    n, h, w, cin = x.shape
    chid = w1.shape[0]
    y = torch.empty((n, (h - 1) // stride + 1, (w - 1) // stride + 1, chid), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_expand_dw(_stream(stream), _dev(x), n, h, w, cin, _dev(w1), _dev(b1), chid, act1, _dev(wd_rsc), _dev(bd), stride, act2,
                                  _dev(y), hp))
    return y


def k_stem3x3s2(x, wf, bias, kout, act=ACT_NONE, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    assert c == 3
    y = torch.empty((n, (h - 1) // 2 + 1, (w - 1) // 2 + 1, kout), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_stem3x3s2(_stream(stream), _dev(x), n, h, w, _dev(wf), _dev(bias), kout, act, _dev(y), hp))
    return y


def k_maxpool2x2s2(x, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    y = torch.empty((n, h // 2, w // 2, c), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_maxpool2x2s2(_stream(stream), _dev(x), n, h, w, c, _dev(y), hp))
    return y


def k_vit_tokens(patch, cls, pos, hp=0, stream=None):
    import torch
    n, t, d = patch.shape
    z = torch.empty((n, t + 1, d), dtype=torch.float16, device=patch.device)
    _check(lib.strait_k_vit_tokens(_stream(stream), _dev(patch), _dev(cls), _dev(pos), n, t, d, _dev(z), hp))
    return z


def k_global_avgpool(x, hp=0, stream=None):
    import torch
    n, h, w, c = x.shape
    y = torch.empty((n, c), dtype=torch.float16, device=x.device)
    _check(lib.strait_k_global_avgpool(_stream(stream), _dev(x), n, h * w, c, _dev(y), hp))
    return y


def k_softmax_top1(logits, hp=0, stream=None):
    import torch
    rows, n = logits.shape
    probs = torch.empty_like(logits)
    top1 = torch.empty((rows,), dtype=torch.int32, device=logits.device)
    _check(lib.strait_k_softmax_top1(_stream(stream), _dev(logits), rows, n, _dev(probs), _dev(top1), hp))
    return probs, top1


def k_layernorm(x, gamma, beta, eps, hp=0, stream=None):
    import torch
    rows, n = x.shape
    y = torch.empty_like(x)
    _check(lib.strait_k_layernorm(_stream(stream), _dev(x), _dev(gamma), _dev(beta), rows, n, eps, _dev(y), hp))
    return y


def k_attention(qkv, valid_len, heads, hp=0, stream=None):
    import torch
    b, s, h3 = qkv.shape
    out = torch.empty((b, s, h3 // 3), dtype=torch.float16, device=qkv.device)
    _check(lib.strait_k_attention(_stream(stream), _dev(qkv), _dev(valid_len), b, s, heads, _dev(out), hp))
    return out


def k_argmax_f16(x, n, row_stride, rows, hp=0, stream=None):
    import torch
    top1 = torch.empty((rows,), dtype=torch.int32, device=x.device)
    _check(lib.strait_k_argmax_f16(_stream(stream), _dev(x), rows, n, row_stride, _dev(top1), hp))
    return top1


class Link:
    """strait_link: the first-in first-out model of the host-to-device link (host only)."""

    def __init__(self):
        self.handle = _vp()
        _check(lib.strait_link_create(C.byref(self.handle)))

    def available(self) -> int:
        v = _i64()
        _check(lib.strait_link_available(self.handle, C.byref(v)))
        return v.value

    def predict(self, t_current_ns: int) -> int:
        v = _i64()
        _check(lib.strait_link_predict(self.handle, t_current_ns, C.byref(v)))
        return v.value

    def schedule(self, t_current_ns: int, t_htod_ns: int):
        tid, v = C.c_uint64(), _i64()
        _check(lib.strait_link_schedule(self.handle, t_current_ns, t_htod_ns, C.byref(tid), C.byref(v)))
        return tid.value, v.value

    def complete(self, transfer_id: int, t_end_ns: int):
        _check(lib.strait_link_complete(self.handle, transfer_id, t_end_ns))

    def close(self):
        if self.handle:
            _check(lib.strait_link_destroy(self.handle))
            self.handle = _vp()


INTF_METRICS = 5


class IntfParams(C.Structure):
    """strait_intf_params."""
    _fields_ = [("k", _f64), ("b", _f64), ("C", _f64), ("w_avg", _f64 * INTF_METRICS), ("w_self_cmp", _f64),
                ("w_self_mem", _f64), ("coeff_p", _f64 * 2)]

    def as_vector(self) -> np.ndarray:
        return np.array([self.k, self.b, self.C, *self.w_avg, self.w_self_cmp, self.w_self_mem, *self.coeff_p])

    @classmethod
    def from_vector(cls, v):
        v = [float(x) for x in v]
        return cls(v[0], v[1], v[2], (_f64 * INTF_METRICS)(*v[3:8]), v[8], v[9], (_f64 * 2)(*v[10:12]))


def _f64v(a, n=INTF_METRICS):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.size != n:
        raise ValueError(f"expected {n} values")
    return a


def intf_demand(v, d) -> np.ndarray:
    d = np.ascontiguousarray(d, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64).reshape(d.size, INTF_METRICS)
    out = np.zeros(INTF_METRICS)
    _check(lib.strait_intf_demand(_np_ptr(v), _np_ptr(d), d.size, _np_ptr(out)))
    return out


class Interference:
    """strait_intf: the kernel-interference predictor with its online update and co-location tracker (host only)."""

    def __init__(self, params=None):
        self.handle = _vp()
        start = None if params is None else IntfParams.from_vector(params)      # must outlive the call
        _check(lib.strait_intf_create(None if start is None else C.cast(C.byref(start), _vp), C.byref(self.handle)))

    def params(self) -> np.ndarray:
        p = IntfParams()
        _check(lib.strait_intf_get_params(self.handle, C.cast(C.byref(p), _vp)))
        return p.as_vector()

    def predict(self, m_avg, self_cmp, self_mem, prio, t_isol=0.0):
        m, intf, tk = _f64v(m_avg), _f64(), _f64()
        _check(lib.strait_intf_predict(self.handle, _np_ptr(m), self_cmp, self_mem, prio, t_isol, C.byref(intf), C.byref(tk)))
        return intf.value, tk.value

    def update(self, m_avg, self_cmp, self_mem, prio, intf_actual) -> float:
        m, loss = _f64v(m_avg), _f64()
        _check(lib.strait_intf_update(self.handle, _np_ptr(m), self_cmp, self_mem, prio, intf_actual, C.byref(loss)))
        return loss.value

    def arrive(self, t_ns, m) -> int:
        mm, bid = _f64v(m), C.c_uint64()
        _check(lib.strait_intf_arrive(self.handle, t_ns, _np_ptr(mm), C.byref(bid)))
        return bid.value

    def depart(self, batch_id, t_ns) -> np.ndarray:
        out = np.zeros(INTF_METRICS)
        _check(lib.strait_intf_depart(self.handle, batch_id, t_ns, _np_ptr(out)))
        return out

    def pressure(self, exclude_id=0) -> np.ndarray:
        out = np.zeros(INTF_METRICS)
        _check(lib.strait_intf_pressure(self.handle, exclude_id, _np_ptr(out)))
        return out

    def close(self):
        if self.handle:
            _check(lib.strait_intf_destroy(self.handle))
            self.handle = _vp()


class BatchProfile(C.Structure):
    """strait_batch_profile."""
    _fields_ = [("t_inf_isol_ns", _f64), ("t_htod_ns", _i64), ("t_kernel_isol_ns", _f64), ("m", _f64 * INTF_METRICS),
                ("m_self_cmp", _f64), ("m_self_mem", _f64)]


class Decision(C.Structure):
    """strait_decision."""
    _fields_ = [("n_dropped", _i32), ("batch", _i32), ("gpu", _i32), ("reserved", _i32), ("t_inf_ns", _f64),
                ("t_data_ns", _i64), ("running_id", C.c_uint64)]


class Completion(C.Structure):
    """strait_completion."""
    _fields_ = [("violated", _i32), ("reserved", _i32), ("loss", _f64), ("m_avg", _f64 * INTF_METRICS), ("c_low", _f64)]


class Scheduler:
    """strait_sched: the scheduling policy over the link and interference models (host only)."""

    def __init__(self, n_gpus: int = 1, params=None):
        self.handle = _vp()
        start = None if params is None else IntfParams.from_vector(params)      # must outlive the call
        _check(lib.strait_sched_create(n_gpus, None if start is None else C.cast(C.byref(start), _vp), C.byref(self.handle)))

    def set_profile(self, model_id: int, priority: int, profiles):
        """profiles: one (t_inf_isol_ns, t_htod_ns, t_kernel_isol_ns, m[5], m_self_cmp, m_self_mem) per batch size 1.."""
        arr = (BatchProfile * len(profiles))()
        for i, (ti, th, tk, m, sc, sm) in enumerate(profiles):
            arr[i] = BatchProfile(float(ti), int(th), float(tk), (_f64 * INTF_METRICS)(*[float(v) for v in m]), float(sc), float(sm))
        _check(lib.strait_sched_set_profile(self.handle, model_id, priority, C.cast(arr, _vp), len(profiles)))

    def tick(self, now_ns: int) -> float:
        c = _f64()
        _check(lib.strait_sched_tick(self.handle, now_ns, C.byref(c)))
        return c.value

    def decide(self, model_id: int, now_ns: int, enqueue_ns, deadline_ns) -> Decision:
        e = np.ascontiguousarray(enqueue_ns, dtype=np.int64)
        d = np.ascontiguousarray(deadline_ns, dtype=np.int64)
        assert e.size == d.size
        out = Decision()
        _check(lib.strait_sched_decide(self.handle, model_id, now_ns, _np_ptr(e) if e.size else None, _np_ptr(d) if d.size else None,
                                       e.size, C.cast(C.byref(out), _vp)))
        return out

    def complete(self, gpu: int, running_id: int, now_ns: int, kernel_ns: float, h2d_end_ns: int = -1) -> Completion:
        out = Completion()
        _check(lib.strait_sched_complete(self.handle, gpu, running_id, now_ns, kernel_ns, h2d_end_ns, C.cast(C.byref(out), _vp)))
        return out

    def params(self) -> np.ndarray:
        p = IntfParams()
        _check(lib.strait_sched_get_params(self.handle, C.cast(C.byref(p), _vp)))
        return p.as_vector()

    def close(self):
        if self.handle:
            _check(lib.strait_sched_destroy(self.handle))
            self.handle = _vp()


class ServerModel(C.Structure):
    """strait_server_model."""
    _fields_ = [("model", _vp), ("model_id", _i32), ("priority", _i32), ("max_batch", _i32), ("n_instances", _i32),
                ("deadline_ns", _i64), ("formation_timeout_ns", _i64)]


_EXEC_SUBMIT = C.CFUNCTYPE(_i32, _vp, C.c_uint64, _i32, _i32, _i32, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_i32))
_EXEC_WAIT = C.CFUNCTYPE(_i32, _vp, C.c_uint64, C.POINTER(_f64), C.POINTER(_f64))


class Executor(C.Structure):
    """strait_executor."""
    _fields_ = [("user", _vp), ("submit", _EXEC_SUBMIT), ("wait", _EXEC_WAIT)]


class RequestRecord(C.Structure):
    """strait_request_record."""
    _fields_ = [("request_id", C.c_uint64), ("batch_seq", C.c_uint64), ("model_id", _i32), ("priority", _i32),
                ("status", _i32), ("batch", _i32), ("position", _i32), ("violated", _i32),
                ("t_enqueue_ns", _i64), ("t_dispatch_ns", _i64), ("t_done_ns", _i64), ("deadline_ns", _i64),
                ("t_inf_pred_ns", _f64), ("kernel_ns", _f64), ("h2d_ns", _f64)]


class ServerStats(C.Structure):
    """strait_server_stats."""
    _fields_ = [(n, _i64) for n in ("requests", "served", "dropped", "failed", "violated_high", "violated_low",
                                    "requests_high", "requests_low", "batches", "batched_requests", "deferrals",
                                    "max_in_flight")]


def profile_model(model: "Model", prio: int, batch: int, reps: int = 30) -> BatchProfile:
    out = BatchProfile()
    _check(lib.strait_model_profile(model.handle, prio, batch, reps, C.cast(C.byref(out), _vp)))
    return out


class Server:
    """strait_server: task queues, batch formation and the scheduling / execution threads."""

    def __init__(self, sched: Scheduler, concurrency: int = 4, retry_ns: int = 200_000, submit=None, wait=None):
        """submit(batch_seq, model_id, priority, batch) / wait(batch_seq) -> (kernel_ns, h2d_ns): a host-side
        executor in place of the library's own (both or neither)."""
        self.sched = sched
        self.handle = _vp()
        self._keep = {}
        self._exec = None
        if submit is not None:
            def _s(user, seq, mid, prio, batch, ins, outs, valid):
                return int(submit(seq, mid, prio, batch) or 0)

            def _w(user, seq, k, h):
                r = wait(seq)
                if r is None:
                    return 1
                k[0], h[0] = float(r[0]), float(r[1])
                return 0
            self._exec = Executor(None, _EXEC_SUBMIT(_s), _EXEC_WAIT(_w))
        _check(lib.strait_server_create(sched.handle, concurrency, retry_ns,
                                        None if self._exec is None else C.cast(C.byref(self._exec), _vp), C.byref(self.handle)))

    def add_model(self, model: Optional["Model"], model_id: int, priority: int, max_batch: int, deadline_ns: int,
                  formation_timeout_ns: int, n_instances: int = 0):
        d = ServerModel(None if model is None else model.handle, model_id, priority, max_batch, n_instances,
                        deadline_ns, formation_timeout_ns)
        _check(lib.strait_server_add_model(self.handle, C.cast(C.byref(d), _vp)))

    def start(self):
        _check(lib.strait_server_start(self.handle))

    def request(self, model_id: int, x: Optional[np.ndarray], out: Optional[np.ndarray], valid_len: int = 0) -> int:
        rid = C.c_uint64()
        _check(lib.strait_server_request(self.handle, model_id, None if x is None else _np_ptr(x), valid_len,
                                         None if out is None else _np_ptr(out), C.byref(rid)))
        self._keep[rid.value] = (x, out)
        return rid.value

    def wait_idle(self, timeout_s: float = 30.0):
        _check(lib.strait_server_wait_idle(self.handle, int(timeout_s * 1e9)))

    def results(self, capacity: int = 4096):
        """Finished request records, oldest first (everything available, in chunks of `capacity`)."""
        out = []
        arr = (RequestRecord * capacity)()
        while True:
            n = _i32()
            _check(lib.strait_server_results(self.handle, C.cast(arr, _vp), capacity, C.byref(n)))
            for i in range(n.value):
                r = RequestRecord.from_buffer_copy(arr[i])
                self._keep.pop(r.request_id, None)
                out.append(r)
            if n.value < capacity:
                return out

    def stats(self) -> ServerStats:
        st = ServerStats()
        _check(lib.strait_server_get_stats(self.handle, C.cast(C.byref(st), _vp)))
        return st

    def stop(self):
        _check(lib.strait_server_stop(self.handle))

    def close(self):
        if self.handle:
            _check(lib.strait_server_destroy(self.handle))
            self.handle = _vp()
