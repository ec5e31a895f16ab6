"""ctypes binding of libdsp_hip.so: same names as the C ABI, argument marshalling only.

PyTorch appears here solely as the owner of device memory and streams (``tensor.data_ptr()``,
``torch.cuda.current_stream().cuda_stream``); no arithmetic of the method runs in Python.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

__all__ = [
    "DSP_FP32", "DSP_BF16", "DSPError", "lib", "lib_path", "check",
    "dsp_layer_desc", "dsp_block_desc", "make_block_desc",
    "dsp_schedule_validate", "dsp_schedule_index", "dsp_schedule_queue_elems", "dsp_schedule_waits",
    "dsp_block_init", "dsp_block_destroy", "dsp_block_forward", "dsp_block_recompute_backward",
    "dsp_param_update", "dsp_param_update_sum", "dsp_pipeline_set_optimizer", "dsp_block_input_slot",
    "dsp_pipeline_attach_gradient_probe", "dsp_pipeline_gradient_difference", "dsp_block_query", "dsp_block_output_shape",
    "dsp_block_input_shape", "dsp_block_memory", "dsp_block_get_params", "dsp_block_set_params",
    "dsp_block_get_momentum", "dsp_block_set_momentum", "dsp_block_get_grads",
    "dsp_pipeline_init", "dsp_pipeline_destroy", "dsp_pipeline_step", "dsp_pipeline_set_delay",
    "dsp_pipeline_set_graph_replay", "dsp_pipeline_set_launch_threads", "dsp_pipeline_set_single_stream", "dsp_pipeline_set_forward_streams",
    "dsp_block_enable_forward_lane", "dsp_block_step", "dsp_pipeline_set_twin_launches",
    "dsp_pipeline_sync", "dsp_pipeline_losses", "dsp_pipeline_ticks",
    "dsp_conv_forward", "dsp_conv_backward_data", "dsp_conv_backward_weight", "dsp_conv_workspace_bytes",
    "dsp_grouped_conv_forward", "dsp_grouped_conv_backward_data", "dsp_grouped_conv_backward_weight",
    "dsp_grouped_conv_workspace_bytes",
    "dsp_conv_backward_weight_static", "dsp_conv_backward_weight_static_bytes",
    "dsp_bn_workspace_bytes", "dsp_bn_forward", "dsp_bn_backward", "dsp_bn_relu_maxpool_forward", "dsp_bn_relu_backward_from_x", "dsp_bn_relu_maxpool_backward", "dsp_bn_relu_bits_bytes", "dsp_bn_forward_bits",
    "dsp_bn_backward_bits", "dsp_maxpool_forward", "dsp_maxpool_backward",
    "dsp_add_forward", "dsp_add_backward", "dsp_gap_forward", "dsp_gap_backward", "dsp_linear_forward",
    "dsp_linear_backward", "dsp_softmax_ce", "dsp_block_get_activation", "dsp_block_get_pool_argmax",
    "dsp_profile_start", "dsp_profile_stop", "dsp_profile_get",
    "dsp_strerror", "dsp_last_error", "dsp_build_id", "EXPORTED_SYMBOLS",
]

DSP_FP32, DSP_BF16 = 0, 1
_OPS = {"conv": 0, "bn": 1, "maxpool": 2, "gap": 3, "linear": 4, "softmax_ce": 5, "add": 6}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class DSPError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().dsp_last_error().decode()
        super().__init__("%s: %s%s" % (where, lib().dsp_strerror(status).decode(), (" -- " + msg) if msg else ""))


class dsp_layer_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "in0", "in1", "cin", "cout", "r", "s", "stride", "pad", "relu", "groups")]


class dsp_block_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(dsp_layer_desc)),
                ("N", C.c_int32), ("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("dtype", C.c_int32), ("k", C.c_int32), ("K", C.c_int32), ("m_k", C.c_int32),
                ("p_prev", C.c_int32), ("needs_input_grad", C.c_int32), ("bn_eps", C.c_float)]


def lib_path():
    return os.path.join(_HERE, "libdsp_hip.so")


def lib():
    """Loads the built library (building it first only if no binary exists at all)."""
    global _LIB
    if _LIB is None:
        # PyTorch owns the device memory and streams handed to the library, so both must talk to ONE
        # HIP runtime: importing torch first makes the loader bind libamdhip64.so.7 to the copy torch
        # ships (two runtimes in a process do not see each other's devices or allocations).
        import torch  # noqa: F401
        path = lib_path()
        if not os.path.exists(path):
            from . import build as _build
            _build.build(force=True)
        _LIB = C.CDLL(path)
        _declare(_LIB)
        from . import build as _build
        have, want = _LIB.dsp_build_id().decode(), _build.source_hash()
        if have != want:
            _LIB = None
            raise RuntimeError("%s was built from other sources (id %s, csrc/ + include/dsp.h now hash to %s): rebuild it "
                               "with `python -m paper_1909_02625_amd.build`" % (path, have, want))
    return _LIB


_vp, _i32, _i64, _sz, _f = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
_pi32, _pi64, _pf = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float)

_SIGNATURES = {
    "dsp_schedule_validate": [_i32, _pi32, _pi32, _pi32],
    "dsp_schedule_index": [_i32, _pi32, _pi32, _i32, _i64, _pi64],
    "dsp_schedule_queue_elems": [_i32, _pi32, _pi32, _pi64, _pi64],
    "dsp_schedule_waits": [_i32, _pi32, _pi32, _pi32, _pi32, _pi32, _pi32],
    "dsp_block_init": [C.POINTER(dsp_block_desc), _pf, _sz, C.POINTER(_vp)],
    "dsp_block_destroy": [_vp],
    "dsp_block_forward": [_vp, _i64, _vp, _vp, _vp, _vp, _vp],
    "dsp_block_recompute_backward": [_vp, _i64, _vp, _vp, _vp],
    "dsp_param_update": [_vp, _f, _f, _f, _vp],
    "dsp_param_update_sum": [_vp, _f, _f, _i32, _f, _vp],
    "dsp_pipeline_set_optimizer": [_vp, _f, _f, _i32, _f],
    "dsp_pipeline_attach_gradient_probe": [_vp, _vp],
    "dsp_pipeline_gradient_difference": [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)],
    "dsp_block_input_slot": [_vp, _i64, C.POINTER(_vp)],
    "dsp_block_query": [_vp, _pi64],
    "dsp_block_output_shape": [_vp, _pi32],
    "dsp_block_input_shape": [_vp, _pi32],
    "dsp_block_memory": [_vp, C.POINTER(_sz), C.POINTER(_sz), C.POINTER(_sz)],
    "dsp_block_get_params": [_vp, _pf, _sz],
    "dsp_block_set_params": [_vp, _pf, _sz],
    "dsp_block_get_momentum": [_vp, _pf, _sz],
    "dsp_block_set_momentum": [_vp, _pf, _sz],
    "dsp_block_get_grads": [_vp, _pf, _sz],
    "dsp_pipeline_init": [_i32, C.POINTER(_vp), _pi32, _pi32, _f, _f, _f, _i64, C.POINTER(_vp)],
    "dsp_pipeline_destroy": [_vp],
    "dsp_pipeline_step": [_vp, _vp, _vp, _pf, _pi64, _vp],
    "dsp_pipeline_set_delay": [_vp, _i32, _i32],
    "dsp_pipeline_set_graph_replay": [_vp, _i32],
    "dsp_pipeline_set_launch_threads": [_vp, _i32],
    "dsp_pipeline_set_single_stream": [_vp, _i32],
    "dsp_pipeline_set_forward_streams": [_vp, _i32],
    "dsp_block_enable_forward_lane": [_vp],
    "dsp_pipeline_set_twin_launches": [_vp, _i32],
    "dsp_block_step": [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _vp],
    "dsp_pipeline_sync": [_vp],
    "dsp_pipeline_losses": [_vp, _pf, _i64, _pi64],
    "dsp_pipeline_ticks": [_vp, _pi64],
    "dsp_conv_forward": [_i32, _vp, _vp, _vp] + [_i32] * 9 + [_vp],
    "dsp_conv_backward_data": [_i32, _vp, _vp, _vp] + [_i32] * 10 + [_vp],
    "dsp_conv_backward_weight": [_i32, _vp, _vp, _vp] + [_i32] * 9 + [_vp, _sz, _vp],
    "dsp_conv_workspace_bytes": [_i32] * 9 + [C.POINTER(_sz)],
    "dsp_grouped_conv_forward": [_i32, _vp, _vp, _vp] + [_i32] * 10 + [_vp],
    "dsp_grouped_conv_backward_data": [_i32, _vp, _vp, _vp] + [_i32] * 11 + [_vp],
    "dsp_grouped_conv_backward_weight": [_i32, _vp, _vp, _vp] + [_i32] * 10 + [_vp, _sz, _vp],
    "dsp_grouped_conv_workspace_bytes": [_i32] * 10 + [C.POINTER(_sz)],
    "dsp_conv_backward_weight_static": [_i32, _vp, _vp, _vp] + [_i32] * 9 + [_vp],
    "dsp_bn_workspace_bytes": [_i32, C.POINTER(_sz)],
    "dsp_bn_forward": [_i32, _vp, _vp, _vp, _vp, _vp, _f, _i64, _i32, _i32, _vp, _vp, _vp, _sz, _vp],
    "dsp_bn_backward": [_i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _sz, _vp],
    "dsp_bn_relu_maxpool_forward": [_i32, _vp, _vp, _vp, _f] + [_i32] * 7 + [_vp] * 6 + [_sz, _vp],
    "dsp_bn_relu_backward_from_x": [_i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _vp, _sz, _vp],
    "dsp_bn_relu_maxpool_backward": [_i32, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp] + [_i32] * 7 + [_vp, _sz, _vp],
    "dsp_bn_relu_bits_bytes": [_i32, _i64, _i32, C.POINTER(C.c_size_t)],
    "dsp_bn_forward_bits": [_i32, _vp, _vp, _vp, _vp, _vp, _f, _i64, _i32, _vp, _vp, _vp, _vp, _sz, _vp],
    "dsp_bn_backward_bits": [_i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _vp, _sz, _vp],
    "dsp_maxpool_forward": [_i32, _vp, _vp, _vp] + [_i32] * 7 + [_vp],
    "dsp_maxpool_backward": [_i32, _vp, _vp, _vp] + [_i32] * 8 + [_vp],
    "dsp_add_forward": [_i32, _vp, _vp, _vp, _i64, _vp],
    "dsp_add_backward": [_i32, _vp, _vp, _i32, _vp, _i32, _i64, _vp],
    "dsp_gap_forward": [_i32, _vp, _vp, _i32, _i32, _i32, _vp],
    "dsp_gap_backward": [_i32, _vp, _vp, _i32, _i32, _i32, _i32, _vp],
    "dsp_linear_forward": [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp],
    "dsp_linear_backward": [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp],
    "dsp_softmax_ce": [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp],
    "dsp_block_get_activation": [_vp, _i32, _vp, _sz],
    "dsp_block_get_pool_argmax": [_vp, _i32, _vp, _sz],
    "dsp_conv_backward_weight_static_bytes": [C.POINTER(_sz)],
    "dsp_profile_start": [_i32],
    "dsp_profile_stop": [_pi32],
    "dsp_profile_get": [_i32, C.c_char_p, _sz, _pi64, C.POINTER(C.c_double), C.POINTER(C.c_double), _pi32],
}
EXPORTED_SYMBOLS = sorted(list(_SIGNATURES) + ["dsp_strerror", "dsp_last_error", "dsp_build_id"])


def _declare(L):
    for name, args in _SIGNATURES.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = C.c_int
    L.dsp_strerror.argtypes = [C.c_int]
    L.dsp_strerror.restype = C.c_char_p
    L.dsp_last_error.argtypes = []
    L.dsp_last_error.restype = C.c_char_p
    L.dsp_build_id.argtypes = []
    L.dsp_build_id.restype = C.c_char_p


def check(status, where):
    if status != 0:
        raise DSPError(status, where)


def _ptr(x):
    """Device/host address of a torch tensor, numpy array, int or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return s if isinstance(s, int) else s.cuda_stream


def _i32arr(v):
    return (C.c_int32 * len(v))(*[int(a) for a in v])


def make_block_desc(layers, in_shape, dtype, k, K, m_k, p_prev=0, needs_input_grad=True, bn_eps=1e-5):
    """Marshals a layer list (dicts, see workloads.configs) and an NCHW input shape into dsp_block_desc.
    Returns (desc, keepalive)."""
    arr = (dsp_layer_desc * len(layers))()
    for d, L in zip(arr, layers):
        d.op, d.in0, d.in1 = _OPS[L["op"]], L["in"], -2
        d.cin = L.get("cin", L.get("c", 0))
        d.cout = L.get("cout", 0)
        d.r, d.s = L.get("r", L.get("k", 0)), L.get("s", L.get("k", 0))
        d.stride, d.pad = L.get("stride", 1), L.get("pad", 0)
        d.relu = int(bool(L.get("relu", False)))
        d.groups = int(L.get("groups", 1))
        if L["op"] in ("bn", "add") and L.get("res") is not None:
            d.in1 = L["res"]
    n, c, h, w = in_shape
    desc = dsp_block_desc(len(layers), arr, n, c, h, w, dtype, k, K, m_k, p_prev, int(bool(needs_input_grad)), bn_eps)
    return desc, arr


# ---- schedule ------------------------------------------------------------------------------------
def dsp_schedule_validate(p, m):
    K = len(m)
    q = (C.c_int32 * K)()
    check(lib().dsp_schedule_validate(K, _i32arr(p), _i32arr(m), q), "dsp_schedule_validate")
    return list(q)


def dsp_schedule_index(p, m, k, tau):
    out = (C.c_int64 * 7)()
    check(lib().dsp_schedule_index(len(m), _i32arr(p), _i32arr(m), k, tau, out), "dsp_schedule_index")
    return dict(zip(("a", "b", "version", "slot_fwd", "slot_bwd", "q_write", "q_read"), list(out)))


def dsp_schedule_queue_elems(p, m, h_elems):
    tot = C.c_int64()
    arr = (C.c_int64 * len(h_elems))(*h_elems)
    check(lib().dsp_schedule_queue_elems(len(m), _i32arr(p), _i32arr(m), arr, C.byref(tot)), "dsp_schedule_queue_elems")
    return tot.value


def dsp_schedule_waits(p, m, spare=None):
    """Returns (wait_down[K], wait_up[K], label_slots)."""
    K = len(m)
    dn, up, lab = (C.c_int32 * K)(), (C.c_int32 * K)(), C.c_int32()
    check(lib().dsp_schedule_waits(K, _i32arr(p), _i32arr(m), None if spare is None else _i32arr(spare), dn, up,
                                   C.byref(lab)), "dsp_schedule_waits")
    return list(dn), list(up), lab.value


# ---- block -----------------------------------------------------------------------------------------
def dsp_block_init(desc, h_params):
    hp = np.ascontiguousarray(h_params, dtype=np.float32)
    out = C.c_void_p()
    check(lib().dsp_block_init(C.byref(desc), hp.ctypes.data_as(_pf), hp.size, C.byref(out)), "dsp_block_init")
    return out.value


def dsp_block_destroy(b):
    check(lib().dsp_block_destroy(b), "dsp_block_destroy")


def dsp_block_forward(b, batch_id, d_in, d_out=None, d_labels=None, d_loss=None, stream=None):
    check(lib().dsp_block_forward(b, batch_id, _ptr(d_in), _ptr(d_out), _ptr(d_labels), _ptr(d_loss), _stream(stream)),
          "dsp_block_forward")


def dsp_block_recompute_backward(b, batch_id, d_grad_out=None, d_grad_in=None, stream=None):
    check(lib().dsp_block_recompute_backward(b, batch_id, _ptr(d_grad_out), _ptr(d_grad_in), _stream(stream)),
          "dsp_block_recompute_backward")


def dsp_block_step(b, batch_fwd, d_in, d_out=None, d_labels=None, d_loss=None, batch_bwd=0, d_grad_out=None,
                   d_grad_in=None, stream=None):
    check(lib().dsp_block_step(b, batch_fwd, _ptr(d_in), _ptr(d_out), _ptr(d_labels), _ptr(d_loss), batch_bwd,
                               _ptr(d_grad_out), _ptr(d_grad_in), _stream(stream)), "dsp_block_step")


def dsp_param_update(b, lr, momentum, weight_decay=0.0, stream=None):
    check(lib().dsp_param_update(b, lr, momentum, weight_decay, _stream(stream)), "dsp_param_update")


def dsp_param_update_sum(b, lr, momentum, s=0, weight_decay=0.0, stream=None):
    check(lib().dsp_param_update_sum(b, lr, momentum, int(s), weight_decay, _stream(stream)), "dsp_param_update_sum")


def dsp_pipeline_set_optimizer(pl, lr, momentum, s=0, weight_decay=0.0):
    check(lib().dsp_pipeline_set_optimizer(pl, lr, momentum, int(s), weight_decay), "dsp_pipeline_set_optimizer")


def dsp_pipeline_attach_gradient_probe(pl, probe):
    check(lib().dsp_pipeline_attach_gradient_probe(pl, probe), "dsp_pipeline_attach_gradient_probe")


def dsp_pipeline_gradient_difference(pl, K):
    """(batch_id, diff_sumsq[K], bp_sumsq[K]) of the latest step; batch_id = -1 while there is none."""
    bid = C.c_int64(-1)
    diff, ref = (C.c_double * K)(), (C.c_double * K)()
    check(lib().dsp_pipeline_gradient_difference(pl, C.byref(bid), diff, ref), "dsp_pipeline_gradient_difference")
    return bid.value, np.array(diff[:], np.float64), np.array(ref[:], np.float64)


def dsp_block_input_slot(b, batch_id):
    out = C.c_void_p()
    check(lib().dsp_block_input_slot(b, batch_id, C.byref(out)), "dsp_block_input_slot")
    return out.value


def dsp_block_query(b):
    out = (C.c_int64 * 8)()
    check(lib().dsp_block_query(b, out), "dsp_block_query")
    return dict(zip(("version", "next_fwd", "next_bwd", "ring_entries", "pending", "n_params", "fwd_version_of_next_bwd",
                     "slot_of_next_bwd"), list(out)))


def dsp_block_output_shape(b):
    out = (C.c_int32 * 5)()
    check(lib().dsp_block_output_shape(b, out), "dsp_block_output_shape")
    return tuple(out[:4]), bool(out[4])


def dsp_block_input_shape(b):
    out = (C.c_int32 * 5)()
    check(lib().dsp_block_input_shape(b, out), "dsp_block_input_shape")
    return tuple(out[:4]), out[4]


def dsp_block_memory(b):
    r, w, p = C.c_size_t(), C.c_size_t(), C.c_size_t()
    check(lib().dsp_block_memory(b, C.byref(r), C.byref(w), C.byref(p)), "dsp_block_memory")
    return {"ring": r.value, "workspace": w.value, "params": p.value}


def _get(fn, name, b):
    n = dsp_block_query(b)["n_params"]
    out = np.empty(n, np.float32)
    check(fn(b, out.ctypes.data_as(_pf), n), name)
    return out


def _set(fn, name, b, h):
    h = np.ascontiguousarray(h, dtype=np.float32)
    check(fn(b, h.ctypes.data_as(_pf), h.size), name)


def dsp_block_get_params(b):
    return _get(lib().dsp_block_get_params, "dsp_block_get_params", b)


def dsp_block_set_params(b, h):
    _set(lib().dsp_block_set_params, "dsp_block_set_params", b, h)


def dsp_block_get_momentum(b):
    return _get(lib().dsp_block_get_momentum, "dsp_block_get_momentum", b)


def dsp_block_set_momentum(b, h):
    _set(lib().dsp_block_set_momentum, "dsp_block_set_momentum", b, h)


def dsp_block_get_grads(b):
    return _get(lib().dsp_block_get_grads, "dsp_block_get_grads", b)


# ---- pipeline --------------------------------------------------------------------------------------
def dsp_pipeline_init(blocks, p, m, lr, momentum, weight_decay, max_ticks):
    K = len(blocks)
    arr = (C.c_void_p * K)(*blocks)
    out = C.c_void_p()
    check(lib().dsp_pipeline_init(K, arr, _i32arr(p), _i32arr(m), lr, momentum, weight_decay, max_ticks, C.byref(out)),
          "dsp_pipeline_init")
    return out.value


def dsp_pipeline_destroy(pl):
    check(lib().dsp_pipeline_destroy(pl), "dsp_pipeline_destroy")


def dsp_pipeline_step(pl, d_batch, d_labels, want_loss=False, stream=None):
    """Returns (loss or None, loss_batch_id)."""
    bid = C.c_int64(-1)
    loss = C.c_float(0.0)
    check(lib().dsp_pipeline_step(pl, _ptr(d_batch), _ptr(d_labels), C.byref(loss) if want_loss else None, C.byref(bid),
                                  _stream(stream)), "dsp_pipeline_step")
    return (loss.value if (want_loss and bid.value >= 0) else None), bid.value


def dsp_pipeline_set_delay(pl, k, microseconds):
    check(lib().dsp_pipeline_set_delay(pl, k, microseconds), "dsp_pipeline_set_delay")


def dsp_pipeline_set_graph_replay(pl, enable):
    check(lib().dsp_pipeline_set_graph_replay(pl, int(bool(enable))), "dsp_pipeline_set_graph_replay")


def dsp_pipeline_set_launch_threads(pl, enable):
    check(lib().dsp_pipeline_set_launch_threads(pl, int(bool(enable))), "dsp_pipeline_set_launch_threads")


def dsp_pipeline_set_single_stream(pl, enable):
    check(lib().dsp_pipeline_set_single_stream(pl, int(bool(enable))), "dsp_pipeline_set_single_stream")


def dsp_pipeline_set_forward_streams(pl, enable):
    check(lib().dsp_pipeline_set_forward_streams(pl, int(bool(enable))), "dsp_pipeline_set_forward_streams")


def dsp_pipeline_set_twin_launches(pl, enable):
    check(lib().dsp_pipeline_set_twin_launches(pl, int(bool(enable))), "dsp_pipeline_set_twin_launches")


def dsp_block_enable_forward_lane(b):
    check(lib().dsp_block_enable_forward_lane(b), "dsp_block_enable_forward_lane")


def dsp_pipeline_sync(pl):
    check(lib().dsp_pipeline_sync(pl), "dsp_pipeline_sync")


def dsp_pipeline_losses(pl):
    avail = C.c_int64()
    check(lib().dsp_pipeline_losses(pl, None, 0, C.byref(avail)), "dsp_pipeline_losses")
    out = np.empty(avail.value, np.float32)
    if avail.value:
        check(lib().dsp_pipeline_losses(pl, out.ctypes.data_as(_pf), avail.value, None), "dsp_pipeline_losses")
    return out


def dsp_pipeline_ticks(pl):
    t = C.c_int64()
    check(lib().dsp_pipeline_ticks(pl, C.byref(t)), "dsp_pipeline_ticks")
    return t.value


# ---- single layers ---------------------------------------------------------------------------------
def dsp_grouped_conv_forward(dtype, d_x, d_w, d_y, N, H, W, cin, cout, r, s, stride, pad, groups, stream=None):
    check(lib().dsp_grouped_conv_forward(dtype, _ptr(d_x), _ptr(d_w), _ptr(d_y), N, H, W, cin, cout, r, s, stride, pad, groups,
                                         _stream(stream)), "dsp_grouped_conv_forward")


def dsp_grouped_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, cin, cout, r, s, stride, pad, groups, accumulate=False,
                                   stream=None):
    check(lib().dsp_grouped_conv_backward_data(dtype, _ptr(d_dy), _ptr(d_wt), _ptr(d_dx), N, H, W, cin, cout, r, s, stride, pad,
                                               groups, int(accumulate), _stream(stream)), "dsp_grouped_conv_backward_data")


def dsp_grouped_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, cin, cout, r, s, stride, pad, groups, d_workspace,
                                     workspace_bytes, stream=None):
    check(lib().dsp_grouped_conv_backward_weight(dtype, _ptr(d_x), _ptr(d_dy), _ptr(d_dw), N, H, W, cin, cout, r, s, stride, pad,
                                                 groups, _ptr(d_workspace), workspace_bytes, _stream(stream)),
          "dsp_grouped_conv_backward_weight")


def dsp_grouped_conv_workspace_bytes(N, H, W, cin, cout, r, s, stride, pad, groups):
    out = C.c_size_t()
    check(lib().dsp_grouped_conv_workspace_bytes(N, H, W, cin, cout, r, s, stride, pad, groups, C.byref(out)),
          "dsp_grouped_conv_workspace_bytes")
    return out.value


def dsp_conv_forward(dtype, d_x, d_w, d_y, N, H, W, cin, cout, r, s, stride, pad, stream=None):
    check(lib().dsp_conv_forward(dtype, _ptr(d_x), _ptr(d_w), _ptr(d_y), N, H, W, cin, cout, r, s, stride, pad,
                                 _stream(stream)), "dsp_conv_forward")


def dsp_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, cin, cout, r, s, stride, pad, accumulate=False, stream=None):
    check(lib().dsp_conv_backward_data(dtype, _ptr(d_dy), _ptr(d_wt), _ptr(d_dx), N, H, W, cin, cout, r, s, stride, pad,
                                       int(accumulate), _stream(stream)), "dsp_conv_backward_data")


def dsp_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, cin, cout, r, s, stride, pad, d_workspace, workspace_bytes,
                             stream=None):
    check(lib().dsp_conv_backward_weight(dtype, _ptr(d_x), _ptr(d_dy), _ptr(d_dw), N, H, W, cin, cout, r, s, stride, pad,
                                         _ptr(d_workspace), workspace_bytes, _stream(stream)), "dsp_conv_backward_weight")


def dsp_conv_workspace_bytes(N, H, W, cin, cout, r, s, stride, pad):
    out = C.c_size_t()
    check(lib().dsp_conv_workspace_bytes(N, H, W, cin, cout, r, s, stride, pad, C.byref(out)), "dsp_conv_workspace_bytes")
    return out.value


def dsp_conv_backward_weight_static(dtype, d_x, d_dy, d_dw, N, H, W, cin, cout, r, s, stride, pad, stream=None):
    check(lib().dsp_conv_backward_weight_static(dtype, _ptr(d_x), _ptr(d_dy), _ptr(d_dw), N, H, W, cin, cout, r, s, stride, pad,
                                                _stream(stream)), "dsp_conv_backward_weight_static")


def dsp_conv_backward_weight_static_bytes():
    out = C.c_size_t()
    check(lib().dsp_conv_backward_weight_static_bytes(C.byref(out)), "dsp_conv_backward_weight_static_bytes")
    return out.value


def dsp_bn_workspace_bytes(C_):
    out = C.c_size_t()
    check(lib().dsp_bn_workspace_bytes(C_, C.byref(out)), "dsp_bn_workspace_bytes")
    return out.value


def dsp_bn_forward(dtype, d_x, d_res, d_y, d_gamma, d_beta, eps, M, C_, relu, d_mean, d_invstd, d_workspace, workspace_bytes,
                   stream=None):
    check(lib().dsp_bn_forward(dtype, _ptr(d_x), _ptr(d_res), _ptr(d_y), _ptr(d_gamma), _ptr(d_beta), eps, M, C_, int(relu),
                               _ptr(d_mean), _ptr(d_invstd), _ptr(d_workspace), workspace_bytes, _stream(stream)),
          "dsp_bn_forward")


def dsp_bn_backward(dtype, d_dy, d_x, d_y, d_dx, d_dres, dres_accumulate, dx_accumulate, d_gamma, d_mean, d_invstd, d_dgamma,
                    d_dbeta, M, C_, relu, d_workspace, workspace_bytes, stream=None):
    check(lib().dsp_bn_backward(dtype, _ptr(d_dy), _ptr(d_x), _ptr(d_y), _ptr(d_dx), _ptr(d_dres), int(dres_accumulate),
                                int(dx_accumulate), _ptr(d_gamma), _ptr(d_mean), _ptr(d_invstd), _ptr(d_dgamma),
                                _ptr(d_dbeta), M, C_, int(relu), _ptr(d_workspace), workspace_bytes, _stream(stream)),
          "dsp_bn_backward")


def dsp_bn_relu_maxpool_forward(dtype, d_x, d_gamma, d_beta, eps, N, H, W, C_, k, stride, pad, d_pool, d_argmax, d_mean, d_invstd,
                                d_scale_shift, d_workspace, workspace_bytes, stream=None):
    check(lib().dsp_bn_relu_maxpool_forward(dtype, _ptr(d_x), _ptr(d_gamma), _ptr(d_beta), eps, N, H, W, C_, k, stride, pad,
                                            _ptr(d_pool), _ptr(d_argmax), _ptr(d_mean), _ptr(d_invstd), _ptr(d_scale_shift),
                                            _ptr(d_workspace), workspace_bytes, _stream(stream)), "dsp_bn_relu_maxpool_forward")


def dsp_bn_relu_backward_from_x(dtype, d_dy, d_x, d_scale_shift, d_dx, dx_accumulate, d_gamma, d_mean, d_invstd, d_dgamma, d_dbeta,
                                M, C_, d_workspace, workspace_bytes, stream=None):
    check(lib().dsp_bn_relu_backward_from_x(dtype, _ptr(d_dy), _ptr(d_x), _ptr(d_scale_shift), _ptr(d_dx), int(dx_accumulate),
                                            _ptr(d_gamma), _ptr(d_mean), _ptr(d_invstd), _ptr(d_dgamma), _ptr(d_dbeta), M, C_,
                                            _ptr(d_workspace), workspace_bytes, _stream(stream)), "dsp_bn_relu_backward_from_x")


def dsp_bn_relu_bits_bytes(dtype, M, C_):
    n = C.c_size_t(0)
    check(lib().dsp_bn_relu_bits_bytes(dtype, M, C_, C.byref(n)), "dsp_bn_relu_bits_bytes")
    return int(n.value)


def dsp_bn_forward_bits(dtype, d_x, d_res, d_y, d_gamma, d_beta, eps, M, C_, d_mean, d_invstd, d_relu_bits, d_workspace,
                        workspace_bytes, stream=None):
    check(lib().dsp_bn_forward_bits(dtype, _ptr(d_x), _ptr(d_res), _ptr(d_y), _ptr(d_gamma), _ptr(d_beta), eps, M, C_, _ptr(d_mean),
                                    _ptr(d_invstd), _ptr(d_relu_bits), _ptr(d_workspace), workspace_bytes, _stream(stream)),
          "dsp_bn_forward_bits")


def dsp_bn_backward_bits(dtype, d_dy, d_x, d_relu_bits, d_dx, d_dres, dres_accumulate, dx_accumulate, d_gamma, d_mean, d_invstd,
                         d_dgamma, d_dbeta, M, C_, d_workspace, workspace_bytes, stream=None):
    check(lib().dsp_bn_backward_bits(dtype, _ptr(d_dy), _ptr(d_x), _ptr(d_relu_bits), _ptr(d_dx), _ptr(d_dres), int(dres_accumulate),
                                     int(dx_accumulate), _ptr(d_gamma), _ptr(d_mean), _ptr(d_invstd), _ptr(d_dgamma), _ptr(d_dbeta),
                                     M, C_, _ptr(d_workspace), workspace_bytes, _stream(stream)), "dsp_bn_backward_bits")


def dsp_bn_relu_maxpool_backward(dtype, d_dpool, d_argmax, d_x, d_scale_shift, d_dx, dx_accumulate, d_gamma, d_mean, d_invstd,
                                 d_dgamma, d_dbeta, N, H, W, C_, k, stride, pad, d_workspace, workspace_bytes, stream=None):
    check(lib().dsp_bn_relu_maxpool_backward(dtype, _ptr(d_dpool), _ptr(d_argmax), _ptr(d_x), _ptr(d_scale_shift), _ptr(d_dx),
                                             int(dx_accumulate), _ptr(d_gamma), _ptr(d_mean), _ptr(d_invstd), _ptr(d_dgamma),
                                             _ptr(d_dbeta), N, H, W, C_, k, stride, pad, _ptr(d_workspace), workspace_bytes,
                                             _stream(stream)), "dsp_bn_relu_maxpool_backward")


def dsp_maxpool_forward(dtype, d_x, d_y, d_argmax, N, H, W, C_, k, stride, pad, stream=None):
    check(lib().dsp_maxpool_forward(dtype, _ptr(d_x), _ptr(d_y), _ptr(d_argmax), N, H, W, C_, k, stride, pad, _stream(stream)),
          "dsp_maxpool_forward")


def dsp_maxpool_backward(dtype, d_dy, d_argmax, d_dx, accumulate, N, H, W, C_, k, stride, pad, stream=None):
    check(lib().dsp_maxpool_backward(dtype, _ptr(d_dy), _ptr(d_argmax), _ptr(d_dx), int(accumulate), N, H, W, C_, k, stride,
                                     pad, _stream(stream)), "dsp_maxpool_backward")


def dsp_add_forward(dtype, d_a, d_b, d_y, n, stream=None):
    check(lib().dsp_add_forward(dtype, _ptr(d_a), _ptr(d_b), _ptr(d_y), n, _stream(stream)), "dsp_add_forward")


def dsp_add_backward(dtype, d_dy, d_da, da_accumulate, d_db, db_accumulate, n, stream=None):
    check(lib().dsp_add_backward(dtype, _ptr(d_dy), _ptr(d_da), int(da_accumulate), _ptr(d_db), int(db_accumulate), n,
                                 _stream(stream)), "dsp_add_backward")


def dsp_gap_forward(dtype, d_x, d_y, N, HW, C_, stream=None):
    check(lib().dsp_gap_forward(dtype, _ptr(d_x), _ptr(d_y), N, HW, C_, _stream(stream)), "dsp_gap_forward")


def dsp_gap_backward(dtype, d_dy, d_dx, accumulate, N, HW, C_, stream=None):
    check(lib().dsp_gap_backward(dtype, _ptr(d_dy), _ptr(d_dx), int(accumulate), N, HW, C_, _stream(stream)), "dsp_gap_backward")


def dsp_linear_forward(d_x, d_w, d_bias, d_z, N, cin, cout, stream=None):
    check(lib().dsp_linear_forward(_ptr(d_x), _ptr(d_w), _ptr(d_bias), _ptr(d_z), N, cin, cout, _stream(stream)),
          "dsp_linear_forward")


def dsp_linear_backward(d_x, d_w, d_dz, d_dx, d_dw, d_dbias, N, cin, cout, stream=None):
    check(lib().dsp_linear_backward(_ptr(d_x), _ptr(d_w), _ptr(d_dz), _ptr(d_dx), _ptr(d_dw), _ptr(d_dbias), N, cin, cout,
                                    _stream(stream)), "dsp_linear_backward")


def dsp_softmax_ce(d_z, d_labels, d_loss, d_dz, d_row_loss, N, C_, stream=None):
    check(lib().dsp_softmax_ce(_ptr(d_z), _ptr(d_labels), _ptr(d_loss), _ptr(d_dz), _ptr(d_row_loss), N, C_, _stream(stream)),
          "dsp_softmax_ce")


def dsp_block_get_activation(b, layer, nbytes):
    """Raw bytes (numpy uint8) of the output layer ``layer`` left in the buffers the backward sweep reads."""
    out = np.empty(nbytes, np.uint8)
    check(lib().dsp_block_get_activation(b, layer, out.ctypes.data, nbytes), "dsp_block_get_activation")
    return out


def dsp_block_get_pool_argmax(b, layer, nbytes):
    out = np.empty(nbytes, np.uint8)
    check(lib().dsp_block_get_pool_argmax(b, layer, out.ctypes.data, nbytes), "dsp_block_get_pool_argmax")
    return out


def dsp_profile_start(max_launches):
    check(lib().dsp_profile_start(max_launches), "dsp_profile_start")


def dsp_profile_stop():
    """Returns the per-kernel table: list of dicts (name, launches, ms, units, unit_kind)."""
    n = C.c_int32()
    check(lib().dsp_profile_stop(C.byref(n)), "dsp_profile_stop")
    return [dsp_profile_get(i) for i in range(n.value)]


def dsp_profile_get(i):
    name = C.create_string_buffer(128)
    launches, ms, units, kind = C.c_int64(), C.c_double(), C.c_double(), C.c_int32()
    check(lib().dsp_profile_get(i, name, 128, C.byref(launches), C.byref(ms), C.byref(units), C.byref(kind)),
          "dsp_profile_get")
    return {"name": name.value.decode(), "launches": launches.value, "ms": ms.value, "units": units.value,
            "unit_kind": "flop" if kind.value == 0 else "byte"}


def dsp_strerror(status):
    return lib().dsp_strerror(status).decode()


def dsp_last_error():
    return lib().dsp_last_error().decode()


def dsp_build_id():
    return lib().dsp_build_id().decode()
