"""ctypes binding of libparle.so: the same names as include/parle.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch appears here only to
allocate device memory and to name the HIP stream.  If the library has not been built the
import of :func:`lib` fails loudly; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libparle.so")

PARLE_OK, PARLE_EINVAL, PARLE_ENOMEM, PARLE_EALIGN, PARLE_ESIZE, PARLE_EHIP, PARLE_ESTATE, PARLE_ENONFINITE = (
    0, -1, -2, -3, -4, -5, -6, -7)
MODEL_FLAT, MODEL_MLP, MODEL_LENET, MODEL_ALLCNN_C, MODEL_WRN = 0, 1, 2, 3, 4
ALG_PARLE, ALG_ELASTIC = 0, 1
SEG_KINDS = {0: "weight", 1: "bias", 2: "bn_gamma", 3: "bn_beta"}


class parle_config(C.Structure):
    _fields_ = [("model", C.c_int32), ("n_replicas", C.c_int32), ("batch", C.c_int32), ("L", C.c_int32),
                ("compute_bf16", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32), ("n_classes", C.c_int32),
                ("arch", C.c_int32 * 4),
                ("n_params", C.c_int64),
                ("eta_inner", C.c_float), ("eta_outer", C.c_float), ("momentum", C.c_float), ("alpha", C.c_float),
                ("weight_decay", C.c_float),
                ("gamma0", C.c_float), ("rho0", C.c_float), ("gamma_max", C.c_float), ("rho_max", C.c_float),
                ("scoping_B", C.c_int64),
                ("xa_mode", C.c_int32), ("xref_mode", C.c_int32), ("reset_flags", C.c_int32),
                ("fuse_outer", C.c_int32), ("algorithm", C.c_int32), ("graph_block", C.c_int32),
                ("dropout", C.c_float), ("lenet_bn", C.c_int32), ("dropout_seed", C.c_int64)]


class parle_sizes(C.Structure):
    _fields_ = [("n_params", C.c_int64), ("n_pad", C.c_int64), ("state_bytes", C.c_int64),
                ("shadow_bytes", C.c_int64), ("bn_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("n_segments", C.c_int32), ("image_elems", C.c_int32),
                ("forward_flops_per_image", C.c_int64)]


class parle_segment(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("offset", C.c_int64), ("size", C.c_int64), ("kind", C.c_int32),
                ("shape", C.c_int32 * 4), ("fan_in", C.c_int32)]


class parle_buffers(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("z", C.c_void_p), ("vy", C.c_void_p), ("vx", C.c_void_p),
                ("grad", C.c_void_p), ("x_ref", C.c_void_p), ("y_bf16", C.c_void_p), ("bn_stats", C.c_void_p),
                ("workspace", C.c_void_p)]


class parle_conv_desc(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("dtype", "n", "batch", "h", "w", "cin", "cout", "k", "stride", "pad")]


class parle_act_desc(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("dtype", "n", "batch", "h", "w", "c")]


_lib = None

_SIGNATURES = {
    "parle_query_sizes": [C.POINTER(parle_config), C.POINTER(parle_sizes)],
    "parle_query_layout": [C.POINTER(parle_config), C.c_int32, C.POINTER(parle_segment)],
    "parle_init": [C.POINTER(parle_config), C.POINTER(parle_buffers), C.c_void_p, C.POINTER(C.c_void_p)],
    "parle_inner_step": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "parle_inner_block": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p],
    "parle_outer_step": [C.c_void_p],
    "parle_eval": [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_float),
                   C.POINTER(C.c_int32), C.POINTER(C.c_float)],
    "parle_get_state": [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_float),
                        C.POINTER(C.c_float)],
    "parle_set_state": [C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_float],
    "parle_k_inner_update": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_float, C.c_float],
    "parle_k_elastic_step": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_float, C.c_float],
    "parle_k_replica_mean": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p],
    "parle_k_outer_update": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float, C.c_float, C.c_float,
                             C.c_int32, C.c_int32, C.c_int32],
    "parle_k_spread": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "parle_k_spread_static": [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p],
    "parle_k_stream_reference": [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p],
    "parle_k_conv_forward": [C.c_void_p, C.POINTER(parle_conv_desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_int32, C.c_void_p],
    "parle_k_conv_forward_colsums": [C.c_void_p, C.POINTER(parle_conv_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)],
    "parle_k_conv_backward_data": [C.c_void_p, C.POINTER(parle_conv_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_int32, C.c_void_p, C.c_void_p],
    "parle_k_conv_backward_weight": [C.c_void_p, C.POINTER(parle_conv_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_void_p],
    "parle_k_conv_backward_weight_bias": [C.c_void_p, C.POINTER(parle_conv_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_int64, C.c_void_p, C.POINTER(C.c_int32)],
    "parle_k_bn_forward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                           C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p],
    "parle_k_bn_backward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "parle_k_maxpool_forward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p],
    "parle_k_maxpool_backward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p],
    "parle_k_gap_forward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_int32, C.c_void_p, C.c_void_p],
    "parle_k_gap_backward": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p],
    "parle_k_dropout": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_int32,
                        C.c_float, C.c_void_p],
    "parle_k_bias_grad": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p],
    "parle_k_softmax_xent": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                             C.c_void_p],
    "parle_k_gap_head": [C.c_void_p, C.POINTER(parle_act_desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                         C.c_void_p, C.c_void_p],
    "parle_k_fc_head": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                        C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
}
EXPORTS = sorted(list(_SIGNATURES) + ["parle_last_error", "parle_destroy", "parle_k_conv_scratch_bytes",
                                         "parle_k_layer_scratch_bytes"])


def lib():
    """The loaded library; raises if it has not been built (run ``python -m paper_1707_00424_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1707_00424_amd.build`; "
                               "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        for name, args in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.parle_last_error.argtypes = [C.c_void_p]
        L.parle_last_error.restype = C.c_char_p
        L.parle_destroy.argtypes = [C.c_void_p]
        L.parle_destroy.restype = None
        L.parle_k_conv_scratch_bytes.argtypes = [C.POINTER(parle_conv_desc)]
        L.parle_k_conv_scratch_bytes.restype = C.c_int64
        L.parle_k_layer_scratch_bytes.argtypes = [C.POINTER(parle_act_desc)]
        L.parle_k_layer_scratch_bytes.restype = C.c_int64
        _lib = L
    return _lib


class ParleError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"parle status {status}: {msg}")
        self.status = status


def _check(status, ctx=None):
    if status != PARLE_OK:
        msg = lib().parle_last_error(ctx)
        raise ParleError(status, msg.decode() if msg else "")


def make_config(model=MODEL_FLAT, n_replicas=1, batch=0, L=25, compute_bf16=0, in_h=0, in_w=0, in_c=0, n_classes=0,
                arch=(0, 0, 0, 0), n_params=0, eta_inner=0.1, eta_outer=0.1, momentum=0.9, alpha=0.75,
                weight_decay=0.0, gamma0=0.01, rho0=1.0, gamma_max=1.0, rho_max=10.0, scoping_B=0, xa_mode=0,
                xref_mode=0, reset_flags=3, fuse_outer=0, algorithm=ALG_PARLE, graph_block=0, dropout=0.0,
                lenet_bn=0, dropout_seed=0) -> parle_config:
    a = list(arch) + [0] * (4 - len(arch))
    return parle_config(model, n_replicas, batch, L, compute_bf16, in_h, in_w, in_c, n_classes, (C.c_int32 * 4)(*a),
                        n_params, eta_inner, eta_outer, momentum, alpha, weight_decay, gamma0, rho0, gamma_max,
                        rho_max, scoping_B, xa_mode, xref_mode, reset_flags, fuse_outer, algorithm, graph_block, dropout,
                        lenet_bn, dropout_seed)


def parle_query_sizes(cfg: parle_config) -> parle_sizes:
    out = parle_sizes()
    _check(lib().parle_query_sizes(C.byref(cfg), C.byref(out)))
    return out


def parle_query_layout(cfg: parle_config):
    """All segments as dicts (name, offset, size, kind, shape, fan_in), in packing order."""
    n = parle_query_sizes(cfg).n_segments
    segs = []
    for i in range(n):
        s = parle_segment()
        _check(lib().parle_query_layout(C.byref(cfg), i, C.byref(s)))
        shape = tuple(int(v) for v in s.shape if v > 0)
        segs.append(dict(name=s.name.decode(), offset=int(s.offset), size=int(s.size), kind=SEG_KINDS[s.kind],
                         shape=shape, fan_in=int(s.fan_in)))
    return segs


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def parle_k_inner_update(grad, x, y, vy, z, y_bf16, eta_inner, momentum, alpha, weight_decay, g, stream=None):
    n, n_pad = x.shape
    _check(lib().parle_k_inner_update(_stream_handle(stream), n, n_pad, _ptr(grad), _ptr(x), _ptr(y), _ptr(vy),
                                      _ptr(z), _ptr(y_bf16), eta_inner, momentum, alpha, weight_decay, g))


def parle_k_elastic_step(grad, xa, v, x_ref, xa_bf16, eta, eta_ref, momentum, weight_decay, r, stream=None):
    n, n_pad = xa.shape
    _check(lib().parle_k_elastic_step(_stream_handle(stream), n, n_pad, _ptr(grad), _ptr(xa), _ptr(v), _ptr(x_ref),
                                      _ptr(xa_bf16), eta, eta_ref, momentum, weight_decay, r))


def parle_k_replica_mean(x, x_ref, stream=None):
    n, n_pad = x.shape
    _check(lib().parle_k_replica_mean(_stream_handle(stream), n, n_pad, _ptr(x), _ptr(x_ref)))


def parle_k_outer_update(x, z, vx, y, vy, x_ref, y_bf16, eta_outer, momentum, c_z, r, reset_flags=3, fuse_mean=0,
                         lagged=0, stream=None):
    n, n_pad = x.shape
    _check(lib().parle_k_outer_update(_stream_handle(stream), n, n_pad, _ptr(x), _ptr(z), _ptr(vx), _ptr(y),
                                      _ptr(vy), _ptr(x_ref), _ptr(y_bf16), eta_outer, momentum, c_z, r, reset_flags,
                                      fuse_mean, lagged))


def parle_k_stream_reference(reads, writes, count, src, dst, stream=None):
    _check(lib().parle_k_stream_reference(_stream_handle(stream), reads, writes, count, _ptr(src), _ptr(dst)))


def parle_k_spread(x, x_ref, partial, out, stream=None):
    n, n_pad = x.shape
    _check(lib().parle_k_spread(_stream_handle(stream), n, n_pad, _ptr(x), _ptr(x_ref), _ptr(partial), _ptr(out)))


def parle_k_spread_static(x, x_ref, out, stream=None):
    n, n_pad = x.shape
    _check(lib().parle_k_spread_static(_stream_handle(stream), n, n_pad, _ptr(x), _ptr(x_ref), _ptr(out)))


def parle_k_conv_forward(desc, x, w, bias, resid, relu, y, stream=None):
    _check(lib().parle_k_conv_forward(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(resid),
                                      int(relu), _ptr(y)))


def parle_k_conv_forward_colsums(desc, x, w, resid, y, partial, capacity, stream=None):
    """Returns S, the number of partial rows per replica written to ``partial`` (0: none taken)."""
    splits = C.c_int32(0)
    _check(lib().parle_k_conv_forward_colsums(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(w), _ptr(resid),
                                              _ptr(y), _ptr(partial), int(capacity), C.byref(splits)))
    return splits.value


def parle_k_conv_backward_data(desc, dy, w, relu_mask, accumulate, wt_scratch, dx, stream=None):
    _check(lib().parle_k_conv_backward_data(_stream_handle(stream), C.byref(desc), _ptr(dy), _ptr(w), _ptr(relu_mask),
                                            int(accumulate), _ptr(wt_scratch), _ptr(dx)))


def parle_k_conv_backward_weight(desc, dy, x, scratch, dw, stream=None):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib().parle_k_conv_backward_weight(_stream_handle(stream), C.byref(desc), _ptr(dy), _ptr(x), _ptr(scratch),
                                              nbytes, _ptr(dw)))


def parle_k_conv_backward_weight_bias(desc, dy, x, scratch, dwb, stream=None) -> bool:
    """Returns whether the bias gradient was written behind each replica's weight gradient."""
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    took = C.c_int32(-1)
    _check(lib().parle_k_conv_backward_weight_bias(_stream_handle(stream), C.byref(desc), _ptr(dy), _ptr(x),
                                                   _ptr(scratch), nbytes, _ptr(dwb), C.byref(took)))
    return bool(took.value)


def parle_k_conv_scratch_bytes(desc) -> int:
    return int(lib().parle_k_conv_scratch_bytes(C.byref(desc)))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def parle_k_layer_scratch_bytes(desc) -> int:
    return int(lib().parle_k_layer_scratch_bytes(C.byref(desc)))


def parle_k_bn_forward(desc, x, gamma, beta, scratch, saved, running, out, stream=None):
    _check(lib().parle_k_bn_forward(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(scratch),
                                    _nbytes(scratch), _ptr(saved), _ptr(running), _ptr(out)))


def parle_k_bn_backward(desc, x, dout, gamma, beta, saved, add, scratch, sums, dgamma, dbeta, dx, stream=None):
    _check(lib().parle_k_bn_backward(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(dout), _ptr(gamma), _ptr(beta),
                                     _ptr(saved), _ptr(add), _ptr(scratch), _nbytes(scratch), _ptr(sums), _ptr(dgamma),
                                     _ptr(dbeta), _ptr(dx)))


def parle_k_maxpool_forward(desc, x, out, stream=None):
    _check(lib().parle_k_maxpool_forward(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(out)))


def parle_k_maxpool_backward(desc, x, dout, relu_mask, din, stream=None):
    _check(lib().parle_k_maxpool_backward(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(dout), int(relu_mask),
                                          _ptr(din)))


def parle_k_gap_forward(desc, out_f32, x, out, stream=None):
    _check(lib().parle_k_gap_forward(_stream_handle(stream), C.byref(desc), int(out_f32), _ptr(x), _ptr(out)))


def parle_k_gap_backward(desc, dout, din, stream=None):
    _check(lib().parle_k_gap_backward(_stream_handle(stream), C.byref(desc), _ptr(dout), _ptr(din)))


def parle_k_dropout(desc, x, relu_src, seed, step_dev, site, p, out, stream=None):
    _check(lib().parle_k_dropout(_stream_handle(stream), C.byref(desc), _ptr(x), _ptr(relu_src), int(seed), _ptr(step_dev),
                                 int(site), float(p), _ptr(out)))


def parle_k_bias_grad(desc, dy, scratch, grad, stream=None):
    _check(lib().parle_k_bias_grad(_stream_handle(stream), C.byref(desc), _ptr(dy), _ptr(scratch), _nbytes(scratch),
                                   _ptr(grad)))


def parle_k_softmax_xent(dtype, logits, labels, loss, dlogits, stream=None):
    n, batch, classes = logits.shape
    _check(lib().parle_k_softmax_xent(_stream_handle(stream), int(dtype), n, batch, classes, _ptr(logits), _ptr(labels),
                                      _ptr(loss), _ptr(dlogits)))


def parle_k_fc_head(dtype, feat, w, bias, labels, relu_mask, loss_img, loss, dlogits, dfeat, stream=None):
    n, batch, features = feat.shape
    classes = w.shape[1]
    _check(lib().parle_k_fc_head(_stream_handle(stream), int(dtype), n, batch, features, classes, _ptr(feat), _ptr(w),
                                 _ptr(bias), _ptr(labels), int(relu_mask), _ptr(loss_img), _ptr(loss), _ptr(dlogits),
                                 _ptr(dfeat)))


def parle_k_gap_head(desc, feat, labels, loss_img, loss, dlogits, dfeat, stream=None):
    _check(lib().parle_k_gap_head(_stream_handle(stream), C.byref(desc), _ptr(feat), _ptr(labels), _ptr(loss_img),
                                  _ptr(loss), _ptr(dlogits), _ptr(dfeat)))


class Parle:
    """A context plus the torch tensors that back its device buffers.

    ``x0``: ``[n, n_params]`` float32 initial replicas (numpy, or a torch tensor on host or device).  Device tensors are
    ``[n, n_pad]``; :meth:`state` returns them trimmed to ``n_params`` as numpy arrays.
    """

    def __init__(self, cfg: parle_config, x0, device="cuda:0", stream=None):
        import numpy as np
        import torch
        self.torch = torch
        self.cfg = cfg
        self.sizes = parle_query_sizes(cfg)
        n, n_pad, N = cfg.n_replicas, self.sizes.n_pad, self.sizes.n_params
        dev = torch.device(device)
        self.device = dev

        def state():
            return torch.zeros((n, n_pad), dtype=torch.float32, device=dev)

        self.x, self.y, self.z, self.vy, self.vx, self.grad = (state() for _ in range(6))
        self.x_ref = torch.zeros(n_pad, dtype=torch.float32, device=dev)
        self.y_bf16 = torch.zeros((n, n_pad), dtype=torch.bfloat16, device=dev) if cfg.compute_bf16 else None
        self.bn_stats = (torch.zeros(self.sizes.bn_bytes // 4, dtype=torch.float32, device=dev)
                         if self.sizes.bn_bytes else None)
        self.workspace = torch.empty(self.sizes.workspace_bytes, dtype=torch.uint8, device=dev)
        if not isinstance(x0, torch.Tensor):
            x0 = torch.as_tensor(np.asarray(x0, dtype=np.float32))
        assert tuple(x0.shape) == (n, N) and x0.dtype == torch.float32, (tuple(x0.shape), (n, N), x0.dtype)
        self.x[:, :N].copy_(x0)
        self.buffers = parle_buffers(*(t.data_ptr() if t is not None else None for t in (
            self.x, self.y, self.z, self.vy, self.vx, self.grad, self.x_ref, self.y_bf16, self.bn_stats,
            self.workspace)))
        self.stream = stream
        h = C.c_void_p()
        with torch.cuda.device(dev):
            _check(lib().parle_init(C.byref(cfg), C.byref(self.buffers), _stream_handle(stream), C.byref(h)))
        self.ctx = h

    def parle_inner_step(self, images=None, labels=None, loss=None):
        _check(lib().parle_inner_step(self.ctx, _ptr(images), _ptr(labels), _ptr(loss)), self.ctx)

    def parle_inner_block(self, images, labels, loss=None):
        """images ``[steps, n, B, H, W, C]``, labels ``[steps, n, B]``, loss ``[steps, n]`` or None."""
        _check(lib().parle_inner_block(self.ctx, _ptr(images), _ptr(labels), int(images.shape[0]), _ptr(loss)),
               self.ctx)

    def parle_outer_step(self):
        _check(lib().parle_outer_step(self.ctx), self.ctx)

    def parle_eval(self, which=-1, images=None, labels=None, want_spread=True):
        loss, nerr, spread = C.c_float(), C.c_int32(), C.c_float()
        count = 0 if images is None else int(images.shape[0])
        _check(lib().parle_eval(self.ctx, which, _ptr(images), _ptr(labels), count, C.byref(loss), C.byref(nerr),
                                C.byref(spread) if want_spread else None), self.ctx)
        return loss.value, nerr.value, (spread.value if want_spread else None)

    def parle_get_state(self):
        k, od, g, r = C.c_int64(), C.c_int64(), C.c_float(), C.c_float()
        _check(lib().parle_get_state(self.ctx, C.byref(k), C.byref(od), C.byref(g), C.byref(r)), self.ctx)
        return k.value, od.value, g.value, r.value

    def parle_set_state(self, k, outer_done, g, r):
        _check(lib().parle_set_state(self.ctx, k, outer_done, g, r), self.ctx)

    def state(self):
        """x, y, z, vy, vx ``[n, n_params]`` and x_ref ``[n_params]`` as numpy (synchronises)."""
        N = self.sizes.n_params
        self.torch.cuda.synchronize(self.device)
        out = {k: getattr(self, k)[:, :N].cpu().numpy() for k in ("x", "y", "z", "vy", "vx", "grad")}
        out["x_ref"] = self.x_ref[:N].cpu().numpy()
        return out

    def close(self):
        if getattr(self, "ctx", None):
            lib().parle_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
