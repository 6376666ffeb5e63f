"""ctypes binding of libsknet.so: the same entry points as include/sknet.h, argument marshalling
only.  Device buffers are torch CUDA tensors (used for memory and streams, nothing else); every
step of the path runs inside the library's HIP kernels.  There is no CPU fallback: if the library
is missing, importing this module raises.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  (imported first so that the library binds to the HIP runtime torch loaded)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsknet.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libsknet.so is not built: run `python -m paper_1509_03371_amd.build` "
                      "(or __graft_entry__.build()) first")
lib = C.CDLL(LIB_PATH)

SK_F32, SK_BF16, SK_F16 = 0, 1, 2
SK_CONV, SK_MAXPOOL = 0, 1
STATUS_NAMES = ["SK_OK", "SK_EINVAL", "SK_ESHAPE", "SK_ESTATE", "SK_ENOMEM", "SK_EDEVICE", "SK_EUNSUPPORTED"]
DTYPES = {"f32": SK_F32, "bf16": SK_BF16, "f16": SK_F16}


class SkLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("c_out", C.c_int32), ("k", C.c_int32), ("d", C.c_int32),
                ("s", C.c_int32), ("relu", C.c_int32)]


class SwLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("c_out", C.c_int32), ("k", C.c_int32), ("s", C.c_int32),
                ("relu", C.c_int32)]


class SknetError(RuntimeError):
    def __init__(self, status, message):
        self.status = status
        self.status_name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__("%s: %s" % (self.status_name, message))


_vp, _i32, _fp, _ip = C.c_void_p, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_int32)
_SIGS = {
    "sknet_convert_sw": [C.POINTER(SwLayer), _i32, _i32, C.POINTER(SkLayer), _ip],
    "sknet_create": [C.POINTER(SkLayer), _i32, _i32, _i32, _i32, _i32, C.POINTER(_vp)],
    "sknet_context": [_vp, _ip],
    "sknet_infer_shapes": [_vp, _i32, _i32, _i32, _ip],
    "sknet_num_convs": [_vp, _ip],
    "sknet_conv_shape": [_vp, _i32, _ip],
    "sknet_set_weights": [_vp, _i32, _fp, _fp],
    "sknet_get_weights": [_vp, _i32, _fp, _fp],
    "sknet_plan": [_vp, _i32, _i32, _i32, _i32, _i32],
    "sknet_forward": [_vp, _vp, _vp, _vp],
    "sknet_time_backward_step": [_vp, _vp, _i32, _i32, _i32, _vp, _fp],
    "sknet_backward_noalloc": [_vp, _vp, _vp, _vp],
    "sknet_backward": [_vp, _vp, _vp, _vp],
    "sknet_sgd_step": [_vp, C.c_float, C.c_float, C.c_float, _vp],
    "sknet_get_grad": [_vp, _i32, _fp, _fp],
    "sknet_get_activation_grad": [_vp, _i32, _vp, _fp],
    "sknet_get_activation": [_vp, _i32, _fp],
    "sknet_get_pool_argmax": [_vp, _i32, _ip],
    "sknet_num_steps": [_vp, _ip],
    "sknet_step_name": [_vp, _i32, C.c_char_p, _i32],
    "sknet_time_step": [_vp, _i32, _i32, _vp, _fp],
    "unet_create": [_i32, _i32, _i32, _i32, _i32, C.POINTER(_vp)],
    "unet_num_params": [_vp, _ip],
    "unet_param_shape": [_vp, _i32, _ip],
    "unet_set_weights": [_vp, _i32, _fp, _fp],
    "unet_output_size": [_vp, _i32, _i32, _ip, _ip],
    "unet_plan": [_vp, _i32, _i32, _i32],
    "unet_forward": [_vp, _vp, _vp, _vp],
    "unet_get_activation": [_vp, C.c_char_p, _fp, _ip],
    "usknet_create": [_i32, _i32, _i32, _i32, C.POINTER(_vp)],
    "unet_plan_training": [_vp, _i32, _i32, _i32],
    "unet_set_merge_backward": [_vp, _i32],
    "unet_backward": [_vp, _vp, _vp, _vp],
    "unet_get_grad": [_vp, _i32, _fp, _fp],
    "unet_param_kind": [_vp, _i32, _ip],
    "unet_sgd_step": [_vp, C.c_float, C.c_float, C.c_float, _vp],
    "unet_get_weights": [_vp, _i32, _fp, _fp],
    "sknet3d_create": [C.POINTER(SkLayer), _i32, _i32, _i32, C.POINTER(_vp)],
    "sknet3d_create_dtype": [C.POINTER(SkLayer), _i32, _i32, _i32, _i32, C.POINTER(_vp)],
    "sknet3d_context": [_vp, _ip],
    "sknet3d_infer_shapes": [_vp, _i32, _i32, _i32, _ip],
    "sknet3d_num_convs": [_vp, _ip],
    "sknet3d_conv_shape": [_vp, _i32, _ip],
    "sknet3d_set_weights": [_vp, _i32, _fp, _fp],
    "sknet3d_plan": [_vp, _i32, _i32, _i32, _i32],
    "sknet3d_forward": [_vp, _vp, _vp, _vp],
    "sknet3d_get_activation": [_vp, _i32, _fp],
    "sknet3d_backward": [_vp, _vp, _vp, _vp],
    "sknet3d_sgd_step": [_vp, C.c_float, C.c_float, C.c_float, _vp],
    "sknet3d_get_grad": [_vp, _i32, _fp, _fp],
    "sknet3d_get_weights": [_vp, _i32, _fp, _fp],
    "sknet3d_get_pool_argmax": [_vp, _i32, _ip],
    "sk_probe_mfma": [_i32, _i32, _i32, _vp, C.POINTER(C.c_double)],
    "sk_probe_copy": [_vp, _vp, C.c_uint64, _i32, _vp, C.POINTER(C.c_double)],
}
for _name, _args in _SIGS.items():
    _f = getattr(lib, _name)
    _f.argtypes = _args
    _f.restype = C.c_int
lib.sknet_destroy.argtypes = [_vp]
lib.sknet_destroy.restype = None
lib.unet_destroy.argtypes = [_vp]
lib.unet_destroy.restype = None
lib.sknet3d_destroy.argtypes = [_vp]
lib.sknet3d_destroy.restype = None
lib.sknet_last_error.argtypes = []
lib.sknet_last_error.restype = C.c_char_p
lib.sknet_conv_flops.argtypes = [C.c_int64] * 4
lib.sknet_conv_flops.restype = C.c_int64

EXPORTED = sorted(list(_SIGS) + ["sknet_destroy", "unet_destroy", "sknet3d_destroy", "sknet_last_error", "sknet_conv_flops"])


def _check(status):
    if status != 0:
        raise SknetError(status, lib.sknet_last_error().decode())


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_fp)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_ptr(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (what, dtype))
    return C.c_void_p(t.data_ptr())


def layers_to_c(layers):
    """[{'type': 'conv'|'pool', 'f_out', 'k', 'd', 's', 'relu'}] -> SkLayer array."""
    arr = (SkLayer * len(layers))()
    for i, l in enumerate(layers):
        if l["type"] == "conv":
            arr[i] = SkLayer(SK_CONV, l["f_out"], l["k"], l.get("d", 1), 1, int(l.get("relu", False)))
        elif l["type"] == "pool":
            arr[i] = SkLayer(SK_MAXPOOL, 0, l["k"], l.get("d", 1), l.get("s", 1), 0)
        else:
            raise ValueError("unknown layer type %r" % (l["type"],))
    return arr


def sk_probe_mfma(dtype, iters=20000, stream=None, varied=False):
    """Sustained TFLOP/s of a bare MFMA issue loop of the shape used for dtype ('f32'|'bf16'|'f16');
    varied=True gives every MFMA operands of its own with hashed bit patterns (real-data switching activity)."""
    out = C.c_double(0.0)
    _check(lib.sk_probe_mfma(DTYPES[dtype], 1 if varied else 0, iters, _stream(stream), C.byref(out)))
    return out.value


def sk_probe_copy(src, dst, reps=10, stream=None):
    """GB/s (read + written) of a streaming copy between two equally sized CUDA tensors."""
    nbytes = src.numel() * src.element_size()
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
            and dst.numel() * dst.element_size() == nbytes):
        raise TypeError("sk_probe_copy: two contiguous CUDA tensors of the same byte size")
    out = C.c_double(0.0)
    _check(lib.sk_probe_copy(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), nbytes, reps, _stream(stream), C.byref(out)))
    return out.value


def sknet_conv_flops(f_in, f_out, k, w_out):
    return int(lib.sknet_conv_flops(f_in, f_out, k, w_out))


def sknet_convert_sw(sw_layers, w0_sw):
    """Algorithm 1. sw_layers: [{'type': 'conv'|'pool'|'ip'|'other', ...}] -> SK layer dicts."""
    kinds = {"conv": 0, "pool": 1, "ip": 2, "other": 3}
    arr = (SwLayer * len(sw_layers))()
    for i, l in enumerate(sw_layers):
        arr[i] = SwLayer(kinds[l["type"]], l.get("f_out", 0), l.get("k", 1), l.get("s", 1), int(l.get("relu", False)))
    out = (SkLayer * len(sw_layers))()
    n_out = C.c_int32(0)
    _check(lib.sknet_convert_sw(arr, len(sw_layers), w0_sw, out, C.byref(n_out)))
    res = []
    for i in range(n_out.value):
        l = out[i]
        if l.kind == SK_CONV:
            res.append({"type": "conv", "f_out": l.c_out, "k": l.k, "d": l.d, "relu": bool(l.relu)})
        else:
            res.append({"type": "pool", "k": l.k, "d": l.d, "s": l.s})
    return res


class SKNet:
    """Owner of one sknet_t handle; methods are the C entry points without the `sknet_` prefix."""

    def __init__(self, layers, c_in, n_classes, dtype="f32", pad_mode=0):
        self.layers = list(layers)
        self._h = _vp()
        arr = layers_to_c(layers)
        _check(lib.sknet_create(arr, len(layers), c_in, n_classes, DTYPES[dtype], pad_mode, C.byref(self._h)))
        self.c_in, self.n_classes = c_in, n_classes
        self._plan = None

    def close(self):
        if self._h:
            lib.sknet_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def context(self):
        v = C.c_int32()
        _check(lib.sknet_context(self._h, C.byref(v)))
        return v.value

    def infer_shapes(self, h, w, pad=True):
        out = (C.c_int32 * (3 * (len(self.layers) + 1)))()
        _check(lib.sknet_infer_shapes(self._h, h, w, int(pad), out))
        return [tuple(out[3 * i:3 * i + 3]) for i in range(len(self.layers) + 1)]

    def num_convs(self):
        c = C.c_int32()
        _check(lib.sknet_num_convs(self._h, C.byref(c)))
        return c.value

    def conv_shape(self, conv_idx):
        s = (C.c_int32 * 4)()
        _check(lib.sknet_conv_shape(self._h, conv_idx, s))
        return tuple(s)

    def set_weights(self, conv_idx, w, b=None):
        shape = self.conv_shape(conv_idx)
        w, wp = _f32(w)
        if w.shape != shape:
            raise ValueError("conv %d expects weights %s, got %s" % (conv_idx, shape, w.shape))
        if b is not None:
            b, bp = _f32(b)
            if b.shape != (shape[0],):
                raise ValueError("conv %d expects %d biases" % (conv_idx, shape[0]))
        else:
            bp = None
        _check(lib.sknet_set_weights(self._h, conv_idx, wp, bp))

    def get_weights(self, conv_idx):
        shape = self.conv_shape(conv_idx)
        w = np.empty(shape, np.float32)
        b = np.empty(shape[0], np.float32)
        _check(lib.sknet_get_weights(self._h, conv_idx, w.ctypes.data_as(_fp), b.ctypes.data_as(_fp)))
        return w, b

    def plan(self, n, h, w, pad=True, training=False, keep=False, fused_head=False):
        """mode 1 if training (3 with fused_head: the head and the loss as one kernel in each direction),
        else 2 if keep (inference, every layer kept), else 0 (inference, fused)."""
        mode = (3 if fused_head else 1) if training else (2 if keep else 0)
        _check(lib.sknet_plan(self._h, n, h, w, int(pad), mode))
        self._plan = (n, h, w, bool(pad), bool(training))
        self._shapes = self.infer_shapes(h, w, pad)

    def out_shape(self):
        n = self._plan[0]
        c, h, w = self._shapes[-1]
        return (n, c, h, w)

    def forward(self, image, prob=None, stream=None):
        n, h, w = self._plan[:3]
        if tuple(image.shape) != (n, self.c_in, h, w):
            raise ValueError("image shape %s does not match the plan %s" % (tuple(image.shape), (n, self.c_in, h, w)))
        if prob is None:
            prob = torch.empty(self.out_shape(), dtype=torch.float32, device=image.device)
        elif tuple(prob.shape) != self.out_shape():
            raise ValueError("prob shape %s does not match %s" % (tuple(prob.shape), self.out_shape()))
        _check(lib.sknet_forward(self._h, _dev_ptr(image, torch.float32, "image"),
                                 _dev_ptr(prob, torch.float32, "prob"), _stream(stream)))
        return prob

    def backward(self, labels, loss=None, stream=None, noalloc=False):
        """noalloc=True: sknet_backward_noalloc (scratch in the library's static device buffer); loss must then
        be given, so that nothing is allocated on the way."""
        n, _, h, w = self.out_shape()
        if tuple(labels.shape) != (n, h, w):
            raise ValueError("labels shape %s does not match %s" % (tuple(labels.shape), (n, h, w)))
        if loss is None:
            if noalloc:
                raise ValueError("noalloc needs a caller-provided loss tensor")
            loss = torch.empty(1, dtype=torch.float32, device=labels.device)
        fn = lib.sknet_backward_noalloc if noalloc else lib.sknet_backward
        _check(fn(self._h, _dev_ptr(labels, torch.int32, "labels"), _dev_ptr(loss, torch.float32, "loss"), _stream(stream)))
        return loss

    def sgd_step(self, lr, momentum=0.0, weight_decay=0.0, stream=None):
        _check(lib.sknet_sgd_step(self._h, lr, momentum, weight_decay, _stream(stream)))

    def get_grad(self, conv_idx):
        shape = self.conv_shape(conv_idx)
        dw = np.empty(shape, np.float32)
        db = np.empty(shape[0], np.float32)
        _check(lib.sknet_get_grad(self._h, conv_idx, dw.ctypes.data_as(_fp), db.ctypes.data_as(_fp)))
        return dw, db

    def get_activation(self, layer_idx):
        c, h, w = self._shapes[layer_idx + 1]
        out = np.empty((self._plan[0], c, h, w), np.float32)
        _check(lib.sknet_get_activation(self._h, layer_idx, out.ctypes.data_as(_fp)))
        return out

    def get_activation_grad(self, layer_idx, labels):
        """Error map of layer layer_idx (fp32 NCHW numpy), recomputed from the last forward with labels."""
        c, h, w = self._shapes[layer_idx + 1]
        out = np.empty((self._plan[0], c, h, w), np.float32)
        _check(lib.sknet_get_activation_grad(self._h, layer_idx, _dev_ptr(labels, torch.int32, "labels"), out.ctypes.data_as(_fp)))
        return out

    def get_pool_argmax(self, pool_idx):
        li = [i for i, l in enumerate(self.layers) if l["type"] == "pool"][pool_idx]
        c, h, w = self._shapes[li + 1]
        out = np.empty((self._plan[0], c, h, w), np.int32)
        _check(lib.sknet_get_pool_argmax(self._h, pool_idx, out.ctypes.data_as(_ip)))
        return out

    def num_steps(self):
        c = C.c_int32()
        _check(lib.sknet_num_steps(self._h, C.byref(c)))
        return c.value

    def step_name(self, step):
        buf = C.create_string_buffer(64)
        _check(lib.sknet_step_name(self._h, step, buf, 64))
        return buf.value.decode()

    def time_backward_step(self, labels, layer_idx, part, iters=10, stream=None):
        """Average ms of one piece of the backward pass: part 0 weight gradient, 1 input gradient, 2 loss."""
        ms = C.c_float()
        _check(lib.sknet_time_backward_step(self._h, _dev_ptr(labels, torch.int32, "labels"), layer_idx, part, iters, _stream(stream), C.byref(ms)))
        return ms.value

    def time_step(self, step, iters=10, stream=None):
        ms = C.c_float()
        _check(lib.sknet_time_step(self._h, step, iters, _stream(stream), C.byref(ms)))
        return ms.value


class UNet:
    """Owner of one unet_t handle."""

    def __init__(self, c_in, n_classes, depth=4, base_ch=64, dtype="f32"):
        self._h = _vp()
        self._create(c_in, n_classes, depth, base_ch, dtype)
        self.c_in, self.n_classes, self.depth = c_in, n_classes, depth
        self._plan = None

    def _create(self, c_in, n_classes, depth, base_ch, dtype):
        _check(lib.unet_create(c_in, n_classes, depth, base_ch, DTYPES[dtype], C.byref(self._h)))

    def close(self):
        if self._h:
            lib.unet_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def num_params(self):
        c = C.c_int32()
        _check(lib.unet_num_params(self._h, C.byref(c)))
        return c.value

    def param_shape(self, idx):
        s = (C.c_int32 * 4)()
        _check(lib.unet_param_shape(self._h, idx, s))
        return tuple(s)

    def set_weights(self, idx, w, b=None):
        shape = self.param_shape(idx)
        w, wp = _f32(w)
        if w.shape != shape:
            raise ValueError("parameter %d expects %s, got %s" % (idx, shape, w.shape))
        bp = None
        if b is not None:
            b, bp = _f32(b)
        _check(lib.unet_set_weights(self._h, idx, wp, bp))

    def output_size(self, h_in, w_in):
        ho, wo = C.c_int32(), C.c_int32()
        _check(lib.unet_output_size(self._h, h_in, w_in, C.byref(ho), C.byref(wo)))
        return ho.value, wo.value

    def plan(self, n, h_in, w_in, training=False):
        _check((lib.unet_plan_training if training else lib.unet_plan)(self._h, n, h_in, w_in))
        self._plan = (n, h_in, w_in)

    def set_merge_backward(self, mode):
        """0: MergeCrop backwards into the up path only (default); 1: into the skip map as well."""
        _check(lib.unet_set_merge_backward(self._h, int(mode)))

    def backward(self, labels, loss=None, stream=None):
        """labels: int32 CUDA tensor [n, h_out, w_out] (-1 = masked pixel); returns the loss (1-element CUDA tensor)."""
        n, h, w = self._plan
        ho, wo = self.output_size(h, w)
        if tuple(labels.shape) != (n, ho, wo):
            raise ValueError("labels shape %s does not match the plan" % (tuple(labels.shape),))
        if loss is None:
            loss = torch.zeros(1, dtype=torch.float32, device=labels.device)
        _check(lib.unet_backward(self._h, _dev_ptr(labels, torch.int32, "labels"), _dev_ptr(loss, torch.float32, "loss"), _stream(stream)))
        return loss

    def sgd_step(self, lr, momentum=0.0, weight_decay=0.0, stream=None):
        _check(lib.unet_sgd_step(self._h, lr, momentum, weight_decay, _stream(stream)))

    def get_weights(self, idx):
        shape = self.param_shape(idx)
        kind = C.c_int32()
        _check(lib.unet_param_kind(self._h, idx, C.byref(kind)))
        w = np.empty(shape, np.float32)
        b = np.empty((shape[1] if kind.value == 1 else shape[0],), np.float32)
        _check(lib.unet_get_weights(self._h, idx, w.ctypes.data_as(_fp), b.ctypes.data_as(_fp)))
        return w, b

    def get_grad(self, idx):
        shape = self.param_shape(idx)
        kind = C.c_int32()
        _check(lib.unet_param_kind(self._h, idx, C.byref(kind)))
        dw = np.empty(shape, np.float32)
        db = np.empty((shape[1] if kind.value == 1 else shape[0],), np.float32)
        _check(lib.unet_get_grad(self._h, idx, dw.ctypes.data_as(_fp), db.ctypes.data_as(_fp)))
        return dw, db

    def forward(self, image, prob=None, stream=None):
        n, h, w = self._plan
        if tuple(image.shape) != (n, self.c_in, h, w):
            raise ValueError("image shape %s does not match the plan" % (tuple(image.shape),))
        ho, wo = self.output_size(h, w)
        if prob is None:
            prob = torch.empty((n, self.n_classes, ho, wo), dtype=torch.float32, device=image.device)
        _check(lib.unet_forward(self._h, _dev_ptr(image, torch.float32, "image"),
                                _dev_ptr(prob, torch.float32, "prob"), _stream(stream)))
        return prob

    def get_activation(self, stage):
        dims = (C.c_int32 * 3)()
        _check(lib.unet_get_activation(self._h, stage.encode(), None, dims))
        out = np.empty((self._plan[0], dims[0], dims[1], dims[2]), np.float32)
        _check(lib.unet_get_activation(self._h, stage.encode(), out.ctypes.data_as(_fp), dims))
        return out


class USKNet(UNet):
    """USK-Net (usknet_create): the same handle type and calls as UNet."""

    def __init__(self, c_in, n_classes, base_ch=64, dtype="f32"):
        super().__init__(c_in, n_classes, 1, base_ch, dtype)

    def _create(self, c_in, n_classes, depth, base_ch, dtype):
        _check(lib.usknet_create(c_in, n_classes, base_ch, DTYPES[dtype], C.byref(self._h)))


class SKNet3D:
    """Owner of one sknet3d_t handle; methods are the C entry points without the `sknet3d_` prefix.
    Volumes are slice-major: [depth][maps][height][width]."""

    def __init__(self, layers, c_in, n_classes, dtype="f32"):
        self.layers = list(layers)
        self._h = _vp()
        _check(lib.sknet3d_create_dtype(layers_to_c(layers), len(layers), c_in, n_classes, DTYPES[dtype], C.byref(self._h)))
        self.c_in, self.n_classes = c_in, n_classes
        self._plan = None

    def close(self):
        if self._h:
            lib.sknet3d_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def context(self):
        v = C.c_int32()
        _check(lib.sknet3d_context(self._h, C.byref(v)))
        return v.value

    def infer_shapes(self, dz, h, w):
        """[(maps, depth, height, width)] for the input volume and every layer's output."""
        out = (C.c_int32 * (4 * (len(self.layers) + 1)))()
        _check(lib.sknet3d_infer_shapes(self._h, dz, h, w, out))
        return [tuple(out[4 * i:4 * i + 4]) for i in range(len(self.layers) + 1)]

    def num_convs(self):
        c = C.c_int32()
        _check(lib.sknet3d_num_convs(self._h, C.byref(c)))
        return c.value

    def conv_shape(self, conv_idx):
        s = (C.c_int32 * 5)()
        _check(lib.sknet3d_conv_shape(self._h, conv_idx, s))
        return tuple(s)

    def set_weights(self, conv_idx, w, b=None):
        shape = self.conv_shape(conv_idx)
        w, wp = _f32(w)
        if w.shape != shape:
            raise ValueError("conv %d expects weights %s, got %s" % (conv_idx, shape, w.shape))
        if b is not None:
            b, bp = _f32(b)
            if b.shape != (shape[0],):
                raise ValueError("conv %d expects %d biases" % (conv_idx, shape[0]))
        else:
            bp = None
        _check(lib.sknet3d_set_weights(self._h, conv_idx, wp, bp))

    def plan(self, dz, h, w, keep=False, training=False):
        """mode 1 if training, else 2 if keep (inference, every layer kept), else 0 (inference, fused head)."""
        _check(lib.sknet3d_plan(self._h, dz, h, w, 1 if training else (2 if keep else 0)))
        self._plan = (dz, h, w)
        self._shapes = self.infer_shapes(dz, h, w)

    def out_shape(self):
        """(depth, classes, height, width) of the probabilities."""
        c, dz, h, w = self._shapes[-1]
        return (dz, c, h, w)

    def forward(self, volume, prob=None, stream=None):
        dz, h, w = self._plan
        if tuple(volume.shape) != (dz, self.c_in, h, w):
            raise ValueError("volume shape %s does not match the plan %s" % (tuple(volume.shape), (dz, self.c_in, h, w)))
        if prob is None:
            prob = torch.empty(self.out_shape(), dtype=torch.float32, device=volume.device)
        elif tuple(prob.shape) != self.out_shape():
            raise ValueError("prob shape %s does not match %s" % (tuple(prob.shape), self.out_shape()))
        _check(lib.sknet3d_forward(self._h, _dev_ptr(volume, torch.float32, "volume"),
                                   _dev_ptr(prob, torch.float32, "prob"), _stream(stream)))
        return prob

    def get_activation(self, layer_idx):
        """Output of layer layer_idx as a numpy array [depth, maps, height, width]."""
        c, dz, h, w = self._shapes[layer_idx + 1]
        out = np.empty((dz, c, h, w), np.float32)
        _check(lib.sknet3d_get_activation(self._h, layer_idx, out.ctypes.data_as(_fp)))
        return out

    def backward(self, labels, loss=None, stream=None):
        dz, _, h, w = self.out_shape()
        if tuple(labels.shape) != (dz, h, w):
            raise ValueError("labels shape %s does not match %s" % (tuple(labels.shape), (dz, h, w)))
        if loss is None:
            loss = torch.empty((), dtype=torch.float32, device=labels.device)
        _check(lib.sknet3d_backward(self._h, _dev_ptr(labels, torch.int32, "labels"), _dev_ptr(loss, torch.float32, "loss"),
                                    _stream(stream)))
        return loss

    def sgd_step(self, lr, momentum=0.0, weight_decay=0.0, stream=None):
        _check(lib.sknet3d_sgd_step(self._h, lr, momentum, weight_decay, _stream(stream)))

    def get_grad(self, conv_idx):
        shape = self.conv_shape(conv_idx)
        dw = np.empty(shape, np.float32)
        db = np.empty(shape[0], np.float32)
        _check(lib.sknet3d_get_grad(self._h, conv_idx, dw.ctypes.data_as(_fp), db.ctypes.data_as(_fp)))
        return dw, db

    def get_weights(self, conv_idx):
        shape = self.conv_shape(conv_idx)
        w = np.empty(shape, np.float32)
        b = np.empty(shape[0], np.float32)
        _check(lib.sknet3d_get_weights(self._h, conv_idx, w.ctypes.data_as(_fp), b.ctypes.data_as(_fp)))
        return w, b

    def get_pool_argmax(self, pool_idx):
        """Winner offsets of max pool number pool_idx as int32 [depth, maps, height, width]."""
        pools = [i for i, l in enumerate(self.layers) if l["type"] == "pool"]
        c, dz, h, w = self._shapes[pools[pool_idx] + 1]
        out = np.empty((dz, c, h, w), np.int32)
        _check(lib.sknet3d_get_pool_argmax(self._h, pool_idx, out.ctypes.data_as(_ip)))
        return out
