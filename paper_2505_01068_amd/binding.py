"""ctypes binding over libimattn.so: same names as the C ABI (include/imattn.h).

Argument marshalling only.  Torch supplies device memory and the current HIP
stream; every step of the computation runs inside the library's kernels.  There
is no fallback: a missing library or a non-zero return code raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

IM_MAX_SEG = 8
IM_DTYPE_F32, IM_DTYPE_BF16 = 0, 1
IM_OK, IM_ERR_INVALID, IM_ERR_UNSUPPORTED, IM_ERR_WORKSPACE, IM_ERR_HIP = 0, -1, -2, -3, -4
IM_IFM_FORWARD, IM_IFM_BACKWARD, IM_IEM, IM_DENSE = 0x062, 0x08C, 0x111, 0x1FF
# the named 3 x 3 patterns of include/imattn.h (segment order t, v, a; bit i*3 + j <=> block (query i, key j) live)
NAMED_MASKS = {
    "ifm_forward": IM_IFM_FORWARD, "ifm_backward": IM_IFM_BACKWARD, "iem": IM_IEM, "dense": IM_DENSE,
    "structure1_a": 0x0A4, "structure1_b": 0x04A, "structure2_a": 0x08A, "structure2_b": 0x064,
    "structure3_a": 0x0A2, "structure3_b": 0x04C, "self_only": 0x0EE,
}

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libimattn.so")


class ImShape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_seg", C.c_int32), ("seg_len", C.c_int32 * IM_MAX_SEG),
                ("d_model", C.c_int32), ("n_heads", C.c_int32), ("live_mask", C.c_uint64),
                ("scale", C.c_float), ("dtype", C.c_int32),
                ("cu_rows", C.c_void_p), ("total_rows", C.c_int64)]


class ImWorkItem(C.Structure):
    _fields_ = [("q_seg", C.c_int32), ("q_start", C.c_int32), ("q_rows", C.c_int32), ("n_key_seg", C.c_int32),
                ("key_seg", C.c_int32 * IM_MAX_SEG), ("pairs", C.c_int64)]


class ImAttnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"imattn error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load the shared library (built in-tree by paper_2505_01068_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} not found: build it with `python -m paper_2505_01068_amd.build` "
                              "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(_LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        shp = C.POINTER(ImShape)
        L.im_last_error.restype = C.c_char_p
        L.im_version.restype = C.c_char_p
        L.im_schedule_build.argtypes = [shp, C.c_int32, C.POINTER(ImWorkItem), C.c_int32, C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int64)]
        L.im_attention_sizes.argtypes = [shp, C.POINTER(sz), C.POINTER(sz)]
        L.im_attention_fwd.argtypes = [shp] + [vp] * 14 + [sz, vp]
        L.im_attention_bwd.argtypes = [shp] + [vp] * 19 + [sz, vp]
        L.im_attention_fwd_noalloc.argtypes = [shp] + [vp] * 13
        L.im_noalloc_init.argtypes = []
        L.im_calibrate_mfma.argtypes = [C.c_int32, vp, C.POINTER(C.c_double), vp]
        L.im_calibrate_copy.argtypes = [vp, vp, sz, vp]
        L.gsit_layer_sizes.argtypes = [shp, C.c_int32, C.POINTER(sz)]
        L.gsit_layer_fwd.argtypes = [shp, C.c_int32] + [vp] * 17 + [C.c_float] + [vp] * 4 + [sz, vp]
        L.im_profile_enable.argtypes = [C.c_int]
        L.im_profile_get.argtypes = [C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.im_profile_enable.restype = C.c_int
        L.im_profile_get.restype = C.c_int
        L.gsit_layer_train_sizes.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.gsit_layer_fwd_train.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.gsit_layer_bwd.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.gsit_model_sizes.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_size_t)]
        L.gsit_model_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p]
        for f in (L.im_schedule_build, L.im_attention_sizes, L.im_attention_fwd, L.im_attention_bwd,
                  L.im_attention_fwd_noalloc, L.im_noalloc_init, L.im_calibrate_mfma, L.im_calibrate_copy,
                  L.gsit_layer_sizes, L.gsit_layer_fwd, L.gsit_model_sizes, L.gsit_model_fwd,
                  L.gsit_layer_train_sizes, L.gsit_layer_fwd_train, L.gsit_layer_bwd):
            f.restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise ImAttnError(rc, lib().im_last_error().decode())


def make_shape(batch, seg_len, d_model, n_heads, live_mask, scale, dtype, cu_rows=None, total_rows=0):
    """The problem statement.  Packed rows: cu_rows = int32 device tensor [batch * n_seg + 1] of row offsets,
    total_rows = its last entry (host int); seg_len then bounds the per-sample segment lengths.  The shape
    keeps a reference to cu_rows, whose device memory it points into."""
    s = ImShape()
    s.cu_rows, s.total_rows = (None, 0) if cu_rows is None else (cu_rows.data_ptr(), int(total_rows))
    s._cu_rows_ref = cu_rows
    s.batch, s.n_seg, s.d_model, s.n_heads = int(batch), len(seg_len), int(d_model), int(n_heads)
    for i, n in enumerate(seg_len):
        s.seg_len[i] = int(n)
    s.live_mask, s.scale = int(live_mask), float(scale)
    s.dtype = {"fp32": IM_DTYPE_F32, "bf16": IM_DTYPE_BF16, torch.float32: IM_DTYPE_F32,
               torch.bfloat16: IM_DTYPE_BF16, 0: 0, 1: 1}[dtype]
    return s


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def im_schedule_build(shape, tile_rows):
    """Host-side listing of the live-block schedule: (items, n_pairs)."""
    n, pairs = C.c_int32(0), C.c_int64(0)
    _check(lib().im_schedule_build(C.byref(shape), tile_rows, None, 0, C.byref(n), C.byref(pairs)))
    items = (ImWorkItem * max(1, n.value))()
    _check(lib().im_schedule_build(C.byref(shape), tile_rows, items, n.value, C.byref(n), C.byref(pairs)))
    return [items[i] for i in range(n.value)], pairs.value


def im_attention_sizes(shape):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().im_attention_sizes(C.byref(shape), C.byref(a), C.byref(b)))
    return a.value, b.value


def gsit_layer_sizes(shape, d_ff):
    a = C.c_size_t(0)
    _check(lib().gsit_layer_sizes(C.byref(shape), int(d_ff), C.byref(a)))
    return a.value


def im_attention_fwd(shape, x, wq, wk, wv, wo, bq=None, bk=None, bv=None, bo=None, valid_len=None, key_pad=None,
                     y=None, saved=None, workspace=None):
    """y = IMAttention(x).  Tensors are CUDA(HIP) tensors; `saved`/`workspace` are uint8 buffers."""
    if y is None:
        y = torch.empty_like(x)
    wbytes = 0 if workspace is None else workspace.numel()
    _check(lib().im_attention_fwd(C.byref(shape), _p(x), _p(wq), _p(wk), _p(wv), _p(wo), _p(bq), _p(bk), _p(bv),
                                  _p(bo), _p(valid_len), _p(key_pad), _p(y), _p(saved), _p(workspace), wbytes,
                                  _stream()))
    return y


IM_NOALLOC_MAX_BYTES = 64 << 20


def im_noalloc_init():
    _check(lib().im_noalloc_init())


def im_attention_fwd_noalloc(shape, x, wq, wk, wv, wo, bq=None, bk=None, bv=None, bo=None, valid_len=None,
                             key_pad=None, y=None):
    """Inference forward on the library's built-in scratch buffer; `y` must be given (nothing is allocated)."""
    _check(lib().im_attention_fwd_noalloc(C.byref(shape), _p(x), _p(wq), _p(wk), _p(wv), _p(wo), _p(bq), _p(bk),
                                          _p(bv), _p(bo), _p(valid_len), _p(key_pad), _p(y), _stream()))
    return y


def im_attention_bwd(shape, x, wq, wk, wv, wo, saved, dy, dx, dwq, dwk, dwv, dwo, dbq=None, dbk=None, dbv=None,
                     dbo=None, valid_len=None, key_pad=None, workspace=None):
    wbytes = 0 if workspace is None else workspace.numel()
    _check(lib().im_attention_bwd(C.byref(shape), _p(x), _p(wq), _p(wk), _p(wv), _p(wo), _p(valid_len), _p(key_pad),
                                  _p(saved), _p(dy), _p(dx), _p(dwq), _p(dwk), _p(dwv), _p(dwo), _p(dbq), _p(dbk),
                                  _p(dbv), _p(dbo), _p(workspace), wbytes, _stream()))
    return dx


def gsit_layer_fwd(shape, d_ff, x, p, ln_eps=1e-5, valid_len=None, key_pad=None, y=None, workspace=None):
    """One encoder layer; `p` maps parameter names (ln1_g, ln1_b, wq, ..., w2, b2) to device tensors."""
    if y is None:
        y = torch.empty_like(x)
    wbytes = 0 if workspace is None else workspace.numel()
    g = p.get
    _check(lib().gsit_layer_fwd(C.byref(shape), int(d_ff), _p(x), _p(p["ln1_g"]), _p(p["ln1_b"]), _p(p["wq"]),
                                _p(p["wk"]), _p(p["wv"]), _p(p["wo"]), _p(g("bq")), _p(g("bk")), _p(g("bv")),
                                _p(g("bo")), _p(p["ln2_g"]), _p(p["ln2_b"]), _p(p["w1"]), _p(g("b1")), _p(p["w2"]),
                                _p(g("b2")), float(ln_eps), _p(valid_len), _p(key_pad), _p(y), _p(workspace), wbytes,
                                _stream()))
    return y


LAYER_FIELDS = ("ln1_g", "ln1_b", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class GsitLayerParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class GsitModel(C.Structure):
    _fields_ = [("n_layers_inter", C.c_int32), ("n_layers_intra", C.c_int32), ("d_ff_inter", C.c_int32),
                ("d_ff_intra", C.c_int32), ("n_heads_intra", C.c_int32), ("n_out", C.c_int32),
                ("scale_intra", C.c_float), ("ln_eps", C.c_float),
                ("mask_fwd", C.c_uint64), ("mask_bwd", C.c_uint64), ("mask_intra", C.c_uint64),
                ("fwd_layers", C.POINTER(GsitLayerParams)), ("bwd_layers", C.POINTER(GsitLayerParams)),
                ("intra_layers", C.POINTER(GsitLayerParams)), ("wf", C.c_void_p), ("bf", C.c_void_p)]


def _layer_array(layers):
    arr = (GsitLayerParams * len(layers))()
    for i, p in enumerate(layers):
        for n in LAYER_FIELDS:
            t = p.get(n)
            setattr(arr[i], n, None if t is None else t.data_ptr())
    return arr


def make_model(model, d_ff_inter, d_ff_intra, n_heads_intra, scale_intra, ln_eps=1e-5,
               mask_fwd=0x062, mask_bwd=0x08C, mask_intra=0x111):
    """gsit_model_t from a dict of device tensors: fwd_layers / bwd_layers / intra_layers (lists of
    layer dicts as for gsit_layer_fwd), wf, bf.  The returned object keeps the arrays alive."""
    m = GsitModel()
    m._keep = (_layer_array(model["fwd_layers"]), _layer_array(model["bwd_layers"]), _layer_array(model["intra_layers"]), model)
    m.n_layers_inter, m.n_layers_intra = len(model["fwd_layers"]), len(model["intra_layers"])
    if len(model["bwd_layers"]) != m.n_layers_inter:
        raise ValueError("the two inter-modal encoders must have the same number of layers")
    m.d_ff_inter, m.d_ff_intra, m.n_heads_intra = int(d_ff_inter), int(d_ff_intra), int(n_heads_intra)
    m.n_out = int(model["wf"].shape[1])
    m.scale_intra, m.ln_eps = float(scale_intra), float(ln_eps)
    m.mask_fwd, m.mask_bwd, m.mask_intra = int(mask_fwd), int(mask_bwd), int(mask_intra)
    m.fwd_layers, m.bwd_layers, m.intra_layers = m._keep[0], m._keep[1], m._keep[2]
    m.wf = model["wf"].data_ptr()
    m.bf = None if model.get("bf") is None else model["bf"].data_ptr()
    return m


def _layer_struct(p):
    st = GsitLayerParams()
    for n in LAYER_FIELDS:
        t = p.get(n)
        setattr(st, n, None if t is None else t.data_ptr())
    return st


def gsit_layer_train_sizes(shape, d_ff):
    a, b = C.c_size_t(0), C.c_size_t(0)
    _check(lib().gsit_layer_train_sizes(C.byref(shape), int(d_ff), C.byref(a), C.byref(b)))
    return a.value, b.value


def gsit_layer_fwd_train(shape, d_ff, x, p, saved, ln_eps=1e-5, valid_len=None, key_pad=None, y=None, workspace=None):
    """Training forward of one encoder layer: y as gsit_layer_fwd, `saved` filled for gsit_layer_bwd."""
    if y is None:
        y = torch.empty_like(x)
    st = _layer_struct(p)
    _check(lib().gsit_layer_fwd_train(C.byref(shape), int(d_ff), _p(x), C.byref(st), float(ln_eps), _p(valid_len),
                                      _p(key_pad), _p(y), _p(saved), _p(workspace), workspace.numel(), _stream()))
    return y


def gsit_layer_bwd(shape, d_ff, x, p, saved, dy, grads, ln_eps=1e-5, valid_len=None, key_pad=None, dx=None, workspace=None):
    """Backward of one encoder layer.  `grads` maps parameter names to fp32 device tensors to overwrite
    (missing / None = not wanted).  Returns dx."""
    if dx is None:
        dx = torch.empty_like(x)
    st, gs = _layer_struct(p), _layer_struct(grads)
    _check(lib().gsit_layer_bwd(C.byref(shape), int(d_ff), _p(x), C.byref(st), float(ln_eps), _p(valid_len), _p(key_pad),
                                _p(saved), _p(dy), _p(dx), C.byref(gs), _p(workspace), workspace.numel(), _stream()))
    return dx


def gsit_model_sizes(shape, model):
    a = C.c_size_t(0)
    _check(lib().gsit_model_sizes(C.byref(shape), C.byref(model), C.byref(a)))
    return a.value


def gsit_model_fwd(shape, model, x, valid_len=None, key_pad=None, out=None, workspace=None):
    """out [B, n_out] = GsiT(x): two IFM encoders, feature concat, IEM encoder, last steps, final linear."""
    if out is None:
        out = torch.empty(x.shape[0], model.n_out, dtype=x.dtype, device=x.device)
    wbytes = 0 if workspace is None else workspace.numel()
    _check(lib().gsit_model_fwd(C.byref(shape), C.byref(model), _p(x), _p(valid_len), _p(key_pad), _p(out),
                                _p(workspace), wbytes, _stream()))
    return out


def im_calibrate_mfma(iters, sink):
    """Enqueue the register-resident MFMA loop; returns the flops it launched."""
    f = C.c_double(0)
    _check(lib().im_calibrate_mfma(int(iters), _p(sink), C.byref(f), _stream()))
    return f.value


def im_calibrate_copy(dst, src):
    """Enqueue a streaming device copy of src (uint8 tensor) into dst."""
    _check(lib().im_calibrate_copy(_p(dst), _p(src), src.numel() * src.element_size(), _stream()))


def im_profile_enable(on, only=None):
    """on: time every kernel family; only=<family name>: time just that one (cheaper)."""
    if only is not None:
        names = im_profile_names()
        lib().im_profile_enable(1 << (names.index(only) + 1))
    else:
        lib().im_profile_enable(1 if on else 0)


def im_profile_names():
    n = lib().im_profile_get(-1, None, None, None)
    out = []
    for i in range(n):
        name = C.c_char_p()
        lib().im_profile_get(i, C.byref(name), None, None)
        out.append(name.value.decode())
    return out


def im_profile_get():
    """{family: (total_ms, launches)} since the last im_profile_enable(True); call after a synchronize."""
    out = {}
    n = lib().im_profile_get(0, None, None, None)
    for i in range(n):
        name, ms, cnt = C.c_char_p(), C.c_double(0), C.c_int64(0)
        lib().im_profile_get(i, C.byref(name), C.byref(ms), C.byref(cnt))
        out[name.value.decode()] = (ms.value, cnt.value)
    return out
