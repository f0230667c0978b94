"""ctypes binding of libwmdec.so: same names as include/wmdec.h, argument
marshalling only (torch tensors -> device pointers, current stream -> void*).
Every computation happens in the library's HIP kernels; there is no fallback:
if the shared library is missing, loading raises."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libwmdec.so")

F32, BF16, F16 = 0, 1, 2
OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_SHAPE, ERR_WORKSPACE, ERR_HIP = -1, -2, -3, -4, -5

_TORCH2ENUM = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}
ENUM2TORCH = {v: k for k, v in _TORCH2ENUM.items()}


class WmdecError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("wmdec status %d: %s" % (status, message))
        self.status = status


class DecoderConfig(ctypes.Structure):
    _fields_ = [("latent_c", ctypes.c_int), ("latent_h", ctypes.c_int), ("latent_w", ctypes.c_int),
                ("num_levels", ctypes.c_int), ("level_channels", ctypes.c_int * 4),
                ("resblocks_per_level", ctypes.c_int), ("groups", ctypes.c_int), ("eps", ctypes.c_float),
                ("out_c", ctypes.c_int), ("act_dtype", ctypes.c_int), ("max_batch", ctypes.c_int),
                ("latent_dtype", ctypes.c_int), ("separate_stats_pass", ctypes.c_int),
                ("separate_merge_launch", ctypes.c_int), ("separate_shortcut", ctypes.c_int)]


_vp, _i, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t

# name -> (restype, argtypes): every symbol include/wmdec.h and include/wmdec_measure.h declare
SIGNATURES = {
    "wmdec_last_error": (ctypes.c_char_p, []),
    "wmdec_status_string": (ctypes.c_char_p, [_i]),
    "wmdec_gn_stats_workspace_bytes": (_sz, [_i] * 5),
    "wmdec_gn_stats": (_i, [_vp, _i, _i, _i, _i, _i, _i, _f, _vp, _vp, _vp, _sz, _vp]),
    "wmdec_gn_stats_noalloc": (_i, [_vp, _i, _i, _i, _i, _i, _i, _f, _vp, _vp, _vp]),
    "wmdec_conv_packed_bytes": (_sz, [_i] * 4),
    "wmdec_pack_conv_weights": (_i, [_vp, _i, _i, _i, _i, _vp, _i, _vp]),
    "wmdec_gn_silu_conv3x3": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "wmdec_gn_silu_conv3x3_shortcut": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _vp, _i, _vp, _vp, _vp, _i,
                                            _i, _i, _i, _i, _i, _vp]),
    "wmdec_conv_stats_workspace_bytes": (_sz, [_i] * 8),
    "wmdec_gn_silu_conv3x3_stats": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i,
                                         _i, _f, _vp, _vp, _vp, _sz, _vp]),
    "wmdec_gn_conv1x1": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "wmdec_upconv_packed_bytes": (_sz, [_i] * 3),
    "wmdec_pack_upconv_weights": (_i, [_vp, _i, _i, _i, _vp, _i, _vp]),
    "wmdec_upsample2x_conv3x3": (_i, [_vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "wmdec_upsample2x_nearest": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "wmdec_nchw_to_nhwc": (_i, [_vp, _i, _vp, _i, _i, _i, _i, _i, _vp]),
    "wmdec_nhwc_to_nchw": (_i, [_vp, _i, _vp, _i, _i, _i, _i, _i, _vp]),
    "wmdec_attention_workspace_bytes": (_sz, [_i] * 4),
    "wmdec_attention": (_i, [_vp, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]),
    "wmdec_adaln_max_batch": (_i, [_i]),
    "wmdec_adaln_fused_projection": (_i, [_vp, _i, _vp, _i, _vp, _vp, _i, _i, _i, _i, _vp]),
    "decoder_default_config": (None, [ctypes.POINTER(DecoderConfig)]),
    "decoder_create": (_i, [ctypes.POINTER(DecoderConfig), ctypes.POINTER(_vp)]),
    "decoder_destroy": (_i, [_vp]),
    "decoder_weights_bytes": (_sz, [_vp]),
    "decoder_num_weights": (_i, [_vp]),
    "decoder_weight_info": (_i, [_vp, _i, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(_sz), ctypes.POINTER(_sz),
                                 ctypes.POINTER(_i), ctypes.POINTER(_i * 4)]),
    "decoder_weight_offset": (_i, [_vp, ctypes.c_char_p, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "decoder_packed_bytes": (_sz, [_vp]),
    "decoder_pack_weights": (_i, [_vp, _vp, _vp, _vp]),
    "decoder_workspace_bytes": (_sz, [_vp, _i]),
    "decoder_set_workspace": (_i, [_vp, _vp, _sz]),
    "decoder_run": (_i, [_vp, _vp, _vp, _vp, _i, _vp]),
    "decoder_run_extrapolated": (_i, [_vp, _vp, _vp, _f, _vp, _vp, _i, _vp]),
    "wmdec_latent_extrapolate": (_i, [_vp, _vp, _i, _f, _i, _vp, _i, _sz, _vp]),
    "decoder_num_launches": (_i, [_vp]),
    "decoder_flops_per_frame": (ctypes.c_double, [_vp]),
    "decoder_dense_flops_per_frame": (ctypes.c_double, [_vp]),
    "decoder_set_profiling": (_i, [_vp, _i]),
    "decoder_num_steps": (_i, [_vp]),
    "decoder_step_info": (_i, [_vp, _i, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                               ctypes.POINTER(ctypes.c_double)]),
    "decoder_step_times": (_i, [_vp, ctypes.POINTER(ctypes.c_float), _i]),
    "decoder_time_step": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, ctypes.POINTER(ctypes.c_float), _vp]),
    "wmdec_measure_copy": (_i, [_vp, _vp, ctypes.c_size_t, _vp]),
}

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libwmdec.so is missing (%s): build it with "
                               "`python -m paper_2602_00608_amd.build`; there is no fallback path" % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def last_error():
    return lib().wmdec_last_error().decode()


def _check(status):
    if status != OK:
        raise WmdecError(status, last_error())


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def dtype_enum(t):
    return _TORCH2ENUM[t.dtype]


# ------------------------------------------------------------------ per-op entry points
def gn_stats_workspace_bytes(n, h, w, c, groups):
    return lib().wmdec_gn_stats_workspace_bytes(n, h, w, c, groups)


def gn_stats(x, groups, eps, mean, rstd, workspace):
    """x: [n,h,w,c] NHWC tensor; mean, rstd: fp32 [n*groups]; workspace: uint8 tensor."""
    n, h, w, c = x.shape
    _check(lib().wmdec_gn_stats(_ptr(x), dtype_enum(x), n, h, w, c, groups, eps, _ptr(mean), _ptr(rstd),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def gn_stats_noalloc(x, groups, eps, mean, rstd):
    """gn_stats on the library's built-in scratch: no workspace argument, no allocation."""
    n, h, w, c = x.shape
    _check(lib().wmdec_gn_stats_noalloc(_ptr(x), dtype_enum(x), n, h, w, c, groups, eps, _ptr(mean), _ptr(rstd), _stream()))


def conv_packed_bytes(cout, cin, k, op_dtype):
    return lib().wmdec_conv_packed_bytes(cout, cin, k, op_dtype)


def pack_conv_weights(src, packed, op_dtype):
    """src: [cout,cin,k,k] fp32 or bf16 tensor; packed: uint8 tensor of conv_packed_bytes."""
    cout, cin, k, _ = src.shape
    _check(lib().wmdec_pack_conv_weights(_ptr(src), dtype_enum(src), cout, cin, k, _ptr(packed), op_dtype, _stream()))


def _conv(fn, x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y, cin, cout):
    n, h, w, _ = y.shape
    _check(fn(_ptr(x), dtype_enum(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(beta), groups, int(apply_silu),
              _ptr(w_packed), _ptr(bias), _ptr(residual), _ptr(y), dtype_enum(y), n, h, w, cin, cout, _stream()))


def gn_silu_conv3x3(x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y):
    _conv(lib().wmdec_gn_silu_conv3x3, x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y,
          x.shape[3], y.shape[3])


def gn_silu_conv3x3_shortcut(x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, x2, w2_packed, bias2, y):
    """y = conv3x3(act(x)) + bias + W2 * x2 + bias2 (the 1x1 shortcut of a channel-changing ResBlock folded in)."""
    n, h, w, _ = y.shape
    _check(lib().wmdec_gn_silu_conv3x3_shortcut(
        _ptr(x), dtype_enum(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(beta), groups, int(apply_silu), _ptr(w_packed),
        _ptr(bias), _ptr(x2), x2.shape[3], _ptr(w2_packed), _ptr(bias2), _ptr(y), dtype_enum(y), n, h, w, x.shape[3],
        y.shape[3], _stream()))


def conv_stats_workspace_bytes(act_dtype, y_dtype, n, h, w, cin, cout, out_groups):
    return lib().wmdec_conv_stats_workspace_bytes(act_dtype, y_dtype, n, h, w, cin, cout, out_groups)


def gn_silu_conv3x3_stats(x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y,
                          out_groups, out_eps, mean_out, rstd_out, workspace):
    """gn_silu_conv3x3 that also returns mean / rstd of its own output y per (sample, output group)."""
    n, h, w, _ = y.shape
    _check(lib().wmdec_gn_silu_conv3x3_stats(
        _ptr(x), dtype_enum(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(beta), groups, int(apply_silu),
        _ptr(w_packed), _ptr(bias), _ptr(residual), _ptr(y), dtype_enum(y), n, h, w, x.shape[3], y.shape[3],
        out_groups, out_eps, _ptr(mean_out), _ptr(rstd_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream()))


def measure_copy(src, dst):
    """Plain copy of src into dst (same byte count, a multiple of 16) by one kernel of known traffic."""
    _check(lib().wmdec_measure_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()))


def gn_conv1x1(x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y):
    _conv(lib().wmdec_gn_conv1x1, x, mean, rstd, gamma, beta, groups, apply_silu, w_packed, bias, residual, y,
          x.shape[3], y.shape[3])


def upconv_packed_bytes(cout, cin, op_dtype):
    return lib().wmdec_upconv_packed_bytes(cout, cin, op_dtype)


def pack_upconv_weights(src, packed, op_dtype):
    """src: [cout,cin,3,3] fp32 or bf16 tensor; packed: uint8 tensor of upconv_packed_bytes (for upsample2x_conv3x3)."""
    cout, cin, _, _ = src.shape
    _check(lib().wmdec_pack_upconv_weights(_ptr(src), dtype_enum(src), cout, cin, _ptr(packed), op_dtype, _stream()))


def upsample2x_conv3x3(x, w_packed, bias, y):
    n, h, w, cin = x.shape
    _check(lib().wmdec_upsample2x_conv3x3(_ptr(x), dtype_enum(x), _ptr(w_packed), _ptr(bias), _ptr(y), dtype_enum(y),
                                          n, h, w, cin, y.shape[3], _stream()))


def upsample2x_nearest(x, y):
    n, h, w, c = x.shape
    _check(lib().wmdec_upsample2x_nearest(_ptr(x), _ptr(y), dtype_enum(x), n, h, w, c, _stream()))


def nchw_to_nhwc(src, dst):
    n, c, h, w = src.shape
    _check(lib().wmdec_nchw_to_nhwc(_ptr(src), dtype_enum(src), _ptr(dst), dtype_enum(dst), n, c, h, w, _stream()))


def nhwc_to_nchw(src, dst):
    n, h, w, c = src.shape
    _check(lib().wmdec_nhwc_to_nchw(_ptr(src), dtype_enum(src), _ptr(dst), dtype_enum(dst), n, c, h, w, _stream()))


def attention_workspace_bytes(n, h, w, c):
    return lib().wmdec_attention_workspace_bytes(n, h, w, c)


def attention(x, mean, rstd, gamma, beta, groups, wqkv_packed, bqkv, wo_packed, bo, y, workspace):
    n, h, w, c = x.shape
    _check(lib().wmdec_attention(_ptr(x), dtype_enum(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(beta), groups,
                                 _ptr(wqkv_packed), _ptr(bqkv), _ptr(wo_packed), _ptr(bo), _ptr(y), n, h, w, c,
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def latent_extrapolate(z_prev, v_prev, lam, steps, z_out):
    """z_out = z_prev + steps * lam * v_prev (fp32 fused multiply-add, one rounding to z_out's type)."""
    _check(lib().wmdec_latent_extrapolate(_ptr(z_prev), _ptr(v_prev), dtype_enum(z_prev), lam, steps, _ptr(z_out),
                                          dtype_enum(z_out), z_prev.numel(), _stream()))


def adaln_max_batch(d_cond):
    return lib().wmdec_adaln_max_batch(d_cond)


def adaln_fused_projection(c, w_fused, bias, out, apply_silu=True):
    """out[b, :] = bias + w_fused @ act(c[b]); c [batch, d_cond], w_fused [rows, d_cond], out fp32 [batch, rows]."""
    batch, d_cond = c.shape
    rows = w_fused.shape[0]
    _check(lib().wmdec_adaln_fused_projection(_ptr(c), dtype_enum(c), _ptr(w_fused), dtype_enum(w_fused), _ptr(bias), _ptr(out),
                                              batch, d_cond, rows, int(apply_silu), _stream()))


# ------------------------------------------------------------------ decoder
def decoder_default_config():
    cfg = DecoderConfig()
    lib().decoder_default_config(ctypes.byref(cfg))
    return cfg


class Decoder:
    """Thin owner of a wmdec_decoder handle; methods mirror the decoder_* entry points."""

    def __init__(self, cfg=None):
        self.cfg = cfg if cfg is not None else decoder_default_config()
        h = _vp()
        _check(lib().decoder_create(ctypes.byref(self.cfg), ctypes.byref(h)))
        self.handle = h
        self._workspace = None

    def close(self):
        if self.handle:
            lib().decoder_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def weights_bytes(self):
        return lib().decoder_weights_bytes(self.handle)

    def packed_bytes(self):
        return lib().decoder_packed_bytes(self.handle)

    def workspace_bytes(self, batch):
        return lib().decoder_workspace_bytes(self.handle, batch)

    def num_launches(self):
        return lib().decoder_num_launches(self.handle)

    def flops_per_frame(self):
        return lib().decoder_flops_per_frame(self.handle)

    def dense_flops_per_frame(self):
        return lib().decoder_dense_flops_per_frame(self.handle)

    def weight_table(self):
        """[(name, offset, bytes, dtype_enum, shape)] of the canonical blob."""
        out = []
        for i in range(lib().decoder_num_weights(self.handle)):
            name, off, nb, dt = ctypes.c_char_p(), _sz(), _sz(), _i()
            shape = (_i * 4)()
            _check(lib().decoder_weight_info(self.handle, i, ctypes.byref(name), ctypes.byref(off), ctypes.byref(nb),
                                             ctypes.byref(dt), ctypes.byref(shape)))
            out.append((name.value.decode(), off.value, nb.value, dt.value, tuple(shape)))
        return out

    def weight_offset(self, name):
        off, nb = _sz(), _sz()
        _check(lib().decoder_weight_offset(self.handle, name.encode(), ctypes.byref(off), ctypes.byref(nb)))
        return off.value, nb.value

    def pack_weights(self, weights, packed):
        _check(lib().decoder_pack_weights(self.handle, _ptr(weights), _ptr(packed), _stream()))

    def set_workspace(self, workspace):
        self._workspace = workspace  # keep the tensor alive
        _check(lib().decoder_set_workspace(self.handle, _ptr(workspace), workspace.numel() * workspace.element_size()))

    def set_profiling(self, enable):
        _check(lib().decoder_set_profiling(self.handle, int(enable)))

    def step_info(self):
        """[(kernel family, algorithmic flops per frame, algorithmic bytes per frame)] per graph step."""
        out = []
        for i in range(lib().decoder_num_steps(self.handle)):
            k, fl, by = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_double()
            _check(lib().decoder_step_info(self.handle, i, ctypes.byref(k), ctypes.byref(fl), ctypes.byref(by)))
            out.append((k.value.decode(), fl.value, by.value))
        return out

    def step_times(self):
        """Milliseconds of every step of the last profiled run (synchronises on its last event)."""
        n = lib().decoder_num_steps(self.handle)
        ms = (ctypes.c_float * n)()
        _check(lib().decoder_step_times(self.handle, ms, n))
        return list(ms)

    def time_step(self, latent, packed, out, step, reps):
        """Mean milliseconds per launch of graph step `step`, `reps` launches back to back (after a run())."""
        ms = ctypes.c_float()
        _check(lib().decoder_time_step(self.handle, _ptr(latent), _ptr(packed), _ptr(out), latent.shape[0], step, reps,
                                       ctypes.byref(ms), _stream()))
        return ms.value

    def run_extrapolated(self, z_prev, v_prev, lam, packed, out):
        """Frame j of out = decode(z_prev + (j + 1) * lam * v_prev), j = 0..out.shape[0]-1."""
        _check(lib().decoder_run_extrapolated(self.handle, _ptr(z_prev), _ptr(v_prev), lam, _ptr(packed), _ptr(out),
                                              out.shape[0], _stream()))

    def run(self, latent, packed, out):
        _check(lib().decoder_run(self.handle, _ptr(latent), _ptr(packed), _ptr(out), latent.shape[0], _stream()))
