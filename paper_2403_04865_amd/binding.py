"""ctypes binding of libslide.so: same names as include/slide.h, argument marshalling only.

torch is used for device memory and streams; every step of the path runs in the library's
HIP kernels.  Missing library => ImportError-like failure at load (no fallback).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libslide.so")


class SlideError(RuntimeError):
    CODES = {-1: "SLIDE_EINVAL", -2: "SLIDE_EARENA", -3: "SLIDE_EUNSUPPORTED", -4: "SLIDE_ESTATE", -5: "SLIDE_EHIP"}

    def __init__(self, code, what, hip=0):
        self.code = code
        super().__init__(f"{what}: {self.CODES.get(code, code)}" + (f" (hipError {hip})" if code == -5 else ""))


class _CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tile", "patch", "dim", "layers", "heads", "mlp_ratio", "mil_hidden",
                                         "n_classes", "dtype", "recompute")] + \
               [("ln_eps", C.c_float), ("reserved", C.c_int32)]


@dataclass
class SlideConfig:
    tile: int
    patch: int
    dim: int
    layers: int
    heads: int
    mlp_ratio: int
    mil_hidden: int
    n_classes: int
    dtype: int = 0          # 0 float32, 1 bfloat16
    recompute: int = 0
    ln_eps: float = 1e-6


def config_from(shape, dtype: int, recompute: int = 0) -> SlideConfig:
    """SlideConfig from any object with the fields tile, patch, dim, layers, heads, mlp_ratio, mil_hidden, n_classes
    and ln_eps (such as a workload description of the input generators)."""
    return SlideConfig(shape.tile, shape.patch, shape.dim, shape.layers, shape.heads, shape.mlp_ratio, shape.mil_hidden,
                       shape.n_classes, dtype=dtype, recompute=recompute, ln_eps=shape.ln_eps)


_SYMS = {
    "slide_ctx_create": (C.c_int, [C.POINTER(_CConfig), C.POINTER(C.c_void_p)]),
    "slide_ctx_destroy": (None, [C.c_void_p]),
    "slide_param_count": (C.c_size_t, [C.c_void_p]),
    "slide_param_tensors": (C.c_int, [C.c_void_p]),
    "slide_param_name": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "slide_param_offset": (C.c_int, [C.c_void_p, C.c_char_p, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "slide_arena_bytes": (C.c_size_t, [C.c_void_p, C.c_int64]),
    "slide_pool_arena_bytes": (C.c_size_t, [C.c_void_p, C.c_int64]),
    "slide_bind": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
    "encoder_fwd_tiles": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_void_p]),
    "encoder_bwd_tiles": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]),
    "mil_pool_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "mil_pool_fwd_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "mil_pool_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int, C.c_void_p]),
    "slide_step_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "slide_step_bwd": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
    "slide_chunked_arena_bytes": (C.c_size_t, [C.c_void_p, C.c_int64, C.c_int64]),
    "slide_step_chunked": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "slide_features": (C.c_void_p, [C.c_void_p]),
    "slide_feature_grads": (C.c_void_p, [C.c_void_p]),
    "slide_last_hip_error": (C.c_int, []),
    "slide_prof_begin": (C.c_int, [C.c_void_p, C.c_int]),
    "slide_prof_end": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "slide_prof_family": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int), C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]),
    "slide_kernel_name": (C.c_char_p, [C.c_int]),
    "slide_calib_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "slide_adamw_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int64, C.c_float,
                                   C.c_float, C.c_float, C.c_float, C.c_float, C.c_void_p]),
}


class _CResNetConfig(C.Structure):
    _fields_ = [("tile", C.c_int32), ("block", C.c_int32), ("depths", C.c_int32 * 4), ("width", C.c_int32),
                ("mil_hidden", C.c_int32), ("n_classes", C.c_int32), ("bn_eps", C.c_float), ("reserved", C.c_int32)]


@dataclass
class ResNetConfig:
    tile: int
    block: int              # 0 basic, 1 bottleneck
    depths: tuple
    width: int
    mil_hidden: int
    n_classes: int
    bn_eps: float = 1e-5


def resnet_config_from(shape) -> ResNetConfig:
    """ResNetConfig from any object with the fields tile, block ("basic" / "bottleneck"), depths, width, mil_hidden,
    n_classes and bn_eps (such as a workload description of the input generators)."""
    return ResNetConfig(shape.tile, 0 if shape.block == "basic" else 1, tuple(shape.depths), shape.width,
                        shape.mil_hidden, shape.n_classes, shape.bn_eps)


_P4 = [C.POINTER(C.c_double), C.POINTER(C.c_int), C.POINTER(C.c_double), C.POINTER(C.c_double)]
_SYMS.update({
    "resnet_ctx_create": (C.c_int, [C.POINTER(_CResNetConfig), C.POINTER(C.c_void_p)]),
    "resnet_ctx_destroy": (None, [C.c_void_p]),
    "resnet_param_count": (C.c_size_t, [C.c_void_p]),
    "resnet_param_tensors": (C.c_int, [C.c_void_p]),
    "resnet_param_name": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "resnet_feature_dim": (C.c_int, [C.c_void_p]),
    "resnet_arena_bytes": (C.c_size_t, [C.c_void_p, C.c_int64]),
    "resnet_bind": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
    "resnet_encoder_fwd_tiles": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]),
    "resnet_encoder_bwd_tiles": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p]),
    "resnet_slide_step_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "resnet_slide_step_bwd": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
    "resnet_features": (C.c_void_p, [C.c_void_p]),
    "resnet_feature_grads": (C.c_void_p, [C.c_void_p]),
    "resnet_saved_activations": (C.c_int, [C.c_void_p]),
    "resnet_saved_activation": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "resnet_prof_begin": (C.c_int, [C.c_void_p, C.c_int]),
    "resnet_prof_end": (C.c_int, [C.c_void_p] + _P4),
    "resnet_prof_family": (C.c_int, [C.c_void_p, C.c_int] + _P4),
    "resnet_kernel_name": (C.c_char_p, [C.c_int]),
})


def load_cdll():
    p = lib_path()
    if not os.path.exists(p):
        raise OSError(f"{p} is not built: run `python -m paper_2403_04865_amd.build` (there is no fallback path)")
    # Device memory and streams come from torch, so the process must run on torch's HIP runtime: with the library
    # loaded first, its own dependency brings up a second runtime and every launch on torch's pointers fails
    # (hipErrorNoDevice).
    import torch  # noqa: F401
    lib = C.CDLL(p)
    for name, (res, args) in _SYMS.items():
        f = getattr(lib, name)
        f.restype = res
        f.argtypes = args
    return lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


class SlideLib:
    """One slide_ctx.  Methods carry the C ABI's names and pass torch tensors' device pointers."""

    def __init__(self, cfg: SlideConfig):
        self.lib = load_cdll()
        self.cfg = cfg
        cc = _CConfig(cfg.tile, cfg.patch, cfg.dim, cfg.layers, cfg.heads, cfg.mlp_ratio, cfg.mil_hidden,
                      cfg.n_classes, cfg.dtype, cfg.recompute, cfg.ln_eps, 0)
        h = C.c_void_p()
        self._check(self.lib.slide_ctx_create(C.byref(cc), C.byref(h)), "slide_ctx_create")
        self.ctx = h
        self._keep = []

    def __del__(self):
        try:
            if getattr(self, "ctx", None):
                self.lib.slide_ctx_destroy(self.ctx)
                self.ctx = None
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != 0:
            raise SlideError(rc, what, self.lib.slide_last_hip_error())

    # ---- layout queries
    def slide_param_count(self):
        return int(self.lib.slide_param_count(self.ctx))

    def param_layout(self):
        """[(name, offset, length)] in layout order."""
        out = []
        buf = C.create_string_buffer(64)
        off, ln = C.c_size_t(), C.c_size_t()
        for i in range(self.lib.slide_param_tensors(self.ctx)):
            self._check(self.lib.slide_param_name(self.ctx, i, buf, 64, C.byref(off), C.byref(ln)), "slide_param_name")
            out.append((buf.value.decode(), off.value, ln.value))
        return out

    def slide_param_offset(self, name):
        off, ln = C.c_size_t(), C.c_size_t()
        self._check(self.lib.slide_param_offset(self.ctx, name.encode(), C.byref(off), C.byref(ln)), "slide_param_offset")
        return off.value, ln.value

    def slide_arena_bytes(self, n_tiles):
        return int(self.lib.slide_arena_bytes(self.ctx, n_tiles))

    def slide_pool_arena_bytes(self, n):
        return int(self.lib.slide_pool_arena_bytes(self.ctx, n))

    # ---- calls
    def slide_bind(self, params, grads, arena):
        self._keep = [params, grads, arena]
        self._check(self.lib.slide_bind(self.ctx, _ptr(params), _ptr(grads), _ptr(arena), arena.numel() * arena.element_size()),
                    "slide_bind")

    def encoder_fwd_tiles(self, pixels, n_tiles, feats_out, save_for_bwd, stream=None):
        self._check(self.lib.encoder_fwd_tiles(self.ctx, _ptr(pixels), n_tiles, _ptr(feats_out), int(save_for_bwd),
                                               _stream(stream)), "encoder_fwd_tiles")

    def encoder_bwd_tiles(self, dfeats, n_tiles, accumulate, pixel_grad=None, stream=None):
        self._check(self.lib.encoder_bwd_tiles(self.ctx, _ptr(dfeats), n_tiles, int(accumulate), _ptr(pixel_grad),
                                               _stream(stream)), "encoder_bwd_tiles")

    def mil_pool_fwd(self, feats, N, label, loss=None, logits=None, alpha=None, stream=None):
        self._check(self.lib.mil_pool_fwd(self.ctx, _ptr(feats), N, label, _ptr(loss), _ptr(logits), _ptr(alpha),
                                          _stream(stream)), "mil_pool_fwd")

    def mil_pool_fwd_static(self, params, feats, N, label, loss=None, logits=None, alpha=None, stream=None):
        self._check(self.lib.mil_pool_fwd_static(self.ctx, _ptr(params), _ptr(feats), N, label, _ptr(loss), _ptr(logits),
                                                 _ptr(alpha), _stream(stream)), "mil_pool_fwd_static")

    def mil_pool_bwd(self, feats, N, label, dfeats_out, accumulate, stream=None):
        self._check(self.lib.mil_pool_bwd(self.ctx, _ptr(feats), N, label, _ptr(dfeats_out), int(accumulate),
                                          _stream(stream)), "mil_pool_bwd")

    def slide_step_fwd(self, pixels, N, label, loss=None, logits=None, alpha=None, stream=None):
        self._check(self.lib.slide_step_fwd(self.ctx, _ptr(pixels), N, label, _ptr(loss), _ptr(logits), _ptr(alpha),
                                            _stream(stream)), "slide_step_fwd")

    def slide_step_bwd(self, accumulate, pixel_grad=None, stream=None):
        self._check(self.lib.slide_step_bwd(self.ctx, int(accumulate), _ptr(pixel_grad), _stream(stream)), "slide_step_bwd")

    def slide_chunked_arena_bytes(self, N, chunk_tiles):
        return int(self.lib.slide_chunked_arena_bytes(self.ctx, N, chunk_tiles))

    def slide_step_chunked(self, pixels, N, chunk_tiles, label, accumulate, loss=None, logits=None, alpha=None,
                           pixel_grad=None, stream=None):
        self._check(self.lib.slide_step_chunked(self.ctx, _ptr(pixels), N, chunk_tiles, label, int(accumulate),
                                                _ptr(loss), _ptr(logits), _ptr(alpha), _ptr(pixel_grad),
                                                _stream(stream)), "slide_step_chunked")

    def slide_features(self):
        return self.lib.slide_features(self.ctx)

    def slide_feature_grads(self):
        return self.lib.slide_feature_grads(self.ctx)

    def slide_prof_begin(self, kernel_id):
        self._check(self.lib.slide_prof_begin(self.ctx, kernel_id), "slide_prof_begin")

    def slide_prof_end(self):
        ms, n, fl, by = C.c_double(), C.c_int(), C.c_double(), C.c_double()
        self._check(self.lib.slide_prof_end(self.ctx, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)), "slide_prof_end")
        return ms.value, n.value, fl.value, by.value

    def slide_prof_family(self, kernel_id):
        ms, n, fl, by = C.c_double(), C.c_int(), C.c_double(), C.c_double()
        self._check(self.lib.slide_prof_family(self.ctx, kernel_id, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)),
                    "slide_prof_family")
        return ms.value, n.value, fl.value, by.value

    def slide_adamw_step(self, params, grads, exp_avg, exp_avg_sq, count, step, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                         weight_decay=0.01, stream=None):
        self._check(self.lib.slide_adamw_step(_ptr(params), _ptr(grads), _ptr(exp_avg), _ptr(exp_avg_sq),
                                              C.c_size_t(count), int(step), lr, beta1, beta2, eps, weight_decay,
                                              _stream(stream)), "slide_adamw_step")

    def slide_calib_copy(self, dst, src, nbytes, stream=None):
        self._check(self.lib.slide_calib_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream(stream)), "slide_calib_copy")

    def kernel_names(self):
        out, i = [], 0
        while True:
            s = self.lib.slide_kernel_name(i)
            if s is None:
                return out
            out.append(s.decode())
            i += 1


class ResNetLib:
    """One resnet_ctx (include/resnet.h).  Methods carry the C ABI's names and pass torch tensors' device pointers."""

    def __init__(self, cfg: ResNetConfig):
        self.lib = load_cdll()
        self.cfg = cfg
        cc = _CResNetConfig(cfg.tile, cfg.block, (C.c_int32 * 4)(*cfg.depths), cfg.width, cfg.mil_hidden, cfg.n_classes,
                            cfg.bn_eps, 0)
        h = C.c_void_p()
        self._check(self.lib.resnet_ctx_create(C.byref(cc), C.byref(h)), "resnet_ctx_create")
        self.ctx = h
        self._keep = []

    def __del__(self):
        try:
            if getattr(self, "ctx", None):
                self.lib.resnet_ctx_destroy(self.ctx)
                self.ctx = None
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != 0:
            raise SlideError(rc, what, self.lib.slide_last_hip_error())

    def resnet_param_count(self):
        return int(self.lib.resnet_param_count(self.ctx))

    def resnet_feature_dim(self):
        return int(self.lib.resnet_feature_dim(self.ctx))

    def param_layout(self):
        """[(name, offset, length)] in layout order."""
        out = []
        buf = C.create_string_buffer(64)
        off, ln = C.c_size_t(), C.c_size_t()
        for i in range(self.lib.resnet_param_tensors(self.ctx)):
            self._check(self.lib.resnet_param_name(self.ctx, i, buf, 64, C.byref(off), C.byref(ln)), "resnet_param_name")
            out.append((buf.value.decode(), off.value, ln.value))
        return out

    def resnet_arena_bytes(self, n_tiles):
        return int(self.lib.resnet_arena_bytes(self.ctx, n_tiles))

    def resnet_bind(self, params, grads, arena):
        self._keep = [params, grads, arena]
        self._check(self.lib.resnet_bind(self.ctx, _ptr(params), _ptr(grads), _ptr(arena),
                                         arena.numel() * arena.element_size()), "resnet_bind")

    def resnet_encoder_fwd_tiles(self, pixels, n_tiles, feats_out, stream=None):
        self._check(self.lib.resnet_encoder_fwd_tiles(self.ctx, _ptr(pixels), n_tiles, _ptr(feats_out), _stream(stream)),
                    "resnet_encoder_fwd_tiles")

    def resnet_encoder_bwd_tiles(self, dfeats, n_tiles, accumulate, stream=None):
        self._check(self.lib.resnet_encoder_bwd_tiles(self.ctx, _ptr(dfeats), n_tiles, int(accumulate), _stream(stream)),
                    "resnet_encoder_bwd_tiles")

    def resnet_slide_step_fwd(self, pixels, N, label, loss=None, logits=None, alpha=None, stream=None):
        self._check(self.lib.resnet_slide_step_fwd(self.ctx, _ptr(pixels), N, label, _ptr(loss), _ptr(logits), _ptr(alpha),
                                                   _stream(stream)), "resnet_slide_step_fwd")

    def resnet_slide_step_bwd(self, accumulate, stream=None):
        self._check(self.lib.resnet_slide_step_bwd(self.ctx, int(accumulate), _stream(stream)), "resnet_slide_step_bwd")

    def resnet_features(self):
        return self.lib.resnet_features(self.ctx)

    def resnet_feature_grads(self):
        return self.lib.resnet_feature_grads(self.ctx)

    def resnet_saved_activations(self):
        return int(self.lib.resnet_saved_activations(self.ctx))

    def resnet_saved_activation(self, index):
        """(device pointer, side, channels) of saved activation `index`."""
        p, side, ch = C.c_void_p(), C.c_int32(), C.c_int32()
        self._check(self.lib.resnet_saved_activation(self.ctx, index, C.byref(p), C.byref(side), C.byref(ch)),
                    "resnet_saved_activation")
        return p.value, side.value, ch.value

    def resnet_prof_begin(self, kernel_id):
        self._check(self.lib.resnet_prof_begin(self.ctx, kernel_id), "resnet_prof_begin")

    def resnet_prof_end(self):
        ms, n, fl, by = C.c_double(), C.c_int(), C.c_double(), C.c_double()
        self._check(self.lib.resnet_prof_end(self.ctx, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)), "resnet_prof_end")
        return ms.value, n.value, fl.value, by.value

    def resnet_prof_family(self, kernel_id):
        ms, n, fl, by = C.c_double(), C.c_int(), C.c_double(), C.c_double()
        self._check(self.lib.resnet_prof_family(self.ctx, kernel_id, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)),
                    "resnet_prof_family")
        return ms.value, n.value, fl.value, by.value

    def kernel_names(self):
        out, i = [], 0
        while True:
            s = self.lib.resnet_kernel_name(i)
            if s is None:
                return out
            out.append(s.decode())
            i += 1
