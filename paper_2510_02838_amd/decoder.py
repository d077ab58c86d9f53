"""ctypes binding of the Decode-stage entry points declared in include/decoder.h (argument
marshalling only; every step of the decoder runs in the HIP library)."""
import ctypes as C

import numpy as np

from .binding import lib, DitError, DIT_OK

_vp, _i, _sz, _fp, _ip = C.c_void_p, C.c_int, C.c_size_t, C.POINTER(C.c_float), C.POINTER(C.c_int)
DEC_MAX_LEVELS = 6


class dec_config(C.Structure):
    _fields_ = [("latent_ch", C.c_int), ("out_ch", C.c_int), ("n_levels", C.c_int),
                ("channels", C.c_int * DEC_MAX_LEVELS), ("n_res", C.c_int), ("temporal", C.c_int), ("t_up", C.c_int)]


_SIGS = {
    "dec_create": (_i, [C.POINTER(dec_config), _i, _vp, C.POINTER(_vp)]),
    "dec_destroy": (None, [_vp]),
    "dec_last_error": (C.c_char_p, [_vp]),
    "dec_frames_out": (_i, [_vp, _i]),
    "dec_weight_bytes": (_sz, [_vp]),
    "dec_workspace_bytes": (_sz, [_vp, _i, _i, _i]),
    "dec_bind": (_i, [_vp, _vp, _sz, _vp, _sz]),
    "dec_init_weights": (_i, [_vp, C.c_uint64, C.c_float]),
    "dec_tensor_count": (_i, [_vp]),
    "dec_tensor_info": (_i, [_vp, _i, C.c_char_p, _sz, _ip, _ip, _ip]),
    "dec_set_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "dec_get_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "dec_forward": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "dec_set_tap": (_i, [_vp, C.c_char_p, _vp, _sz]),
    "dec_clear_taps": (None, [_vp]),
}
EXPORTS = sorted(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
    globals()[_name] = _f


def make_config(arch):
    ch = list(arch["channels"])
    if not 1 <= len(ch) <= DEC_MAX_LEVELS:
        raise DitError(1, "1..6 levels")
    arr = (C.c_int * DEC_MAX_LEVELS)(*(ch + [0] * (DEC_MAX_LEVELS - len(ch))))
    # a "t_up" entry makes it the causal video decoder
    return dec_config(arch["latent_ch"], arch["out_ch"], len(ch), arr, arch["n_res"], int("t_up" in arch), arch.get("t_up", 0))


class Decoder:
    """One decoder instance; weights and workspace are torch tensors owned by this object."""

    def __init__(self, arch, device=0, bind=True, stream=None):
        self.cfg = make_config(arch)
        self.arch = arch
        self.ctx = _vp()
        st = dec_create(C.byref(self.cfg), device, stream, C.byref(self.ctx))    # stream: HIP stream handle or None (default stream)
        if st != DIT_OK:
            raise DitError(st, "dec_create rejected the configuration")
        self.device = device
        self.weights = self.workspace = None
        self._keep = {}
        if bind:
            import torch
            self.torch = torch
            self.weights = torch.empty(self.weight_bytes(), dtype=torch.uint8, device=f"cuda:{device}")

    def close(self):
        if self.ctx:
            dec_destroy(self.ctx)
            self.ctx = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st):
        if st != DIT_OK:
            raise DitError(st, dec_last_error(self.ctx).decode())

    def weight_bytes(self):
        return dec_weight_bytes(self.ctx)

    def workspace_bytes(self, h, w, n=1):
        return dec_workspace_bytes(self.ctx, n, h, w)

    def frames_out(self, n):
        return dec_frames_out(self.ctx, n)

    def up_factor(self):
        return 1 << (self.cfg.n_levels - 1)

    def ensure_workspace(self, h, w, n=1):
        need = self.workspace_bytes(h, w, n)
        if need == 0:
            raise DitError(2, "invalid latent size")
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = self.torch.empty(need, dtype=self.torch.uint8, device=f"cuda:{self.device}")
        self.check(dec_bind(self.ctx, self.weights.data_ptr(), self.weights.numel(), self.workspace.data_ptr(),
                            self.workspace.numel()))

    def tensors(self):
        out = []
        buf = C.create_string_buffer(128)
        r, c, k = C.c_int(), C.c_int(), C.c_int()
        for i in range(dec_tensor_count(self.ctx)):
            self.check(dec_tensor_info(self.ctx, i, buf, 128, C.byref(r), C.byref(c), C.byref(k)))
            out.append((buf.value.decode(), r.value, c.value, k.value))
        return out

    def init_weights(self, seed, std=0.02):
        self.check(dec_init_weights(self.ctx, seed, std))

    def set_tensor(self, name, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32)
        self.check(dec_set_tensor(self.ctx, name.encode(), a.ctypes.data_as(_fp), a.size))

    def get_tensor(self, name, shape):
        a = np.empty(shape, dtype=np.float32)
        self.check(dec_get_tensor(self.ctx, name.encode(), a.ctypes.data_as(_fp), a.size))
        return a

    def set_params(self, params):
        for name, arr in params.items():
            self.set_tensor(name, arr)

    def forward(self, h, w, latent, image, n=1):
        """latent: fp32 [n][latent_ch][h][w]; image: fp32 [n][h*f][w*f][out_ch], f = up_factor().
        Video decoder: latent [latent_ch][n][h][w] of one video, image [frames_out(n)][h*f][w*f][out_ch]."""
        self.check(dec_forward(self.ctx, n, h, w, latent.data_ptr(), image.data_ptr()))

    def set_tap(self, point, tensor):
        self._keep[point] = tensor
        self.check(dec_set_tap(self.ctx, point.encode(), tensor.data_ptr(), tensor.numel() * tensor.element_size()))

    def clear_taps(self):
        dec_clear_taps(self.ctx)
        self._keep.clear()
