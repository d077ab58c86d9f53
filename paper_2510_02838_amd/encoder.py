"""ctypes binding of the Encode-stage entry points declared in include/encoder.h (argument
marshalling only; every step of the encoder runs in the HIP library)."""
import ctypes as C

import numpy as np

from .binding import lib, DitError, DIT_OK

_vp, _i, _sz, _fp, _ip = C.c_void_p, C.c_int, C.c_size_t, C.POINTER(C.c_float), C.POINTER(C.c_int)


class enc_config(C.Structure):
    _fields_ = [("vocab", C.c_int), ("d_model", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int),
                ("d_ff", C.c_int), ("n_layers", C.c_int)]


_SIGS = {
    "enc_create": (_i, [C.POINTER(enc_config), _i, _vp, C.POINTER(_vp)]),
    "enc_destroy": (None, [_vp]),
    "enc_last_error": (C.c_char_p, [_vp]),
    "enc_weight_bytes": (_sz, [_vp]),
    "enc_workspace_bytes": (_sz, [_vp, _i, _ip]),
    "enc_bind": (_i, [_vp, _vp, _sz, _vp, _sz]),
    "enc_init_weights": (_i, [_vp, C.c_uint64, C.c_float]),
    "enc_tensor_count": (_i, [_vp]),
    "enc_tensor_info": (_i, [_vp, _i, C.c_char_p, _sz, _ip, _ip, _ip]),
    "enc_set_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "enc_get_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "enc_forward": (_i, [_vp, _i, _ip, _vp, _vp, _vp]),
    "enc_set_tap": (_i, [_vp, C.c_char_p, _vp, _sz]),
    "enc_clear_taps": (None, [_vp]),
}
EXPORTS = sorted(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
    globals()[_name] = _f


def _lens(lens):
    a = np.ascontiguousarray(lens, dtype=np.int32)
    return a, a.ctypes.data_as(_ip)


class Encoder:
    """One encoder instance; weights and workspace are torch tensors owned by this object."""

    def __init__(self, arch, device=0, bind=True, stream=None):
        self.cfg = enc_config(arch["vocab"], arch["d_model"], arch["n_heads"], arch["head_dim"], arch["d_ff"],
                              arch["n_layers"])
        self.arch = arch
        self.ctx = _vp()
        st = enc_create(C.byref(self.cfg), device, stream, C.byref(self.ctx))    # stream: HIP stream handle or None (default stream)
        if st != DIT_OK:
            raise DitError(st, "enc_create rejected the configuration")
        self.device = device
        self.weights = self.workspace = None
        self._keep = {}
        if bind:
            import torch
            self.torch = torch
            self.weights = torch.empty(self.weight_bytes(), dtype=torch.uint8, device=f"cuda:{device}")

    def close(self):
        if self.ctx:
            enc_destroy(self.ctx)
            self.ctx = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st):
        if st != DIT_OK:
            raise DitError(st, enc_last_error(self.ctx).decode())

    def weight_bytes(self):
        return enc_weight_bytes(self.ctx)

    def workspace_bytes(self, lens):
        a, p = _lens(lens)
        return enc_workspace_bytes(self.ctx, len(a), p)

    def ensure_workspace(self, lens):
        need = self.workspace_bytes(lens)
        if need == 0:
            raise DitError(2, "invalid sequence lengths")
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = self.torch.empty(need, dtype=self.torch.uint8, device=f"cuda:{self.device}")
        self.check(enc_bind(self.ctx, self.weights.data_ptr(), self.weights.numel(), self.workspace.data_ptr(),
                            self.workspace.numel()))

    def tensors(self):
        out = []
        buf = C.create_string_buffer(128)
        r, c, k = C.c_int(), C.c_int(), C.c_int()
        for i in range(enc_tensor_count(self.ctx)):
            self.check(enc_tensor_info(self.ctx, i, buf, 128, C.byref(r), C.byref(c), C.byref(k)))
            out.append((buf.value.decode(), r.value, c.value, k.value))
        return out

    def init_weights(self, seed, std=0.02):
        self.check(enc_init_weights(self.ctx, seed, std))

    def set_tensor(self, name, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32)
        self.check(enc_set_tensor(self.ctx, name.encode(), a.ctypes.data_as(_fp), a.size))

    def get_tensor(self, name, shape):
        a = np.empty(shape, dtype=np.float32)
        self.check(enc_get_tensor(self.ctx, name.encode(), a.ctypes.data_as(_fp), a.size))
        return a

    def set_params(self, params):
        for name, arr in params.items():
            self.set_tensor(name, arr)

    def forward(self, lens, tokens, out_bf16=None, out_f32=None):
        a, p = _lens(lens)
        self.check(enc_forward(self.ctx, len(a), p, tokens.data_ptr(),
                               out_bf16.data_ptr() if out_bf16 is not None else None,
                               out_f32.data_ptr() if out_f32 is not None else None))

    def set_tap(self, point, tensor):
        self._keep[point] = tensor
        self.check(enc_set_tap(self.ctx, point.encode(), tensor.data_ptr(), tensor.numel() * tensor.element_size()))

    def clear_taps(self):
        enc_clear_taps(self.ctx)
        self._keep.clear()
