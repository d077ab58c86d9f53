"""ctypes binding of libdit.so: the same names as include/dit.h, argument marshalling only.

Nothing is computed here.  Device buffers are torch tensors (torch is used for device
memory and streams); `DiT` bundles a context with its weight arena and workspace.
The import fails loudly when the built library is missing: there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DIT_LIB_PATH: another build of the same library (A/B timing of two builds in one session)
LIB_PATH = os.environ.get("DIT_LIB_PATH") or os.path.join(_HERE, "libdit.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2510_02838_amd.build` "
                      "(or __graft_entry__.build()) first")
lib = C.CDLL(LIB_PATH)

DIT_OK = 0
STATUS_NAMES = {0: "DIT_OK", 1: "DIT_EINVAL", 2: "DIT_ESHAPE", 3: "DIT_ENOMEM", 4: "DIT_EDEVICE",
                5: "DIT_EUNSUPPORTED", 6: "DIT_ENOTFOUND"}
FAMILY = {"J": 0, "F": 1, "W": 2}
PROF_CLASSES = ["gemm", "attention", "ln_modulate", "qknorm_rope_vt", "update", "other"]


class dit_config(C.Structure):
    _fields_ = [("family", C.c_int), ("n_blocks", C.c_int), ("n_single", C.c_int), ("hidden", C.c_int),
                ("n_heads", C.c_int), ("head_dim", C.c_int), ("mlp_hidden", C.c_int), ("latent_ch", C.c_int),
                ("patch_t", C.c_int), ("patch_h", C.c_int), ("patch_w", C.c_int), ("cond_dim", C.c_int),
                ("rope_axes", C.c_int * 3), ("rope_theta", C.c_float), ("act_dtype", C.c_int)]


class dit_req(C.Structure):
    _fields_ = [("frames", C.c_int), ("height", C.c_int), ("width", C.c_int), ("n_cond", C.c_int)]


_vp, _i, _sz, _fp = C.c_void_p, C.c_int, C.c_size_t, C.POINTER(C.c_float)
_ip = C.POINTER(C.c_int)
_SIGS = {
    "dit_create": (_i, [C.POINTER(dit_config), _i, _vp, C.POINTER(_vp)]),
    "dit_destroy": (None, [_vp]),
    "dit_set_stream": (_i, [_vp, _vp]),
    "dit_last_error": (C.c_char_p, [_vp]),
    "dit_weight_bytes": (_sz, [_vp]),
    "dit_workspace_bytes": (_sz, [_vp, _i, C.POINTER(dit_req), _i]),
    "dit_attention_plan": (_i, [_vp, _i, C.POINTER(dit_req), C.POINTER(C.c_int)]),
    "dit_bind": (_i, [_vp, _vp, _sz, _vp, _sz]),
    "dit_init_weights": (_i, [_vp, C.c_uint64, C.c_float]),
    "dit_tensor_count": (_i, [_vp]),
    "dit_tensor_info": (_i, [_vp, _i, C.c_char_p, _sz, _ip, _ip, _ip]),
    "dit_set_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "dit_get_tensor": (_i, [_vp, C.c_char_p, _fp, _sz]),
    "dit_denoise_step": (_i, [_vp, _i, C.POINTER(dit_req), _vp, _vp, _fp, _fp, _i, _vp]),
    "dit_sample": (_i, [_vp, _i, C.POINTER(dit_req), _vp, _vp, _fp, _i, _i]),
    "dit_set_tap": (_i, [_vp, C.c_char_p, _vp, _sz]),
    "dit_tap_info": (_i, [_vp, C.c_char_p, _ip, _ip, _ip]),
    "dit_clear_taps": (None, [_vp]),
    "dit_profile_enable": (_i, [_vp, _i]),
    "dit_profile_read": (_i, [_vp, _i, C.POINTER(C.c_double), C.POINTER(C.c_longlong),
                              C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "dit_op_gemm": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp]),
    "dit_op_gemm_qknorm": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _i, _i, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp,
                                _i, C.c_float]),
    "dit_op_gemm_splitk": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp, _i, _vp, _sz]),
    "dit_op_gemm_splitk_static": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _vp, _i, _vp, _i]),
    "dit_op_gemm_variant": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _i]),
    "dit_op_attention_work_bytes": (_sz, [_i, _ip]),
    "dit_op_attention": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _vp, _i, _i, _i, _i, _ip, _ip, _ip, _vp, _sz, _i, C.c_float]),
    "dit_op_ln_modulate": (_i, [_vp, _vp, _vp, _i, _i, _vp, _vp, _i, _vp]),
    "dit_op_latent_update": (_i, [_vp, _vp, _vp, C.c_longlong, C.c_float, C.c_float]),
}
EXPORTS = sorted(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
    globals()[_name] = _f


class DitError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


def make_config(arch):
    cfg = dit_config()
    cfg.family = FAMILY[arch["family"]]
    cfg.n_blocks, cfg.n_single = arch["n_blocks"], arch["n_single"]
    cfg.hidden, cfg.n_heads, cfg.head_dim = arch["hidden"], arch["n_heads"], arch["head_dim"]
    cfg.mlp_hidden, cfg.latent_ch = arch["mlp_hidden"], arch["latent_ch"]
    cfg.patch_t, cfg.patch_h, cfg.patch_w = arch["patch"]
    cfg.cond_dim = arch["cond_dim"]
    for a in range(3):
        cfg.rope_axes[a] = arch["rope_axes"][a]
    cfg.rope_theta = arch["rope_theta"]
    cfg.act_dtype = {"f32": 0, "bf16": 1}[arch.get("act_dtype", "bf16")]
    return cfg


def make_reqs(reqs):
    arr = (dit_req * len(reqs))()
    for i, (f, h, w, nc) in enumerate(reqs):
        arr[i].frames, arr[i].height, arr[i].width, arr[i].n_cond = f, h, w, nc
    return arr


def _fptr(a):
    return a.ctypes.data_as(_fp)


class DiT:
    """A context plus its torch-allocated weight arena and workspace."""

    def __init__(self, arch, device=0, stream=None, bind=True):
        self.arch = dict(arch)
        self.cfg = make_config(arch)
        self.device = device
        self.ctx = _vp()
        st = dit_create(C.byref(self.cfg), device, stream, C.byref(self.ctx))
        if st != DIT_OK:
            raise DitError(st, "dit_create rejected the configuration")
        self.weights = None
        self.workspace = None
        self._keep = {}
        if bind:
            import torch
            self.torch = torch
            self.weights = torch.empty(self.weight_bytes(), dtype=torch.uint8, device=f"cuda:{device}")

    def close(self):
        if self.ctx:
            dit_destroy(self.ctx)
            self.ctx = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st):
        if st != DIT_OK:
            raise DitError(st, dit_last_error(self.ctx).decode())

    def weight_bytes(self):
        return dit_weight_bytes(self.ctx)

    def workspace_bytes(self, reqs, max_steps):
        return dit_workspace_bytes(self.ctx, len(reqs), make_reqs(reqs), max_steps)

    def attention_plan(self, reqs):
        """(queries per workgroup, query blocks per head, blocks run as key-split shares, shares each)."""
        out = (C.c_int * 4)()
        self.check(dit_attention_plan(self.ctx, len(reqs), make_reqs(reqs), out))
        return tuple(out)

    def ensure_workspace(self, reqs, max_steps):
        need = self.workspace_bytes(reqs, max_steps)
        if need == 0:
            raise DitError(2, "invalid request list")
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = self.torch.empty(need, dtype=self.torch.uint8, device=f"cuda:{self.device}")
        self.check(dit_bind(self.ctx, self.weights.data_ptr(), self.weights.numel(),
                            self.workspace.data_ptr(), self.workspace.numel()))

    def tensors(self):
        out = []
        buf = C.create_string_buffer(128)
        r, c, k = C.c_int(), C.c_int(), C.c_int()
        for i in range(dit_tensor_count(self.ctx)):
            self.check(dit_tensor_info(self.ctx, i, buf, 128, C.byref(r), C.byref(c), C.byref(k)))
            out.append((buf.value.decode(), r.value, c.value, k.value))
        return out

    def init_weights(self, seed, std=0.02):
        self.check(dit_init_weights(self.ctx, seed, std))

    def set_tensor(self, name, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32)
        self.check(dit_set_tensor(self.ctx, name.encode(), _fptr(a), a.size))

    def get_tensor(self, name, shape):
        a = np.empty(shape, dtype=np.float32)
        self.check(dit_get_tensor(self.ctx, name.encode(), _fptr(a), a.size))
        return a

    def set_params(self, params):
        for name, arr in params.items():
            self.set_tensor(name, arr)

    def denoise_step(self, reqs, latents, cond, sigma_cur, sigma_next, kind=0, v_out=None):
        sc = np.ascontiguousarray(sigma_cur, dtype=np.float32)
        sn = np.ascontiguousarray(sigma_next, dtype=np.float32)
        self.check(dit_denoise_step(self.ctx, len(reqs), make_reqs(reqs), latents.data_ptr(), cond.data_ptr(),
                                    _fptr(sc), _fptr(sn), kind, v_out.data_ptr() if v_out is not None else None))

    def sample(self, reqs, latents, cond, sigmas, kind=0):
        sg = np.ascontiguousarray(sigmas, dtype=np.float32)
        T = sg.shape[1] - 1
        self.check(dit_sample(self.ctx, len(reqs), make_reqs(reqs), latents.data_ptr(), cond.data_ptr(),
                              _fptr(sg), T, kind))

    def set_tap(self, point, tensor):
        self._keep[point] = tensor
        self.check(dit_set_tap(self.ctx, point.encode(), tensor.data_ptr(), tensor.numel() * tensor.element_size()))

    def tap_info(self, point):
        r, c, e = C.c_int(), C.c_int(), C.c_int()
        self.check(dit_tap_info(self.ctx, point.encode(), C.byref(r), C.byref(c), C.byref(e)))
        return r.value, c.value, e.value

    def clear_taps(self):
        dit_clear_taps(self.ctx)
        self._keep.clear()

    def profile_enable(self, on=True):
        self.check(dit_profile_enable(self.ctx, 1 if on else 0))

    def profile_read(self):
        out = {}
        for k, name in enumerate(PROF_CLASSES):
            ms, n, fl, by = C.c_double(), C.c_longlong(), C.c_double(), C.c_double()
            self.check(dit_profile_read(self.ctx, k, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)))
            out[name] = dict(ms=ms.value, launches=n.value, flop=fl.value, bytes=by.value)
        return out
