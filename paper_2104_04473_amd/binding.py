"""ctypes binding of libptdp.so: same names as include/ptdp.h, argument marshalling only.

Pointers are passed as integers (``tensor.data_ptr()``), streams as the integer handle of a
``torch.cuda.Stream`` (``stream.cuda_stream``).  Functions return the library's status code;
``check`` turns a negative status into ``PtdpError``.
"""
import ctypes as C
import os

# torch ships its own HIP runtime; it must be the one already loaded when libptdp.so is opened, so
# that the library and the tensors / streams it is handed live in the same runtime.
import torch  # noqa: F401  (device memory and streams only)

_HERE = os.path.dirname(os.path.abspath(__file__))
# PTDP_LIB names another build of the same library (e.g. the host-sanitizer build of `build.py --sanitize`)
LIB_PATH = os.environ.get("PTDP_LIB") or os.path.join(_HERE, "libptdp.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libptdp.so is not built (expected at %s); run `python -m paper_2104_04473_amd.build`. "
        "There is no fallback path." % LIB_PATH)
lib = C.CDLL(LIB_PATH)

OK, E_INVALID_ARG, E_UNSUPPORTED, E_NULL_PTR, E_TOO_SMALL, E_HIP, E_STATE = 0, -1, -2, -3, -4, -5, -6
F32, BF16 = 0, 1
GELU_ERF, GELU_TANH = 0, 1
GEMM_NN, GEMM_NT, GEMM_TN = 0, 1, 2
STASH_FIELDS = ("X", "U", "QKV", "CTX", "X1", "U2", "Z", "G", "MU1", "RSTD1", "MU2", "RSTD2", "LSE")
WS_FIELDS = ("DO", "DU", "DX1", "CHAIN", "DZ", "DCTX", "DQKV", "DMO")
PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")
PROF_FAMILIES = 15


class PtdpError(RuntimeError):
    def __init__(self, status, where=""):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


class LayerCfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("h", C.c_int32), ("a", C.c_int32), ("t", C.c_int32),
                ("s", C.c_int32), ("b", C.c_int32), ("dtype", C.c_int32), ("causal", C.c_int32),
                ("gelu_mode", C.c_int32), ("p_hidden", C.c_float), ("ln_eps", C.c_float), ("seed", C.c_uint64)]


class LayerParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class LayerGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class Step(C.Structure):
    _fields_ = [("kind", C.c_int32), ("chunk", C.c_int32), ("microbatch", C.c_int32)]


class ProfEntry(C.Structure):
    _fields_ = [("ms", C.c_double), ("work", C.c_double), ("launches", C.c_int64)]


def make_cfg(h, a, t, s, b, dtype=BF16, p_hidden=0.0, ln_eps=1e-5, seed=0, gelu_mode=GELU_ERF, causal=1):
    return LayerCfg(C.sizeof(LayerCfg), h, a, t, s, b, dtype, causal, gelu_mode, p_hidden, ln_eps, seed)


_vp, _i, _i64, _u64, _u32, _f, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_uint32, C.c_float, C.c_size_t
_cfgp = C.POINTER(LayerCfg)

# name -> (restype, argtypes); one entry per declaration in include/ptdp.h
SIGNATURES = {
    "ptdp_status_string": (C.c_char_p, [_i]),
    "ptdp_cfg_validate": (_i, [_cfgp]),
    "ptdp_layer_stash_bytes": (_sz, [_cfgp]),
    "ptdp_stash_offset": (_sz, [_cfgp, _i]),
    "ptdp_workspace_bytes": (_sz, [_cfgp]),
    "ptdp_workspace_offset": (_sz, [_cfgp, _i]),
    "ptdp_layer_flops_fwd": (_i64, [_cfgp]),
    "ptdp_batch_time": (C.c_double, [_i64, _i64, _i, C.c_double, C.c_double]),
    "ptdp_hash": (_u64, [_u64, _u32, _u32, _u64, _u64]),
    "ptdp_chunk_create": (_i, [_cfgp, _i, _i, C.POINTER(_vp)]),
    "ptdp_chunk_destroy": (None, [_vp]),
    "ptdp_chunk_n_layers": (_i, [_vp]),
    "ptdp_chunk_bind_params": (_i, [_vp, _i, C.POINTER(LayerParams)]),
    "ptdp_chunk_bind_grads": (_i, [_vp, _i, C.POINTER(LayerGrads)]),
    "ptdp_layer_forward": (_i, [_vp, _i, _i64, _vp, _vp, _vp, _vp, _vp]),
    "ptdp_layer_backward": (_i, [_vp, _i, _i64, _vp, _vp, _vp, _vp, _vp]),
    "ptdp_chunk_forward": (_i, [_vp, _i64, _vp, _vp, _vp, _vp, _vp]),
    "ptdp_chunk_backward": (_i, [_vp, _i64, _vp, _vp, _vp, _vp, _vp]),
    "ptdp_checkpoint_bytes": (_sz, [_cfgp]),
    "ptdp_chunk_n_checkpoints": (_i, [_vp, _i]),
    "ptdp_chunk_forward_ckpt": (_i, [_vp, _i64, _vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "ptdp_chunk_backward_ckpt": (_i, [_vp, _i64, _vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "ptdp_schedule_build": (_i, [_i, _i, _i, _i, C.POINTER(Step), _i, C.POINTER(_i)]),
    "ptdp_schedule_peak_inflight": (_i, [_i, _i, _i, _i]),
    "ptdp_schedule_run": (_i, [C.POINTER(_vp), _i, _i, C.POINTER(Step), _i, C.POINTER(_vp), C.POINTER(_vp),
                               C.POINTER(_vp), C.POINTER(_vp), _vp, _sz, _i, _vp, _vp]),
    "ptdp_schedule_run_ckpt": (_i, [C.POINTER(_vp), _i, _i, C.POINTER(Step), _i, C.POINTER(_vp), C.POINTER(_vp),
                                    C.POINTER(_vp), C.POINTER(_vp), _vp, _sz, _i, _i, _vp, _vp, _vp]),
    "ptdp_lm_workspace_bytes": (_sz, [_cfgp, _i]),
    "ptdp_logit_flops_fwd": (_i64, [_cfgp, _i]),
    "ptdp_embedding_forward": (_i, [_cfgp, _i, _i, _vp, _vp, _vp, _vp, _i64, _vp]),
    "ptdp_embedding_backward": (_i, [_cfgp, _i, _i, _vp, _vp, _vp, _vp, _vp, _i64, _vp]),
    "ptdp_lm_head_step": (_i, [_cfgp, _i, _i, _vp, _vp, _vp, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "ptdp_layernorm_fwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _f, _vp]),
    "ptdp_layernorm_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _vp]),
    "ptdp_bias_gelu_fwd": (_i, [_i, _i, _vp, _vp, _vp, _i, _i, _vp]),
    "ptdp_bias_gelu_bwd": (_i, [_i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _vp]),
    "ptdp_bias_dropout_add_fwd": (_i, [_i, _vp, _vp, _vp, _vp, _i, _i, _f, _u64, _u32, _u32, _u64, _vp]),
    "ptdp_bias_dropout_add_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _i, _i, _f, _u64, _u32, _u32, _u64, _vp]),
    "ptdp_bias_dropout_add_bwd_noalloc": (_i, [_i, _vp, _vp, _vp, _i, _i, _f, _u64, _u32, _u32, _u64, _vp]),
    "ptdp_noalloc_scratch_bytes": (_sz, []),
    "ptdp_colsum_scratch_bytes": (_sz, [_i, _i]),
    "ptdp_layernorm_bwd_scratch_bytes": (_sz, [_i, _i]),
    "ptdp_dropout_mask": (_i, [_vp, _i64, _f, _u64, _u32, _u32, _u64, _vp]),
    "ptdp_gemm": (_i, [_i, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _sz, _vp]),
    "ptdp_gemm_workspace_bytes": (_sz, []),
    "ptdp_gemm_plan": (_i, [_i, _i, _i, _i, _i, _i, _sz, C.POINTER(_i), C.POINTER(_i), C.POINTER(_i), C.POINTER(_i)]),
    "ptdp_attn_fwd": (_i, [_i, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "ptdp_attn_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "ptdp_attn_masked_fwd": (_i, [_i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "ptdp_attn_masked_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "ptdp_chunk_set_mask": (_i, [_vp, _vp]),
    "ptdp_ceiling_mfma": (_i, [_vp, _i, _i, _i, C.POINTER(C.c_double), _vp]),
    "ptdp_ceiling_copy": (_i, [_vp, _vp, _sz, _vp]),
    "ptdp_prof_enable": (_i, [_i]),
    "ptdp_prof_collect": (_i, [C.POINTER(ProfEntry)]),
    "ptdp_prof_family_name": (C.c_char_p, [_i]),
}

for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args
    globals()[_name] = _fn


def status_string(status):
    return lib.ptdp_status_string(status).decode()


def check(status, where=""):
    if status != OK:
        raise PtdpError(status, where)
    return status


def stream_handle(stream=None):
    """Integer hipStream_t of a torch stream (default: torch's current stream)."""
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class Chunk:
    """Owner of a ptdp_chunk handle plus the torch tensors whose pointers it borrows."""

    def __init__(self, cfg, n_layers, first_global_layer=0):
        self.cfg = cfg
        self.n_layers = n_layers
        self.handle = _vp()
        check(lib.ptdp_chunk_create(C.byref(cfg), n_layers, first_global_layer, C.byref(self.handle)), "chunk_create")
        self._keep = []

    def bind(self, layer, params, grads=None):
        """params / grads: dict name -> torch tensor on the GPU."""
        P = LayerParams(*[params[n].data_ptr() for n in PARAM_NAMES])
        check(lib.ptdp_chunk_bind_params(self.handle, layer, C.byref(P)), "bind_params")
        self._keep.append(params)
        if grads is not None:
            G = LayerGrads(*[grads[n].data_ptr() for n in PARAM_NAMES])
            check(lib.ptdp_chunk_bind_grads(self.handle, layer, C.byref(G)), "bind_grads")
            self._keep.append(grads)

    def stash_bytes(self):
        return lib.ptdp_layer_stash_bytes(C.byref(self.cfg)) * self.n_layers

    def workspace_bytes(self):
        return lib.ptdp_workspace_bytes(C.byref(self.cfg))

    def layer_forward(self, layer, mb, x, y, stash, ws, stream=None):
        return lib.ptdp_layer_forward(self.handle, layer, mb, x, y, stash, ws, stream_handle(stream))

    def layer_backward(self, layer, mb, dy, dx, stash, ws, stream=None):
        return lib.ptdp_layer_backward(self.handle, layer, mb, dy, dx, stash, ws, stream_handle(stream))

    def forward(self, mb, x, y, stash, ws, stream=None):
        return lib.ptdp_chunk_forward(self.handle, mb, x, y, stash, ws, stream_handle(stream))

    def backward(self, mb, dy, dx, stash, ws, stream=None):
        return lib.ptdp_chunk_backward(self.handle, mb, dy, dx, stash, ws, stream_handle(stream))

    def checkpoint_bytes(self, seg_layers):
        return lib.ptdp_chunk_n_checkpoints(self.handle, seg_layers) * lib.ptdp_checkpoint_bytes(C.byref(self.cfg))

    def forward_ckpt(self, mb, x, y, ckpt, seg_layers, seg_stash, ws, stream=None):
        return lib.ptdp_chunk_forward_ckpt(self.handle, mb, x, y, ckpt, seg_layers, seg_stash, ws,
                                           stream_handle(stream))

    def backward_ckpt(self, mb, dy, dx, ckpt, seg_layers, seg_stash, ws, stream=None):
        return lib.ptdp_chunk_backward_ckpt(self.handle, mb, dy, dx, ckpt, seg_layers, seg_stash, ws,
                                            stream_handle(stream))

    def close(self):
        if self.handle:
            lib.ptdp_chunk_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def schedule_build(p, v, m, rank):
    n = _i(0)
    check(lib.ptdp_schedule_build(p, v, m, rank, None, 0, C.byref(n)), "schedule_build")
    steps = (Step * n.value)()
    check(lib.ptdp_schedule_build(p, v, m, rank, steps, n.value, C.byref(n)), "schedule_build")
    return steps


def stash_offsets(cfg):
    return {name: lib.ptdp_stash_offset(C.byref(cfg), i) for i, name in enumerate(STASH_FIELDS)}


def workspace_offsets(cfg):
    return {name: lib.ptdp_workspace_offset(C.byref(cfg), i) for i, name in enumerate(WS_FIELDS)}


def prof_collect():
    arr = (ProfEntry * PROF_FAMILIES)()
    check(lib.ptdp_prof_collect(arr), "prof_collect")
    return {lib.ptdp_prof_family_name(i).decode(): (arr[i].ms, arr[i].work, arr[i].launches)
            for i in range(PROF_FAMILIES)}
