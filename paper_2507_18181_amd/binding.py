"""Thin ctypes binding of libspecasr.so: the same entry points as include/specasr.h.

Argument marshalling only -- every step of the verification path runs in the HIP
library.  Device buffers are passed as integer addresses (``tensor.data_ptr()``),
host arrays as contiguous numpy int32/uint8 arrays.  Importing this module does
not need a GPU; calling anything that computes does.  There is no CPU fallback:
if the library is missing, loading raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecasr.so")

SPECASR_OK = 0
SPECASR_E_NULL = -1
SPECASR_E_CONFIG = -2
SPECASR_E_TREE = -3
SPECASR_E_KV_OVERFLOW = -4
SPECASR_E_WORKSPACE = -5
SPECASR_E_HIP = -6
SPECASR_E_UNSUPPORTED = -7
SPECASR_E_PATH = -8
SPECASR_F32, SPECASR_BF16 = 0, 1
SPECASR_FLAG_GENERIC_KERNELS = 1
SPECASR_FLAG_NO_REPACK = 2
SPECASR_FLAG_NO_WIDE = 4
SPECASR_MAX_NODES = 64
SPECASR_STATIC_MAX_BATCH = 16

EXPORTS = ("specasr_create", "specasr_destroy", "specasr_workspace_bytes", "specasr_verify_tree",
           "specasr_tree_forward", "specasr_tree_forward_top2", "specasr_prefill", "specasr_accept",
           "specasr_accept_from_logits", "specasr_accept_from_logits_static",
           "specasr_commit", "specasr_strerror", "specasr_last_hip_error", "specasr_abi_version",
           "specasr_uses_mfma", "specasr_profile_stage", "specasr_stage_time",
           "specasr_stage_rows", "specasr_read_ceiling")
SPECASR_STAGE_QKV, SPECASR_STAGE_O, SPECASR_STAGE_GATE_UP, SPECASR_STAGE_DOWN, SPECASR_STAGE_LM_HEAD = range(5)


class specasr_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads",
                                          "head_dim", "d_ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("max_nodes", C.c_int32), ("max_batch", C.c_int32), ("flags", C.c_uint32)]


LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class specasr_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class specasr_weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(specasr_layer_weights))]


class specasr_kv(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("capacity", C.c_int64),
                ("batch", C.c_int32), ("kv_len", C.POINTER(C.c_int32))]


class specasr_tree(C.Structure):
    _fields_ = [("tokens", C.POINTER(C.c_int32)), ("parents", C.POINTER(C.c_int32)),
                ("n_nodes", C.POINTER(C.c_int32)), ("input_embeds", C.c_void_p),
                ("use_embed", C.POINTER(C.c_uint8))]


class specasr_out(C.Structure):
    _fields_ = [("argmax", C.POINTER(C.c_int32)), ("path", C.POINTER(C.c_int32)),
                ("accept_len", C.POINTER(C.c_int32)), ("next_token", C.POINTER(C.c_int32)),
                ("logits", C.c_void_p)]


_lib = None


def load_library(path=None):
    """dlopen the HIP library (fails loudly if it has not been built) and set signatures."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError("libspecasr.so not built: run `python -m paper_2507_18181_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(p)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.specasr_create.restype = C.c_int
    lib.specasr_create.argtypes = [C.POINTER(specasr_config), C.POINTER(specasr_weights), C.POINTER(vp)]
    lib.specasr_destroy.restype = None
    lib.specasr_destroy.argtypes = [vp]
    lib.specasr_workspace_bytes.restype = C.c_size_t
    lib.specasr_workspace_bytes.argtypes = [vp, C.c_int32]
    lib.specasr_verify_tree.restype = C.c_int
    lib.specasr_verify_tree.argtypes = [vp, C.POINTER(specasr_kv), C.POINTER(specasr_tree),
                                        C.POINTER(specasr_out), vp, C.c_size_t, vp]
    lib.specasr_tree_forward.restype = C.c_int
    lib.specasr_tree_forward.argtypes = [vp, C.POINTER(specasr_kv), C.POINTER(specasr_tree), vp, vp,
                                         vp, C.c_size_t, vp]
    lib.specasr_tree_forward_top2.restype = C.c_int
    lib.specasr_tree_forward_top2.argtypes = [vp, C.POINTER(specasr_kv), C.POINTER(specasr_tree), vp,
                                              vp, vp, vp, C.c_size_t, vp]
    lib.specasr_prefill.restype = C.c_int
    lib.specasr_prefill.argtypes = [vp, C.POINTER(specasr_kv), i32p, vp, C.POINTER(C.c_uint8), i32p,
                                    C.c_int32, i32p, vp, C.c_size_t, vp]
    lib.specasr_accept.restype = C.c_int
    lib.specasr_accept.argtypes = [vp, C.POINTER(specasr_tree), C.c_int32, vp, vp, vp, vp, vp,
                                   C.c_size_t, vp]
    lib.specasr_accept_from_logits.restype = C.c_int
    lib.specasr_accept_from_logits.argtypes = [vp, C.POINTER(specasr_tree), C.c_int32, vp, vp, vp,
                                               vp, vp, vp, C.c_size_t, vp]
    lib.specasr_accept_from_logits_static.restype = C.c_int
    lib.specasr_accept_from_logits_static.argtypes = [vp, C.POINTER(specasr_tree), C.c_int32, vp, vp,
                                                      vp, vp, vp, vp]
    lib.specasr_commit.restype = C.c_int
    lib.specasr_commit.argtypes = [vp, C.POINTER(specasr_kv), i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.specasr_strerror.restype = C.c_char_p
    lib.specasr_strerror.argtypes = [C.c_int]
    lib.specasr_last_hip_error.restype = C.c_int32
    lib.specasr_last_hip_error.argtypes = [vp]
    lib.specasr_abi_version.restype = C.c_int32
    lib.specasr_uses_mfma.restype = C.c_int32
    lib.specasr_uses_mfma.argtypes = [vp, C.c_int32]
    lib.specasr_profile_stage.restype = C.c_int
    lib.specasr_profile_stage.argtypes = [vp, C.c_int32, C.c_int32]
    lib.specasr_stage_time.restype = C.c_int
    lib.specasr_stage_time.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_double)]
    lib.specasr_stage_rows.restype = C.c_int
    lib.specasr_stage_rows.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.specasr_read_ceiling.restype = C.c_int
    lib.specasr_read_ceiling.argtypes = [vp, vp, C.c_size_t, C.c_int32, vp, C.POINTER(C.c_double)]
    if path is None:
        _lib = lib
    return lib


class SpecasrError(RuntimeError):
    def __init__(self, status, hip=0):
        self.status = status
        msg = load_library().specasr_strerror(status).decode()
        super().__init__("specasr status %d: %s%s" % (status, msg, (" (hipError %d)" % hip) if hip else ""))


def _i32(a):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _ptr(x):
    """torch tensor / int address / None -> c_void_p value."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def make_config(cfg, dtype, max_nodes, max_batch=1, flags=0):
    return specasr_config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["n_kv_heads"],
                          cfg["head_dim"], cfg["d_ffn"], cfg["vocab"], cfg.get("rms_eps", 1e-5),
                          cfg.get("rope_theta", 10000.0), dtype, max_nodes, max_batch, flags)


def make_weights(w):
    """dict of device tensors (same keys as the workload generator) -> (struct, keepalive)."""
    nl = len(w["layers"])
    arr = (specasr_layer_weights * nl)()
    for l in range(nl):
        for f in LAYER_FIELDS:
            setattr(arr[l], f, _ptr(w["layers"][l][f]))
    sw = specasr_weights(_ptr(w["tok_embed"]), _ptr(w["final_norm"]), _ptr(w["lm_head"]), arr)
    return sw, arr


def specasr_abi_version():
    return int(load_library().specasr_abi_version())


def specasr_strerror(status):
    return load_library().specasr_strerror(status).decode()


def specasr_create(config, weights):
    """-> (status, ctx handle)."""
    ctx = C.c_void_p()
    rc = load_library().specasr_create(C.byref(config) if config is not None else None,
                                       C.byref(weights) if weights is not None else None,
                                       C.byref(ctx))
    return rc, ctx


def specasr_destroy(ctx):
    load_library().specasr_destroy(ctx)


def specasr_workspace_bytes(ctx, batch):
    return int(load_library().specasr_workspace_bytes(ctx, batch))


def specasr_uses_mfma(ctx, rows):
    return int(load_library().specasr_uses_mfma(ctx, rows))


def specasr_profile_stage(ctx, stage, enable):
    """enable: False/0 off, True/1 every launch of the stage, 2 only the wide (prefill) kernel."""
    return load_library().specasr_profile_stage(ctx, stage, int(enable))


def specasr_stage_rows(ctx):
    """-> (status, activation rows summed over the timed launches)."""
    n = C.c_int64(0)
    rc = load_library().specasr_stage_rows(ctx, C.byref(n))
    return rc, n.value


def specasr_stage_time(ctx):
    """-> (status, total_ms, launches, weight_bytes_per_launch)."""
    ms, n, b = C.c_double(0), C.c_int64(0), C.c_double(0)
    rc = load_library().specasr_stage_time(ctx, C.byref(ms), C.byref(n), C.byref(b))
    return rc, ms.value, n.value, b.value


def specasr_read_ceiling(ctx, buf_dev, nbytes, reps=3, stream=None):
    """-> (status, GB/s) of a pure read stream over a device buffer."""
    g = C.c_double(0)
    rc = load_library().specasr_read_ceiling(ctx, _ptr(buf_dev), nbytes, reps, _ptr(stream), C.byref(g))
    return rc, g.value


def specasr_last_hip_error(ctx):
    return int(load_library().specasr_last_hip_error(ctx))


def make_kv(k, v, capacity, kv_len):
    """kv_len: contiguous numpy int32 [batch] (updated in place by verify/commit)."""
    assert kv_len.dtype == np.int32 and kv_len.flags.c_contiguous
    return specasr_kv(_ptr(k), _ptr(v), capacity, kv_len.shape[0], _i32(kv_len))


def make_tree(tokens, parents, n_nodes, input_embeds=None, use_embed=None):
    """tokens/parents: numpy int32 [batch][max_nodes]; n_nodes: numpy int32 [batch]."""
    for a in (tokens, parents, n_nodes):
        assert a.dtype == np.int32 and a.flags.c_contiguous
    ue = None
    if use_embed is not None:
        assert use_embed.dtype == np.uint8 and use_embed.flags.c_contiguous
        ue = use_embed.ctypes.data_as(C.POINTER(C.c_uint8))
    return specasr_tree(_i32(tokens), _i32(parents), _i32(n_nodes), _ptr(input_embeds), ue)


def make_out(argmax, path, accept_len, next_token, logits=None):
    return specasr_out(_i32(argmax), _i32(path), _i32(accept_len), _i32(next_token), _ptr(logits))


def specasr_verify_tree(ctx, kv, tree, out, workspace, workspace_bytes, stream=None):
    return load_library().specasr_verify_tree(ctx, C.byref(kv), C.byref(tree), C.byref(out),
                                              _ptr(workspace), workspace_bytes, _ptr(stream))


def specasr_tree_forward(ctx, kv, tree, argmax_dev, logits_dev, workspace, workspace_bytes,
                         stream=None):
    return load_library().specasr_tree_forward(ctx, C.byref(kv), C.byref(tree), _ptr(argmax_dev),
                                               _ptr(logits_dev), _ptr(workspace), workspace_bytes,
                                               _ptr(stream))


def specasr_tree_forward_top2(ctx, kv, tree, top2_dev, top1_prob_dev, logits_dev, workspace,
                              workspace_bytes, stream=None):
    return load_library().specasr_tree_forward_top2(ctx, C.byref(kv), C.byref(tree), _ptr(top2_dev),
                                                    _ptr(top1_prob_dev), _ptr(logits_dev),
                                                    _ptr(workspace), workspace_bytes, _ptr(stream))


def specasr_prefill(ctx, kv, tokens, input_embeds, use_embed, n_pos, max_pos, next_token, workspace,
                    workspace_bytes, stream=None):
    ue = None if use_embed is None else use_embed.ctypes.data_as(C.POINTER(C.c_uint8))
    return load_library().specasr_prefill(ctx, C.byref(kv), _i32(tokens), _ptr(input_embeds), ue,
                                          _i32(n_pos), max_pos, _i32(next_token), _ptr(workspace),
                                          workspace_bytes, _ptr(stream))


def specasr_accept(ctx, tree, batch, argmax_dev, path_dev, accept_len_dev, next_token_dev,
                   workspace, workspace_bytes, stream=None):
    return load_library().specasr_accept(ctx, C.byref(tree), batch, _ptr(argmax_dev),
                                         _ptr(path_dev), _ptr(accept_len_dev),
                                         _ptr(next_token_dev), _ptr(workspace), workspace_bytes,
                                         _ptr(stream))


def specasr_accept_from_logits(ctx, tree, batch, logits_dev, argmax_dev, path_dev, accept_len_dev,
                               next_token_dev, workspace, workspace_bytes, stream=None):
    return load_library().specasr_accept_from_logits(ctx, C.byref(tree), batch, _ptr(logits_dev),
                                                     _ptr(argmax_dev), _ptr(path_dev),
                                                     _ptr(accept_len_dev), _ptr(next_token_dev),
                                                     _ptr(workspace), workspace_bytes,
                                                     _ptr(stream))


def specasr_accept_from_logits_static(ctx, tree, batch, logits_dev, argmax_dev, path_dev,
                                      accept_len_dev, next_token_dev, stream=None):
    return load_library().specasr_accept_from_logits_static(ctx, C.byref(tree), batch,
                                                            _ptr(logits_dev), _ptr(argmax_dev),
                                                            _ptr(path_dev), _ptr(accept_len_dev),
                                                            _ptr(next_token_dev), _ptr(stream))


def specasr_commit(ctx, kv, n_nodes, path, accept_len, workspace, workspace_bytes, stream=None):
    for a in (n_nodes, path, accept_len):
        assert a.dtype == np.int32 and a.flags.c_contiguous
    return load_library().specasr_commit(ctx, C.byref(kv), _i32(n_nodes), _i32(path),
                                         _i32(accept_len), _ptr(workspace), workspace_bytes,
                                         _ptr(stream))
