"""ctypes front end of the C oracle (specasr_oracle.c).  Test infrastructure only.

Holds no arithmetic of its own beyond array bookkeeping: building the cache
after a commit is a row gather (the definition of "append the accepted path").
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specasr_oracle.c")
_SO = os.path.join(_HERE, "_build", "libspecasr_oracle.so")

F32, BF16, F64 = 0, 1, 2
_lib = None


def build_oracle(force=False):
    """Compile the C oracle with gcc (OpenMP, no fast-math) and return the .so path."""
    os.makedirs(os.path.dirname(_SO), exist_ok=True)
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads",
                                          "head_dim", "d_ffn", "vocab", "wdtype")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double)]


_LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class _Weights(C.Structure):
    _fields_ = [("tok_embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(_Layer))]


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build_oracle())
        lib.oracle_tree_meta.restype = C.c_int
        lib.oracle_tree_forward.restype = C.c_int
        lib.oracle_accept.restype = C.c_int
        lib.oracle_top2.restype = C.c_int
        lib.oracle_silu.restype = C.c_double
        lib.oracle_silu.argtypes = [C.c_double]
        lib.oracle_num_threads.restype = C.c_int
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float64:
        return F64
    raise TypeError("unsupported storage dtype %s" % a.dtype)


def num_threads():
    return int(_load().oracle_num_threads())


def tree_meta(parents):
    """depth[n] and the n x n ancestor-or-self matrix of a parent array."""
    par = np.ascontiguousarray(parents, dtype=np.int32)
    n = par.shape[0]
    depth = np.zeros(n, np.int32)
    anc = np.zeros((n, n), np.uint8)
    rc = _load().oracle_tree_meta(_p(par), C.c_int(n), _p(depth), _p(anc))
    if rc != 0:
        raise ValueError("parents is not a rooted topological order")
    return depth, anc


def accept(tokens, parents, amax):
    """Greedy acceptance: (path, accept_len, next_token)."""
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    par = np.ascontiguousarray(parents, dtype=np.int32)
    am = np.ascontiguousarray(amax, dtype=np.int32)
    n = tok.shape[0]
    path = np.full(n, -1, np.int32)
    alen = C.c_int32(0)
    nxt = C.c_int32(0)
    rc = _load().oracle_accept(_p(tok), _p(par), _p(am), C.c_int(n), _p(path), C.byref(alen),
                               C.byref(nxt))
    if rc != 0:
        raise ValueError("invalid tree")
    return path[:alen.value].copy(), int(alen.value), int(nxt.value)


def top2(logits):
    """Draft-side read-out of logit rows [n][V]: (top int32 [n][2], p1 float64 [n]) = the ids of
    the largest and second largest logit (lowest id on ties, -1 if there is no second) and the
    softmax probability of the largest."""
    x = np.ascontiguousarray(logits, np.float64)
    n, V = x.shape
    top = np.full((n, 2), -7, np.int32)
    p1 = np.zeros(n, np.float64)
    rc = _load().oracle_top2(_p(x), C.c_int(n), C.c_int(V), _p(top), _p(p1))
    if rc != 0:
        raise ValueError("invalid shape")
    return top, p1


def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(x, np.float64)
    g = np.ascontiguousarray(g, np.float64)
    y = np.empty_like(x)
    _load().oracle_rmsnorm(_p(x), _p(g), C.c_int(x.shape[0]), C.c_double(eps), _p(y))
    return y


def rope(x, pos, theta):
    y = np.array(x, np.float64, copy=True)
    _load().oracle_rope(_p(y), C.c_int(y.shape[0]), C.c_int64(int(pos)), C.c_double(theta))
    return y


def softmax(s):
    y = np.array(s, np.float64, copy=True)
    _load().oracle_softmax(_p(y), C.c_int(y.shape[0]))
    return y


def silu(z):
    return float(_load().oracle_silu(C.c_double(z)))


class OracleModel:
    """A decoder held as numpy arrays in storage dtype (float32, or uint16 bf16 bits).

    ``weights`` is a dict: tok_embed [V,d], final_norm [d], lm_head [V,d], and
    ``layers`` = list of dicts with attn_norm, wq, wk, wv, wo, ffn_norm, w_gate,
    w_up, w_down, every matrix row-major [out, in].
    """

    def __init__(self, cfg, weights):
        self.cfg = dict(cfg)
        self.w = weights
        wd = _dtype_code(weights["tok_embed"])
        self._keep = []

        def ptr(a):
            a = np.ascontiguousarray(a)
            if _dtype_code(a) != wd:
                raise TypeError("all weights must share one storage dtype")
            self._keep.append(a)
            return a.ctypes.data

        nl = cfg["n_layers"]
        self._layers = (_Layer * nl)()
        for l in range(nl):
            for f in _LAYER_FIELDS:
                setattr(self._layers[l], f, ptr(weights["layers"][l][f]))
        self._w = _Weights(ptr(weights["tok_embed"]), ptr(weights["final_norm"]),
                           ptr(weights["lm_head"]), self._layers)
        self._cfg = _Cfg(nl, cfg["d_model"], cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                         cfg["d_ffn"], cfg["vocab"], wd, cfg.get("rms_eps", 1e-5),
                         cfg.get("rope_theta", 10000.0))

    # -- cache helpers ------------------------------------------------------
    def empty_cache(self, capacity, dtype=np.float64):
        c = self.cfg
        shape = (c["n_layers"], c["n_kv_heads"], capacity, c["head_dim"])
        return np.zeros(shape, dtype), np.zeros(shape, dtype)

    # -- steps 0-8 ------------------------------------------------------------
    def tree_forward(self, kc, vc, L, tokens, parents, embeds=None, use_embed=None,
                     want_logits=True, want_kv=True):
        c = self.cfg
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        par = np.ascontiguousarray(parents, dtype=np.int32)
        n = tok.shape[0]
        assert kc.flags.c_contiguous and vc.flags.c_contiguous and kc.dtype == vc.dtype
        assert kc.shape == vc.shape == (c["n_layers"], c["n_kv_heads"], kc.shape[2], c["head_dim"])
        cap = kc.shape[2]
        logits = np.empty((n, c["vocab"]), np.float64) if want_logits else None
        amax = np.empty(n, np.int32)
        kt = vt = None
        if want_kv:
            kt = np.empty((c["n_layers"], c["n_kv_heads"], n, c["head_dim"]), np.float64)
            vt = np.empty_like(kt)
        emb = ue = None
        if embeds is not None:
            emb = np.ascontiguousarray(embeds, np.float64)
            ue = np.ascontiguousarray(use_embed if use_embed is not None else np.ones(n), np.uint8)
            assert emb.shape == (n, c["d_model"]) and ue.shape == (n,)
        rc = _load().oracle_tree_forward(
            C.byref(self._cfg), C.byref(self._w), _p(kc), _p(vc), C.c_int(_dtype_code(kc)),
            C.c_int64(cap), C.c_int64(int(L)), _p(tok), _p(par), C.c_int(n), _p(emb), _p(ue),
            _p(logits), _p(amax), _p(kt), _p(vt))
        if rc != 0:
            raise ValueError("oracle_tree_forward failed: %d" % rc)
        return {"logits": logits, "amax": amax, "ktree": kt, "vtree": vt}

    # -- step 10: commit = gather the accepted nodes' rows behind the prefix --
    @staticmethod
    def commit(kc, vc, L, ktree, vtree, path):
        """Write rows L+k <- node path[k]; returns the new length.  The rows come from a forward
        over this very cache, so they already hold values of its storage type (fp64, fp32, or
        bf16 bit patterns in uint16): the conversion below is exact, and checked to be."""
        def stored(rows):
            if kc.dtype == np.float64:
                return rows
            f32 = rows.astype(np.float32)
            assert np.array_equal(f32.astype(np.float64), rows), "rows not representable in fp32"
            if kc.dtype == np.float32:
                return f32
            assert kc.dtype == np.uint16
            bits = np.ascontiguousarray(f32).view(np.uint32)
            assert not np.any(bits & np.uint32(0xFFFF)), "rows not representable in bf16"
            return (bits >> np.uint32(16)).astype(np.uint16)
        for k, node in enumerate(path):
            kc[:, :, L + k, :] = stored(ktree[:, :, node, :])
            vc[:, :, L + k, :] = stored(vtree[:, :, node, :])
        return L + len(path)

    def prefill(self, kc, vc, L, embeds, tokens, chunk=64):
        """Extend a cache (any storage type) by a chain of inputs: first the rows of ``embeds``
        ([A,d] audio-embedding vectors, may be empty), then ``tokens``.  A chain is
        the tree in which every node's parent is its predecessor, so this is plain
        causal prefill.  Returns (new length, logits of the last position)."""
        A = 0 if embeds is None else embeds.shape[0]
        T = A + len(tokens)
        d = self.cfg["d_model"]
        last = None
        for s in range(0, T, chunk):
            e = min(T, s + chunk)
            n = e - s
            par = np.arange(-1, n - 1, dtype=np.int32)
            tok = np.zeros(n, np.int32)
            emb = np.zeros((n, d), np.float64)
            ue = np.zeros(n, np.uint8)
            for i in range(n):
                g = s + i
                if g < A:
                    emb[i] = embeds[g]
                    ue[i] = 1
                else:
                    tok[i] = tokens[g - A]
            r = self.tree_forward(kc, vc, L, tok, par, emb, ue)
            L = self.commit(kc, vc, L, r["ktree"], r["vtree"], list(range(n)))
            last = r["logits"][-1]
        return L, last
