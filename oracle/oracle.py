"""ctypes wrapper over the C oracle (test infrastructure only).

`OracleModel` takes host fp32 tensors in the oracle's own naming (separate q/k/v and
gate/up matrices per layer); nothing here does arithmetic of the method.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_f32p = C.POINTER(C.c_float)
_i32p = C.POINTER(C.c_int32)
_u32p = C.POINTER(C.c_uint32)


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("qkv_bias", C.c_int32), ("max_seq", C.c_int32)]


_PER_LAYER = ("wq", "wk", "wv", "bq", "bk", "bv", "wo", "wg", "wu", "wd", "norm_attn", "norm_mlp")


class _Weights(C.Structure):
    _fields_ = [("embed", _f32p), ("lm_head", _f32p), ("final_norm", _f32p)] + \
               [(n, C.POINTER(_f32p)) for n in _PER_LAYER]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        L = C.CDLL(path)
        L.orc_create.restype = C.c_void_p
        L.orc_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights)]
        L.orc_destroy.argtypes = [C.c_void_p]
        L.orc_kv_len.argtypes = [C.c_void_p]
        L.orc_kv_len.restype = C.c_int32
        L.orc_kv_truncate.argtypes = [C.c_void_p, C.c_int32]
        for f in (L.orc_feed, L.orc_feed_block):
            f.argtypes = [C.c_void_p, _i32p, C.c_int32, _f32p, _f32p]
            f.restype = C.c_int
        L.orc_threads.restype = C.c_int
        L.orc_rmsnorm.argtypes = [_f32p, _f32p, C.c_int32, C.c_float, _f32p]
        L.orc_rope.argtypes = [_f32p, C.c_int32, C.c_int32, C.c_float]
        L.orc_softmax.argtypes = [_f32p, C.c_int32]
        L.orc_silu.argtypes = [C.c_float]
        L.orc_silu.restype = C.c_float
        L.orc_argmax.argtypes = [_f32p, C.c_int32]
        L.orc_argmax.restype = C.c_int32
        L.orc_attention.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _f32p]
        L.orc_trigger_scan.argtypes = [_i32p, C.c_int32, C.c_int32, C.c_int32, _u32p, _u32p, C.c_int32,
                                       _i32p, C.c_int32]
        L.orc_trigger_scan.restype = C.c_int32
        _lib = L
    return _lib


def _fp(a):
    return a.ctypes.data_as(_f32p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


class OracleModel:
    """cfg: dict with the orc_config fields.  w: dict with 'embed', 'lm_head' (or None when tied),
    'final_norm' and per-layer lists wq, wk, wv, bq, bk, bv, wo, wg, wu, wd, norm_attn, norm_mlp."""

    def __init__(self, cfg, w):
        self.cfg = dict(cfg)
        self._keep = []
        ws = _Weights()
        emb = _f32(w["embed"])
        head = emb if w.get("lm_head") is None else _f32(w["lm_head"])
        fin = _f32(w["final_norm"])
        self._keep += [emb, head, fin]
        ws.embed, ws.lm_head, ws.final_norm = _fp(emb), _fp(head), _fp(fin)
        L = cfg["n_layers"]
        for name in _PER_LAYER:
            arr = (_f32p * L)()
            if name in ("bq", "bk", "bv") and not cfg.get("qkv_bias", 1):
                pass
            else:
                for l in range(L):
                    a = _f32(w[name][l])
                    self._keep.append(a)
                    arr[l] = _fp(a)
            self._keep.append(arr)
            setattr(ws, name, arr)
        c = _Config(cfg["n_layers"], cfg["hidden"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                    cfg["intermediate"], cfg["vocab"], cfg["rms_eps"], cfg["rope_theta"],
                    int(cfg.get("qkv_bias", 1)), cfg["max_seq"])
        self._h = lib().orc_create(C.byref(c), C.byref(ws))
        if not self._h:
            raise ValueError("orc_create rejected the configuration")
        self.vocab = cfg["vocab"]

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the library wrapper may already be gone
            pass

    @property
    def kv_len(self):
        return lib().orc_kv_len(self._h)

    def truncate(self, n):
        if lib().orc_kv_truncate(self._h, n) != 0:
            raise ValueError("bad truncate length")

    def _run(self, fn, tokens, all_logits):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        n = t.shape[0]
        last = np.empty(self.vocab, dtype=np.float32)
        full = np.empty((n, self.vocab), dtype=np.float32) if all_logits else None
        rc = fn(self._h, t.ctypes.data_as(_i32p), n, _fp(last), _fp(full) if all_logits else None)
        if rc != 0:
            raise ValueError("oracle feed rejected its input (overflow, empty, or token id out of range)")
        return full if all_logits else last

    def feed(self, tokens, all_logits=False):
        """n successive single-token steps; logits of the last (or every) position."""
        return self._run(lib().orc_feed, tokens, all_logits)

    def feed_block(self, tokens, all_logits=False):
        return self._run(lib().orc_feed_block, tokens, all_logits)


def rmsnorm(x, g, eps):
    x, g = _f32(x), _f32(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_fp(x), _fp(g), x.size, eps, _fp(out))
    return out


def rope(v, pos, theta):
    v = _f32(v).copy()
    lib().orc_rope(_fp(v), v.size, pos, theta)
    return v


def softmax(s):
    s = _f32(s).copy()
    lib().orc_softmax(_fp(s), s.size)
    return s


def silu(z):
    return float(lib().orc_silu(float(z)))


def argmax(v):
    v = _f32(v)
    return int(lib().orc_argmax(_fp(v), v.size))


def attention(q, K, V):
    """q [nq][d], K/V [t][nkv][d] -> [nq][d]."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    nq, d = q.shape
    t, nkv, _ = K.shape
    out = np.empty_like(q)
    lib().orc_attention(_fp(q), _fp(K), _fp(V), t, nq, nkv, d, _fp(out))
    return out


def trigger_scan(tokens, lo, hi, vocab, kw, delim, window, cap):
    """Returns (total_count, positions[:min(count,cap)]); raises on a token id outside the vocabulary."""
    t = np.ascontiguousarray(tokens, dtype=np.int32)
    kw = np.ascontiguousarray(kw, dtype=np.uint32)
    delim = np.ascontiguousarray(delim if delim is not None else kw, dtype=np.uint32)
    pos = np.empty(max(cap, 1), dtype=np.int32)
    n = lib().orc_trigger_scan(t.ctypes.data_as(_i32p), lo, hi, vocab, kw.ctypes.data_as(_u32p),
                               delim.ctypes.data_as(_u32p), window, pos.ctypes.data_as(_i32p), cap)
    if n < 0:
        raise ValueError("token id outside the vocabulary")
    return n, pos[:min(n, cap)].copy()
