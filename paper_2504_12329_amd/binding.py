"""Thin ctypes binding over libst.so: same names as include/st.h, argument marshalling only.

PyTorch supplies device memory (weights, KV cache, workspace) and the stream handle; every
step of the path runs in the library's HIP kernels.  Loading fails loudly when the library has
not been built -- there is no fallback.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libst.so")

ST_OK, ST_EINVAL, ST_ENOMEM, ST_ERANGE, ST_EHIP = 0, -1, -2, -3, -4
ST_TOKENS_DEVICE, ST_OUT_DEVICE, ST_TOKEN_CHAINED, ST_PREFILL_TWO_TERM, ST_PREFILL_FAST = 1, 2, 4, 8, 16

EXPORTS = ("st_query_sizes", "st_prefill_plan_check", "st_model_create", "st_model_destroy", "st_kv_len", "st_kv_truncate", "st_prefill",
           "st_query_f16_bytes", "st_model_attach_f16", "st_batch_attach_f16", "st_decode_step", "st_decode_graph_state", "st_decode_step_kind", "st_decode_persist_plan", "st_decode_step_timed", "st_decode_greedy", "st_trigger_scan", "st_trigger_scan_static", "st_handoff", "st_generate",
           "st_generate_policy", "st_batch_query_sizes", "st_batch_create", "st_batch_destroy", "st_batch_kv_len",
           "st_batch_truncate", "st_batch_prefill", "st_batch_prefill_many", "st_batch_decode_step", "st_generate_batch",
           "st_last_error")


class StError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"st error {code}: {msg}")
        self.code = code


class st_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("tie_embeddings", "qkv_bias", "max_seq", "max_chunk")]


_vpp = C.POINTER(C.c_void_p)


class st_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, _vpp) for n in ("wqkv", "bqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp")]


class st_trigger_rule(C.Structure):
    _fields_ = [("kw_bitmap", C.c_void_p), ("delim_bitmap", C.c_void_p), ("window", C.c_int32), ("vocab", C.c_int32)]


class st_spans(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("large_prefill_lo", "large_prefill_hi", "large_decode_lo", "large_decode_hi",
                                         "small_prefill_lo", "small_prefill_hi")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class st_gen_stats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_out", "n_handoffs", "n_large", "n_spans")] + \
               [(n, C.c_double) for n in ("ms_small_decode", "ms_large_decode", "ms_small_prefill", "ms_large_prefill")]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2504_12329_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_12329_amd.build`")
        L = C.CDLL(LIB_PATH)
        i32p, f32p = C.POINTER(C.c_int32), C.POINTER(C.c_float)
        L.st_last_error.restype = C.c_char_p
        L.st_query_sizes.argtypes = [C.POINTER(st_config), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.st_prefill_plan_check.argtypes = [C.POINTER(st_config), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.st_model_create.argtypes = [C.POINTER(st_config), C.POINTER(st_weights), C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
        L.st_model_destroy.argtypes = [C.c_void_p]
        L.st_model_destroy.restype = None
        L.st_kv_len.argtypes = [C.c_void_p, i32p]
        L.st_kv_truncate.argtypes = [C.c_void_p, C.c_int32]
        L.st_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32]
        L.st_decode_step.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32]
        L.st_decode_step_timed.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.st_decode_graph_state.argtypes = [C.c_void_p, i32p, i32p]
        L.st_decode_step_kind.argtypes = [C.c_void_p, i32p]
        L.st_decode_persist_plan.argtypes = [C.POINTER(st_config), C.c_int32, C.POINTER(C.c_size_t),
                                             C.POINTER(C.c_size_t), i32p, i32p]
        L.st_query_f16_bytes.argtypes = [C.POINTER(st_config), C.POINTER(C.c_size_t)]
        L.st_model_attach_f16.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.st_batch_attach_f16.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
        L.st_decode_greedy.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_uint32]
        L.st_trigger_scan.argtypes = [C.POINTER(st_trigger_rule), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]
        L.st_trigger_scan_static.argtypes = [C.POINTER(st_trigger_rule), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                             C.c_int32, C.c_void_p, C.c_void_p]
        L.st_handoff.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, i32p, C.c_int32, C.c_int32, C.c_void_p,
                                 i32p, C.POINTER(st_spans), C.c_uint32]
        L.st_generate.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(st_trigger_rule), C.c_int32, C.c_void_p,
                                  C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(st_spans),
                                  C.c_int32, C.POINTER(st_gen_stats)]
        L.st_generate_policy.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(st_policy), C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_void_p, C.c_void_p, C.POINTER(st_action), C.c_int32,
                                         C.POINTER(st_gen_stats)]
        L.st_batch_query_sizes.argtypes = [C.POINTER(st_config), C.c_int32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.st_batch_create.argtypes = [C.POINTER(st_config), C.POINTER(st_weights), C.c_int32, C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
        L.st_batch_destroy.argtypes = [C.c_void_p]
        L.st_batch_destroy.restype = None
        L.st_batch_kv_len.argtypes = [C.c_void_p, C.c_int32, i32p]
        L.st_batch_truncate.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.st_batch_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.st_batch_decode_step.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.st_batch_prefill_many.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
        L.st_generate_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.POINTER(st_gen_stats)]
        _lib = L
    return _lib


def _check(rc):
    if rc != ST_OK:
        raise StError(rc, lib().st_last_error().decode())


def make_config(cfg):
    return st_config(*(cfg[n] for n, _ in st_config._fields_))


def st_query_sizes(cfg):
    kv, ws = C.c_size_t(), C.c_size_t()
    _check(lib().st_query_sizes(C.byref(make_config(cfg)), C.byref(kv), C.byref(ws)))
    return kv.value, ws.value


def st_prefill_plan_check(cfg, rows):
    """Host-only walk over the launch plan of a catch-up pass of `rows` rows; returns (launches, blocks) of a layer."""
    nl, nb = C.c_int32(), C.c_int32()
    _check(lib().st_prefill_plan_check(C.byref(make_config(cfg)), int(rows), C.byref(nl), C.byref(nb)))
    return nl.value, nb.value


def st_decode_persist_plan(cfg, n_cu):
    """Host-only plan of the single-kernel decode step: dict(lds_bytes, handover_words, regions[7], parts[5])."""
    lds, words = C.c_size_t(), C.c_size_t()
    regions, parts = (C.c_int32 * 7)(), (C.c_int32 * 5)()
    _check(lib().st_decode_persist_plan(C.byref(make_config(cfg)), int(n_cu), C.byref(lds), C.byref(words), regions, parts))
    return dict(lds_bytes=lds.value, handover_words=words.value, regions=list(regions), parts=list(parts))


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


class TriggerRule:
    """Device bitmaps of the keyword and delimiter token sets."""

    def __init__(self, vocab, kw_bitmap, delim_bitmap=None, window=1, device="cuda"):
        self.kw = torch.from_numpy(np.ascontiguousarray(kw_bitmap).view(np.int32)).to(device)
        self.delim = None if delim_bitmap is None else \
            torch.from_numpy(np.ascontiguousarray(delim_bitmap).view(np.int32)).to(device)
        self.c = st_trigger_rule(self.kw.data_ptr(), 0 if self.delim is None else self.delim.data_ptr(), window, vocab)


def st_trigger_scan(rule, tokens_dev, lo, hi, cap, stream=None):
    """tokens_dev: int32 CUDA tensor.  Returns (total_count, positions ndarray)."""
    scratch = torch.empty(cap + 1, dtype=torch.int32, device=tokens_dev.device)
    pos = np.empty(max(cap, 1), dtype=np.int32)
    n = C.c_int32()
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(lib().st_trigger_scan(C.byref(rule.c), tokens_dev.data_ptr(), lo, hi, _np_ptr(pos), cap, C.byref(n),
                                 scratch.data_ptr(), s, 0))
    return n.value, pos[:min(n.value, cap)].copy()


ST_SCAN_STATIC_MAX_CAP = 4096


def st_trigger_scan_static(rule, tokens_dev, lo, hi, cap, stream=None):
    """st_trigger_scan without a caller-provided device scratch (the library's static staging array; allocates
    nothing on the device).  Returns (total_count, positions ndarray)."""
    pos = np.empty(max(cap, 1), dtype=np.int32)
    n = C.c_int32()
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(lib().st_trigger_scan_static(C.byref(rule.c), tokens_dev.data_ptr(), lo, hi, _np_ptr(pos), cap, C.byref(n), s))
    return n.value, pos[:min(n.value, cap)].copy()


def _pass_flags(two_term, fast):
    return (ST_PREFILL_TWO_TERM if two_term else 0) | (ST_PREFILL_FAST if fast else 0)


class Model:
    """st_model over torch-owned device buffers.  `weights` is the dict made by synth.make_weights on the GPU."""

    def __init__(self, cfg, weights, stream=None):
        self.cfg = dict(cfg)
        self.weights = weights                      # keeps the tensors alive
        dev = weights["embed"].device
        if dev.type != "cuda":
            raise RuntimeError("weights must live on the GPU")
        kv_bytes, ws_bytes = st_query_sizes(cfg)
        self.kv = torch.empty(kv_bytes, dtype=torch.uint8, device=dev)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        L = cfg["n_layers"]
        w = st_weights()
        w.embed = weights["embed"].data_ptr()
        w.lm_head = 0 if weights.get("lm_head") is None else weights["lm_head"].data_ptr()
        w.final_norm = weights["final_norm"].data_ptr()
        self._arrays = []
        for name in ("wqkv", "bqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp"):
            arr = (C.c_void_p * L)(*[lw[name].data_ptr() for lw in weights["layers"]])
            self._arrays.append(arr)
            setattr(w, name, C.cast(arr, _vpp))
        self.stream = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        h = C.c_void_p()
        _check(lib().st_model_create(C.byref(make_config(cfg)), C.byref(w), self.kv.data_ptr(), kv_bytes,
                                     self.ws.data_ptr(), ws_bytes, self.stream, C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().st_model_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the library wrapper may already be gone
            pass

    @property
    def kv_len(self):
        n = C.c_int32()
        _check(lib().st_kv_len(self._h, C.byref(n)))
        return n.value

    def truncate(self, n):
        _check(lib().st_kv_truncate(self._h, n))

    def prefill(self, tokens, want_logits=True, two_term=False, fast=False):
        """tokens: host int array; two_term: passes of at most 256 rows (ST_PREFILL_TWO_TERM); fast: single-bf16 GEMM
        inputs in passes of more than 256 rows (ST_PREFILL_FAST).  Returns (logits ndarray or None, greedy token)."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.empty(self.cfg["vocab"], dtype=np.float32) if want_logits else None
        nt = C.c_int32()
        _check(lib().st_prefill(self._h, _np_ptr(t), t.size, _np_ptr(lg) if want_logits else None,
                                C.addressof(nt), _pass_flags(two_term, fast)))
        return lg, nt.value

    def prefill_device(self, tokens_dev, two_term=False, fast=False):
        """tokens_dev: int32 CUDA tensor; enqueues only (no outputs, no synchronisation)."""
        _check(lib().st_prefill(self._h, tokens_dev.data_ptr(), tokens_dev.numel(), None, None,
                                ST_TOKENS_DEVICE | ST_OUT_DEVICE | _pass_flags(two_term, fast)))

    def decode_step(self, token, want_logits=True):
        lg = np.empty(self.cfg["vocab"], dtype=np.float32) if want_logits else None
        nt = C.c_int32()
        _check(lib().st_decode_step(self._h, int(token), _np_ptr(lg) if want_logits else None, C.addressof(nt), 0))
        return lg, nt.value

    def attach_f16(self, on=True):
        """Gives the model an fp16 copy of its projection weights (torch-owned buffer): long default-precision passes
        then run on the fp16 MFMA with single fp16 activations.  on=False detaches and frees the buffer."""
        if not on:
            _check(lib().st_model_attach_f16(self._h, None, 0))
            self.f16_buf = None
            return
        n = C.c_size_t()
        _check(lib().st_query_f16_bytes(C.byref(make_config(self.cfg)), C.byref(n)))
        self.f16_buf = torch.empty(n.value, dtype=torch.uint8, device=self.kv.device)
        _check(lib().st_model_attach_f16(self._h, self.f16_buf.data_ptr(), n.value))

    def graph_state(self):
        """(step graphs captured so far, mode): mode 0 = graphs replayed, 1 = off by ST_NO_GRAPH, 2 = capture failed."""
        n, mode = C.c_int32(), C.c_int32()
        _check(lib().st_decode_graph_state(self._h, C.byref(n), C.byref(mode)))
        return n.value, mode.value

    def step_kind(self):
        """1 = the decode step is one persistent kernel, 0 = one kernel per stage."""
        k = C.c_int32()
        _check(lib().st_decode_step_kind(self._h, C.byref(k)))
        return k.value

    def decode_step_timed(self):
        """One chained step with per-launch events; returns (mean gate/up kernel us, whole step us)."""
        a, b = C.c_double(), C.c_double()
        _check(lib().st_decode_step_timed(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def decode_greedy(self, first_token, n, chained=False, out_dev=None):
        """n chained greedy steps.  Returns the tokens (host) unless out_dev (int32 CUDA tensor) is given."""
        flags = ST_TOKEN_CHAINED if chained else 0
        if out_dev is not None:
            _check(lib().st_decode_greedy(self._h, int(first_token), n, out_dev.data_ptr(), flags | ST_OUT_DEVICE))
            return None
        out = np.empty(n, dtype=np.int32)
        _check(lib().st_decode_greedy(self._h, int(first_token), n, _np_ptr(out), flags))
        return out


def st_handoff(small, large, seq, T, n_large, budget, want_logits=False):
    """seq: host int32 ndarray with room for the segment.  Returns (new_T, small_next_tok, spans dict, logits)."""
    t = C.c_int32(T)
    nt = C.c_int32(-1)
    sp = st_spans()
    lg = np.empty(small.cfg["vocab"], dtype=np.float32) if want_logits else None
    _check(lib().st_handoff(small._h, large._h, _np_ptr(seq), C.byref(t), n_large, budget,
                            _np_ptr(lg) if want_logits else None, C.byref(nt), C.byref(sp), 0))
    return t.value, nt.value, sp.as_dict(), lg


def st_generate(small, large, rule, prompt, n_out, n_seg, forced_period=0, span_cap=4096):
    """Runs the whole loop.  Returns dict(seq, src, spans, stats)."""
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    seq = np.zeros(p.size + n_out, dtype=np.int32)
    src = np.zeros(max(n_out, 1), dtype=np.uint8)
    spans = (st_spans * max(span_cap, 1))()
    stats = st_gen_stats()
    _check(lib().st_generate(small._h, large._h, C.byref(rule.c) if rule is not None else None, forced_period,
                             _np_ptr(p), p.size, n_out, n_seg, _np_ptr(seq), _np_ptr(src),
                             C.cast(spans, C.POINTER(st_spans)), span_cap, C.byref(stats)))
    return dict(seq=seq[:p.size + stats.n_out], src=src[:stats.n_out],
                spans=[spans[i].as_dict() for i in range(stats.n_spans)],
                stats={n: getattr(stats, n) for n, _ in st_gen_stats._fields_})


class st_policy(C.Structure):
    _fields_ = [("delim_bitmap", C.c_void_p), ("ar_bitmap", C.c_void_p), ("verify_bitmap", C.c_void_p),
                ("neg_bitmap", C.c_void_p), ("vocab", C.c_int32), ("sentence_len", C.c_int32), ("n1", C.c_int32),
                ("n2", C.c_int32), ("n3", C.c_int32), ("neg_threshold", C.c_int32), ("aux_tokens", C.c_void_p),
                ("n_aux", C.c_int32), ("replace", C.c_int32), ("unconditional", C.c_int32),
                ("initial_target", C.c_int32)]


class st_action(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "sentence_end", "dropped", "aux_lo", "aux_hi", "granted")]


def host_bitmap(vocab, ids):
    """Host bitmap of `vocab` bits with the given token ids set (uint32 words, bit t of word t // 32)."""
    bm = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    ids = np.asarray(list(ids), dtype=np.int64)
    np.bitwise_or.at(bm, ids >> 5, (np.uint32(1) << (ids & 31).astype(np.uint32)))
    return bm


def st_generate_policy(small, large, prompt, n_out, vocab, delim, sentence_len=1, ar=None, n1=20, verify=None, n2=125,
                       neg=None, neg_threshold=15, aux=(), n3=125, replace=False, unconditional=False,
                       initial_target=0, action_cap=4096):
    """Runs the full takeover policy; delim / ar / verify / neg are host bitmaps (see host_bitmap) or None.
    Returns dict(seq, src, actions, stats)."""
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    seq = np.zeros(p.size + n_out, dtype=np.int32)
    src = np.zeros(max(n_out, 1), dtype=np.uint8)
    keep = [np.ascontiguousarray(b, dtype=np.uint32) if b is not None else None for b in (delim, ar, verify, neg)]
    auxa = np.ascontiguousarray(list(aux), dtype=np.int32)
    ptr = lambda a: a.ctypes.data if a is not None and a.size else None
    pol = st_policy(ptr(keep[0]), ptr(keep[1]), ptr(keep[2]), ptr(keep[3]), vocab, sentence_len, n1, n2, n3,
                    neg_threshold, ptr(auxa), auxa.size, int(replace), int(unconditional), initial_target)
    acts = (st_action * max(action_cap, 1))()
    stats = st_gen_stats()
    _check(lib().st_generate_policy(small._h, large._h, C.byref(pol), _np_ptr(p), p.size, n_out, _np_ptr(seq),
                                    _np_ptr(src), C.cast(acts, C.POINTER(st_action)), action_cap, C.byref(stats)))
    return dict(seq=seq[:p.size + stats.n_out], src=src[:stats.n_out],
                actions=[tuple(getattr(acts[i], n) for n, _ in st_action._fields_) for i in range(stats.n_spans)],
                stats={n: getattr(stats, n) for n, _ in st_gen_stats._fields_})


def _weights_struct(cfg, weights):
    """st_weights over the tensors of synth.make_weights; returns (struct, objects to keep alive)."""
    L = cfg["n_layers"]
    w = st_weights()
    w.embed = weights["embed"].data_ptr()
    w.lm_head = 0 if weights.get("lm_head") is None else weights["lm_head"].data_ptr()
    w.final_norm = weights["final_norm"].data_ptr()
    keep = []
    for name in ("wqkv", "bqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp"):
        arr = (C.c_void_p * L)(*[lw[name].data_ptr() for lw in weights["layers"]])
        keep.append(arr)
        setattr(w, name, C.cast(arr, _vpp))
    return w, keep


class Batch:
    """st_batch: n_seq independent sequences over one set of weights, torch-owned device buffers."""

    def __init__(self, cfg, weights, n_seq, stream=None):
        self.cfg, self.weights, self.n_seq = dict(cfg), weights, n_seq
        dev = weights["embed"].device
        if dev.type != "cuda":
            raise RuntimeError("weights must live on the GPU")
        kv, ws = C.c_size_t(), C.c_size_t()
        _check(lib().st_batch_query_sizes(C.byref(make_config(cfg)), n_seq, C.byref(kv), C.byref(ws)))
        self.kv = torch.empty(kv.value, dtype=torch.uint8, device=dev)
        self.ws = torch.empty(ws.value, dtype=torch.uint8, device=dev)
        w, self._arrays = _weights_struct(cfg, weights)
        self.stream = torch.cuda.current_stream(dev).cuda_stream if stream is None else stream
        h = C.c_void_p()
        _check(lib().st_batch_create(C.byref(make_config(cfg)), C.byref(w), n_seq, self.kv.data_ptr(), kv.value,
                                     self.ws.data_ptr(), ws.value, self.stream, C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().st_batch_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_len(self, seq):
        n = C.c_int32()
        _check(lib().st_batch_kv_len(self._h, seq, C.byref(n)))
        return n.value

    def truncate(self, seq, n):
        _check(lib().st_batch_truncate(self._h, seq, n))

    def attach_f16(self):
        """fp16 copy of the shared projection weights (see Model.attach_f16)."""
        n = C.c_size_t()
        _check(lib().st_query_f16_bytes(C.byref(make_config(self.cfg)), C.byref(n)))
        self.f16_buf = torch.empty(n.value, dtype=torch.uint8, device=self.kv.device)
        _check(lib().st_batch_attach_f16(self._h, self.f16_buf.data_ptr(), n.value))

    def prefill(self, seq, tokens, want_logits=True):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.empty(self.cfg["vocab"], dtype=np.float32) if want_logits else None
        tok = C.c_int32()
        _check(lib().st_batch_prefill(self._h, seq, _np_ptr(t), t.size, _np_ptr(lg) if want_logits else None,
                                      C.byref(tok)))
        return lg, tok.value

    def prefill_many(self, seqs, token_lists, want_logits=False):
        """One ragged catch-up pass: token_lists[j] goes to sequence seqs[j].  Returns (logits [n][V] or None, next)."""
        s = np.ascontiguousarray(seqs, dtype=np.int32)
        ts = [np.ascontiguousarray(t, dtype=np.int32) for t in token_lists]
        lens = np.array([t.size for t in ts], dtype=np.int32)
        ptrs = (C.c_void_p * len(ts))(*[t.ctypes.data for t in ts])
        lg = np.empty((s.size, self.cfg["vocab"]), dtype=np.float32) if want_logits else None
        nxt = np.empty(s.size, dtype=np.int32)
        _check(lib().st_batch_prefill_many(self._h, s.size, _np_ptr(s), ptrs, _np_ptr(lens),
                                           _np_ptr(lg) if want_logits else None, _np_ptr(nxt)))
        return lg, nxt

    def decode_step(self, seqs, tokens, want_logits=False):
        s = np.ascontiguousarray(seqs, dtype=np.int32)
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        assert s.size == t.size
        lg = np.empty((s.size, self.cfg["vocab"]), dtype=np.float32) if want_logits else None
        nxt = np.empty(s.size, dtype=np.int32)
        _check(lib().st_batch_decode_step(self._h, s.size, _np_ptr(s), _np_ptr(t),
                                          _np_ptr(lg) if want_logits else None, _np_ptr(nxt)))
        return lg, nxt


class st_host_rule(C.Structure):
    _fields_ = [("kw_bitmap", C.c_void_p), ("delim_bitmap", C.c_void_p), ("window", C.c_int32), ("vocab", C.c_int32)]


def st_generate_batch(small, large, prompts, n_out, n_seg, vocab, kw=None, delim=None, window=1, forced_period=0,
                      forced_phase=None, gather=0):
    """The st_generate loop for len(prompts) sequences at once on two Batch objects; kw / delim are host bitmaps,
    forced_phase the per-sequence start of the forced-period count, gather the number of waiting sequences the
    target's passes are held for.  Returns dict(seqs, srcs, stats)."""
    n = len(prompts)
    ps = [np.ascontiguousarray(p, dtype=np.int32) for p in prompts]
    lens = np.array([p.size for p in ps], dtype=np.int32)
    seqs = [np.zeros(p.size + n_out, dtype=np.int32) for p in ps]
    srcs = [np.zeros(max(n_out, 1), dtype=np.uint8) for _ in ps]
    arr = lambda xs: (C.c_void_p * n)(*[x.ctypes.data for x in xs])
    kwa = None if kw is None else np.ascontiguousarray(kw, dtype=np.uint32)
    dla = None if delim is None else np.ascontiguousarray(delim, dtype=np.uint32)
    rule = st_host_rule(None if kwa is None else kwa.ctypes.data, None if dla is None else dla.ctypes.data, window, vocab)
    stats = st_gen_stats()
    phase = None if forced_phase is None else np.ascontiguousarray(forced_phase, dtype=np.int32)
    _check(lib().st_generate_batch(small._h, large._h, C.byref(rule) if kwa is not None else None, forced_period,
                                   None if phase is None else _np_ptr(phase), gather, n,
                                   arr(ps), _np_ptr(lens), n_out, n_seg, arr(seqs), arr(srcs), C.byref(stats)))
    return dict(seqs=seqs, srcs=srcs, stats={k: getattr(stats, k) for k, _ in st_gen_stats._fields_})
