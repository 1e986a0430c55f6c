"""Thin ctypes binding of ``libkvq.so``: same names as the C ABI, argument marshalling only.

Every step of the hot path runs in the library's HIP kernels.  PyTorch appears here only as the owner
of device memory (``tensor.data_ptr()``) and of the stream the work is enqueued on.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvq.so")

KVQ_OK = 0
KVQ_ERR_INVALID_ARG, KVQ_ERR_CAPACITY, KVQ_ERR_UNSUPPORTED, KVQ_ERR_DEVICE, KVQ_ERR_OOM = 1, 2, 3, 4, 5
FLAG_POOL_EXHAUSTED = 1
FLAG_CONTEXT_FULL = 2
FLAG_BAD_BITS = 4
EXPORT_REC = 128

EXPORTED_SYMBOLS = (
    "kvq_version", "kvq_last_error", "kvq_cache_arena_bytes", "kvq_cache_create", "kvq_cache_destroy",
    "kvq_cache_reset", "kvq_cache_free_seqs", "kvq_cache_set_length_hint", "kvq_cache_status", "kvq_cache_counts", "kvq_cache_usage_of", "kvq_cache_export", "kvq_cache_import", "kvq_cache_set_k_channel_quant",
    "kvq_features_workspace", "kvq_features", "kvq_features_typed", "kvq_controller", "kvq_features_controller", "kvq_features_controller_typed", "kvq_rule_policy", "kvq_controller_param_count", "kvq_controller_train_workspace",
    "kvq_controller_train_step", "kvq_append", "kvq_decode_attn_workspace",
    "kvq_decode_attn", "kvq_decode_attn_static_capacity", "kvq_decode_attn_static", "kvq_append_decode_attn", "kvq_tuning_set", "kvq_tuning_get",
)


class KvqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("kvq status %d: %s" % (code, msg))
        self.code = code


class CacheDesc(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("max_seqs", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("page_tokens", ctypes.c_int32),
        ("max_context", ctypes.c_int64), ("pool_pages", ctypes.c_int64 * 4),
        ("arena", ctypes.c_void_p), ("arena_bytes", ctypes.c_size_t),
    ]


class Mlp(ctypes.Structure):
    _fields_ = [("n_linear", ctypes.c_int32), ("dims", ctypes.c_int32 * 5),
                ("W", ctypes.c_void_p * 4), ("b", ctypes.c_void_p * 4)]


class CacheUsage(ctypes.Structure):
    _fields_ = [("tokens", ctypes.c_int64 * 4), ("expected_bits", ctypes.c_double), ("effective_bits", ctypes.c_double),
                ("payload_bytes", ctypes.c_int64), ("pages_in_use", ctypes.c_int64 * 4), ("page_bytes_in_use", ctypes.c_int64)]


class Rule(ctypes.Structure):
    _fields_ = [("w", ctypes.c_float * 4), ("bias", ctypes.c_float), ("thr", ctypes.c_float * 3)]


class TrainHparams(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_float), ("beta", ctypes.c_float), ("gamma", ctypes.c_float),
                ("c", ctypes.c_float * 4), ("q", ctypes.c_float * 4),
                ("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float)]


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """Load the built library.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.kvq_version.restype = ctypes.c_char_p
    lib.kvq_last_error.restype = ctypes.c_char_p
    lib.kvq_cache_arena_bytes.restype = sz
    lib.kvq_cache_arena_bytes.argtypes = [ctypes.POINTER(CacheDesc)]
    lib.kvq_cache_create.argtypes = [ctypes.POINTER(CacheDesc), ctypes.POINTER(vp)]
    lib.kvq_cache_destroy.argtypes = [vp]
    lib.kvq_cache_reset.argtypes = [vp, vp]
    lib.kvq_cache_free_seqs.argtypes = [vp, vp, i32, vp]
    lib.kvq_cache_set_length_hint.argtypes = [vp, i64]
    lib.kvq_cache_status.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(i64), vp]
    lib.kvq_cache_counts.argtypes = [vp, vp, vp]
    lib.kvq_cache_usage_of.argtypes = [vp, ctypes.POINTER(CacheUsage), vp]
    lib.kvq_cache_export.argtypes = [vp, i32, i32, vp, vp, vp, i64, vp]
    lib.kvq_cache_import.argtypes = [vp, i32, i32, vp, vp, vp, i64, vp]
    lib.kvq_cache_set_k_channel_quant.argtypes = [vp, vp, vp, vp]
    lib.kvq_features_workspace.restype = sz
    lib.kvq_features_workspace.argtypes = [i64, i64]
    lib.kvq_features.argtypes = [vp, i64, i64, vp, vp, vp, i32, vp, vp, vp, i32, i64, vp, vp, sz, vp]
    lib.kvq_features_typed.argtypes = [vp, i32, i64, i64, vp, vp, vp, i32, vp, vp, vp, i32, i64, vp, vp, sz, vp]
    lib.kvq_features_controller_typed.argtypes = [vp, i32, i64, i64, vp, vp, vp, i32, vp, vp, i32, ctypes.POINTER(Mlp), vp, vp, vp, vp,
                                                  vp, vp, sz, vp]
    lib.kvq_controller.argtypes = [vp, i64, ctypes.POINTER(Mlp), vp, vp, vp]
    lib.kvq_features_controller.argtypes = [vp, i64, i64, vp, vp, vp, i32, vp, vp, i32, ctypes.POINTER(Mlp), vp, vp, vp, vp,
                                            vp, vp, sz, vp]
    lib.kvq_rule_policy.argtypes = [vp, i64, ctypes.POINTER(Rule), vp, vp, vp]
    lib.kvq_controller_param_count.restype = i64
    lib.kvq_controller_param_count.argtypes = [ctypes.POINTER(Mlp)]
    lib.kvq_controller_train_workspace.restype = sz
    lib.kvq_controller_train_workspace.argtypes = [ctypes.POINTER(Mlp), i64]
    lib.kvq_controller_train_step.argtypes = [vp, vp, i64, ctypes.POINTER(Mlp), ctypes.POINTER(Mlp), ctypes.POINTER(Mlp),
                                              ctypes.POINTER(TrainHparams), i64, vp, vp, vp, sz, vp]
    lib.kvq_append.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32, vp]
    lib.kvq_decode_attn_workspace.restype = sz
    lib.kvq_decode_attn_workspace.argtypes = [vp, i32]
    lib.kvq_decode_attn.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.kvq_decode_attn_static_capacity.restype = sz
    lib.kvq_decode_attn_static_capacity.argtypes = []
    lib.kvq_decode_attn_static.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.kvq_append_decode_attn.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.kvq_tuning_set.argtypes = [ctypes.c_char_p, i32]
    lib.kvq_tuning_get.argtypes = [ctypes.c_char_p, ctypes.POINTER(i32)]
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != KVQ_OK:
        raise KvqError(rc, load_library().kvq_last_error().decode())


# torch.cuda.current_stream() builds a Stream object on every call (2.7 us, more than half of what a call through this
# binding costs on the host); the raw getter returns the same handle in 0.1 us.
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_raw_device = getattr(torch._C, "_cuda_getDevice", None)


def _stream(stream) -> int:
    if stream is None:
        if _raw_stream is not None and _raw_device is not None:
            return _raw_stream(_raw_device())
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def kvq_version() -> str:
    return load_library().kvq_version().decode()


class Cache:
    """Owner of one ``kvq_cache`` handle."""

    def __init__(self, n_layers: int, max_seqs: int, n_q_heads: int, n_kv_heads: int, max_context: int,
                 page_tokens: int = 0, pool_pages: Sequence[int] = (0, 0, 0, 0), head_dim: int = 64,
                 arena: Optional[torch.Tensor] = None):
        lib = load_library()
        self.desc = CacheDesc()
        self.desc.n_layers, self.desc.max_seqs = n_layers, max_seqs
        self.desc.n_q_heads, self.desc.n_kv_heads, self.desc.head_dim = n_q_heads, n_kv_heads, head_dim
        self.desc.page_tokens, self.desc.max_context = page_tokens, max_context
        for c in range(4):
            self.desc.pool_pages[c] = int(pool_pages[c])
        self._arena = arena
        if arena is not None:
            self.desc.arena = _ptr(arena, torch.uint8, "arena")
            self.desc.arena_bytes = arena.numel()
        self.handle = ctypes.c_void_p(None)
        _check(lib.kvq_cache_create(ctypes.byref(self.desc), ctypes.byref(self.handle)))
        self.n_layers, self.max_seqs, self.Hq, self.Hkv, self.max_context = n_layers, max_seqs, n_q_heads, n_kv_heads, max_context

    @staticmethod
    def arena_bytes(n_layers, max_seqs, n_q_heads, n_kv_heads, max_context, page_tokens=0, pool_pages=(0, 0, 0, 0)) -> int:
        d = CacheDesc()
        d.n_layers, d.max_seqs, d.n_q_heads, d.n_kv_heads, d.head_dim = n_layers, max_seqs, n_q_heads, n_kv_heads, 64
        d.page_tokens, d.max_context = page_tokens, max_context
        for c in range(4):
            d.pool_pages[c] = int(pool_pages[c])
        return int(load_library().kvq_cache_arena_bytes(ctypes.byref(d)))

    def destroy(self) -> None:
        if self.handle:
            _check(load_library().kvq_cache_destroy(self.handle))
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reset(self, stream=None) -> None:
        _check(load_library().kvq_cache_reset(self.handle, _stream(stream)))

    def free_seqs(self, seq_ids: Optional[torch.Tensor], n_seq: int, stream=None) -> None:
        _check(load_library().kvq_cache_free_seqs(self.handle, _ptr(seq_ids, torch.int32, "seq_ids"), n_seq, _stream(stream)))

    def set_length_hint(self, longest_live_length: int) -> None:
        _check(load_library().kvq_cache_set_length_hint(self.handle, int(longest_live_length)))

    def status(self, stream=None):
        flags = ctypes.c_uint32(0)
        free = (ctypes.c_int64 * 4)()
        _check(load_library().kvq_cache_status(self.handle, ctypes.byref(flags), free, _stream(stream)))
        return int(flags.value), [int(x) for x in free]

    def counts(self, stream=None) -> torch.Tensor:
        """int32 [max_seqs, 5] on the host: tokens per class and total length."""
        out = torch.zeros((self.max_seqs, 5), dtype=torch.int32)
        _check(load_library().kvq_cache_counts(self.handle, out.data_ptr(), _stream(stream)))
        return out

    def set_k_channel_quant(self, kmin: Optional[torch.Tensor], krange: Optional[torch.Tensor], stream=None) -> None:
        """Static per-channel key quantizer: fp16 device tensors [n_layers, Hkv, 64] (None, None: back to per-token)."""
        for t in (kmin, krange):
            assert t is None or (t.is_cuda and t.dtype == torch.float16 and t.is_contiguous() and
                                 tuple(t.shape) == (self.desc.n_layers, self.Hkv, 64))
        _check(load_library().kvq_cache_set_k_channel_quant(self.handle, kmin.data_ptr() if kmin is not None else None,
                                                            krange.data_ptr() if krange is not None else None, _stream(stream)))

    def usage(self, stream=None) -> dict:
        """Tokens per class, E[b], stored bits per element, payload and page bytes (host values)."""
        u = CacheUsage()
        _check(load_library().kvq_cache_usage_of(self.handle, ctypes.byref(u), _stream(stream)))
        return {"tokens": [int(x) for x in u.tokens], "expected_bits": float(u.expected_bits),
                "effective_bits": float(u.effective_bits), "payload_bytes": int(u.payload_bytes),
                "pages_in_use": [int(x) for x in u.pages_in_use], "page_bytes_in_use": int(u.page_bytes_in_use)}

    def export(self, layer: int, seq: int, max_tokens: int, stream=None):
        dev = torch.device("cuda")
        bits = torch.zeros(max_tokens, dtype=torch.uint8, device=dev)
        codes = torch.zeros((max_tokens, self.Hkv, 2, EXPORT_REC), dtype=torch.uint8, device=dev)
        meta = torch.zeros((max_tokens, self.Hkv, 2, 2), dtype=torch.int16, device=dev)
        _check(load_library().kvq_cache_export(self.handle, layer, seq, bits.data_ptr(), codes.data_ptr(),
                                               meta.data_ptr(), max_tokens, _stream(stream)))
        return bits, codes, meta


def kvq_cache_import(cache: Cache, layer: int, seq: int, bits: Optional[torch.Tensor], codes: torch.Tensor, meta: torch.Tensor,
                     n_tokens: int, stream=None) -> None:
    """Appends n_tokens tokens to `seq` from the arrays Cache.export returned (device tensors)."""
    assert codes.is_cuda and meta.is_cuda and codes.is_contiguous() and meta.is_contiguous()
    assert codes.numel() >= n_tokens * cache.Hkv * 2 * EXPORT_REC and meta.numel() >= n_tokens * cache.Hkv * 4
    _check(load_library().kvq_cache_import(cache.handle, layer, seq, _ptr(bits, torch.uint8, "bits"), codes.data_ptr(),
                                           meta.data_ptr(), n_tokens, _stream(stream)))


def kvq_features_workspace(n: int, vocab: int) -> int:
    return int(load_library().kvq_features_workspace(n, vocab))


def kvq_features(logits: torch.Tensor, token_ids: torch.Tensor, counts: torch.Tensor, totals: torch.Tensor,
                 update_counts: bool, attn_len: torch.Tensor, n_q_heads: int, feats_out: torch.Tensor,
                 workspace: torch.Tensor, attn_probs: Optional[torch.Tensor] = None,
                 sum_p2: Optional[torch.Tensor] = None, stream=None) -> None:
    n, vocab = logits.shape
    ld = attn_probs.shape[-1] if attn_probs is not None else 0
    _check(load_library().kvq_features(
        _ptr(logits, torch.float32, "logits"), n, vocab, _ptr(token_ids, torch.int32, "token_ids"),
        _ptr(counts, torch.int64, "counts"), _ptr(totals, torch.int64, "totals"), int(bool(update_counts)),
        _ptr(attn_probs, torch.float32, "attn_probs"), _ptr(sum_p2, torch.float32, "sum_p2"),
        _ptr(attn_len, torch.int32, "attn_len"), n_q_heads, ld, _ptr(feats_out, torch.float32, "feats_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


def kvq_features_controller(logits: torch.Tensor, token_ids: torch.Tensor, counts: torch.Tensor, totals: torch.Tensor,
                            update_counts: bool, sum_p2: torch.Tensor, attn_len: torch.Tensor, n_q_heads: int,
                            mlp: "MlpWeights", feats_out: torch.Tensor, bits_out: torch.Tensor, workspace: torch.Tensor,
                            cache: Optional["Cache"] = None, seq_ids: Optional[torch.Tensor] = None,
                            logits_out: Optional[torch.Tensor] = None, stream=None) -> None:
    n, vocab = logits.shape
    _check(load_library().kvq_features_controller(
        _ptr(logits, torch.float32, "logits"), n, vocab, _ptr(token_ids, torch.int32, "token_ids"),
        _ptr(counts, torch.int64, "counts"), _ptr(totals, torch.int64, "totals"), int(bool(update_counts)),
        _ptr(sum_p2, torch.float32, "sum_p2"), _ptr(attn_len, torch.int32, "attn_len"), n_q_heads,
        ctypes.byref(mlp.c), cache.handle if cache is not None else None, _ptr(seq_ids, torch.int32, "seq_ids"),
        _ptr(feats_out, torch.float32, "feats_out"), _ptr(bits_out, torch.uint8, "bits_out"),
        _ptr(logits_out, torch.float32, "logits_out"), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


DTYPE_F32, DTYPE_F16, DTYPE_BF16 = 0, 1, 2


def _logits_dtype(logits: torch.Tensor) -> int:
    codes = {torch.float32: DTYPE_F32, torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16}
    if logits.dtype not in codes:
        raise ValueError("logits must be float32, float16 or bfloat16, got %s" % logits.dtype)
    return codes[logits.dtype]


def kvq_features_typed(logits: torch.Tensor, token_ids: torch.Tensor, counts: torch.Tensor, totals: torch.Tensor,
                       update_counts: bool, attn_len: torch.Tensor, n_q_heads: int, feats_out: torch.Tensor,
                       workspace: torch.Tensor, attn_probs: Optional[torch.Tensor] = None,
                       sum_p2: Optional[torch.Tensor] = None, stream=None) -> None:
    """kvq_features for float32, float16 or bfloat16 logits (the type code is taken from the tensor)."""
    n, vocab = logits.shape
    ld = attn_probs.shape[-1] if attn_probs is not None else 0
    _check(load_library().kvq_features_typed(
        _ptr(logits, None, "logits"), _logits_dtype(logits), n, vocab, _ptr(token_ids, torch.int32, "token_ids"),
        _ptr(counts, torch.int64, "counts"), _ptr(totals, torch.int64, "totals"), int(bool(update_counts)),
        _ptr(attn_probs, torch.float32, "attn_probs"), _ptr(sum_p2, torch.float32, "sum_p2"),
        _ptr(attn_len, torch.int32, "attn_len"), n_q_heads, ld, _ptr(feats_out, torch.float32, "feats_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


def kvq_features_controller_typed(logits: torch.Tensor, token_ids: torch.Tensor, counts: torch.Tensor, totals: torch.Tensor,
                                  update_counts: bool, sum_p2: torch.Tensor, attn_len: torch.Tensor, n_q_heads: int,
                                  mlp: "MlpWeights", feats_out: torch.Tensor, bits_out: torch.Tensor, workspace: torch.Tensor,
                                  cache: Optional["Cache"] = None, seq_ids: Optional[torch.Tensor] = None,
                                  logits_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """kvq_features_controller for float32, float16 or bfloat16 logits."""
    n, vocab = logits.shape
    _check(load_library().kvq_features_controller_typed(
        _ptr(logits, None, "logits"), _logits_dtype(logits), n, vocab, _ptr(token_ids, torch.int32, "token_ids"),
        _ptr(counts, torch.int64, "counts"), _ptr(totals, torch.int64, "totals"), int(bool(update_counts)),
        _ptr(sum_p2, torch.float32, "sum_p2"), _ptr(attn_len, torch.int32, "attn_len"), n_q_heads,
        ctypes.byref(mlp.c), cache.handle if cache is not None else None, _ptr(seq_ids, torch.int32, "seq_ids"),
        _ptr(feats_out, torch.float32, "feats_out"), _ptr(bits_out, torch.uint8, "bits_out"),
        _ptr(logits_out, torch.float32, "logits_out"), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


class MlpWeights:
    """Device weights of the controller plus the C struct that points at them."""

    def __init__(self, weights: Sequence[torch.Tensor], biases: Sequence[torch.Tensor]):
        assert len(weights) == len(biases) and 2 <= len(weights) <= 3
        self.W = [w.contiguous() for w in weights]
        self.b = [b.contiguous() for b in biases]
        self.c = Mlp()
        self.c.n_linear = len(self.W)
        self.c.dims[0] = self.W[0].shape[1]
        for l, (w, b) in enumerate(zip(self.W, self.b)):
            assert w.dtype == torch.float32 and b.dtype == torch.float32 and w.is_cuda and b.is_cuda
            assert w.shape[1] == self.c.dims[l] and b.shape == (w.shape[0],)
            self.c.dims[l + 1] = w.shape[0]
            self.c.W[l] = w.data_ptr()
            self.c.b[l] = b.data_ptr()


def kvq_controller(feats: torch.Tensor, mlp: MlpWeights, bits_out: torch.Tensor,
                   logits_out: Optional[torch.Tensor] = None, stream=None) -> None:
    n = feats.shape[0]
    _check(load_library().kvq_controller(_ptr(feats, torch.float32, "feats"), n, ctypes.byref(mlp.c),
                                         _ptr(bits_out, torch.uint8, "bits_out"),
                                         _ptr(logits_out, torch.float32, "logits_out"), _stream(stream)))


def make_rule(w: Sequence[float], bias: float, thr: Sequence[float]) -> Rule:
    r = Rule()
    for i in range(4):
        r.w[i] = w[i]
    r.bias = bias
    for k in range(3):
        r.thr[k] = thr[k]
    return r


def kvq_rule_policy(feats: torch.Tensor, rule: Rule, bits_out: torch.Tensor, score_out: Optional[torch.Tensor] = None,
                    stream=None) -> None:
    _check(load_library().kvq_rule_policy(_ptr(feats, torch.float32, "feats"), feats.shape[0], ctypes.byref(rule),
                                          _ptr(bits_out, torch.uint8, "bits_out"), _ptr(score_out, torch.float32, "score_out"),
                                          _stream(stream)))


def make_train_hparams(alpha: float, beta: float, gamma: float, c: Sequence[float], q: Sequence[float], lr: float = 1e-3,
                       beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> TrainHparams:
    hp = TrainHparams()
    hp.alpha, hp.beta, hp.gamma, hp.lr, hp.beta1, hp.beta2, hp.eps = alpha, beta, gamma, lr, beta1, beta2, eps
    for k in range(4):
        hp.c[k], hp.q[k] = c[k], q[k]
    return hp


def kvq_controller_param_count(mlp: MlpWeights) -> int:
    return int(load_library().kvq_controller_param_count(ctypes.byref(mlp.c)))


def kvq_controller_train_workspace(mlp: MlpWeights, n: int) -> int:
    return int(load_library().kvq_controller_train_workspace(ctypes.byref(mlp.c), n))


def kvq_controller_train_step(feats: torch.Tensor, label_bits: torch.Tensor, mlp: MlpWeights, adam_m: MlpWeights,
                              adam_v: MlpWeights, hp: TrainHparams, step: int, workspace: torch.Tensor,
                              losses_out: Optional[torch.Tensor] = None, grads_out: Optional[torch.Tensor] = None,
                              stream=None) -> None:
    """Updates mlp's weights and the Adam moments (adam_m, adam_v: MlpWeights of the same shape) in place."""
    n = feats.shape[0]
    _check(load_library().kvq_controller_train_step(
        _ptr(feats, torch.float32, "feats"), _ptr(label_bits, torch.uint8, "label_bits"), n, ctypes.byref(mlp.c),
        ctypes.byref(adam_m.c), ctypes.byref(adam_v.c), ctypes.byref(hp), step, _ptr(losses_out, torch.float32, "losses_out"),
        _ptr(grads_out, torch.float32, "grads_out"), _ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream(stream)))


def kvq_append(cache: Cache, layer: int, k: torch.Tensor, v: torch.Tensor, bits: Optional[torch.Tensor],
               seq_ids: Optional[torch.Tensor], n_seq: int, T: int, stream=None) -> None:
    _check(load_library().kvq_append(cache.handle, layer, _ptr(k, torch.float16, "k"), _ptr(v, torch.float16, "v"),
                                     _ptr(bits, torch.uint8, "bits"), _ptr(seq_ids, torch.int32, "seq_ids"),
                                     n_seq, T, _stream(stream)))


def kvq_decode_attn_workspace(cache: Cache, n_seq: int) -> int:
    return int(load_library().kvq_decode_attn_workspace(cache.handle, n_seq))


def kvq_decode_attn(cache: Cache, layer: int, q: torch.Tensor, seq_ids: Optional[torch.Tensor], n_seq: int,
                    out: torch.Tensor, workspace: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                    sum_p2_out: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(load_library().kvq_decode_attn(cache.handle, layer, _ptr(q, torch.float16, "q"),
                                          _ptr(seq_ids, torch.int32, "seq_ids"), n_seq,
                                          _ptr(out, torch.float32, "out"), _ptr(lse_out, torch.float32, "lse_out"),
                                          _ptr(sum_p2_out, torch.float32, "sum_p2_out"),
                                          _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


def kvq_decode_attn_static_capacity() -> int:
    return int(load_library().kvq_decode_attn_static_capacity())


def kvq_decode_attn_static(cache: Cache, layer: int, q: torch.Tensor, seq_ids: Optional[torch.Tensor], n_seq: int,
                           out: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                           sum_p2_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """kvq_decode_attn without a workspace argument (the library's fixed scratch array); allocates nothing."""
    _check(load_library().kvq_decode_attn_static(cache.handle, layer, _ptr(q, torch.float16, "q"),
                                                 _ptr(seq_ids, torch.int32, "seq_ids"), n_seq,
                                                 _ptr(out, torch.float32, "out"), _ptr(lse_out, torch.float32, "lse_out"),
                                                 _ptr(sum_p2_out, torch.float32, "sum_p2_out"), _stream(stream)))


def kvq_append_decode_attn(cache: Cache, layer: int, k: torch.Tensor, v: torch.Tensor, bits: Optional[torch.Tensor],
                           q: torch.Tensor, seq_ids: Optional[torch.Tensor], n_seq: int, out: torch.Tensor,
                           workspace: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                           sum_p2_out: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(load_library().kvq_append_decode_attn(
        cache.handle, layer, _ptr(k, torch.float16, "k"), _ptr(v, torch.float16, "v"), _ptr(bits, torch.uint8, "bits"),
        _ptr(q, torch.float16, "q"), _ptr(seq_ids, torch.int32, "seq_ids"), n_seq, _ptr(out, torch.float32, "out"),
        _ptr(lse_out, torch.float32, "lse_out"), _ptr(sum_p2_out, torch.float32, "sum_p2_out"),
        _ptr(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


def kvq_tuning_set(name: str, value: int) -> None:
    _check(load_library().kvq_tuning_set(name.encode(), int(value)))


def kvq_tuning_get(name: str) -> int:
    v = ctypes.c_int32(0)
    _check(load_library().kvq_tuning_get(name.encode(), ctypes.byref(v)))
    return int(v.value)


class tuning:
    """Context manager: set entries of the library's launch-shape table, restore them on exit (tests and sweeps)."""

    def __init__(self, **kw):
        self.kw = kw

    def __enter__(self):
        self.old = {k: kvq_tuning_get(k) for k in self.kw}
        for k, v in self.kw.items():
            kvq_tuning_set(k, v)
        return self

    def __exit__(self, *a):
        for k, v in self.old.items():
            kvq_tuning_set(k, v)
