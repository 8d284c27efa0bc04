"""ctypes binding of include/first.h.  Argument marshalling only: tensors are used for
device memory and the stream, nothing is computed here."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
DTYPE_CODES = {"fp32": 0, "bf16": 1}
OPT_USE_GRAPH, OPT_ATTN_SPLITS, OPT_DECODE_PATH = 1, 2, 3

EXPORTS = ["first_create", "first_destroy", "first_prefill_route", "first_set_mask", "first_get_kept",
           "first_decode_step", "first_set_option", "first_sync", "first_last_error", "first_seq_len",
           "first_batch", "first_kv_read", "first_kv_write", "first_get_hidden", "first_set_page_order", "first_sample_top_k",
           "first_num_pages", "first_op_gemv", "first_op_gemm_nt", "first_op_gateup", "first_step_timing", "first_op_gemm_nt_f32a", "first_set_seq_len", "first_kv_usage", "first_soft_forward",
           "first_lora_merge", "first_sample_top_k_static", "first_decode_step_sampled"]


class FirstError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libfirst error {code}: {msg}")
        self.code = code


class _Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rope_base", C.c_float),
                ("rms_eps", C.c_float), ("kv_page_tokens", C.c_int32), ("max_batch", C.c_int32),
                ("max_seq_len", C.c_int32), ("kv_layer_slots", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wq", C.POINTER(C.c_void_p)),
                ("wk", C.POINTER(C.c_void_p)), ("wv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("mlp_norm", C.POINTER(C.c_void_p)), ("w_gate", C.POINTER(C.c_void_p)),
                ("w_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p)), ("router", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(HERE, "libfirst.so")


_LIB = None


def load_library():
    """Loads libfirst.so.  Fails loudly when it has not been built: there is no fallback."""
    global _LIB
    if _LIB is None:
        p = lib_path()
        if not os.path.exists(p):
            raise FileNotFoundError(f"{p} is missing: run `python -m paper_2410_12513_amd.build` "
                                    "(or __graft_entry__.build()) first; there is no CPU fallback")
        lib = C.CDLL(p)
        lib.first_last_error.restype = C.c_char_p
        lib.first_last_error.argtypes = [C.c_void_p]
        for name in EXPORTS:
            if name != "first_last_error":
                getattr(lib, name).restype = C.c_int
        _LIB = lib
    return _LIB


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _check_dev(t: torch.Tensor, dtype: torch.dtype, name: str, numel: Optional[int] = None) -> None:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous device tensor of {dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: needs at least {numel} elements")


class FirstContext:
    """One context per stream.  `weights` is the dict made by synth.make_weights (already on
    the device); `router` a device fp32 [L, D] tensor."""

    def __init__(self, desc, weights: dict, router: torch.Tensor, max_batch: int, max_seq_len: int,
                 kv_page_tokens: int = 16, stream: Optional[torch.cuda.Stream] = None, kv_layer_slots: int = 0):
        self.lib = load_library()
        self.desc = desc
        self.stream = stream
        self.max_batch, self.max_seq_len = int(max_batch), int(max_seq_len)
        wdt = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
        L = desc.n_layers
        self._keep = [weights, router]                       # keep the borrowed tensors alive
        d = _Desc(L, desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.d_ffn, desc.vocab,
                  DTYPE_CODES[desc.dtype], desc.rope_base, desc.rms_eps, kv_page_tokens, max_batch, max_seq_len,
                  kv_layer_slots)
        w = _Weights()
        for name in ("embed", "lm_head"):
            _check_dev(weights[name], wdt, name, desc.vocab * desc.d_model)
            setattr(w, name, weights[name].data_ptr())
        _check_dev(weights["final_norm"], torch.float32, "final_norm", desc.d_model)
        w.final_norm = weights["final_norm"].data_ptr()
        _check_dev(router, torch.float32, "router", L * desc.d_model)
        w.router = router.data_ptr()
        arrays = {}
        for field, key, dt in (("attn_norm", "attn_norm", torch.float32), ("wq", "wq", wdt), ("wk", "wk", wdt),
                               ("wv", "wv", wdt), ("wo", "wo", wdt), ("mlp_norm", "mlp_norm", torch.float32),
                               ("w_gate", "w_gate", wdt), ("w_up", "w_up", wdt), ("w_down", "w_down", wdt)):
            arr = (C.c_void_p * L)()
            for i in range(L):
                _check_dev(weights["layers"][i][key], dt, f"layers[{i}].{key}")
                arr[i] = weights["layers"][i][key].data_ptr()
            arrays[field] = arr
            setattr(w, field, C.cast(arr, C.POINTER(C.c_void_p)))
        self._arrays = arrays
        handle = C.c_void_p()
        sp = C.c_void_p(stream.cuda_stream if stream is not None else 0)
        rc = self.lib.first_create(C.byref(d), C.byref(w), sp, C.byref(handle))
        if rc != 0:
            raise FirstError(rc, self.lib.first_last_error(None).decode())
        self.h = handle

    # -- helpers
    def _chk(self, rc: int) -> None:
        if rc != 0:
            raise FirstError(rc, self.lib.first_last_error(self.h).decode())

    def close(self) -> None:
        if getattr(self, "h", None):
            self.lib.first_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the path
    def prefill_route(self, ids: torch.Tensor, lens: Sequence[int], rho=None, mask=None, hidden=None,
                      logits=None, token=None) -> None:
        B = len(lens)
        _check_dev(ids, torch.int32, "ids", int(sum(lens)))
        L, D, V = self.desc.n_layers, self.desc.d_model, self.desc.vocab
        for t, dt, nm, n in ((rho, torch.float32, "rho", B * L), (mask, torch.uint8, "mask", B * L),
                             (hidden, torch.float32, "hidden", B * D), (logits, torch.float32, "logits", B * V),
                             (token, torch.int32, "token", B)):
            if t is not None:
                _check_dev(t, dt, nm, n)
        lens_a = (C.c_int32 * B)(*[int(x) for x in lens])
        self._chk(self.lib.first_prefill_route(self.h, C.c_int32(B), _ptr(ids), lens_a, _ptr(rho), _ptr(mask),
                                               _ptr(hidden), _ptr(logits), _ptr(token)))

    def soft_forward(self, ids: torch.Tensor, lens: Sequence[int], targets: torch.Tensor, lam: float, alpha: float,
                     terms: torch.Tensor, rho=None, hidden=None) -> None:
        B, n = len(lens), int(sum(lens))
        L, D = self.desc.n_layers, self.desc.d_model
        _check_dev(ids, torch.int32, "ids", n)
        _check_dev(targets, torch.int32, "targets", n)
        _check_dev(terms, torch.float32, "terms", B * 4)
        if rho is not None:
            _check_dev(rho, torch.float32, "rho", B * L)
        if hidden is not None:
            _check_dev(hidden, torch.float32, "hidden", n * D)
        lens_a = (C.c_int32 * B)(*[int(x) for x in lens])
        self._chk(self.lib.first_soft_forward(self.h, C.c_int32(B), _ptr(ids), lens_a, _ptr(targets), C.c_float(lam),
                                              C.c_float(alpha), _ptr(rho), _ptr(terms), _ptr(hidden)))

    def set_mask(self, seq: int, mask: Sequence[int]) -> None:
        L = self.desc.n_layers
        if len(mask) != L:
            raise ValueError("mask must have one entry per layer")
        arr = (C.c_uint8 * L)(*[int(bool(m)) for m in mask])
        self._chk(self.lib.first_set_mask(self.h, C.c_int32(seq), arr))

    def get_kept(self, seq: int) -> List[int]:
        L = self.desc.n_layers
        arr = (C.c_int32 * L)()
        n = C.c_int32()
        self._chk(self.lib.first_get_kept(self.h, C.c_int32(seq), arr, C.byref(n)))
        return list(arr[: n.value])

    def decode_step(self, last_tokens: torch.Tensor, logits: Optional[torch.Tensor], token: torch.Tensor) -> None:
        _check_dev(last_tokens, torch.int32, "last_tokens")
        _check_dev(token, torch.int32, "token")
        if logits is not None:
            _check_dev(logits, torch.float32, "logits")
        self._chk(self.lib.first_decode_step(self.h, _ptr(last_tokens), _ptr(logits), _ptr(token)))

    def decode_step_sampled(self, last_tokens: torch.Tensor, uniforms: torch.Tensor, temperature: float, top_k: int,
                            logits: Optional[torch.Tensor], token: torch.Tensor,
                            candidates_out: Optional[torch.Tensor] = None) -> None:
        B = self.batch()
        _check_dev(last_tokens, torch.int32, "last_tokens")
        _check_dev(uniforms, torch.float32, "uniforms", B)
        _check_dev(token, torch.int32, "token")
        if logits is not None:
            _check_dev(logits, torch.float32, "logits")
        if candidates_out is not None:
            _check_dev(candidates_out, torch.int32, "candidates_out", B * top_k)
        self._chk(self.lib.first_decode_step_sampled(self.h, _ptr(last_tokens), _ptr(uniforms), C.c_float(temperature),
                                                     C.c_int32(top_k), _ptr(logits), _ptr(token), _ptr(candidates_out)))

    def set_option(self, option: int, value: int) -> None:
        self._chk(self.lib.first_set_option(self.h, C.c_int32(option), C.c_int32(value)))

    def sync(self) -> None:
        self._chk(self.lib.first_sync(self.h))

    # -- taps
    def seq_len(self, seq: int) -> int:
        n = C.c_int32()
        self._chk(self.lib.first_seq_len(self.h, C.c_int32(seq), C.byref(n)))
        return n.value

    def batch(self) -> int:
        n = C.c_int32()
        self._chk(self.lib.first_batch(self.h, C.byref(n)))
        return n.value

    def kv_read(self, seq: int, layer: int, pos0: int, n: int):
        shape = (n, self.desc.n_kv_heads, self.desc.head_dim)
        k = torch.empty(shape, dtype=torch.float32, device="cuda")
        v = torch.empty(shape, dtype=torch.float32, device="cuda")
        self._chk(self.lib.first_kv_read(self.h, C.c_int32(seq), C.c_int32(layer), C.c_int32(pos0), C.c_int32(n),
                                         _ptr(k), _ptr(v)))
        return k, v

    def kv_write(self, seq: int, layer: int, pos0: int, k: torch.Tensor, v: torch.Tensor) -> None:
        n = k.shape[0]
        _check_dev(k, torch.float32, "k", n * self.desc.n_kv_heads * self.desc.head_dim)
        _check_dev(v, torch.float32, "v", n * self.desc.n_kv_heads * self.desc.head_dim)
        self._chk(self.lib.first_kv_write(self.h, C.c_int32(seq), C.c_int32(layer), C.c_int32(pos0), C.c_int32(n),
                                          _ptr(k), _ptr(v)))

    def set_seq_len(self, seq: int, length: int) -> None:
        self._chk(self.lib.first_set_seq_len(self.h, C.c_int32(seq), C.c_int32(length)))

    def sample_top_k(self, logits: torch.Tensor, uniforms: torch.Tensor, temperature: float, top_k: int,
                     token_out: torch.Tensor, candidates_out: Optional[torch.Tensor] = None) -> None:
        B = self.batch()
        _check_dev(logits, torch.float32, "logits", B * self.desc.vocab)
        _check_dev(uniforms, torch.float32, "uniforms", B)
        _check_dev(token_out, torch.int32, "token_out", B)
        if candidates_out is not None:
            _check_dev(candidates_out, torch.int32, "candidates_out", B * top_k)
        self._chk(self.lib.first_sample_top_k(self.h, _ptr(logits), _ptr(uniforms), C.c_float(temperature),
                                              C.c_int32(top_k), _ptr(token_out), _ptr(candidates_out)))

    def get_hidden(self) -> torch.Tensor:
        out = torch.empty((self.batch(), self.desc.d_model), dtype=torch.float32, device="cuda")
        self._chk(self.lib.first_get_hidden(self.h, _ptr(out)))
        return out

    def op_gateup(self, layer: int, seq: int = 0) -> None:
        self._chk(self.lib.first_op_gateup(self.h, C.c_int32(layer), C.c_int32(seq)))

    def step_timing(self):
        """Timestamps [phases, 6] (100 MHz ticks) of the last persistent-kernel step."""
        cap = (4 * self.desc.n_layers + 1) * 12
        arr = (C.c_uint64 * cap)()
        n = C.c_int32()
        self._chk(self.lib.first_step_timing(self.h, arr, C.c_int32(cap), C.byref(n)))
        return [list(arr[i:i + 12]) for i in range(0, n.value, 12)]

    def num_pages(self) -> int:
        n = C.c_int32()
        self._chk(self.lib.first_num_pages(self.h, C.byref(n)))
        return n.value

    def kv_usage(self):
        """(bytes of the KV page pool, layer slices available, layer slices in use)."""
        nbytes, slots, used = C.c_int64(), C.c_int32(), C.c_int32()
        self._chk(self.lib.first_kv_usage(self.h, C.byref(nbytes), C.byref(slots), C.byref(used)))
        return nbytes.value, slots.value, used.value

    def set_page_order(self, perm: Sequence[int]) -> None:
        arr = (C.c_int32 * len(perm))(*[int(x) for x in perm])
        if len(perm) != self.num_pages():
            raise ValueError("perm must list every page once")
        self._chk(self.lib.first_set_page_order(self.h, arr))


def _stream_ptr(stream) -> C.c_void_p:
    return C.c_void_p(stream.cuda_stream if stream is not None else 0)


def op_gemv(W: torch.Tensor, x: torch.Tensor, y: torch.Tensor, accumulate: bool = False, stream=None) -> None:
    lib = load_library()
    code = DTYPE_CODES["bf16" if W.dtype == torch.bfloat16 else "fp32"]
    n, k = W.shape
    _check_dev(W, W.dtype, "W"); _check_dev(x, torch.float32, "x", k); _check_dev(y, torch.float32, "y", n)
    rc = lib.first_op_gemv(_stream_ptr(stream), C.c_int32(code), _ptr(W), _ptr(x), _ptr(y), C.c_int32(n),
                           C.c_int32(k), C.c_int32(int(accumulate)))
    if rc != 0:
        raise FirstError(rc, lib.first_last_error(None).decode())


def lora_merge(W: torch.Tensor, A: torch.Tensor, Bm: torch.Tensor, scale: float, stream=None) -> None:
    """In place W += scale * Bm @ A on the device (W [n, k] bf16 or fp32; A [r, k], Bm [n, r] fp32)."""
    lib = load_library()
    code = DTYPE_CODES["bf16" if W.dtype == torch.bfloat16 else "fp32"]
    n, k = W.shape
    r = A.shape[0]
    _check_dev(W, W.dtype, "W"); _check_dev(A, torch.float32, "A", r * k); _check_dev(Bm, torch.float32, "Bm", n * r)
    rc = lib.first_lora_merge(_stream_ptr(stream), C.c_int32(code), _ptr(W), _ptr(A), _ptr(Bm), C.c_int32(n), C.c_int32(k),
                              C.c_int32(r), C.c_float(scale))
    if rc != 0:
        raise FirstError(rc, lib.first_last_error(None).decode())


def op_gemm_nt(A: torch.Tensor, W: torch.Tensor, Cm: torch.Tensor, accumulate: bool = False, stream=None) -> None:
    lib = load_library()
    code = DTYPE_CODES["bf16" if W.dtype == torch.bfloat16 else "fp32"]
    m, k = A.shape
    n = W.shape[0]
    _check_dev(A, W.dtype, "A"); _check_dev(W, W.dtype, "W"); _check_dev(Cm, torch.float32, "C", m * n)
    rc = lib.first_op_gemm_nt(_stream_ptr(stream), C.c_int32(code), _ptr(A), _ptr(W), _ptr(Cm), C.c_int32(m),
                              C.c_int32(n), C.c_int32(k), C.c_int32(int(accumulate)))
    if rc != 0:
        raise FirstError(rc, lib.first_last_error(None).decode())


def op_gemm_nt_f32a(A: torch.Tensor, W: torch.Tensor, Cm: torch.Tensor, accumulate: bool = False, stream=None) -> None:
    """fp32 activations x bf16 weights (split-precision matrix-core kernel of the prefill path)."""
    lib = load_library()
    m, k = A.shape
    n = W.shape[0]
    _check_dev(A, torch.float32, "A"); _check_dev(W, torch.bfloat16, "W"); _check_dev(Cm, torch.float32, "C", m * n)
    rc = lib.first_op_gemm_nt_f32a(_stream_ptr(stream), _ptr(A), _ptr(W), _ptr(Cm), C.c_int32(m), C.c_int32(n),
                                   C.c_int32(k), C.c_int32(int(accumulate)))
    if rc != 0:
        raise FirstError(rc, lib.first_last_error(None).decode())


def sample_top_k_static(logits: torch.Tensor, uniforms: torch.Tensor, temperature: float, top_k: int,
                        token_out: torch.Tensor, candidates_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """first_sample_top_k without a context and without any allocation (static scratch inside the library)."""
    lib = load_library()
    n_seq, vocab = logits.shape
    _check_dev(logits, torch.float32, "logits"); _check_dev(uniforms, torch.float32, "uniforms", n_seq)
    _check_dev(token_out, torch.int32, "token_out", n_seq)
    if candidates_out is not None:
        _check_dev(candidates_out, torch.int32, "candidates_out", n_seq * top_k)
    rc = lib.first_sample_top_k_static(_stream_ptr(stream), _ptr(logits), C.c_int32(n_seq), C.c_int32(vocab), _ptr(uniforms),
                                       C.c_float(temperature), C.c_int32(top_k), _ptr(token_out), _ptr(candidates_out))
    if rc != 0:
        raise FirstError(rc, lib.first_last_error(None).decode())
