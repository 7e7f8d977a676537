"""Thin ctypes binding of libbd.so (include/bd.h, include/bd_kernels.h).

Argument marshalling only: every step of the decode path runs inside the library's HIP kernels.
PyTorch tensors are used as device buffers; their data pointers are handed over as plain pointers.
There is no fallback: if the shared library is missing, importing `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbd.so")

BD_OK, BD_E_ARG, BD_E_STATE, BD_E_CAPACITY, BD_E_DTYPE, BD_E_HIP = 0, -1, -2, -3, -4, -5
BD_F32, BD_BF16, BD_FP8_E4M3 = 0, 1, 2
BD_MODE_BIDIR, BD_MODE_CAUSAL = 0, 1
BD_FLAG_CHIP_WIDE_HANDOVER, BD_FLAG_REGISTER_RING, BD_FLAG_PREFILL_DECODE, BD_FLAG_PREFILL_STAGED = 1, 2, 4, 8
BD_FLAG_ATTENTION_KEY_SPLIT = 16
BD_FLAG_MEASURE_NO_WEIGHTS = 32

# every symbol the two headers declare
EXPORTS = [
    "bd_create", "bd_destroy", "bd_load_weight", "bd_prefill", "bd_denoise_step", "bd_commit_block",
    "bd_verify_block", "bd_decode_block", "bd_speculative_step", "bd_quad_draft", "bd_quad_step", "bd_crop", "bd_cache_len", "bd_status", "bd_debug_logits", "bd_read_logits", "bd_read_kv",
    "bd_read_carry", "bd_read_rows", "bd_forward_bytes", "bd_strerror", "bd_last_error",
    "bd_k_attention", "bd_k_attention_static", "bd_k_profile", "bd_k_profile_read", "bd_k_class_count", "bd_k_class_name",
    "bd_k_class_bytes", "bd_k_trace", "bd_k_trace_read", "bd_k_stream_floor", "bd_kv_page_order", "bd_kv_pages", "bd_k_raise_device_error",
]


class bd_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("max_seq", "max_block", "mask_token_id", "weight_dtype", "flags")]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
    L.bd_create.argtypes = [C.POINTER(bd_config), vp, C.POINTER(vp)]
    L.bd_destroy.argtypes = [vp]
    L.bd_destroy.restype = None
    L.bd_load_weight.argtypes = [vp, C.c_char_p, vp, C.c_size_t, i32, vp]
    L.bd_prefill.argtypes = [vp, vp, i32, vp, i32]
    L.bd_denoise_step.argtypes = [vp, vp, vp, i32, f32, i32, vp, vp]
    L.bd_commit_block.argtypes = [vp, vp, i32]
    L.bd_verify_block.argtypes = [vp, vp, i32, i32, vp, vp]
    L.bd_decode_block.argtypes = [vp, i32, f32, i32, vp, vp]
    L.bd_quad_draft.argtypes = [vp, i32, vp]
    L.bd_quad_step.argtypes = [vp, i32, vp, vp, C.POINTER(C.c_int32)]
    L.bd_speculative_step.argtypes = [vp, i32, vp, C.POINTER(C.c_int32)]
    L.bd_crop.argtypes = [vp, i32]
    L.bd_cache_len.argtypes = [vp]
    L.bd_status.argtypes = [vp]
    L.bd_debug_logits.argtypes = [vp, i32]
    L.bd_read_logits.argtypes = [vp, vp, i32]
    L.bd_read_kv.argtypes = [vp, i32, i32, i32, vp, vp]
    L.bd_read_carry.argtypes = [vp, vp, vp]
    L.bd_read_rows.argtypes = [vp, vp, vp, i32]
    L.bd_forward_bytes.argtypes = [vp]
    L.bd_forward_bytes.restype = C.c_int64
    L.bd_strerror.argtypes = [i32]
    L.bd_strerror.restype = C.c_char_p
    L.bd_last_error.argtypes = []
    L.bd_last_error.restype = C.c_char_p
    L.bd_k_attention.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, C.POINTER(f32)]
    L.bd_k_attention_static.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
    L.bd_k_profile.argtypes = [vp, i32]
    L.bd_k_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i32)]
    L.bd_k_class_count.argtypes = []
    L.bd_k_class_name.argtypes = [i32]
    L.bd_k_class_name.restype = C.c_char_p
    L.bd_k_class_bytes.argtypes = [vp, i32]
    L.bd_k_class_bytes.restype = C.c_int64
    L.bd_k_trace.argtypes = [vp, i32]
    L.bd_kv_page_order.argtypes = [vp, vp, i32]
    L.bd_kv_pages.argtypes = [vp, vp, i32]
    L.bd_k_raise_device_error.argtypes = [vp]
    L.bd_k_stream_floor.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.bd_k_trace_read.argtypes = [vp, vp, i32, C.POINTER(i32), C.POINTER(i32)]
    _lib = L
    return L


class BdError(RuntimeError):
    def __init__(self, code: int):
        L = lib()
        msg = L.bd_strerror(code).decode()
        if code == BD_E_HIP:
            msg += ": " + L.bd_last_error().decode()
        super().__init__(f"bd error {code}: {msg}")
        self.code = code


def _check(code: int) -> int:
    if code < 0:
        raise BdError(code)
    return code


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (None passes NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


class Context:
    """One decode context = one bd_ctx.  Methods carry the names of the C calls they wrap."""

    def __init__(self, shape, max_seq: int, max_block: int, weight_dtype: int = BD_BF16, stream=None, flags: int = 0):
        import torch
        self.shape = shape
        cfg = bd_config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                        shape.vocab, shape.rope_theta, shape.rms_eps, max_seq, max_block, shape.mask_token_id,
                        weight_dtype, flags)
        self._stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        _check(lib().bd_create(C.byref(cfg), C.c_void_p(self._stream.cuda_stream), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().bd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the module globals may already be gone
            pass

    # -- weights ------------------------------------------------------------------------------------------
    def bd_load_weight(self, name: str, arr: np.ndarray, scales: Optional[np.ndarray] = None):
        arr = np.ascontiguousarray(arr)
        dt = {np.dtype(np.float32): BD_F32, np.dtype(np.uint16): BD_BF16, np.dtype(np.uint8): BD_FP8_E4M3}[arr.dtype]
        sp = None
        if scales is not None:
            scales = np.ascontiguousarray(scales, dtype=np.float32)
            sp = scales.ctypes.data
        _check(lib().bd_load_weight(self._h, name.encode(), arr.ctypes.data, arr.nbytes, dt, sp))

    def load_model(self, weights: Dict[str, np.ndarray], as_bf16_bits: bool = True):
        """Upload every tensor of an inputs.make_weights() dict (matrices as bf16 bit patterns when they are
        already bf16-representable, else as fp32, which the library rounds)."""
        from . import inputs
        # gain vectors first: the library folds each into the matrices it feeds
        order = sorted(weights.items(), key=lambda kv: kv[1].ndim != 1)
        for name, w in order:
            if name.endswith(".scale"):
                continue
            if w.dtype == np.uint8:
                self.bd_load_weight(name, w, weights[name + ".scale"])
            elif w.ndim == 1 or not as_bf16_bits:
                self.bd_load_weight(name, w.astype(np.float32, copy=False))
            else:
                self.bd_load_weight(name, inputs.bf16_bits(w))

    # -- decode calls --------------------------------------------------------------------------------------
    def bd_prefill(self, embeds, ids):
        n_e = 0 if embeds is None else embeds.shape[0]
        n_i = 0 if ids is None else ids.shape[0]
        _check(lib().bd_prefill(self._h, _ptr(embeds), n_e, _ptr(ids), n_i))

    def bd_denoise_step(self, tokens, mask, threshold: float, fixed_k: int = 0, n_unmasked=None, conf_out=None):
        _check(lib().bd_denoise_step(self._h, _ptr(tokens), _ptr(mask), tokens.shape[0], threshold, fixed_k,
                                     _ptr(n_unmasked), _ptr(conf_out)))

    def bd_commit_block(self, tokens):
        _check(lib().bd_commit_block(self._h, _ptr(tokens), tokens.shape[0]))

    def bd_verify_block(self, draft, commit: bool, ar_pred=None, n_accept=None):
        _check(lib().bd_verify_block(self._h, _ptr(draft), draft.shape[0], int(commit), _ptr(ar_pred), _ptr(n_accept)))

    def bd_decode_block(self, B: int, threshold: float, fixed_k: int, tokens_out, steps_out=None):
        _check(lib().bd_decode_block(self._h, B, threshold, fixed_k, _ptr(tokens_out), _ptr(steps_out)))

    def bd_quad_draft(self, B: int, draft_out):
        _check(lib().bd_quad_draft(self._h, B, _ptr(draft_out)))

    def bd_quad_step(self, B: int, draft, next_draft) -> int:
        k = C.c_int32(0)
        _check(lib().bd_quad_step(self._h, B, _ptr(draft), _ptr(next_draft), C.byref(k)))
        return int(k.value)

    def bd_speculative_step(self, B: int, tokens_out) -> int:
        k = C.c_int32(0)
        _check(lib().bd_speculative_step(self._h, B, _ptr(tokens_out), C.byref(k)))
        return int(k.value)

    def bd_crop(self, new_len: int):
        _check(lib().bd_crop(self._h, new_len))

    def bd_cache_len(self) -> int:
        return _check(lib().bd_cache_len(self._h))

    def bd_status(self):
        _check(lib().bd_status(self._h))

    # -- inspection ----------------------------------------------------------------------------------------
    def bd_debug_logits(self, enable: bool):
        _check(lib().bd_debug_logits(self._h, int(enable)))

    def bd_read_logits(self, rows: int):
        import torch
        out = torch.empty((rows, self.shape.vocab), dtype=torch.float32, device="cuda")
        _check(lib().bd_read_logits(self._h, _ptr(out), rows))
        return out

    def bd_read_kv(self, layer: int, pos0: int, count: int):
        import torch
        k = torch.empty((count, self.shape.n_kv_heads, self.shape.head_dim), dtype=torch.float32, device="cuda")
        v = torch.empty_like(k)
        _check(lib().bd_read_kv(self._h, layer, pos0, count, _ptr(k), _ptr(v)))
        return k, v

    def bd_read_carry(self):
        import torch
        cand = torch.empty(1, dtype=torch.int32, device="cuda")
        conf = torch.empty(1, dtype=torch.float32, device="cuda")
        _check(lib().bd_read_carry(self._h, _ptr(cand), _ptr(conf)))
        return int(cand.item()), float(conf.item())

    def bd_read_rows(self, rows: int):
        import torch
        cand = torch.empty(rows, dtype=torch.int32, device="cuda")
        conf = torch.empty(rows, dtype=torch.float32, device="cuda")
        _check(lib().bd_read_rows(self._h, _ptr(cand), _ptr(conf), rows))
        return cand, conf

    def bd_forward_bytes(self) -> int:
        return _check(lib().bd_forward_bytes(self._h))

    # -- per-kernel timing ---------------------------------------------------------------------------------
    def bd_k_profile(self, enable: bool):
        _check(lib().bd_k_profile(self._h, int(enable)))

    def bd_k_profile_read(self):
        """{class name: (total ms, launches, algorithmic bytes per launch)}"""
        L = lib()
        out = {}
        for k in range(L.bd_k_class_count()):
            ms, cnt = C.c_double(), C.c_int()
            _check(L.bd_k_profile_read(self._h, k, C.byref(ms), C.byref(cnt)))
            out[L.bd_k_class_name(k).decode()] = (ms.value, cnt.value, int(L.bd_k_class_bytes(self._h, k)))
        return out


def _trace_methods():
    def bd_k_trace(self, enable: bool):
        _check(lib().bd_k_trace(self._h, int(enable)))

    def bd_kv_page_order(self, order):
        """Order in which free cache pages are handed out: a permutation of range(ceil(max_seq / 32))."""
        o = np.ascontiguousarray(order, dtype=np.int32)
        _check(lib().bd_kv_page_order(self._h, o.ctypes.data, int(o.size)))

    def bd_kv_pages(self):
        """Pages of the blocks in use, in sequence order."""
        n = lib().bd_kv_pages(self._h, None, 0)
        _check(min(n, 0))
        out = np.zeros(max(n, 1), dtype=np.int32)
        lib().bd_kv_pages(self._h, out.ctypes.data, n)
        return out[:n]

    def bd_k_raise_device_error(self):
        _check(lib().bd_k_raise_device_error(self._h))

    def bd_k_stream_floor(self, repeats: int = 10):
        """(milliseconds, bytes) of reading one forward's layer weights with no consumer, hand-over or barrier."""
        ms, nb = C.c_double(0), C.c_int64(0)
        _check(lib().bd_k_stream_floor(self._h, repeats, C.byref(ms), C.byref(nb)))
        return ms.value, nb.value

    def bd_k_trace_read(self):
        """Timestamps (100 MHz ticks) of the last forward, array [n_wg, per_wg]."""
        n_layers = self.shape.n_layers
        cap = 4096 * (10 * n_layers + 4 + 64)
        buf = np.zeros(cap, dtype=np.uint64)
        n_wg, per = C.c_int(), C.c_int()
        _check(lib().bd_k_trace_read(self._h, buf.ctypes.data, cap, C.byref(n_wg), C.byref(per)))
        n1 = n_wg.value * per.value
        self.last_subtrace = buf[n1:n1 + n_wg.value * 64].reshape(n_wg.value, 64)
        return buf[:n1].reshape(n_wg.value, per.value)

    Context.bd_k_trace = bd_k_trace
    Context.bd_k_stream_floor = bd_k_stream_floor
    Context.bd_k_raise_device_error = bd_k_raise_device_error
    Context.bd_kv_page_order = bd_kv_page_order
    Context.bd_kv_pages = bd_kv_pages
    Context.bd_k_trace_read = bd_k_trace_read


_trace_methods()


def bd_k_attention(q, k, v, n_prefix: int, mode: int, iters: int = 1):
    """Block-causal GQA attention on explicit fp32 cuda operands (see include/bd_kernels.h)."""
    import torch
    M, n_q, D = q.shape
    n_kv = k.shape[1]
    out = torch.empty((M, n_q * D), dtype=torch.float32, device="cuda")
    ms = C.c_float(0)
    _check(lib().bd_k_attention(C.c_void_p(torch.cuda.current_stream().cuda_stream), _ptr(q), _ptr(k), _ptr(v), n_prefix,
                                M, n_q, n_kv, D, mode, _ptr(out), iters, C.byref(ms)))
    return out, ms.value


def bd_k_attention_static(q, k, v, n_prefix: int, mode: int, out=None):
    """The same operation through the entry point that allocates nothing (its working buffers are a static device
    array).  `out` (fp32 [M, n_q*D], cuda) is allocated here when not given; the call only enqueues."""
    import torch
    M, n_q, D = q.shape
    n_kv = k.shape[1]
    if out is None:
        out = torch.empty((M, n_q * D), dtype=torch.float32, device="cuda")
    _check(lib().bd_k_attention_static(C.c_void_p(torch.cuda.current_stream().cuda_stream), _ptr(q), _ptr(k), _ptr(v),
                                       n_prefix, M, n_q, n_kv, D, mode, _ptr(out)))
    return out
