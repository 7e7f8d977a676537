"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds no arithmetic of the decoding method: it only draws random
tensors (weights, visual embeddings, prompt ids, draft corruption) and rounds
them to the storage type a configuration names.  Both sides read the same
values; neither side's forward code lives here.

Every tensor is drawn from its own Philox stream keyed by (seed, tensor tag), so
tensors can be generated in any order and in parallel with identical results.
"""
from __future__ import annotations

import dataclasses
import zlib
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder-only language backbone shape (pre-RMSNorm, GQA, SwiGLU, RoPE)."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6

    @property
    def mask_token_id(self) -> int:
        return self.vocab - 1

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def weight_elements(self) -> int:
        """Elements of the matrices one forward streams (norm gains excluded)."""
        per_layer = (self.hidden * (self.q_dim + 2 * self.kv_dim) + self.q_dim * self.hidden
                     + 3 * self.hidden * self.ffn)
        return self.n_layers * per_layer + self.vocab * self.hidden

    def with_layers(self, n_layers: int) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers)


# The 2-layer plumbing model and the Qwen2.5-VL-3B-shaped language backbone.
TINY = ModelShape(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=688, vocab=1024)
QWEN3B = ModelShape(n_layers=36, hidden=2048, n_q_heads=16, n_kv_heads=2, head_dim=128, ffn=11008,
                    vocab=151936)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable; call round_to_bf16 first")
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --- OCP fp8 e4m3fn (1-4-3, bias 7, max 448, no infinities) -----------------------------------------

def _e4m3_table() -> np.ndarray:
    vals = np.empty(256, dtype=np.float32)
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            v = np.nan
        elif e == 0:
            v = s * (m / 8.0) * 2.0 ** (-6)
        else:
            v = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
        vals[code] = v
    return vals


E4M3_VALUES = _e4m3_table()


def quantize_e4m3(a: np.ndarray) -> np.ndarray:
    """Nearest e4m3fn code (ties to even mantissa), saturating at +-448."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    pos = E4M3_VALUES[:0x7F].astype(np.float64)           # 0 .. 448, ascending, codes 0..126
    mag = np.minimum(np.abs(a).astype(np.float64), 448.0)
    hi = np.searchsorted(pos, mag, side="left").clip(1, len(pos) - 1)
    lo = hi - 1
    dlo = mag - pos[lo]
    dhi = pos[hi] - mag
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((hi & 1) == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    exact0 = mag == 0.0
    code = np.where(exact0, 0, code).astype(np.uint8)
    return (code | (np.signbit(a).astype(np.uint8) << 7)).astype(np.uint8)


def dequantize_e4m3(codes: np.ndarray) -> np.ndarray:
    return E4M3_VALUES[np.ascontiguousarray(codes, dtype=np.uint8)]


# --- weights --------------------------------------------------------------------------------------

def _rng(seed: int, tag: str) -> np.random.Generator:
    key = zlib.crc32(tag.encode("utf-8"))
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(key)]))


def weight_names(shape: ModelShape) -> List[Tuple[str, Tuple[int, ...]]]:
    """(name, shape) of every tensor of the model; matrices are [out_features, in_features]."""
    out: List[Tuple[str, Tuple[int, ...]]] = [("embed", (shape.vocab, shape.hidden))]
    for l in range(shape.n_layers):
        p = f"l{l}."
        out += [
            (p + "attn_norm", (shape.hidden,)),
            (p + "wq", (shape.q_dim, shape.hidden)),
            (p + "wk", (shape.kv_dim, shape.hidden)),
            (p + "wv", (shape.kv_dim, shape.hidden)),
            (p + "wo", (shape.hidden, shape.q_dim)),
            (p + "ffn_norm", (shape.hidden,)),
            (p + "w_gate", (shape.ffn, shape.hidden)),
            (p + "w_up", (shape.ffn, shape.hidden)),
            (p + "w_down", (shape.hidden, shape.ffn)),
        ]
    out += [("final_norm", (shape.hidden,)), ("lm_head", (shape.vocab, shape.hidden))]
    return out


FP8_LINEARS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def make_weights(shape: ModelShape, seed: int, storage: str = "f32", std: float = 0.02,
                 norm_gain_jitter: float = 0.0, lm_head_scale: float = 1.0,
                 threads: int = 8) -> Dict[str, np.ndarray]:
    """Random-init model.

    storage: "f32"  - fp32 values as drawn;
             "bf16" - every matrix rounded to bf16 (returned as fp32 holding bf16 values);
             "fp8"  - the seven decoder linears become e4m3 codes with one fp32 scale per output
                      channel (amax/448); entries "<name>" (uint8 codes) and "<name>.scale"
                      (fp32 [out]); embedding table and LM head are rounded to bf16.
    Norm gains are 1 (plus an optional jitter used only by tests, so that a dropped gain shows).
    lm_head_scale multiplies the LM head before rounding (tests use it to spread confidences).
    """
    if storage not in ("f32", "bf16", "fp8"):
        raise ValueError(storage)

    def one(item):
        name, shp = item
        base = name.split(".")[-1]
        g = _rng(seed, name)
        if len(shp) == 1:
            w = np.ones(shp, dtype=np.float32)
            if norm_gain_jitter:
                w = w + np.float32(norm_gain_jitter) * g.standard_normal(shp, dtype=np.float32)
            return [(name, w)]
        w = g.standard_normal(shp, dtype=np.float32)
        w *= np.float32(std * (lm_head_scale if name == "lm_head" else 1.0))
        if storage == "f32":
            return [(name, w)]
        if storage == "bf16" or base not in FP8_LINEARS:
            return [(name, round_to_bf16(w))]
        amax = np.abs(w).max(axis=1)
        scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
        codes = quantize_e4m3(w / scale[:, None])
        return [(name, codes), (name + ".scale", scale)]

    items = weight_names(shape)
    out: Dict[str, np.ndarray] = {}
    if threads <= 1:
        res = [one(it) for it in items]
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            res = list(ex.map(one, items))
    for lst in res:
        for k, v in lst:
            out[k] = v
    return out


# --- prompts and drafts ---------------------------------------------------------------------------

def make_prompt(shape: ModelShape, n_embed: int, n_ids: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Prefix = n_embed continuous 'visual' embeddings ~N(0,1)/16 followed by n_ids uniform text ids.

    Ids are drawn from [0, vocab-1) so that none equals the mask token (the last id).
    """
    ge = _rng(seed, "prompt.embeds")
    gi = _rng(seed, "prompt.ids")
    embeds = (ge.standard_normal((n_embed, shape.hidden), dtype=np.float32) / np.float32(16.0)).astype(np.float32)
    ids = gi.integers(0, shape.vocab - 1, size=n_ids, dtype=np.int64).astype(np.int32)
    return embeds, ids


def corrupt_draft(shape: ModelShape, draft: np.ndarray, seed: int, p: float = 0.2) -> Tuple[np.ndarray, np.ndarray]:
    """Replace each drafted id independently with probability p by a uniform id in [0, vocab-1).

    Returns (corrupted draft, boolean array of replaced positions).
    """
    g = _rng(seed, "draft.corrupt")
    draft = np.asarray(draft, dtype=np.int32)
    hit = g.random(draft.shape[0]) < p
    repl = g.integers(0, shape.vocab - 1, size=draft.shape[0], dtype=np.int64).astype(np.int32)
    return np.where(hit, repl, draft).astype(np.int32), hit


def random_qkv(n_keys: int, n_rows: int, n_q_heads: int, n_kv_heads: int, head_dim: int, seed: int,
               bf16: bool = True):
    """Random attention operands for kernel-level tests: Q [rows,n_q,d], K,V [keys,n_kv,d]."""
    g = _rng(seed, "attn.qkv")
    q = g.standard_normal((n_rows, n_q_heads, head_dim), dtype=np.float32)
    k = g.standard_normal((n_keys, n_kv_heads, head_dim), dtype=np.float32)
    v = g.standard_normal((n_keys, n_kv_heads, head_dim), dtype=np.float32)
    if bf16:
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k, v
