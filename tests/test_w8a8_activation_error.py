"""What the paper's "W8A8 (FP8)" would cost in accuracy on this path, measured on the oracle (CPU only).

The GPU path keeps the activations in bf16 and multiplies them with the e4m3 weights widened to bf16 (W8A16).  Running
the seven decoder linears on the fp8 matrix cores instead would need the activations in e4m3 as well: a dynamic scale
per token (max |x| of the row mapped to 448, the largest e4m3 value) and round-to-nearest into e4m3.  This file applies
exactly that to the inputs of the seven linears inside the oracle's forward (through its own weight accessor, nothing
else changed) and compares the logits with the oracle's own: the error that such a kernel would add before any
arithmetic of its own.  The test holds the reduced-depth figure to the bar of the e4m3 configuration (1e-1 of the logit
range) and prints it; run as a script it prints the figure for any depth:

    python tests/test_w8a8_activation_error.py --layers 36 --prefix 256
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle.bd_oracle import BIDIR, BlockDiffusionOracle, _decode_e4m3   # noqa: E402
from paper_2604_06832_amd import inputs                                  # noqa: E402

_POS = np.sort(np.unique(_decode_e4m3(np.arange(0, 127, dtype=np.uint8))))     # the non-negative e4m3 values, ascending
_MID = (_POS[1:] + _POS[:-1]) / 2.0


def quantise_rows_e4m3(x):
    """Per-row dynamic e4m3: row / scale rounded to the nearest representable value (scale = max|row| / 448)."""
    x = np.asarray(x, np.float64)
    scale = np.abs(x).max(axis=-1, keepdims=True) / 448.0
    scale = np.where(scale == 0.0, 1.0, scale)
    a = np.abs(x) / scale
    q = _POS[np.searchsorted(_MID, a)]                   # nearest value (ties go up: immaterial here)
    return np.sign(x) * q * scale


class _QuantisedInput:
    """Stands for W^T in `x @ W.T`: quantises x per row first."""
    __array_ufunc__ = None

    def __init__(self, wt):
        self.wt = wt

    def __rmatmul__(self, x):
        return (quantise_rows_e4m3(x).astype(self.wt.dtype)) @ self.wt


class _Mat:
    def __init__(self, w):
        self.w = w

    @property
    def T(self):
        return _QuantisedInput(self.w.T)


class W8A8Oracle(BlockDiffusionOracle):
    """The oracle with e4m3 activations in front of the seven decoder linears (the LM head stays as it is)."""

    def _mat(self, name):
        w = super()._mat(name)
        return _Mat(w) if name != "lm_head" else w


def measure(n_layers, prefix, B, seed=2, say=lambda m: None):
    shape = inputs.QWEN3B.with_layers(n_layers)
    w = inputs.make_weights(shape, seed, "fp8", threads=min(16, os.cpu_count() or 8))
    n_embed = prefix * 3 // 4
    emb, ids = inputs.make_prompt(shape, n_embed, prefix - n_embed, seed=104)
    # codes x scales -> real values once, with the oracle's own routine (it would otherwise redo that on every use)
    dec = BlockDiffusionOracle(shape, w, dtype=np.float32)
    wd = {}
    for k, v in w.items():
        if not k.endswith(".scale"):
            wd[k] = dec._mat(k) if v.dtype == np.uint8 else v
            if k.endswith("w_down"):
                say(f"decoded {k}")
    w = wd
    out = []
    for cls in (BlockDiffusionOracle, W8A8Oracle):
        o = cls(shape, w, dtype=np.float32)
        say(f"{cls.__name__}: prompt pass")
        o.prefill(emb, ids, chunk=256)
        say(f"{cls.__name__}: block forward")
        lg, _, _ = o.forward(o.embed(np.full(B, o.mask_id, np.int32)), BIDIR)
        out.append((np.asarray(lg, np.float64), np.asarray(o.carry, np.float64)))
    (a, ca), (b, cb) = out
    rng = float(a.max() - a.min())
    return {"max_abs_err": float(np.abs(a - b).max()), "range": rng, "err_over_range": float(np.abs(a - b).max()) / rng,
            "rms_err_over_sigma": float(np.sqrt(np.mean((a - b) ** 2)) / a.std()),
            "argmax_changed": int((a.argmax(-1) != b.argmax(-1)).sum()), "rows": int(a.shape[0]),
            "carry_err_over_range": float(np.abs(ca - cb).max()) / float(ca.max() - ca.min())}


def test_quantiser_is_exact_on_representable_values_and_within_half_a_step():
    vals = _decode_e4m3(np.arange(256, dtype=np.uint8))
    vals = vals[np.isfinite(vals)]
    row = np.concatenate([vals, [448.0]])                 # max 448: scale 1
    assert np.array_equal(quantise_rows_e4m3(row[None, :])[0], row)
    x = np.random.default_rng(0).normal(size=(4, 4096))
    q = quantise_rows_e4m3(x)
    rel = np.abs(q - x) / np.maximum(np.abs(x), 1e-30)
    big = np.abs(x) > np.abs(x).max(axis=-1, keepdims=True) * 2.0 ** -6     # normal range of the scaled row
    assert rel[big].max() <= 2.0 ** -4 + 1e-12            # 3 mantissa bits: half a step of 2^-3


def test_w8a8_activations_at_reduced_depth_stay_within_the_e4m3_bar():
    r = measure(n_layers=2, prefix=64, B=32)
    print(f"[w8a8] 2 layers: logits differ by {r['err_over_range']:.4f} of their range (rms {r['rms_err_over_sigma']:.4f} sigma), "
          f"{r['argmax_changed']}/{r['rows']} argmax ids change")
    assert r["err_over_range"] <= 1e-1


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=36)
    ap.add_argument("--prefix", type=int, default=256)
    ap.add_argument("--block", type=int, default=32)
    a = ap.parse_args()
    print(measure(a.layers, a.prefix, a.block, say=lambda m: print(m, flush=True)), flush=True)
