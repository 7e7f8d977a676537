"""The seeded input generators: storage rounding against PyTorch's own casts, determinism, shapes."""
import numpy as np
import torch

from oracle.bd_oracle import _decode_e4m3
from paper_2604_06832_amd import inputs


def test_bf16_rounding_matches_torch_cast():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 0.02
    x = np.concatenate([x, np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38])])
    got = inputs.round_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    bits = inputs.bf16_bits(got)
    np.testing.assert_array_equal(inputs.bf16_bits_to_f32(bits), got)


def test_e4m3_quantisation_and_both_decoders_match_torch():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for dec in (inputs.dequantize_e4m3(codes), _decode_e4m3(codes)):
        np.testing.assert_array_equal(np.nan_to_num(np.asarray(dec, np.float32), nan=7777.0),
                                      np.nan_to_num(want, nan=7777.0))
    x = np.random.default_rng(1).standard_normal(200000).astype(np.float32) * 100
    x = np.concatenate([x, np.float32([0, 448, 500, -1000, 0.001, 2 ** -9, 2 ** -10, 17.0, 18.0, 19.0, 22.0])])
    got = inputs.quantize_e4m3(x)
    want = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    same = (got == want) | ((inputs.dequantize_e4m3(got) == 0) & (inputs.dequantize_e4m3(want) == 0))
    assert same.all()


def test_weights_are_deterministic_and_order_independent():
    a = inputs.make_weights(inputs.TINY, 0, "bf16", threads=1)
    b = inputs.make_weights(inputs.TINY, 0, "bf16", threads=4)
    assert a.keys() == b.keys()
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    c = inputs.make_weights(inputs.TINY, 1, "bf16", threads=1)
    assert not np.array_equal(a["l0.wq"], c["l0.wq"])
    assert abs(a["l1.w_down"].std() - 0.02) < 1e-3 and np.all(a["final_norm"] == 1)
    assert inputs.TINY.weight_elements() == 2 * (256 * 512 + 256 * 256 + 3 * 256 * 688) + 1024 * 256
    assert inputs.QWEN3B.weight_elements() == 3085697024


def test_fp8_storage_round_trip():
    w = inputs.make_weights(inputs.TINY, 2, "fp8", threads=1)
    f = inputs.make_weights(inputs.TINY, 2, "f32", threads=1)
    q, s = w["l0.w_gate"], w["l0.w_gate.scale"]
    assert q.dtype == np.uint8 and s.shape == (688,)
    deq = inputs.dequantize_e4m3(q) * s[:, None]
    assert np.abs(deq - f["l0.w_gate"]).max() <= np.abs(f["l0.w_gate"]).max() / 448 * 16 + 1e-9
    assert np.abs(inputs.dequantize_e4m3(q)).max() == 448
    assert w["lm_head"].dtype == np.float32


def test_prompt_never_holds_mask_id():
    e, ids = inputs.make_prompt(inputs.TINY, 64, 64, seed=100)
    assert e.shape == (64, 256) and ids.shape == (64,) and ids.max() < inputs.TINY.mask_token_id
    assert abs(e.std() - 1 / 16) < 2e-3
