"""Kernel-level parity on the GPU: block-causal attention on caller tensors against the oracle's dense-softmax
definition on seeded operands, through the C ABI (include/bd_kernels.h)."""
import numpy as np
import pytest
import torch

from oracle.bd_oracle import BIDIR, CAUSAL, BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_prefix,M,n_q,n_kv,D,mode", [
    (128, 4, 4, 2, 64, BIDIR), (128, 4, 4, 2, 64, CAUSAL), (0, 5, 4, 2, 64, CAUSAL), (1, 1, 4, 2, 64, CAUSAL),
    (1024, 32, 16, 2, 128, BIDIR), (1024, 32, 16, 2, 128, CAUSAL), (1000, 32, 16, 2, 128, CAUSAL),
    (1013, 17, 16, 2, 128, BIDIR), (2048, 64, 16, 2, 128, CAUSAL), (2048, 8, 16, 2, 128, BIDIR),
    (8192, 32, 16, 2, 128, BIDIR), (8704 - 32, 32, 16, 2, 128, CAUSAL), (31, 48, 16, 2, 128, CAUSAL),
    (300, 16, 8, 8, 64, BIDIR),
])
def test_attention_matches_dense_softmax(n_prefix, M, n_q, n_kv, D, mode):
    print(f"attention n={n_prefix} M={M} heads={n_q}/{n_kv} D={D} mode={mode}", flush=True)
    q, k, v = inputs.random_qkv(n_prefix + M, M, n_q, n_kv, D, seed=n_prefix + M)
    shape = inputs.ModelShape(1, n_q * D, n_q, n_kv, D, 16, 16)
    want = BlockDiffusionOracle(shape, {}).attention(q.astype(np.float64), k.astype(np.float64),
                                                     v.astype(np.float64), n_prefix, mode)
    got, _ = binding.bd_k_attention(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(),
                                    torch.from_numpy(v).cuda(), n_prefix, mode)
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    # probabilities are rounded to bf16 before the PV product and the output is stored in bf16
    err = np.abs(got - want).max()
    assert err <= 2e-2, err


def test_attention_first_causal_row_with_empty_prefix_sees_only_itself():
    q, k, v = inputs.random_qkv(6, 6, 4, 2, 64, seed=9)
    got, _ = binding.bd_k_attention(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(),
                                    torch.from_numpy(v).cuda(), 0, CAUSAL)
    got = got.cpu().numpy().reshape(6, 4, 64)
    for h in range(4):
        np.testing.assert_allclose(got[0, h], v[0, h // 2], atol=1e-2)


def test_stream_floor_reads_the_layers_weight_stream():
    """bd_k_stream_floor reads exactly the bytes of the decoder layers' weight stream (every wavefront its own share)
    and reports a time that corresponds to a plausible memory rate."""
    from paper_2604_06832_amd import inputs
    shape = inputs.QWEN3B.with_layers(2)
    ctx = binding.Context(shape, max_seq=256, max_block=32)
    ms, nbytes = ctx.bd_k_stream_floor(5)
    per_layer = shape.hidden * (shape.q_dim + 2 * shape.kv_dim) + shape.q_dim * shape.hidden + 3 * shape.hidden * shape.ffn
    assert nbytes == 2 * 2 * per_layer, (nbytes, per_layer)
    rate = nbytes / (ms * 1e-3) / 1e12
    print(f"stream floor: {nbytes / 1e6:.1f} MB in {ms * 1e3:.1f} us = {rate:.2f} TB/s", flush=True)
    assert 0.2 < rate < 8.0
    ctx.close()
