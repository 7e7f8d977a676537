"""Kernel-level parity on the GPU: the skinny GEMM and the block-causal attention against the oracle's
definitions on seeded operands, through the C ABI (include/bd_kernels.h)."""
import numpy as np
import pytest
import torch

from oracle.bd_oracle import BIDIR, CAUSAL, BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _bits_cuda(w):
    return torch.from_numpy(inputs.bf16_bits(w).view(np.int16)).cuda()


# shapes: every 3B projection (some with fewer output rows to keep the host matmul short), ragged K,
# the tiny model's shapes, M from 1 to 64 including non-multiples of 16
@pytest.mark.parametrize("M,N,K", [
    (32, 2560, 2048), (32, 2048, 2048), (32, 2048, 11008), (32, 4096, 2048), (64, 2560, 2048),
    (1, 2048, 2048), (4, 512, 256), (4, 256, 688), (7, 1376, 256), (33, 1024, 256), (48, 2048, 2048),
    (17, 16, 32), (64, 2048, 11008),
])
def test_gemm_matches_matmul(M, N, K):
    print(f"gemm M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M * 1000003 + N * 101 + K)
    w = inputs.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32) * 0.02)
    x = inputs.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    y, _ = binding.bd_k_gemm(_bits_cuda(w), torch.from_numpy(x).cuda())
    want = x.astype(np.float64) @ w.astype(np.float64).T
    err = np.abs(y.cpu().numpy() - want).max()
    assert err <= 2e-5 * np.sqrt(K) * 0.02 * 4 + 1e-6, err       # fp32 accumulation of exact bf16 products


def test_gemm_identity_pattern_pins_operand_layout():
    # W = [I | 0]: row r of W picks x[:, r]; any mix-up of the packed row/k order or of the accumulator
    # layout moves values to the wrong place
    K, N, M = 96, 64, 20
    w = np.zeros((N, K), np.float32)
    w[np.arange(N), np.arange(N)] = 1.0
    x = inputs.round_to_bf16(np.arange(M * K, dtype=np.float32).reshape(M, K) % 251)
    y, _ = binding.bd_k_gemm(_bits_cuda(w), torch.from_numpy(x).cuda())
    np.testing.assert_array_equal(y.cpu().numpy(), x[:, :N])


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
