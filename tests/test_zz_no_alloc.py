"""The attention entry point that allocates nothing (bd_k_attention_static: its working buffers are one static
device array) against the allocating entry point and the oracle, through the C ABI: two calls in a row, the second
on a smaller input, so that whatever the first call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

from oracle.bd_oracle import BIDIR, CAUSAL, BlockDiffusionOracle
from paper_2604_06832_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _case(n_prefix, M, n_q, n_kv, D, mode, seed):
    q, k, v = inputs.random_qkv(n_prefix + M, M, n_q, n_kv, D, seed=seed)
    shape = inputs.ModelShape(1, n_q * D, n_q, n_kv, D, 16, 16)
    want = BlockDiffusionOracle(shape, {}).attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64),
                                                     n_prefix, mode)
    return [torch.from_numpy(a).cuda() for a in (q, k, v)], want


def test_static_attention_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    cases = [(1024, 32, 16, 2, 128, BIDIR, 1), (77, 5, 4, 2, 64, CAUSAL, 2), (300, 17, 16, 2, 128, CAUSAL, 3)]
    prepared = [(_case(*c), c) for c in cases]
    outs = [torch.empty((c[1], c[2] * c[4]), dtype=torch.float32, device="cuda") for c in cases]
    # the first call on a device makes the runtime load the library's code object, and with it the static array itself;
    # what is measured is that the calls after it leave the amount of free device memory alone
    binding.bd_k_attention_static(*prepared[1][0][0], cases[1][0], cases[1][5], out=outs[1])
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for ((qkv, _), c), out in zip(prepared, outs):
        print(f"static attention n={c[0]} M={c[1]} heads={c[2]}/{c[3]} D={c[4]} mode={c[5]}", flush=True)
        binding.bd_k_attention_static(*qkv, c[0], c[5], out=out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "the static entry point changed the amount of free device memory"
    for ((qkv, want), c), out in zip(prepared, outs):
        ref, _ = binding.bd_k_attention(*qkv, c[0], c[5])
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        assert np.array_equal(got, ref.cpu().numpy()), "static and allocating entry points differ"
        # bar of the attention tests: probabilities rounded to bf16 before the PV product, output stored in bf16
        assert np.abs(got - want).max() <= 2e-2


def test_static_attention_rejects_what_does_not_fit():
    q = torch.zeros((32, 16, 128), dtype=torch.float32, device="cuda")
    n = 40000                                    # packed K/V of 40032 keys x 8 kv heads exceed the 32 MiB array
    k = torch.zeros((n + 32, 8, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.BdError) as e:
        binding.bd_k_attention_static(q, k, k, n, BIDIR)
    assert e.value.code == binding.BD_E_CAPACITY
    with pytest.raises(binding.BdError) as e:
        binding.bd_k_attention_static(q[:, :, :48].contiguous(), k[:64, :, :48].contiguous(), k[:64, :, :48].contiguous(), 32, BIDIR)
    assert e.value.code == binding.BD_E_ARG
