"""GPU tests of bf16 output (shape.out_dtype = PA_OUT_BF16): every element must be the float32
result of the same call rounded to nearest even, bit for bit.  Against the float64 CPU oracle the
relative-L2 gate holds as it stands; the max-abs gate is widened by what the output format itself
costs, half a bf16 unit in the last place (|x| / 256 at most)."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import BF16_REL_L2, errors

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pa():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2605_06068_amd import binding

    binding.lib()
    return binding


def run_gpu(pa, batch, **kw):
    import torch

    dev = pa.DeviceBatch(batch, **kw)
    out = dev.decode()
    torch.cuda.synchronize()
    return out.cpu().numpy(), dev


CASES = {
    "head_dim 64": lambda: W.make_config(1),
    "head_dim 64, groups of 8, fp8": lambda: W.make_batch("o0", 699, [0, 1, 33, 700, 16], 16, 2, 64, 16, W.KV_FP8_E4M3),
    "matrix-core kernel, groups of 2": lambda: W.make_batch("o1", 700, [0, 1, 33, 700, 16], 4, 2, 128, 16, W.KV_BF16),
    "matrix-core kernel": lambda: W.make_batch("o2", 701, [0, 1, 33, 700, 16, 2000], 16, 4, 128, 16, W.KV_BF16),
    "matrix-core kernel, fp8": lambda: W.make_batch("o3", 702, [513, 40, 0], 16, 2, 128, 16, W.KV_FP8_E4M3),
    "verification, one wave": lambda: W.make_batch("o4", 703, [600, 2, 90], 8, 2, 128, 16, W.KV_BF16, q_len=4),
    "verification, one wave, two column tiles": lambda: W.make_batch("o7", 706, [600, 2, 90, 33], 8, 2, 128, 16, W.KV_BF16, q_len=7),
    "verification, multi-wave": lambda: W.make_batch("o5", 704, [600, 3, 90, 0], 8, 2, 128, 16, W.KV_BF16, q_len=16),
    "shared prefix": lambda: W.make_batch("o8", 707, [160, 161, 200, 700, 175], 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=10),
    "shared prefix, multi-token, fp8": lambda: W.make_batch("o9", 708, [180, 164, 200, 700], 8, 2, 128, 16, W.KV_FP8_E4M3, q_len=4,
                                                            shared_prefix_blocks=10),
    "sliding window": lambda: W.make_batch("o6", 705, [700, 50, 1], 8, 2, 128, 16, W.KV_BF16, window=100),
    "reduced 8B-shaped batch": lambda: W.make_config(2, length_scale=0.25),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("P", [0, 1, 5])
def test_bf16_output_is_the_rounded_float32_output(pa, oracle, name, P):
    b = CASES[name]()
    print(f"[case] bf16 output: {name} P={P}", flush=True)
    f32, _ = run_gpu(pa, b, num_partitions=P)
    bits, dev = run_gpu(pa, b, num_partitions=P, out_dtype=pa.PA_OUT_BF16)
    assert bits.dtype == np.int16 and bits.shape == f32.shape
    assert np.array_equal(bits.view(np.uint16), W.f32_to_bf16_bits(f32))  # every element written, every rounding RNE
    got = W.bf16_bits_to_f32(bits.view(np.uint16))
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert np.isfinite(got).all()
    # half a bf16 ulp of the value on top of what the float32 result of the same path may be off by:
    # next to nothing where the softmax weights enter the PV product with their rounding remainder
    # (bf16 KV, up to 16 columns, no shared prefix), the path's own bar where they enter as one bf16 number
    columns = b.q_len * (b.num_q_heads // b.num_kv_heads)
    full_weights = b.kv_dtype == W.KV_BF16 and columns <= 16 and b.shared_prefix_blocks == 0
    slack = 1e-5 if full_weights else 1e-2
    assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) / 256 + slack)
    err = errors(flat(got), flat(want))
    assert err[1] <= BF16_REL_L2
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e}", flush=True)
