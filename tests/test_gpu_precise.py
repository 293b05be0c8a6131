"""shape.precise_weights on the GPU: with the flag set the softmax weights enter the PV product
with 16 significant bits on every path (fp8 KV, wide column tiles, the multi-wave kernel, the
shared-prefix pass), so every kind of call meets the tight bound plain bf16 decode meets by
default; without it those calls stay inside the method's tolerance for values of unit size, but
not for larger ones."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity, errors

pytestmark = pytest.mark.gpu

# bound with the flag set: weights to 2^-17 relative, fp32 accumulation; measured ~1e-5 for values of unit size
PRECISE_MAX_ABS_PER_UNIT = 6e-5


@pytest.fixture(scope="module")
def pa():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2605_06068_amd import binding

    binding.lib()
    return binding


def run(pa, batch, **kw):
    import torch

    dev = pa.DeviceBatch(batch, **kw)
    out = dev.decode()
    torch.cuda.synchronize()
    return out.cpu().numpy(), dev


def flat(a):
    return a.reshape(a.shape[0], -1, a.shape[-1])


CASES = [
    # what, kv, lens, Hq, Hkv, D, q_len, prefix_blocks, window
    ("fp8 decode", W.KV_FP8_E4M3, [513, 40, 1, 2000, 77], 16, 2, 128, 1, 0, 0),
    ("fp8 decode, head_dim 64", W.KV_FP8_E4M3, [513, 40, 1, 2000, 77], 16, 2, 64, 1, 0, 0),
    ("two column tiles in one wave", W.KV_BF16, [700, 90, 33, 1500], 8, 2, 128, 8, 0, 0),
    ("multi-wave, 64 columns", W.KV_BF16, [600, 90, 40, 1300], 8, 2, 128, 16, 0, 0),
    ("multi-wave, 128 columns", W.KV_BF16, [600, 90, 40, 1300], 16, 2, 128, 16, 0, 0),
    ("multi-wave, 128 columns, fp8", W.KV_FP8_E4M3, [600, 90, 40, 1300], 16, 2, 128, 16, 0, 0),
    ("multi-wave, head_dim 64", W.KV_BF16, [600, 90, 40, 1300], 8, 1, 64, 16, 0, 0),
    ("shared prefix", W.KV_BF16, [400, 330, 321, 900], 8, 2, 128, 1, 20, 0),
    ("shared prefix, 4 query tokens, fp8", W.KV_FP8_E4M3, [400, 330, 324, 900], 8, 2, 128, 4, 20, 0),
    ("sliding window, 16 query tokens", W.KV_BF16, [700, 50, 300], 8, 2, 128, 16, 0, 100),
    ("wide group", W.KV_BF16, [300, 257, 31], 64, 1, 128, 1, 0, 0),
]


@pytest.mark.parametrize("what,kv,lens,Hq,Hkv,D,Q,prefix,window", CASES)
@pytest.mark.parametrize("P", [0, 3])
def test_every_path_meets_the_tight_bound_with_the_flag(pa, oracle, what, kv, lens, Hq, Hkv, D, Q, prefix, window, P):
    b = W.make_batch("precise", 700 + len(what), lens, Hq, Hkv, D, 16, kv, q_len=Q, shared_prefix_blocks=prefix, window=window)
    want = oracle.decode_batch(b)["out"]
    print(f"[case] precise weights: {what} P={P}", flush=True)
    got, dev = run(pa, b, num_partitions=P, precise_weights=1)
    assert np.isfinite(got).all()
    err, rel = errors(flat(got), flat(want))
    loose, _ = run(pa, b, num_partitions=P)
    err0, rel0 = errors(flat(loose), flat(want))
    print(f"        flag set: max_abs={err:.2e} rel_l2={rel:.2e}   default: max_abs={err0:.2e} rel_l2={rel0:.2e}", flush=True)
    vmax = 4.0  # N(0, 1) values: a handful of sigmas
    assert err <= PRECISE_MAX_ABS_PER_UNIT * vmax and rel <= 2e-5, (what, err, rel)
    assert_parity(flat(loose), flat(want), kv, what + " (default)")


def test_plain_bf16_decode_is_the_same_call_either_way(pa):
    b = W.make_config(2, length_scale=0.25)
    a, _ = run(pa, b)
    c, _ = run(pa, b, precise_weights=1)
    assert np.array_equal(a, c)


@pytest.mark.parametrize("what,kv,Hq,Hkv,Q,prefix", [("multi-wave", W.KV_BF16, 8, 2, 16, 0), ("fp8", W.KV_FP8_E4M3, 16, 2, 1, 0),
                                                  ("shared prefix", W.KV_BF16, 8, 2, 1, 20)])
def test_values_twice_the_unit_size_need_the_flag(pa, oracle, what, kv, Hq, Hkv, Q, prefix):
    """sigma = 2: the default's error scales with |v| and is no longer guaranteed to stay inside the
    1e-2 gate for bf16 KV (its bound is 2^-9 max|v|, about 1.6e-2 here); the flag restores it with a
    wide margin.  The default's figures are printed, not gated."""
    lens = [900, 330, 324, 2000, 650, 1200]
    b = W.make_batch("sigma2", 750, lens, Hq, Hkv, 128, 16, kv, sigma=2.0, q_len=Q, shared_prefix_blocks=prefix)
    want = oracle.decode_batch(b)["out"]
    got, _ = run(pa, b, precise_weights=1)
    err, rel = errors(flat(got), flat(want))
    loose, _ = run(pa, b)
    err0, rel0 = errors(flat(loose), flat(want))
    print(f"[case] sigma=2 {what}: flag set max_abs={err:.2e} rel_l2={rel:.2e}; default max_abs={err0:.2e} rel_l2={rel0:.2e} "
          f"(default bound 2^-9 max|v| = {np.float32(2.0 ** -9 * 8.0):.2e})", flush=True)
    assert_parity(flat(got), flat(want), kv, what + " with the flag")
    assert err <= PRECISE_MAX_ABS_PER_UNIT * 8.0
    assert np.isfinite(loose).all() and err0 <= 2.0 ** -9 * 10.0


def test_trace_and_static_entries_honour_the_flag(pa):
    import torch

    b = W.make_batch("precise-entries", 760, [600, 90, 40], 8, 2, 128, 16, W.KV_BF16, q_len=16)
    ref, dev = run(pa, b, precise_weights=1)
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), -7, dtype=torch.int32, device="cuda")
    dev.out.fill_(float("nan"))
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    assert np.array_equal(dev.out.cpu().numpy(), ref)
    dev.out.fill_(float("nan"))
    pa.pa_decode_static(*dev.args(), shape=dev.shape)
    torch.cuda.synchronize()
    assert np.array_equal(dev.out.cpu().numpy(), ref)
