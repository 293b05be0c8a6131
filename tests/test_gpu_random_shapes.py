"""GPU parity on seeded random combinations of everything a call can vary: batch size and context
lengths, head counts, head_dim, KV type, query tokens, sliding window, shared prefix, output type,
forced partition counts.  Each case is small enough for the float64 CPU oracle to finish at once;
the point is the combinations the hand-picked cases of the other files do not list."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity

pytestmark = pytest.mark.gpu

MAX_COLS = 512


@pytest.fixture(scope="module")
def pa():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2605_06068_amd import binding

    binding.lib()
    return binding


def draw_case(seed):
    """A valid call, drawn from the seed alone."""
    rng = np.random.default_rng(10_000 + seed)
    D = int(rng.choice([64, 128]))
    kv = int(rng.choice([W.KV_BF16, W.KV_FP8_E4M3]))
    Hkv = int(rng.choice([1, 2, 3, 4]))
    kind = rng.choice(["decode", "verify", "window", "prefix", "prefix-verify", "wide-group"])
    Q, window, prefix_blocks = 1, 0, 0
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
    if kind == "wide-group":
        G = int(rng.choice([17, 24, 32, 48, 64, 100, 128]))
    if kind in ("verify", "window") and rng.random() < 0.8:
        Q = int(rng.integers(2, 1 + max(2, min(64, MAX_COLS // G))))
    if kind == "window":
        window = int(rng.choice([1, 2, 15, 16, 17, 31, 32, 33, 64, 100, 257, 1000]))
    if kind in ("prefix", "prefix-verify"):
        G = int(rng.choice([1, 2, 4, 8, 16, 32]))
        prefix_blocks = int(rng.choice([1, 2, 3, 4, 7, 8, 21, 40]))
        if kind == "prefix-verify":
            Q = int(rng.integers(2, 1 + max(2, 128 // G)))  # up to 128 columns per KV head behind a shared prefix
    B = int(rng.choice([1, 2, 3, 5, 8, 17, 40]))
    style = rng.choice(["short", "mixed", "long"])
    hi = {"short": 70, "mixed": 600, "long": 1500}[style]
    lens = rng.integers(0 if prefix_blocks == 0 else 1, hi, size=B)
    if prefix_blocks == 0:
        lens[rng.random(B) < 0.15] = 0           # empty contexts
    else:
        lens = prefix_blocks * 16 + Q - 1 + rng.integers(0, hi // 4 + 1, size=B)   # every query token after the prefix
    P = int(rng.choice([0, 0, 0, 1, 2, 3, 7, 33, 500]))
    out_bf16 = bool(rng.random() < 0.25)
    return dict(kind=str(kind), D=D, kv=kv, Hkv=Hkv, G=G, Q=Q, window=window, prefix_blocks=prefix_blocks,
                lens=[int(x) for x in lens], P=P, out_bf16=out_bf16)


def seeds():
    """400 seeds by default; PA_EXTRA_SEEDS=first:last adds a range of further ones (a longer run by hand)."""
    import os

    extra = os.environ.get("PA_EXTRA_SEEDS", "")
    more = []
    if extra:
        first, last = (int(x) for x in extra.split(":"))
        more = list(range(first, last))
    return list(range(400)) + more


@pytest.mark.parametrize("seed", seeds())
def test_random_call(pa, oracle, seed):
    import torch

    c = draw_case(seed)
    print(f"[case] seed={seed} {c}", flush=True)
    b = W.make_batch("random", 20_000 + seed, c["lens"], c["G"] * c["Hkv"], c["Hkv"], c["D"], 16, c["kv"], q_len=c["Q"],
                     window=c["window"], shared_prefix_blocks=c["prefix_blocks"])
    dev = pa.DeviceBatch(b, num_partitions=c["P"], out_dtype=pa.PA_OUT_BF16 if c["out_bf16"] else pa.PA_OUT_F32)
    out = dev.decode()
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    if c["out_bf16"]:
        got = W.bf16_bits_to_f32(got.view(np.uint16))
    want = oracle.decode_batch(b)["out"]
    assert got.shape == want.shape
    assert np.isfinite(got).all()
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    if c["out_bf16"]:
        slack = 1e-2 if c["kv"] == W.KV_BF16 else 5e-2   # the path's own bar, on top of half a bf16 ulp of the value
        assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) / 256 + slack)
    else:
        err = assert_parity(flat(got), flat(want), c["kv"], f"random call {seed}")
        print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)} "
              f"{pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)
