"""GPU parity of the stage-split partition kernel (17 .. 128 columns per KV head: score waves and
value waves; at head_dim 128 fp8 scores on the fp8 matrix instruction with the query rows split in
two) against the float64 CPU oracle: query rows of wide dynamic range, and context lengths that
put the ends of its runs of plain steps on every side of a tile boundary."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity

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


def flat(a):
    return a.reshape(a.shape[0], -1, a.shape[-1])


def rescale_queries(batch, rng, lo_exp, hi_exp):
    """Every query element times a power of two of its own (exact in bf16), and a few special rows:
    all zeros, one spike among tiny elements, one constant magnitude."""
    q = W.bf16_bits_to_f32(batch.q).astype(np.float32)
    q *= np.exp2(rng.integers(lo_exp, hi_exp + 1, size=q.shape)).astype(np.float32)
    rows = q.reshape(-1, q.shape[-1])
    rows[0] = 0.0
    rows[1] = np.float32(2.0 ** -10) * np.sign(rows[1])
    rows[1, 7] = 96.0
    rows[2] = np.float32(0.5) * np.where(rows[2] >= 0, 1, -1)
    batch.q = W.f32_to_bf16_bits(q).reshape(batch.q.shape)
    assert np.array_equal(W.bf16_bits_to_f32(batch.q), q), "powers of two keep bf16 numbers exact"


# (Q, Hq, Hkv): 64 columns (one column tile per wave), 96 / 128 (two), 24 / 32 (fp8: two score and two value waves)
SHAPES = [(16, 4, 1), (16, 8, 1), (12, 16, 2), (8, 16, 1), (4, 8, 1), (3, 16, 2), (2, 9, 1)]


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", SHAPES)
@pytest.mark.parametrize("lo_exp,hi_exp", [(-12, 0), (-3, 3), (-20, -8)])
def test_query_rows_of_wide_dynamic_range(pa, oracle, kv, Q, Hq, Hkv, lo_exp, hi_exp):
    """fp8 KV: the kernel splits every query row into two e4m3 operands after scaling it by a power of
    two of the row's own; elements many binades below the row's largest, zero rows and rows that are
    one spike must come through (bf16 KV runs the same cases on the bf16 path)."""
    rng = np.random.default_rng(9000 + 31 * Q + Hq + hi_exp)
    lens = [int(x) for x in rng.integers(Q, 700, size=5)] + [Q, 33 + Q, 1024]
    b = W.make_batch("staged-dynamic-range", 9100 + Q + Hq + hi_exp - lo_exp, lens, Hq, Hkv, 128, 16, kv, q_len=Q)
    rescale_queries(b, rng, lo_exp, hi_exp)
    print(f"[case] dynamic range 2^{lo_exp}..2^{hi_exp} Q={Q} Hq={Hq} Hkv={Hkv} kv={kv}", flush=True)
    got, dev = run_gpu(pa, b)
    cols = Q * (Hq // Hkv)
    if cols > 32:
        staged = kv == W.KV_FP8_E4M3 or cols <= 64
        assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == ("mfma-staged" if staged else "mfma-wide")
    elif kv == W.KV_FP8_E4M3:
        assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == "mfma-staged"
    want = oracle.decode_batch(b)["out"]
    err = assert_parity(flat(got), flat(want), kv, "query rows of wide dynamic range")
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e}", flush=True)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(16, 4, 1), (16, 8, 1), (4, 8, 1)])
@pytest.mark.parametrize("P", [0, 1, 3, 7])
def test_lengths_around_the_ends_of_runs(pa, oracle, kv, Q, Hq, Hkv, P):
    """A run of plain steps ends before the first tile that needs a causal mask and before a sequence's
    last tile; lengths that put L and L - Q + 1 just below, on and just above multiples of 32, with range
    starts in the middle of sequences (odd partition counts)."""
    lens = []
    for base in (64, 96, 128, 160, 1024):
        for d in (-1, 0, 1):
            lens += [base + d, base + Q - 1 + d]
    lens += [Q, Q + 1, 31 + Q, 2048]
    b = W.make_batch("staged-run-ends", 9300 + Q + Hq, lens, Hq, Hkv, 128, 16, kv, q_len=Q)
    print(f"[case] run ends Q={Q} Hq={Hq} Hkv={Hkv} kv={kv} P={P}", flush=True)
    got, dev = run_gpu(pa, b, num_partitions=P)
    cols = Q * (Hq // Hkv)
    if kv == W.KV_FP8_E4M3 or 32 < cols <= 64:
        assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == "mfma-staged"
    want = oracle.decode_batch(b)["out"]
    err = assert_parity(flat(got), flat(want), kv, "lengths around the ends of runs")
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)}", flush=True)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(16, 4, 1), (16, 8, 1), (5, 8, 1), (12, 16, 2)])
@pytest.mark.parametrize("P", [0, 3])
def test_head_dim_64(pa, oracle, kv, Q, Hq, Hkv, P):
    """head_dim 64: a tile has half the load instructions, so four score waves exist for bf16 KV only
    (128 fp8 columns stay on the multi-wave kernel), and fp8 scores go through K converted to bf16."""
    lens = []
    for base in (64, 96, 160, 1024):
        for d in (-1, 0, 1):
            lens += [base + d, base + Q - 1 + d]
    lens += [Q, 31 + Q, 2048, 700]
    b = W.make_batch("staged-d64", 9700 + Q + Hq, lens, Hq, Hkv, 64, 16, kv, q_len=Q)
    rescale_queries(b, np.random.default_rng(9700 + Q), -6, 2)
    print(f"[case] head_dim 64 Q={Q} Hq={Hq} Hkv={Hkv} kv={kv} P={P}", flush=True)
    got, dev = run_gpu(pa, b, num_partitions=P)
    cols = Q * (Hq // Hkv)
    if cols > 32:
        staged = cols <= 64 or kv == W.KV_BF16
        assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == ("mfma-staged" if staged else "mfma-wide")
    want = oracle.decode_batch(b)["out"]
    err = assert_parity(flat(got), flat(want), kv, "head_dim 64")
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} {pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_negative_softmax_scale(pa, oracle, kv):
    """A negative scale turns the search for the largest exponent into one for the smallest raw score."""
    b = W.make_batch("staged-negative-scale", 9400, [100, 257, 40, 16, 512], 8, 1, 128, 16, kv, q_len=8)
    b.scale = np.float32(-b.scale)
    got, dev = run_gpu(pa, b)
    assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == "mfma-staged"
    want = oracle.decode_batch(b)["out"]
    assert_parity(flat(got), flat(want), kv, "negative scale")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(16, 4, 1), (4, 8, 1)])
def test_query_rows_at_the_ends_of_the_bf16_range(pa, oracle, kv, Q, Hq, Hkv):
    """Rows of magnitude 2^-118 (all scores vanish: the output is the mean of the visible values) and
    2^8 (scores of a few thousand: one token takes nearly all the weight) beside ordinary ones: the
    per-row power of two of the fp8 split stays finite at the low end, and the exponents keep their
    accuracy at the upper end of what the 8-bit paths are specified for."""
    b = W.make_batch("staged-range-ends", 9500 + Q, [200, 77, 512, 33 + Q], Hq, Hkv, 128, 16, kv, q_len=Q)
    q = W.bf16_bits_to_f32(b.q).astype(np.float32)
    rows = q.reshape(-1, q.shape[-1])
    rows[0::5] *= np.float32(2.0 ** -118)
    rows[1::5] *= np.float32(2.0 ** 8)
    b.q = W.f32_to_bf16_bits(q).reshape(b.q.shape)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all()
    want = oracle.decode_batch(b)["out"]
    assert_parity(flat(got), flat(want), kv, "query rows at the ends of the bf16 range")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 1), (16, 4, 1), (16, 8, 1)])
def test_verification_call_in_a_hip_graph(pa, oracle, kv, Q, Hq, Hkv):
    """A multi-token call captured once and replayed with queries and lengths updated in place: every
    replay equals the eager call on the same state bit for bit and the oracle within tolerance, with
    host work and synchronisations between the replays."""
    import torch

    rng = np.random.default_rng(9600 + Q + Hq)
    full = np.array([700, 40 + Q, 1030, 333, 96 + Q], dtype=np.int32)
    b = W.make_batch("staged-graph", 9600 + Q, full.tolist(), Hq, Hkv, 128, 16, kv, poison=False, q_len=Q)
    dev = pa.DeviceBatch(b, max_context_len=int(full.max()))
    out_eager = torch.empty_like(dev.out)

    def enqueue(out):
        pa.pa_decode(dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype, out,
                     dev.k_scale, dev.v_scale, shape=dev.shape, workspace=dev.workspace)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(dev.out)  # warm-up outside capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(dev.out)
    torch.cuda.synchronize()

    for i in range(4):
        b.context_lens = np.maximum(full - rng.integers(0, 40, size=full.shape), Q).astype(np.int32)
        q_new = W.f32_to_bf16_bits(rng.standard_normal(b.q.shape).astype(np.float32)).reshape(b.q.shape)
        b.q = q_new
        dev.q.copy_(torch.from_numpy(q_new.view(np.int16)))
        dev.context_lens.copy_(torch.from_numpy(b.context_lens))
        dev.out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = dev.out.cpu().numpy()
        want = oracle.decode_batch(b)["out"]
        assert_parity(flat(got), flat(want), kv, f"graph replay {i}")
        enqueue(out_eager)
        torch.cuda.synchronize()
        assert np.array_equal(out_eager.cpu().numpy(), got)
        _ = (torch.randn(1 << 16, device="cuda") * 2).sum().item()  # unrelated eager work between replays
