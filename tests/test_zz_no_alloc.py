"""pa_decode_static, the entry point that allocates nothing (its partials live in a static device
array inside the library), against pa_decode on the same inputs: bit-identical output, on calls in
a row that share the array, a smaller call after a larger one included; and against the oracle."""
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


def both(pa, batch, **kw):
    """(pa_decode_static output, pa_decode output) for the same device batch."""
    import torch

    dev = pa.DeviceBatch(batch, **kw)
    dev.out.fill_(float("nan"))
    pa.pa_decode_static(*dev.args(), shape=dev.shape)
    torch.cuda.synchronize()
    got = dev.out.cpu().numpy().copy()
    dev.out.fill_(float("nan"))
    dev.decode()
    torch.cuda.synchronize()
    return got, dev.out.cpu().numpy(), dev


def test_static_scratch_calls_in_a_row_match_the_workspace_calls(pa, oracle):
    """A large call, then a smaller one (fewer sequences, fewer partitions: it finds the first
    call's partials in the array and must not read them), then other kinds of call, then the first
    one again."""
    cases = [
        ("config 2, quarter lengths", W.make_config(2, length_scale=0.25), {}),
        ("smaller: 5 sequences, P=3", W.make_batch("small", 91, [700, 33, 1, 300, 0], 8, 2, 128, 16, W.KV_BF16), dict(num_partitions=3)),
        ("fp8", W.make_config(5, length_scale=1 / 16, batch_limit=16), {}),
        ("16 query tokens", W.make_batch("verify", 92, [600, 90, 40], 8, 2, 128, 16, W.KV_BF16, q_len=16), {}),
        ("shared prefix", W.make_batch("prefix", 93, [400, 330, 321], 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=20), {}),
        ("sliding window", W.make_batch("window", 94, [700, 50], 8, 2, 128, 16, W.KV_BF16, window=100), {}),
        ("one partition: no scratch at all", W.make_config(1), dict(num_partitions=1)),
        ("config 2 again", W.make_config(2, length_scale=0.25), {}),
    ]
    for what, batch, kw in cases:
        print(f"[case] static scratch: {what}", flush=True)
        got, ref, dev = both(pa, batch, **kw)
        assert np.array_equal(got, ref), what
        want = oracle.decode_batch(batch)["out"]
        flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
        assert_parity(flat(got), flat(want), batch.kv_dtype, what)


def test_static_scratch_full_size_config(pa):
    """The 8B-shaped batch at full size, default plan (the launch configuration the benchmark times)."""
    b = W.make_config(2)
    got, ref, dev = both(pa, b)
    assert pa.pa_decode_workspace_size(dev.shape, dev.kv_dtype) <= pa.PA_STATIC_SCRATCH_BYTES
    assert np.isfinite(got).all() and np.array_equal(got, ref)


def test_static_scratch_refuses_what_does_not_fit(pa):
    b = W.make_batch("wide", 95, [64, 64], 64, 8, 128, 16, W.KV_BF16, q_len=16)
    dev = pa.DeviceBatch(b, num_partitions=400)
    assert pa.pa_decode_workspace_size(dev.shape, dev.kv_dtype) > pa.PA_STATIC_SCRATCH_BYTES
    with pytest.raises(pa.PaError) as e:
        pa.pa_decode_static(*dev.args(), shape=dev.shape)
    assert e.value.status == pa.PA_ERR_WORKSPACE_TOO_SMALL
    # the same rules as pa_decode for everything else
    small = pa.DeviceBatch(W.make_config(1))
    with pytest.raises(pa.PaError) as e:
        pa.pa_decode_static(None, *small.args()[1:], shape=small.shape)
    assert e.value.status == pa.PA_ERR_INVALID_ARG


def test_static_scratch_call_replayed_from_a_hip_graph(pa, oracle):
    """What the entry point is for: a caller under graph capture.  After one eager call on the
    device (which looks the array's address up), the call is captured once and replayed with q
    updated in place; every replay is checked against the oracle and against pa_decode run eagerly
    on the same inputs, with unrelated eager work and synchronisations between the replays."""
    import torch

    rng = np.random.default_rng(21)
    b = W.make_config(2, length_scale=0.25, poison=False)
    dev = pa.DeviceBatch(b)
    out_eager = torch.empty_like(dev.out)

    def enqueue():
        pa.pa_decode_static(*dev.args(), shape=dev.shape)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()  # warm-up outside capture: the first call on a device resolves the array's address
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for i in range(4):
        q_new = W.f32_to_bf16_bits((rng.standard_normal(b.q.shape) * 0.5).astype(np.float32))
        b.q = q_new
        dev.q.copy_(torch.from_numpy(q_new.view(np.int16)))
        dev.out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = dev.out.cpu().numpy().copy()
        want = oracle.decode_batch(b)["out"]
        assert_parity(got, want, b.kv_dtype, f"static scratch, graph replay {i}")
        pa.pa_decode(dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype,
                     out_eager, dev.k_scale, dev.v_scale, shape=dev.shape, workspace=dev.workspace)
        torch.cuda.synchronize()
        assert np.array_equal(out_eager.cpu().numpy(), got)
        _ = (torch.randn(1 << 16, device="cuda") * 2).sum().item()  # unrelated eager work between replays
