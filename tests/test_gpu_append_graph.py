"""GPU tests of the KV append entry point and of append -> decode captured in a HIP graph."""
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


def bf16(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def new_rows(rng, B, Hkv, D, scale=1.0, edge=False):
    x = rng.standard_normal((B, Hkv, D)).astype(np.float32) * np.float32(scale)
    if edge:  # rounding ties, subnormals, zeros of both signs, saturation
        specials = np.array([0.0, -0.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, 1.1875, 448.0, 464.0, 1e4, -1e4,
                             -2.0 ** -10, 0.0009765625, 240.0, 248.0], dtype=np.float32)
        x.reshape(-1)[:specials.size] = specials
    return bf16(x)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 128), (4, 2, 64), (32, 8, 128)])
def test_append_is_byte_exact(pa, oracle, kv, Hq, Hkv, D):
    import torch

    rng = np.random.default_rng(7 + D + Hq)
    lens = [17, 0, 32, 1, 100, 16, 33, 0, 255]
    b = W.make_batch("append", 70 + Hq, lens, Hq, Hkv, D, 16, kv, poison=False)
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0  # so that the special values below hit the ties exactly
        b.v_scale[:] = np.linspace(0.01, 0.05, Hkv, dtype=np.float32)
    k_new = new_rows(rng, len(lens), Hkv, D, edge=True)
    v_new = new_rows(rng, len(lens), Hkv, D, scale=0.5)
    dev = pa.DeviceBatch(b)
    dk = torch.from_numpy(k_new.view(np.int16)).cuda()
    dv = torch.from_numpy(v_new.view(np.int16)).cuda()
    pa.pa_kv_append(dk, dv, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.kv_dtype, dev.k_scale,
                    dev.v_scale, shape=dev.shape)
    torch.cuda.synchronize()
    oracle.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.context_lens, kv, b.k_scale, b.v_scale)
    view = np.int16 if kv == W.KV_BF16 else np.uint8
    assert np.array_equal(dev.k_cache.cpu().numpy(), b.k_cache.view(view))
    assert np.array_equal(dev.v_cache.cpu().numpy(), b.v_cache.view(view))
    # and the decode step over the appended cache agrees with the oracle over its appended cache
    got = dev.decode().cpu().numpy()
    assert_parity(got, oracle.decode_batch(b)["out"], kv, "decode after append")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 2), (16, 8, 2), (16, 8, 1)])
def test_window_append_is_byte_exact_and_feeds_verification(pa, oracle, kv, Q, Hq, Hkv):
    """Q proposed tokens per sequence are appended in one call (byte-exact against the oracle, contexts
    shorter than the window included) and the verification call then attends over them."""
    import torch

    rng = np.random.default_rng(17 + Q + Hkv)
    lens = [17, 0, 32, 3, 100, 16, 33, 255, Q, Q - 1, Q + 1]
    b = W.make_batch("append-window", 75 + Q, lens, Hq, Hkv, 128, 16, kv, poison=False, q_len=Q)
    k_new = np.stack([new_rows(rng, len(lens), Hkv, 128, edge=(i == 0)) for i in range(Q)], axis=1)
    v_new = np.stack([new_rows(rng, len(lens), Hkv, 128, scale=0.5) for i in range(Q)], axis=1)
    dev = pa.DeviceBatch(b)
    dk = torch.from_numpy(np.ascontiguousarray(k_new).view(np.int16)).cuda()
    dv = torch.from_numpy(np.ascontiguousarray(v_new).view(np.int16)).cuda()
    pa.pa_kv_append(dk, dv, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.kv_dtype, dev.k_scale,
                    dev.v_scale, shape=dev.shape)
    torch.cuda.synchronize()
    oracle.kv_append(np.ascontiguousarray(k_new), np.ascontiguousarray(v_new), b.k_cache, b.v_cache, b.block_tables,
                     b.context_lens, kv, b.k_scale, b.v_scale)
    view = np.int16 if kv == W.KV_BF16 else np.uint8
    assert np.array_equal(dev.k_cache.cpu().numpy(), b.k_cache.view(view))
    assert np.array_equal(dev.v_cache.cpu().numpy(), b.v_cache.view(view))
    got = dev.decode().cpu().numpy()
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert_parity(flat(got), flat(want), kv, "verification after the window append")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_append_and_decode_in_a_hip_graph(pa, oracle, kv):
    """Five decode steps: append the new token's K/V, attend over the grown context.  The two
    library calls are captured once into a HIP graph and replayed with the inputs updated in
    place; every replay is checked against the eager calls and against the oracle, with host
    work and synchronisations in between."""
    import torch

    rng = np.random.default_rng(11)
    B, Hq, Hkv, D = 6, 16, 4, 128
    lens0 = np.array([30, 1, 500, 15, 16, 700], dtype=np.int32)
    steps = 5
    final = lens0 + steps
    b = W.make_batch("graph", 80, final.tolist(), Hq, Hkv, D, 16, kv, poison=False)  # blocks for the final lengths
    b.context_lens = lens0.copy()
    dev = pa.DeviceBatch(b, max_context_len=int(final.max()))
    dk = torch.zeros((B, Hkv, D), dtype=torch.int16, device="cuda")
    dv = torch.zeros((B, Hkv, D), dtype=torch.int16, device="cuda")
    out_eager = torch.empty_like(dev.out)

    def enqueue(out):
        pa.pa_kv_append(dk, dv, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.kv_dtype,
                        dev.k_scale, dev.v_scale, shape=dev.shape)
        pa.pa_decode(dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype, out,
                     dev.k_scale, dev.v_scale, shape=dev.shape, workspace=dev.workspace)

    # capture on a side stream (default priority), as torch requires
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(dev.out)  # warm-up outside capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(dev.out)
    torch.cuda.synchronize()
    # the warm-up and the capture-time call must not count as steps: restore the caches
    view = np.int16 if kv == W.KV_BF16 else np.uint8
    dev.k_cache.copy_(torch.from_numpy(b.k_cache.view(view)))
    dev.v_cache.copy_(torch.from_numpy(b.v_cache.view(view)))

    for i in range(steps):
        k_new = new_rows(rng, B, Hkv, D)
        v_new = new_rows(rng, B, Hkv, D)
        q_new = new_rows(rng, B, Hq, D)
        b.context_lens = (lens0 + i + 1).astype(np.int32)
        b.q = q_new
        dk.copy_(torch.from_numpy(k_new.view(np.int16)))
        dv.copy_(torch.from_numpy(v_new.view(np.int16)))
        dev.q.copy_(torch.from_numpy(q_new.view(np.int16)))
        dev.context_lens.copy_(torch.from_numpy(b.context_lens))
        dev.out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = dev.out.cpu().numpy()
        oracle.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.context_lens, kv, b.k_scale, b.v_scale)
        want = oracle.decode_batch(b)["out"]
        assert_parity(got, want, kv, f"graph replay {i}")
        assert np.array_equal(dev.k_cache.cpu().numpy(), b.k_cache.view(view))
        # eager calls on the same state (the append rewrites the same slot with the same bytes)
        enqueue(out_eager)
        torch.cuda.synchronize()
        assert np.array_equal(out_eager.cpu().numpy(), got)
        _ = (torch.randn(1 << 16, device="cuda") * 2).sum().item()  # unrelated eager work between replays
