"""GPU parity of sliding-window calls (shape.window > 0, plain decode and multi-token): the HIP path
through the C ABI against the float64 CPU oracle.  The generated batches treat everything before
the earliest window of a sequence as evicted: table entries -1, NaN patterns in the slots."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity

pytestmark = pytest.mark.gpu

EDGE_LENS = [1, 2, 3, 15, 16, 17, 0, 31, 32, 33, 47, 48, 49, 300, 257, 512, 5, 64, 65, 1000]


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


def check(pa, oracle, batch, what, **kw):
    print(f"[case] {what} seed={batch.seed} B={batch.batch} Q={batch.q_len} W={batch.window} Hq={batch.num_q_heads} "
          f"Hkv={batch.num_kv_heads} kv={batch.kv_dtype} tokens={batch.total_tokens} {kw}", flush=True)
    got, dev = run_gpu(pa, batch, **kw)
    assert got.shape == batch.q.shape
    want = oracle.decode_batch(batch)["out"]
    err = assert_parity(flat(got), flat(want), batch.kv_dtype, what)
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)} "
          f"{pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)
    return got, want


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 8, 2), (1, 16, 1), (4, 8, 2), (16, 4, 1), (16, 8, 1), (3, 5, 1), (1, 2, 2),
                                      (1, 4, 2), (2, 1, 1), (8, 4, 1), (5, 5, 1), (16, 2, 1), (1, 32, 1), (2, 48, 2), (16, 10, 1)])
@pytest.mark.parametrize("window", [1, 5, 16, 31, 32, 33, 100, 5000])
def test_sliding_window_shapes(pa, oracle, kv, Q, Hq, Hkv, window):
    b = W.make_batch("sliding", 600 + 13 * Q + Hq + window, EDGE_LENS, Hq, Hkv, 128, 16, kv, q_len=Q, window=window)
    check(pa, oracle, b, "sliding-window")
    check(pa, oracle, b, "sliding-window P=5", num_partitions=5)


@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 8, 2), (8, 8, 2)])
@pytest.mark.parametrize("P", [1, 2, 7, 64, 1000])
def test_sliding_window_partition_sweep(pa, oracle, Q, Hq, Hkv, P):
    lens = [33, 34, 47, 48, 49, 0, 255, 256, 257, 1023, 1025, 2000, 31, 32, 64, 65, 66]
    b = W.make_batch("sliding-splits", 660, lens, Hq, Hkv, 128, 16, W.KV_BF16, q_len=Q, window=300)
    got, _ = check(pa, oracle, b, f"sliding-sweep P={P}", num_partitions=P)
    ref, _ = run_gpu(pa, b, num_partitions=1)
    assert_parity(flat(got), flat(ref), b.kv_dtype, "against the unsplit run")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 8, 2), (4, 8, 2), (16, 4, 1), (8, 4, 1), (6, 5, 1)])
@pytest.mark.parametrize("window", [1, 15, 16, 17, 32, 40])
def test_sliding_window_edges_are_exact(pa, kv, Q, Hq, Hkv, window):
    """For query token i (position pos = L - Q + i) the token just before its window, pos - W, carries
    the strongest key (32 e_i), the first token inside, pos - W + 1, the second strongest (16 e_i),
    all other keys are zero along e_i, and the query is 128 e_i: the right answer is exactly the
    value row of pos - W + 1 (base-16 digits of the position); a window one token too wide returns
    the row of pos - W, one too narrow an average.  Nothing is evicted here (the probe writes a key
    outside the window)."""
    lens = [60, 64, 65, 95, 96, 97, 128, 700]
    b = W.make_batch("sliding-onehot", 670, lens, Hq, Hkv, 128, 16, kv, q_len=Q, window=window, poison=False)
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    q4 = b.q if b.q.ndim == 4 else b.q[:, None]
    q4[:] = 0
    b.k_cache[:] = 0
    b.v_cache[:] = 0
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
        b.v_scale[:] = 1.0
    for s, L in enumerate(lens):
        for t in range(L):
            phys, slot = b.block_tables[s, t // 16], t % 16
            for d in range(4):
                b.v_cache[phys, :, slot, 64 + d] = enc((t >> (4 * d)) & 15)
        for i in range(Q):
            pos = L - Q + i
            outside, inside = pos - window, pos - window + 1
            b.k_cache[b.block_tables[s, outside // 16], :, outside % 16, i] = enc(32)
            b.k_cache[b.block_tables[s, inside // 16], :, inside % 16, i] = enc(16)
            q4[s, i, :, i] = W.f32_to_bf16_bits(np.float32(128))
    for P in (0, 1, 6):
        got, _ = run_gpu(pa, b, num_partitions=P)
        got = got if got.ndim == 4 else got[:, None]
        for s, L in enumerate(lens):
            for i in range(Q):
                t = L - Q + i - window + 1
                want = np.array([(t >> (4 * d)) & 15 for d in range(4)], dtype=np.float32)
                digits = got[s, i, :, 64:68]
                assert np.array_equal(digits, np.broadcast_to(want, digits.shape)), (P, s, L, i, digits[0])


@pytest.mark.parametrize("Q,window,P", [(1, 100, 0), (1, 20, 5), (8, 33, 0), (16, 300, 11), (1, 10 ** 6, 0)])
def test_sliding_window_trace_touches_only_live_blocks(pa, oracle, Q, window, P):
    """The instrumented kernels report every block they load: exactly the blocks that hold a token some
    query can see, with the ids of the table and the partitions of the plan; evicted entries (-1)
    are never read."""
    import torch

    b = W.make_config(4, length_scale=1 / 8, q_len=Q, window=window)
    dev = pa.DeviceBatch(b, num_partitions=P)
    Pr = pa.pa_num_partitions(dev.shape, dev.kv_dtype)
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), -7, dtype=torch.int32, device="cuda")
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    visited = visited.cpu().numpy()
    reach = window + Q - 1
    T, owner = oracle.block_partition(b.context_lens, b.max_blocks_per_seq, 16, Pr, reach=reach)
    Th, owner_host = pa.pa_split_plan(dev.shape, dev.kv_dtype, b.context_lens)
    assert Th == T and np.array_equal(owner_host, owner)
    for s in range(b.batch):
        first, ids = oracle.window_blocks(b.block_tables, b.context_lens, 16, s, reach)
        n = len(ids)
        for g in range(b.num_kv_heads):
            assert np.array_equal(visited[s, g, first:first + n, 0], ids)
            assert np.array_equal(visited[s, g, first:first + n, 1], ids)
            assert np.array_equal(visited[s, g, first:first + n, 2], owner[s, first:first + n])
            assert np.all(visited[s, g, :first] == -7) and np.all(visited[s, g, first + n:] == -7)
    want = oracle.decode_batch(b)["out"]
    assert_parity(flat(dev.out.cpu().numpy()), flat(want), b.kv_dtype, "sliding trace-run")


@pytest.mark.parametrize("config,Q,window", [(2, 1, 1024), (2, 16, 512), (5, 1, 4096), (3, 1, 8192)])
def test_sliding_window_full_size_sampled_rows(pa, oracle, config, Q, window):
    b = W.make_config(config, q_len=Q, window=window)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all()
    got = got if got.ndim == 4 else got[:, None]
    rng = np.random.default_rng(config * 100 + Q)
    rows = [(s, i, int(rng.integers(0, b.num_q_heads))) for s in range(b.batch) for i in {0, Q - 1}]
    view = type("V", (), dict(vars(b), q=b.q if b.q.ndim == 4 else b.q[:, None]))()
    want = oracle.decode_batch(view, rows=rows)["out"]
    sel = np.stack([got[s, i, h] for s, i, h in rows])
    err = assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, f"config{config} sliding Q={Q} W={window}")
    print(f"        {len(rows)} sampled rows max_abs={err[0]:.3e} worst row rel_l2={err[1]:.3e} "
          f"P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)}", flush=True)


@pytest.mark.parametrize("B", [65, 130])
@pytest.mark.parametrize("Q", [1, 8])
def test_sliding_window_many_short_sequences(pa, oracle, B, Q):
    rng = np.random.default_rng(B + Q)
    lens = rng.integers(1, 200, size=B)
    lens[rng.random(B) < 0.2] = 0
    lens[0] = 0
    b = W.make_batch("sliding-many", 680 + B, lens.tolist(), 8, 2, 128, 16, W.KV_BF16, max_blocks_per_seq=13, q_len=Q,
                     window=40)
    for P in (0, 1, 7, 50):
        check(pa, oracle, b, f"sliding many-sequences P={P}", num_partitions=P)
