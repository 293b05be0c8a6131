"""GPU parity of multi-token verification calls (q_len > 1, causal inside the window of new tokens):
the HIP path through the C ABI against the float64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity

pytestmark = pytest.mark.gpu

EDGE_LENS = [1, 2, 3, 15, 16, 17, 0, 31, 32, 33, 47, 48, 49, 300, 257, 512, 5, 64, 65]


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
    """[B, Q, Hq, D] -> [B, Q*Hq, D] so the per-sequence error gates apply unchanged."""
    return a.reshape(a.shape[0], -1, a.shape[-1])


def check(pa, oracle, batch, what, **kw):
    print(f"[case] {what} seed={batch.seed} B={batch.batch} Q={batch.q_len} Hq={batch.num_q_heads} "
          f"Hkv={batch.num_kv_heads} kv={batch.kv_dtype} tokens={batch.total_tokens} {kw}", flush=True)
    got, dev = run_gpu(pa, batch, **kw)
    assert got.shape == batch.q.shape
    want = oracle.decode_batch(batch)["out"]
    err = assert_parity(flat(got), flat(want), batch.kv_dtype, what)
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)} "
          f"{pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)
    return got, want


# (Q, Hq, Hkv): columns per KV head Q*G = 2 .. 128: up to 32 one wave (padded to 4 / 8 / 16 / 32), above that a
# workgroup of 4 / 8 waves with 16 columns each
WINDOW_SHAPES = [(4, 4, 4), (2, 8, 2), (2, 4, 1), (3, 6, 2), (2, 16, 2), (16, 2, 2), (7, 3, 1), (2, 16, 1),
                 (16, 4, 2), (5, 16, 2), (16, 4, 1), (4, 16, 1), (9, 7, 1), (16, 8, 1), (16, 16, 2), (8, 16, 1),
                 (13, 9, 1), (5, 13, 1), (2, 1, 1), (3, 2, 2), (2, 4, 2), (5, 4, 1), (2, 9, 1), (3, 8, 1), (16, 2, 1),
                 (6, 5, 1), (3, 11, 1), (16, 4, 2), (4, 32, 1), (2, 40, 1), (3, 17, 1), (32, 4, 1), (128, 1, 1), (64, 2, 1), (24, 5, 1), (17, 2, 2), (40, 3, 1), (16, 16, 1), (32, 5, 1), (128, 4, 1),
                 (16, 32, 2), (9, 16, 1), (3, 43, 1)]


@pytest.mark.parametrize("Q,Hq,Hkv", WINDOW_SHAPES)
@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_window_shapes(pa, oracle, Q, Hq, Hkv, kv):
    b = W.make_batch("window", 300 + 17 * Q + Hq, EDGE_LENS, Hq, Hkv, 128, 16, kv, num_blocks=160,
                     max_blocks_per_seq=40, q_len=Q)
    got, _ = check(pa, oracle, b, "window-shapes")
    # contexts shorter than the window: the first Q - L query tokens see nothing
    for s, L in enumerate(EDGE_LENS):
        if L < Q:
            assert np.all(got[s, :Q - L] == 0), (s, L)
    check(pa, oracle, b, "window-shapes P=5", num_partitions=5)
    check(pa, oracle, b, "window-shapes P=1", num_partitions=1)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 2), (16, 8, 2), (6, 10, 2), (16, 16, 2), (5, 8, 2), (8, 8, 2), (20, 16, 2)])
@pytest.mark.parametrize("P", [2, 3, 7, 64, 1000])
def test_window_partition_sweep(pa, oracle, kv, Q, Hq, Hkv, P):
    """Boundaries anywhere, including ones that leave a partition only the last tile of a sequence,
    of which the early query tokens of the window see nothing."""
    lens = [33, 34, 47, 48, 49, 0, 255, 256, 257, 1023, 1025, 2000, 31, 32, 64, 65, 66]
    b = W.make_batch("window-splits", 360, lens, Hq, Hkv, 128, 16, kv, q_len=Q)
    got, _ = check(pa, oracle, b, f"window-sweep P={P}", num_partitions=P)
    ref, _ = run_gpu(pa, b, num_partitions=1)
    assert_parity(flat(got), flat(ref), kv, "against the unsplit run")


def test_window_one_sequence_cut_by_every_partition(pa, oracle):
    b = W.make_batch("window-long1", 361, [5000], 8, 2, 128, 16, W.KV_BF16, q_len=16)
    for P in (2, 9, 100, 157):
        check(pa, oracle, b, f"window-single-sequence P={P}", num_partitions=P)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 2), (16, 4, 1), (16, 1, 1), (6, 10, 2), (16, 8, 1), (8, 4, 1), (5, 8, 2), (16, 12, 1)])
@pytest.mark.parametrize("P", [0, 1, 6])
def test_window_mask_is_exact(pa, kv, Q, Hq, Hkv, P):
    """Window token j (logical position L - Q + j) has the key 16 (j + 1) e_0, every other token the
    zero key, and every query is 128 e_0: among the tokens query i may see, window token i outweighs
    all others by a factor that underflows them, so query i must return exactly the value row of
    position L - Q + i, which spells that position in base-16 digits.  A mask that is off by one in
    either direction returns a neighbour's digits."""
    lens = [16, 17, 31, 32, 33, 48, 49, 700, 257, 40]
    b = W.make_batch("window-onehot", 370, lens, Hq, Hkv, 128, 16, kv, q_len=Q)
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    b.q[:] = 0
    b.q[..., 0] = W.f32_to_bf16_bits(np.float32(128))  # one window step = 181 nats: the rest underflows to 0
    b.k_cache[:] = 0
    b.v_cache[:] = 0
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
        b.v_scale[:] = 1.0
    for s, L in enumerate(lens):
        for t in range(L):
            phys, slot = b.block_tables[s, t // 16], t % 16
            for d in range(4):
                b.v_cache[phys, :, slot, d] = enc((t >> (4 * d)) & 15)
            b.v_cache[phys, :, slot, 4] = enc(s % 16)
            j = t - (L - Q)
            if j >= 0:
                b.k_cache[phys, :, slot, 0] = enc(16 * (j + 1))
    got, _ = run_gpu(pa, b, num_partitions=P)
    for s, L in enumerate(lens):
        for i in range(Q):
            t = L - Q + i
            want = np.array([(t >> (4 * d)) & 15 for d in range(4)] + [s % 16], dtype=np.float32)
            digits = got[s, i, :, :5]
            assert np.array_equal(digits, np.broadcast_to(want, digits.shape)), (s, L, i, digits[0])


@pytest.mark.parametrize("config,kwargs,Q", [
    (2, dict(length_scale=0.25), 4), (2, dict(length_scale=0.25), 16), (4, dict(length_scale=1 / 8), 8),
    (5, dict(length_scale=1 / 16, batch_limit=16), 8), (5, dict(length_scale=1 / 16, batch_limit=16), 16),
    (4, dict(length_scale=1 / 8), 16),
])
def test_window_on_reduced_configs(pa, oracle, config, kwargs, Q):
    b = W.make_config(config, q_len=Q, **kwargs)
    check(pa, oracle, b, f"config{config}-reduced window Q={Q}")


@pytest.mark.parametrize("config,Q", [(2, 4), (2, 5), (2, 8), (2, 16), (5, 4), (5, 8), (5, 16), (4, 16)])
def test_window_full_size_sampled_rows(pa, oracle, config, Q):
    """Full-size batches in the default launch configuration; the oracle computes a seeded sample of
    output rows one by one (every sequence, both ends of the window and a random interior token)."""
    b = W.make_config(config, q_len=Q)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(config * 100 + Q)
    rows = []
    for s in range(b.batch):
        for i in (0, Q - 1, int(rng.integers(0, Q))):
            rows.append((s, i, int(rng.integers(0, b.num_q_heads))))
    want = oracle.decode_batch(b, rows=rows)["out"]
    sel = np.stack([got[s, i, h] for s, i, h in rows])
    err = assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, f"config{config} window Q={Q}")
    print(f"        {len(rows)} sampled rows max_abs={err[0]:.3e} worst row rel_l2={err[1]:.3e} "
          f"P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)}", flush=True)


def test_window_trace_matches_block_tables_and_split_plan(pa, oracle):
    import torch

    b = W.make_config(4, length_scale=1 / 8, q_len=8)
    dev = pa.DeviceBatch(b, num_partitions=37)
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), -7, dtype=torch.int32, device="cuda")
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    visited = visited.cpu().numpy()
    T, owner = oracle.block_partition(b.context_lens, b.max_blocks_per_seq, 16, 37)
    for s in range(b.batch):
        ids = oracle.visited_blocks(b.block_tables, b.context_lens, 16, s)
        n = len(ids)
        for g in range(b.num_kv_heads):
            assert np.array_equal(visited[s, g, :n, 0], ids) and np.array_equal(visited[s, g, :n, 1], ids)
            assert np.array_equal(visited[s, g, :n, 2], owner[s, :n])
            assert np.all(visited[s, g, n:] == -7)
    want = oracle.decode_batch(b)["out"]
    assert_parity(flat(dev.out.cpu().numpy()), flat(want), b.kv_dtype, "window trace-run")


def test_window_repeated_calls_share_one_workspace(pa, oracle):
    b = W.make_config(2, length_scale=0.25, q_len=16)
    dev = pa.DeviceBatch(b)
    want = oracle.decode_batch(b)["out"]
    first = None
    for i in range(3):
        dev.out.fill_(float("nan"))
        dev.workspace.fill_(float("nan"))
        got = dev.decode().cpu().numpy()
        assert_parity(flat(got), flat(want), b.kv_dtype, f"call {i}")
        first = got if first is None else first
        assert np.array_equal(got, first)


@pytest.mark.parametrize("B", [65, 130])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 2), (16, 8, 2)])
def test_window_many_short_sequences(pa, oracle, B, Q, Hq, Hkv):
    """More sequences than lanes (the length scan runs in 64-sequence chunks), empty ones sprinkled in."""
    rng = np.random.default_rng(B + Q)
    lens = rng.integers(1, 120, size=B)
    lens[rng.random(B) < 0.2] = 0
    lens[0] = 0
    b = W.make_batch("window-many", 380 + B, lens.tolist(), Hq, Hkv, 128, 16, W.KV_BF16, max_blocks_per_seq=8, q_len=Q)
    for P in (0, 1, 7, 50):
        check(pa, oracle, b, f"window many-sequences P={P}", num_partitions=P)
