"""GPU parity at head_dim 64 for every kind of call (plain decode, multi-token verification, shared
prefix, sliding window, bf16 output, instrumented run): rows of the cache are half as long as at
head_dim 128, which changes the tile geometry in LDS, the swizzle and how the loads of a tile divide
over the waves of a workgroup.  The HIP path through the C ABI against the float64 CPU oracle."""
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
          f"Hkv={batch.num_kv_heads} D={batch.head_dim} kv={batch.kv_dtype} prefix={batch.shared_prefix_blocks} "
          f"tokens={batch.total_tokens} {kw}", flush=True)
    got, dev = run_gpu(pa, batch, **kw)
    assert got.shape == batch.q.shape
    want = oracle.decode_batch(batch)["out"]
    err = assert_parity(flat(got), flat(want), batch.kv_dtype, what)
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)} "
          f"{pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)
    return got, want


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (2, 1), (3, 1), (8, 2), (5, 1), (12, 4), (16, 2), (16, 1), (9, 1)])
def test_decode_groups(pa, oracle, kv, Hq, Hkv):
    b = W.make_batch("d64", 900 + Hq, EDGE_LENS, Hq, Hkv, 64, 16, kv)
    check(pa, oracle, b, "head_dim 64 decode")
    for P in (1, 5, 1000):
        check(pa, oracle, b, f"head_dim 64 decode P={P}", num_partitions=P)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(2, 8, 2), (4, 4, 4), (16, 1, 1), (3, 6, 2), (2, 16, 2), (16, 2, 2), (16, 4, 2),
                                      (5, 16, 2), (16, 4, 1), (9, 7, 1), (16, 8, 1), (16, 16, 2), (13, 9, 1), (5, 4, 1),
                                      (2, 9, 1), (16, 2, 1), (6, 5, 1), (8, 8, 2), (16, 16, 1), (40, 8, 1)])
def test_verification_shapes(pa, oracle, kv, Q, Hq, Hkv):
    """2 .. 128 columns per KV head: one wave with one or two column tiles, and 4 and 8 waves per
    workgroup (with fp8 rows a tile is four loads, so only four of eight waves load)."""
    b = W.make_batch("d64-verify", 910 + 17 * Q + Hq, EDGE_LENS, Hq, Hkv, 64, 16, kv, q_len=Q)
    got, _ = check(pa, oracle, b, "head_dim 64 verify")
    for s, L in enumerate(EDGE_LENS):
        if L < Q:
            assert np.all(got[s, :Q - L] == 0), (s, L)
    check(pa, oracle, b, "head_dim 64 verify P=5", num_partitions=5)
    check(pa, oracle, b, "head_dim 64 verify P=1", num_partitions=1)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 8, 2), (4, 8, 2), (16, 8, 2), (16, 16, 2)])
@pytest.mark.parametrize("P", [2, 7, 64, 1000])
def test_partition_sweep(pa, oracle, kv, Q, Hq, Hkv, P):
    lens = [33, 34, 47, 48, 49, 0, 255, 256, 257, 1023, 1025, 2000, 31, 32, 64, 65, 66]
    b = W.make_batch("d64-splits", 920, lens, Hq, Hkv, 64, 16, kv, q_len=Q)
    got, _ = check(pa, oracle, b, f"head_dim 64 sweep P={P}", num_partitions=P)
    ref, _ = run_gpu(pa, b, num_partitions=1)
    assert_parity(flat(got), flat(ref), kv, "against the unsplit run")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 4, 1), (4, 8, 2), (16, 4, 1), (16, 8, 1), (8, 4, 1), (6, 5, 1)])
def test_every_dim_and_token_lands_in_its_place(pa, kv, Q, Hq, Hkv):
    """Query token i of a sequence sees, with all its weight, its own position (key 16 (i + 1) e_0
    against a query of 128 e_0: the others underflow); the value row of position t holds t's base-16
    digits in dims 4 d' .. 4 d' + 3 for every d' (all 64 dims, each with a digit that depends on d'),
    so a swapped piece, dim tile or token row of V shows as a wrong digit."""
    lens = [16, 17, 31, 32, 33, 48, 49, 700, 257, 40]
    b = W.make_batch("d64-onehot", 930, lens, Hq, Hkv, 64, 16, kv, q_len=Q)
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    q4 = b.q if b.q.ndim == 4 else b.q[:, None]
    q4[:] = 0
    q4[..., 0] = W.f32_to_bf16_bits(np.float32(128))
    b.k_cache[:] = 0
    b.v_cache[:] = 0
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
        b.v_scale[:] = 1.0

    def row_of(t):
        return np.array([((t + d // 4) >> (4 * (d % 4))) & 15 for d in range(64)], dtype=np.float32)

    for s, L in enumerate(lens):
        for t in range(L):
            phys, slot = b.block_tables[s, t // 16], t % 16
            r = row_of(t)
            for d in range(64):
                b.v_cache[phys, :, slot, d] = enc(r[d])
            j = t - (L - Q)
            if j >= 0:
                b.k_cache[phys, :, slot, 0] = enc(16 * (j + 1))
    for P in (0, 1, 6):
        got, _ = run_gpu(pa, b, num_partitions=P)
        got = got if got.ndim == 4 else got[:, None]
        for s, L in enumerate(lens):
            for i in range(Q):
                want = row_of(L - Q + i)
                assert np.array_equal(got[s, i], np.broadcast_to(want, got[s, i].shape)), (P, s, L, i)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_every_key_dim_counts(pa, oracle, kv):
    """Keys that differ in one dim only: a K piece read from the wrong place changes which token wins."""
    lens = [64] * 64
    b = W.make_batch("d64-keydims", 940, lens, 4, 1, 64, 16, kv)
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    b.q[:] = 0
    b.k_cache[:] = 0
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
    for s in range(64):  # sequence s asks along dim s; token t has its key along dim t
        b.q[s, :, s] = W.f32_to_bf16_bits(np.float32(128))
        for t in range(64):
            b.k_cache[b.block_tables[s, t // 16], :, t % 16, t] = enc(16)
    got, want = check(pa, oracle, b, "head_dim 64 key dims")
    # the winner's value row, exactly (the other 63 weights underflow)
    v = W.bf16_bits_to_f32(b.v_cache) if kv == W.KV_BF16 else None
    if v is not None:
        for s in range(64):
            row = v[b.block_tables[s, s // 16], 0, s % 16]
            assert np.array_equal(got[s, 0], row), s


def suffix_lens(prefix_blocks, B, seed):
    rng = np.random.default_rng(seed)
    base = prefix_blocks * 16
    extra = [0, 1, 15, 16, 17, 31, 32, 33, 128, 129, 700, 40, 64, 5, 300, 2]
    lens = [base + extra[i % len(extra)] for i in range(B)]
    rng.shuffle(lens)
    return lens


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 1), (5, 1), (2, 2)])
@pytest.mark.parametrize("B,prefix_blocks", [(1, 8), (5, 3), (20, 64), (40, 10)])
def test_shared_prefix(pa, oracle, kv, Hq, Hkv, B, prefix_blocks):
    b = W.make_batch("d64-prefix", 950 + 7 * B + Hq, suffix_lens(prefix_blocks, B, B), Hq, Hkv, 64, 16, kv,
                     shared_prefix_blocks=prefix_blocks)
    got, _ = check(pa, oracle, b, "head_dim 64 shared-prefix")
    check(pa, oracle, b, "head_dim 64 shared-prefix P=3", num_partitions=3)
    plain, _ = run_gpu(pa, b, shared_prefix_blocks=0)
    assert_parity(got, plain, b.kv_dtype, "against the call without a shared prefix")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv", [(1, 8, 2), (1, 16, 1), (4, 8, 2), (16, 4, 1), (16, 8, 1), (1, 2, 2), (8, 4, 1), (5, 5, 1)])
@pytest.mark.parametrize("window", [1, 16, 33, 100, 5000])
def test_sliding_window(pa, oracle, kv, Q, Hq, Hkv, window):
    b = W.make_batch("d64-sliding", 960 + 13 * Q + Hq + window, EDGE_LENS, Hq, Hkv, 64, 16, kv, q_len=Q, window=window)
    check(pa, oracle, b, "head_dim 64 sliding-window")
    check(pa, oracle, b, "head_dim 64 sliding-window P=5", num_partitions=5)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q", [1, 8])
def test_bf16_output(pa, oracle, kv, Q):
    b = W.make_batch("d64-obf16", 970 + Q, EDGE_LENS, 8, 2, 64, 16, kv, q_len=Q)
    f32, _ = run_gpu(pa, b)
    bits, _ = run_gpu(pa, b, out_dtype=pa.PA_OUT_BF16)
    assert bits.dtype == np.int16 and bits.shape == f32.shape
    assert np.array_equal(bits.view(np.uint16), W.f32_to_bf16_bits(f32))  # the same numbers, rounded once
    got = W.bf16_bits_to_f32(bits.view(np.uint16))
    want = oracle.decode_batch(b)["out"]
    assert np.all(np.abs(got.astype(np.float64) - want) <= np.abs(want) / 256 + (1e-2 if kv == W.KV_BF16 else 5e-2))


@pytest.mark.parametrize("Q,P", [(1, 37), (8, 11), (16, 0)])
def test_trace_matches_block_tables_and_split_plan(pa, oracle, Q, P):
    import torch

    rng = np.random.default_rng(Q)
    lens = rng.integers(0, 900, size=24).tolist()
    b = W.make_batch("d64-trace", 980 + Q, lens, 8, 2, 64, 16, W.KV_FP8_E4M3, q_len=Q)
    dev = pa.DeviceBatch(b, num_partitions=P)
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), -7, dtype=torch.int32, device="cuda")
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    visited = visited.cpu().numpy()
    nparts = pa.pa_num_partitions(dev.shape, dev.kv_dtype)
    T, owner = oracle.block_partition(b.context_lens, b.max_blocks_per_seq, 16, nparts)
    for s in range(b.batch):
        ids = oracle.visited_blocks(b.block_tables, b.context_lens, 16, s)
        n = len(ids)
        for g in range(b.num_kv_heads):
            assert np.array_equal(visited[s, g, :n, 0], ids) and np.array_equal(visited[s, g, :n, 1], ids)
            assert np.array_equal(visited[s, g, :n, 2], owner[s, :n])
            assert np.all(visited[s, g, n:] == -7)
    want = oracle.decode_batch(b)["out"]
    assert_parity(flat(dev.out.cpu().numpy()), flat(want), b.kv_dtype, "head_dim 64 trace-run")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q", [1, 16])
def test_serving_sized_batch_sampled_rows(pa, oracle, kv, Q):
    """64 sequences of 1k-8k tokens, 32 query / 8 KV heads of 64 dims, default launch configuration;
    the oracle computes a seeded sample of rows."""
    lens = (W.config_context_lens(2, 1002) * 2).tolist()
    b = W.make_batch("d64-serving", 990, lens, 32, 8, 64, 16, kv, 0.5, q_len=Q)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all()
    got = got if got.ndim == 4 else got[:, None]
    rng = np.random.default_rng(Q)
    rows = [(s, int(rng.integers(0, Q)), int(rng.integers(0, 32))) for s in range(b.batch)]
    if Q == 1:
        want = oracle.decode_batch(b, rows=[(s, h) for s, _, h in rows])["out"]
    else:
        want = oracle.decode_batch(b, rows=rows)["out"]
    sel = np.stack([got[s, i, h] for s, i, h in rows])
    err = assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, f"head_dim 64 serving Q={Q}")
    print(f"        {len(rows)} sampled rows max_abs={err[0]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)}", flush=True)
