"""GPU parity: the HIP path (through the C ABI) against the float64 CPU oracle on the same
seeded inputs, plus bit-exact checks of the block-table walk and the split boundaries."""
import time

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


def check(pa, oracle, batch, what, **kw):
    print(f"[case] {what} seed={batch.seed} B={batch.batch} Hq={batch.num_q_heads} Hkv={batch.num_kv_heads} "
          f"D={batch.head_dim} kv={batch.kv_dtype} tokens={batch.total_tokens} {kw}", flush=True)
    got, dev = run_gpu(pa, batch, **kw)
    want = oracle.decode_batch(batch)["out"]
    err = assert_parity(got, want, batch.kv_dtype, what)
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)} "
          f"{pa.pa_kernel_variant(dev.shape, dev.kv_dtype)}", flush=True)
    return got, want


# ------------------------------------------------------------------ the five configs
@pytest.mark.parametrize("seed", [1001, 2001, 3001, None])
def test_config1_tiny(pa, oracle, seed):
    seed = int(time.time()) % 100000 + 10 if seed is None else seed
    check(pa, oracle, W.make_config(1, seed=seed), "config1")


@pytest.mark.parametrize("config,kwargs", [
    (2, dict(length_scale=0.25)),
    (3, dict(length_scale=1 / 32, batch_limit=4)),
    (4, dict(length_scale=1 / 8)),
    (5, dict(length_scale=1 / 16, batch_limit=16)),
])
@pytest.mark.parametrize("seed_base", [1000, 2000])
def test_configs_reduced_lengths(pa, oracle, config, kwargs, seed_base):
    b = W.make_config(config, seed=seed_base + config, **kwargs)
    check(pa, oracle, b, f"config{config}-reduced")


@pytest.mark.parametrize("config", [2, 3, 4, 5])
def test_configs_full_size(pa, oracle, config):
    """Full-size batches in the launch configuration the benchmark times (default plan,
    max_context_len = the batch maximum); the oracle covers every output row."""
    b = W.make_config(config)
    check(pa, oracle, b, f"config{config}-full")


# ------------------------------------------------------------------ shapes and edges
@pytest.mark.parametrize("Hq,Hkv,D", [(1, 1, 64), (1, 1, 128), (4, 4, 128), (2, 1, 64), (6, 2, 128), (8, 1, 128),
                                      (16, 2, 64), (5, 1, 128), (12, 4, 64), (16, 1, 128), (24, 2, 128), (4, 1, 128),
                                      (32, 1, 128), (64, 1, 64), (128, 1, 128), (64, 2, 128), (40, 1, 64), (17, 1, 128)])
@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_head_shapes(pa, oracle, Hq, Hkv, D, kv):
    b = W.make_batch("shapes", 50 + Hq + D, [1, 15, 16, 17, 300, 257, 512, 31, 32, 33], Hq, Hkv, D, 16, kv,
                     num_blocks=100, max_blocks_per_seq=40)
    check(pa, oracle, b, "head-shapes")
    check(pa, oracle, b, "head-shapes P=5", num_partitions=5)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("P", [1, 2, 3, 7, 64, 1000])
def test_forced_partition_sweep(pa, oracle, kv, P):
    """Any number of partitions gives the same answer: one (no split, no merge), a few (long
    sequences cut several times), more than there are tiles (empty partitions)."""
    lens = [1, 16, 47, 48, 49, 0, 255, 256, 257, 1023, 1025, 2000, 31, 32, 33, 64, 65]
    b = W.make_batch("splits", 60, lens, 8, 2, 128, 16, kv)
    got, want = check(pa, oracle, b, f"partition-sweep P={P}", num_partitions=P)
    ref, _ = run_gpu(pa, b, num_partitions=1)
    assert_parity(got, ref, kv, "against the unsplit run")  # partition counts agree with each other too


def test_one_sequence_cut_by_every_partition(pa, oracle):
    b = W.make_batch("long1", 61, [5000], 8, 2, 128, 16, W.KV_BF16)
    for P in (2, 9, 100, 157):
        check(pa, oracle, b, f"single-sequence P={P}", num_partitions=P)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 64), (8, 2, 128), (2, 2, 128), (16, 1, 128)])
@pytest.mark.parametrize("P", [16, 40, 300])
def test_few_sequences_cut_many_times(pa, oracle, kv, Hq, Hkv, D, P):
    """Eight or more partitions per sequence: the merge runs as a workgroup of waves per output row
    (both head sizes, both partition kernels, empty partitions when P exceeds the tile count)."""
    b = W.make_batch("fewlong", 65 + P, [3000, 0, 1500], Hq, Hkv, D, 16, kv)
    got, want = check(pa, oracle, b, f"few-long P={P}", num_partitions=P)
    ref, _ = run_gpu(pa, b, num_partitions=1)
    assert_parity(got, ref, kv, "against the unsplit run")


@pytest.mark.parametrize("B", [63, 64, 65, 130, 300])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (2, 2)])
def test_many_short_sequences_with_gaps(pa, oracle, B, Hq, Hkv):
    """More sequences than lanes (the length scan runs in 64-sequence chunks), empty sequences
    sprinkled in, ranges that span dozens of sequences; several partition counts."""
    rng = np.random.default_rng(B)
    lens = rng.integers(1, 120, size=B)
    lens[rng.random(B) < 0.2] = 0
    lens[0] = 0
    lens[B - 1] = 0 if B % 2 else 77
    b = W.make_batch("many", 90 + B, lens.tolist(), Hq, Hkv, 128, 16, W.KV_BF16, max_blocks_per_seq=8)
    for P in (0, 1, 7, 50):
        check(pa, oracle, b, f"many-sequences P={P}", num_partitions=P)


def test_single_token_context_returns_v_exactly(pa):
    for kv in (W.KV_BF16, W.KV_FP8_E4M3):
        b = W.make_batch("l1", 70, [1, 1, 1, 1], 8, 2, 128, 16, kv, num_blocks=9)
        if kv == W.KV_FP8_E4M3:
            # every finite e4m3 byte once: 254 values over the two KV heads of sequence 0
            vals = np.array([x for x in range(256) if x not in (0x7F, 0xFF)] + [0, 0x80], dtype=np.uint8)
            b.v_cache[b.block_tables[0, 0], :, 0, :] = vals.reshape(2, 128)
            b.v_scale[:] = [0.5, 2.0]  # powers of two keep the product exact in float32
        got, _ = run_gpu(pa, b)
        for s in range(4):
            for h in range(8):
                raw = b.v_cache[b.block_tables[s, 0], h // 4, 0]
                if kv == W.KV_BF16:
                    want = W.bf16_bits_to_f32(raw)
                else:
                    import torch

                    want = torch.from_numpy(raw.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy() \
                        * b.v_scale[h // 4]
                assert np.array_equal(got[s, h], want), (kv, s, h)


def test_zero_length_and_poisoned_inputs(pa, oracle):
    for kv in (W.KV_BF16, W.KV_FP8_E4M3):
        b = W.make_batch("edge", 71, [0, 33, 0, 700, 16, 0], 8, 2, 128, 16, kv, num_blocks=60, max_blocks_per_seq=50)
        b.block_tables[b.block_tables < 0] = 2 ** 30  # garbage ids behind the valid prefix
        got, want = check(pa, oracle, b, "zero-length+poison")
        assert np.all(got[0] == 0) and np.all(got[2] == 0) and np.all(got[5] == 0)
        # a host bound above the real maximum may change the plan, not the result
        got2, _ = run_gpu(pa, b, max_context_len=800)
        assert_parity(got2, want, kv, "loose host bound")
        # an all-empty batch
        e = W.make_batch("empty", 72, [0, 0, 0], 8, 2, 128, 16, kv, num_blocks=2, max_blocks_per_seq=2)
        got3, _ = run_gpu(pa, e, num_partitions=4)
        assert np.all(got3 == 0)


def test_runs_are_bit_identical(pa):
    b = W.make_config(2, length_scale=0.25)
    a1, _ = run_gpu(pa, b)
    a2, _ = run_gpu(pa, b)
    assert np.array_equal(a1, a2)


@pytest.mark.parametrize("config,kwargs,P", [(2, dict(length_scale=0.25), 0), (1, {}, 3),
                                             (5, dict(length_scale=1 / 16, batch_limit=16), 0)])
def test_repeated_calls_share_one_workspace(pa, oracle, config, kwargs, P):
    """The workspace carries nothing from one call to the next: poison it (and the output)
    between calls and every call must still produce the same bits."""
    b = W.make_config(config, **kwargs)
    dev = pa.DeviceBatch(b, num_partitions=P)
    want = oracle.decode_batch(b)["out"]
    first = None
    for i in range(3):
        dev.out.fill_(float("nan"))
        if dev.workspace is not None:
            dev.workspace.fill_(float("nan"))
        got = dev.decode().cpu().numpy()
        assert_parity(got, want, b.kv_dtype, f"call {i}")
        first = got if first is None else first
        assert np.array_equal(got, first)


# ------------------------------------------------------------------ bit-exact indexing
def one_hot_batch(kv, lens, Hq, Hkv, D, targets, seed):
    """q = 64*e_0 for every head; the target token's K row is 64*e_0 (all others 0), so the target
    outweighs every other token by exp(4096*scale) and all other weights underflow to 0.  V rows
    hold their own logical position as base-16 digits in dims 0..3 (exact in bf16 and e4m3) and
    the sequence index in dim 4."""
    b = W.make_batch("onehot", seed, lens, Hq, Hkv, D, 16, kv)
    b.q[:] = 0
    b.q[:, :, 0] = W.f32_to_bf16_bits(np.float32(64))
    b.k_cache[:] = 0
    b.v_cache[:] = 0
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
        b.v_scale[:] = 1.0
    for s, L in enumerate(lens):
        for t in range(L):
            phys, slot = b.block_tables[s, t // 16], t % 16
            for d in range(4):
                b.v_cache[phys, :, slot, d] = enc((t >> (4 * d)) & 15)
            b.v_cache[phys, :, slot, 4] = enc(s % 16)
        t = targets[s]
        b.k_cache[b.block_tables[s, t // 16], :, t % 16, 0] = enc(64)
    return b


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (2, 2)])
@pytest.mark.parametrize("P", [0, 1, 6, 29])
def test_one_hot_probe_reads_exactly_the_target_slot(pa, kv, Hq, Hkv, P):
    L = 700
    edge = sorted({0, 15, 16, 17, 31, 32, 33, 255, 256, 257, 351, 352, L - 17, L - 16, L - 2, L - 1})
    lens = [L] * len(edge)
    b = one_hot_batch(kv, lens, Hq, Hkv, 128, edge, 80)
    got, _ = run_gpu(pa, b, num_partitions=P)
    for s, t in enumerate(edge):
        digits = got[s, :, :5]
        want = np.array([(t >> (4 * d)) & 15 for d in range(4)] + [s % 16], dtype=np.float32)
        assert np.array_equal(digits, np.broadcast_to(want, digits.shape)), (s, t, digits[0])


@pytest.mark.parametrize("config,kwargs,P", [
    (1, {}, 0), (1, {}, 3), (2, dict(length_scale=0.25), 0), (4, dict(length_scale=1 / 8), 0),
    (4, dict(length_scale=1 / 8), 37), (5, dict(length_scale=1 / 16, batch_limit=8), 0), (2, {}, 0), (4, {}, 0),
])
def test_trace_matches_block_tables_and_split_plan(pa, oracle, config, kwargs, P):
    """The instrumented production kernels report which physical block they read for every logical
    block (K and V) and which partition processed it: both must equal, bit for bit, the oracle's
    block-table walk and the split plan written from its definition (and the host plan)."""
    import torch

    b = W.make_config(config, **kwargs)
    dev = pa.DeviceBatch(b, num_partitions=P)
    Pr = pa.pa_num_partitions(dev.shape, dev.kv_dtype)
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), -7, dtype=torch.int32, device="cuda")
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    visited = visited.cpu().numpy()
    T, owner = oracle.block_partition(b.context_lens, b.max_blocks_per_seq, 16, Pr)
    Th, owner_host = pa.pa_split_plan(dev.shape, dev.kv_dtype, b.context_lens)
    assert Th == T and np.array_equal(owner_host, owner)
    for s in range(b.batch):
        ids = oracle.visited_blocks(b.block_tables, b.context_lens, 16, s)
        n = len(ids)
        for g in range(b.num_kv_heads):
            assert np.array_equal(visited[s, g, :n, 0], ids) and np.array_equal(visited[s, g, :n, 1], ids)
            assert np.array_equal(visited[s, g, :n, 2], owner[s, :n])
            assert np.all(visited[s, g, n:] == -7)  # nothing past the context was dereferenced
    # the instrumented run computes the same output as the plain one
    want = oracle.decode_batch(b)["out"]
    assert_parity(dev.out.cpu().numpy(), want, b.kv_dtype, "trace-run")


def test_profile_entry_reports_kernel_times(pa):
    b = W.make_config(2, length_scale=0.25)
    dev = pa.DeviceBatch(b)
    part_ms, merge_ms = pa.pa_decode_profile(*dev.args(), shape=dev.shape, workspace=dev.workspace, steps=5)
    assert part_ms > 0 and merge_ms >= 0


@pytest.mark.parametrize("B,hi,Hq,Hkv", [(5000, 40, 8, 2), (20000, 9, 4, 1), (3000, 300, 32, 8), (65535, 4, 8, 2)])
def test_thousands_of_sequences(pa, oracle, B, hi, Hq, Hkv):
    """Batches far larger than a wave: the search for a partition's first sequence goes through groups
    of 1024 sequences, the zero rows of empty contexts are dealt out over all partitions, and the
    merge finds its sequences by boundary.  The oracle checks a seeded sample of rows, every empty
    context must give exact zeros.  The last case is the largest batch the interface takes."""
    rng = np.random.default_rng(B)
    lens = rng.integers(0, hi, size=B)
    lens[rng.random(B) < 0.1] = 0
    b = W.make_batch("thousands", 800 + B % 97, lens.tolist(), Hq, Hkv, 128, 16, W.KV_BF16)
    for P in (0, 37):
        got, dev = run_gpu(pa, b, num_partitions=P)
        assert np.isfinite(got).all()
        assert np.all(got[lens == 0] == 0)
        rows = [(int(s), int(rng.integers(0, Hq))) for s in rng.integers(0, B, size=300)]
        want = oracle.decode_batch(b, rows=rows)["out"]
        sel = np.stack([got[r] for r in rows])
        assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, f"B={B} P={P}")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_one_very_long_context_beside_short_ones(pa, oracle, kv):
    """300,000 tokens in one sequence (18,750 table entries), cut by nearly every partition, next to
    a 17-token and a 100,000-token one; the oracle checks every row."""
    lens = [300_000, 17, 100_000]
    b = W.make_batch("long-one", 812, lens, 8, 2, 128, 16, kv)
    got, dev = run_gpu(pa, b)
    want = oracle.decode_batch(b)["out"]
    assert_parity(got, want, kv, "very long context")
    assert pa.pa_num_partitions(dev.shape, dev.kv_dtype) > 100
