"""GPU parity of decode calls that declare a shared prefix (the same physical blocks at the head of
every block table): the result must be the plain decode attention the float64 CPU oracle computes;
only the way the prefix is read differs."""
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
          f"kv={batch.kv_dtype} prefix_blocks={batch.shared_prefix_blocks} tokens={batch.total_tokens} {kw}", flush=True)
    got, dev = run_gpu(pa, batch, **kw)
    want = oracle.decode_batch(batch)["out"]
    err = assert_parity(got, want, batch.kv_dtype, what)
    print(f"        max_abs={err[0]:.3e} rel_l2={err[1]:.3e} P={pa.pa_num_partitions(dev.shape, dev.kv_dtype)}", flush=True)
    return got, want


def suffix_lens(prefix_blocks, B, seed):
    """Contexts that cover the prefix: some end exactly with it, some inside the next block or tile,
    some hundreds of tokens later."""
    rng = np.random.default_rng(seed)
    base = prefix_blocks * 16
    extra = [0, 1, 15, 16, 17, 31, 32, 33, 128, 129, 700, 40, 64, 5, 300, 2]
    lens = [base + extra[i % len(extra)] for i in range(B)]
    rng.shuffle(lens)
    return lens


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 2), (16, 1), (5, 1), (2, 2), (4, 2), (32, 1), (40, 2), (17, 1)])
@pytest.mark.parametrize("B,prefix_blocks", [(1, 8), (3, 2), (5, 3), (20, 64), (16, 9), (40, 10)])
def test_shared_prefix_shapes(pa, oracle, kv, Hq, Hkv, B, prefix_blocks):
    """Column counts B*G from 1 to 640: 2, 4 and 8 waves per workgroup, padded and idle waves, several
    column groups; odd block counts leave the last prefix block to the per-sequence pass."""
    b = W.make_batch("prefix", 500 + 7 * B + Hq, suffix_lens(prefix_blocks, B, B), Hq, Hkv, 128, 16, kv,
                     shared_prefix_blocks=prefix_blocks)
    check(pa, oracle, b, "shared-prefix")
    check(pa, oracle, b, "shared-prefix P=3", num_partitions=3)


@pytest.mark.parametrize("P", [1, 2, 7, 50])
def test_shared_prefix_partition_sweep(pa, oracle, P):
    b = W.make_batch("prefix-sweep", 520, suffix_lens(40, 12, 3), 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=40)
    got, want = check(pa, oracle, b, f"shared-prefix sweep P={P}", num_partitions=P)
    plain, _ = run_gpu(pa, b, shared_prefix_blocks=0)  # the same batch without the promise
    assert_parity(got, plain, b.kv_dtype, "against the call without a shared prefix")


def test_prefix_of_one_block_is_the_plain_call(pa, oracle):
    b = W.make_batch("prefix-1", 521, [16, 40, 100], 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=1)
    got, _ = check(pa, oracle, b, "one shared block")
    plain, _ = run_gpu(pa, b, shared_prefix_blocks=0)
    assert np.array_equal(got, plain)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("P", [0, 1, 5])
def test_shared_prefix_one_hot_probe(pa, kv, P):
    """Sequence s has a target token whose key is 32 e_s, every other key of the cache is zero, and
    its query is 128 e_s: queries and target keys of different sequences are orthogonal, so sequence
    s puts all its weight on its own target (the rest underflows) whether the target lies in the
    shared prefix or in its own blocks.  V rows spell their logical position in base-16 digits.
    Targets sit at both ends of the prefix, around tile and range boundaries, and after the prefix."""
    prefix_blocks = 24
    base = prefix_blocks * 16
    targets = [0, 15, 16, 31, 32, 33, 191, 192, 193, base - 33, base - 32, base - 1, base, base + 1, base + 15,
               base + 16, base + 31, base + 32, base + 99]
    B = len(targets)
    lens = [base + 100] * B
    b = W.make_batch("prefix-onehot", 530, lens, 8, 2, 128, 16, kv, shared_prefix_blocks=prefix_blocks)
    enc = (lambda x: W.f32_to_bf16_bits(np.float32(x))) if kv == W.KV_BF16 else \
        (lambda x: W.f32_to_e4m3_bytes(np.array([x], np.float32))[0])
    b.q[:] = 0
    b.k_cache[:] = 0
    b.v_cache[:] = 0
    if kv == W.KV_FP8_E4M3:
        b.k_scale[:] = 1.0
        b.v_scale[:] = 1.0
    for s in range(B):
        for t in range(lens[s]):
            phys, slot = b.block_tables[s, t // 16], t % 16
            for d in range(4):
                b.v_cache[phys, :, slot, d] = enc((t >> (4 * d)) & 15)
        t = targets[s]
        b.k_cache[b.block_tables[s, t // 16], :, t % 16, s] = enc(32)
        b.q[s, :, s] = W.f32_to_bf16_bits(np.float32(128))
    got, _ = run_gpu(pa, b, num_partitions=P)
    for s, t in enumerate(targets):
        want = np.array([(t >> (4 * d)) & 15 for d in range(4)], dtype=np.float32)
        digits = got[s, :, :4]
        assert np.array_equal(digits, np.broadcast_to(want, digits.shape)), (s, t, digits[0])


def test_shared_prefix_repeated_calls_share_one_workspace(pa, oracle):
    b = W.make_batch("prefix-ws", 540, suffix_lens(32, 20, 9), 32, 8, 128, 16, W.KV_BF16, shared_prefix_blocks=32)
    dev = pa.DeviceBatch(b)
    want = oracle.decode_batch(b)["out"]
    first = None
    for i in range(3):
        dev.out.fill_(float("nan"))
        dev.workspace.fill_(float("nan"))
        got = dev.decode().cpu().numpy()
        assert_parity(got, want, b.kv_dtype, f"call {i}")
        first = got if first is None else first
        assert np.array_equal(got, first)


def test_prompt_cache_workload_sampled_rows(pa, oracle):
    """The prompt-caching shape at full size (20 sequences over one 32k-token prefix, 128..255 own
    tokens each) in the default launch configuration; the oracle computes sampled output rows."""
    b = W.make_config(6)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(6)
    rows = [(s, int(rng.integers(0, b.num_q_heads))) for s in range(b.batch)] + [(0, 0), (b.batch - 1, b.num_q_heads - 1)]
    want = oracle.decode_batch(b, rows=rows)["out"]
    sel = np.stack([got[s, h] for s, h in rows])
    err = assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, "prompt-cache workload")
    print(f"        {len(rows)} sampled rows max_abs={err[0]:.3e} worst row rel_l2={err[1]:.3e}", flush=True)


@pytest.mark.parametrize("B", [65, 130])
def test_shared_prefix_many_sequences(pa, oracle, B):
    """More sequences than lanes: several column groups in the prefix pass, chunked scans in the
    per-sequence pass and in the merge."""
    b = W.make_batch("prefix-many", 550 + B, suffix_lens(6, B, B), 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=6)
    for P in (0, 1, 9):
        check(pa, oracle, b, f"shared-prefix many-sequences P={P}", num_partitions=P)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("Q,Hq,Hkv", [(4, 8, 2), (8, 4, 1), (2, 16, 1), (16, 2, 1), (3, 5, 1), (2, 2, 2), (16, 4, 2)])
@pytest.mark.parametrize("B,prefix_blocks", [(1, 8), (5, 3), (20, 64), (9, 10)])
def test_multi_token_calls_over_a_shared_prefix(pa, oracle, kv, D, Q, Hq, Hkv, B, prefix_blocks):
    """Verification windows whose tokens all lie after the shared prefix (the shortest context ends
    Q - 1 tokens after it): the prefix pass sees B * Q * G columns, the per-sequence pass is causal
    inside the window, the merge joins them row by row."""
    lens = [L + Q - 1 for L in suffix_lens(prefix_blocks, B, B + Q)]
    b = W.make_batch("prefix-verify", 560 + 7 * B + Hq + Q, lens, Hq, Hkv, D, 16, kv, q_len=Q,
                     shared_prefix_blocks=prefix_blocks)
    print(f"[case] Q={Q} D={D}", flush=True)
    got, dev = run_gpu(pa, b)
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert_parity(flat(got), flat(want), kv, "shared prefix, multi-token")
    got3, _ = run_gpu(pa, b, num_partitions=3)
    assert_parity(flat(got3), flat(want), kv, "shared prefix, multi-token, P=3")
    plain, _ = run_gpu(pa, b, shared_prefix_blocks=0)
    assert_parity(flat(got), flat(plain), kv, "against the call without a shared prefix")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv,D", [(16, 8, 2, 128), (16, 16, 2, 128), (12, 4, 1, 64), (8, 8, 1, 128), (3, 40, 1, 128), (16, 3, 1, 64)])
@pytest.mark.parametrize("B,prefix_blocks", [(3, 8), (20, 64), (7, 5)])
def test_wide_multi_token_calls_over_a_shared_prefix(pa, oracle, kv, Q, Hq, Hkv, D, B, prefix_blocks):
    """33 .. 128 columns per KV head behind a shared prefix: the per-sequence pass runs on the
    multi-wave kernels (stage-split at head_dim 128), which leave the prefix tiles out of their plan as the
    one-wave kernel does."""
    lens = [L + Q - 1 for L in suffix_lens(prefix_blocks, B, B + Q)]
    b = W.make_batch("prefix-verify-wide", 580 + 7 * B + Hq + Q, lens, Hq, Hkv, D, 16, kv, q_len=Q,
                     shared_prefix_blocks=prefix_blocks)
    print(f"[case] wide prefix verify Q={Q} Hq={Hq} Hkv={Hkv} D={D} B={B} prefix={prefix_blocks} kv={kv}", flush=True)
    got, dev = run_gpu(pa, b)
    staged = Q * (Hq // Hkv) <= 64 or (D == 128) == (kv == W.KV_FP8_E4M3)
    assert pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == ("mfma-staged" if staged else "mfma-wide")
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert_parity(flat(got), flat(want), kv, "shared prefix, wide multi-token")
    got3, _ = run_gpu(pa, b, num_partitions=3)
    assert_parity(flat(got3), flat(want), kv, "shared prefix, wide multi-token, P=3")
    plain, _ = run_gpu(pa, b, shared_prefix_blocks=0)
    assert_parity(flat(got), flat(plain), kv, "against the call without a shared prefix")


def test_prompt_cache_workload_with_16_token_verification(pa, oracle):
    """Speculative verification over a cached prompt: 20 sequences over one 32k-token prefix, a window
    of 16 proposed tokens each, 4 query heads per KV head (64 columns); the oracle computes sampled rows."""
    b = W.make_config(6, q_len=16)
    got, dev = run_gpu(pa, b)
    assert np.isfinite(got).all() and pa.pa_kernel_variant(dev.shape, dev.kv_dtype) == "mfma-staged"
    rng = np.random.default_rng(66)
    rows = [(s, int(rng.integers(0, 16)), int(rng.integers(0, b.num_q_heads))) for s in range(b.batch)] + \
           [(0, 0, 0), (b.batch - 1, 15, b.num_q_heads - 1)]
    want = oracle.decode_batch(b, rows=rows)["out"]
    sel = np.stack([got[s, i, h] for s, i, h in rows])
    err = assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, "prompt-cache workload, 16-token verification")
    print(f"        {len(rows)} sampled rows max_abs={err[0]:.3e} worst row rel_l2={err[1]:.3e}", flush=True)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv,D", [(1, 8, 2, 128), (4, 8, 2, 128), (16, 4, 1, 128), (3, 16, 2, 64), (16, 8, 1, 64)])
@pytest.mark.parametrize("window", [1, 33, 200, 1000])
def test_sliding_window_over_a_shared_prefix(pa, oracle, kv, Q, Hq, Hkv, D, window):
    """A window and the promise of a shared prefix in one call: the promise goes unused, every sequence
    reads its own last window + Q - 1 tokens (inside the prefix for some sequences, behind it for others)
    and no block before them: the batch's evicted prefix blocks are poisoned and their table entries,
    row 0's included, are -1."""
    prefix_blocks = 24
    lens = [L + Q - 1 for L in suffix_lens(prefix_blocks, 18, 60 + Q)]
    b = W.make_batch("prefix-window", 640 + Q + Hq + window, lens, Hq, Hkv, D, 16, kv, q_len=Q,
                     shared_prefix_blocks=prefix_blocks, window=window)
    assert (b.block_tables[:, :prefix_blocks] == -1).any(axis=1).all() == (window + Q - 1 <= prefix_blocks * 16 - 16)
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    for P in (0, 3):
        print(f"[case] window over a shared prefix Q={Q} Hq={Hq} Hkv={Hkv} D={D} W={window} kv={kv} P={P}", flush=True)
        got, dev = run_gpu(pa, b, num_partitions=P)
        assert dev.shape.window == window and dev.shape.shared_prefix_blocks == prefix_blocks
        want = oracle.decode_batch(b)["out"]
        assert_parity(flat(got), flat(want), kv, "window over a shared prefix")
