"""The debug path of the C ABI on the GPU: pa_check_tables (tables and lengths held against the
pool without following an id), pa_decode_trace refusing ids outside the pool, and the
instrumented shared-prefix pass.  Expected values come from the CPU oracle's table check and
block-table walk, compared with ==."""
import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.parity import assert_parity

pytestmark = pytest.mark.gpu

UNTOUCHED = -7


@pytest.fixture(scope="module")
def pa():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2605_06068_amd import binding

    binding.lib()
    return binding


def gpu_check(pa, tables, lens, shape):
    """pa_check_tables on device copies of the arrays -> (count, (kind, b, j, value))."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(tables, dtype=np.int32)).cuda()
    l = torch.from_numpy(np.ascontiguousarray(lens, dtype=np.int32)).cuda()
    report = torch.full((8,), 12345, dtype=torch.int32, device="cuda")
    pa.pa_check_tables(t, l, shape=shape, report=report)
    torch.cuda.synchronize()
    r = report.cpu().numpy()
    return int(r[4]), tuple(int(x) for x in r[:4])


def shape_of(pa, b, **kw):
    args = dict(batch=b.batch, num_q_heads=b.num_q_heads, num_kv_heads=b.num_kv_heads, head_dim=b.head_dim,
                block_size=16, max_blocks_per_seq=b.max_blocks_per_seq, num_blocks=b.num_blocks,
                max_context_len=int(b.context_lens.max(initial=0)), q_len=b.q_len,
                shared_prefix_blocks=b.shared_prefix_blocks, window=b.window)
    args.update(kw)
    return pa.make_shape(**args)


def oracle_check(oracle, tables, lens, shape):
    Q = max(1, shape.q_len)
    max_ctx = shape.max_context_len if shape.max_context_len > 0 else shape.max_blocks_per_seq * 16
    return oracle.check_tables(tables, lens, 16, shape.num_blocks, max_ctx,
                               reach=shape.window + Q - 1 if shape.window > 0 else 0,
                               shared_prefix_blocks=shape.shared_prefix_blocks, q_len=Q)


# ------------------------------------------------------------------ pa_check_tables
@pytest.mark.parametrize("config,kwargs", [(1, {}), (2, dict(length_scale=0.25)), (4, dict(length_scale=1 / 8)), (2, {}),
                                           (3, dict(length_scale=1 / 32)), (5, dict(length_scale=1 / 16))])
def test_clean_tables_pass(pa, oracle, config, kwargs):
    b = W.make_config(config, **kwargs)
    s = shape_of(pa, b)
    print(f"[case] clean tables config {config} {kwargs}", flush=True)
    assert gpu_check(pa, b.block_tables, b.context_lens, s) == (0, (0, -1, -1, 0))
    assert oracle_check(oracle, b.block_tables, b.context_lens, s) == (0, (0, -1, -1, 0))


@pytest.mark.parametrize("bad", [-1, None, 2 ** 30, -2 ** 31, 2 ** 31 - 1])
def test_one_bad_id_at_a_valid_position_is_reported_there(pa, oracle, bad):
    """None stands for id == num_blocks, the smallest id outside the pool.  The check reads the
    tables only, so no id is followed and the call completes whatever they hold."""
    rng = np.random.default_rng(abs(bad or 3) % 1000)
    b = W.make_config(4, length_scale=1 / 8)
    s = shape_of(pa, b)
    bad = b.num_blocks if bad is None else bad
    for _ in range(6):
        seq = int(rng.integers(0, b.batch))
        j = int(rng.integers(0, (int(b.context_lens[seq]) + 15) // 16))
        t = b.block_tables.copy()
        t[seq, j] = bad
        t[seq, (int(b.context_lens[seq]) + 15) // 16:] = bad  # behind the context: may hold anything
        print(f"[case] bad id {bad} at ({seq}, {j})", flush=True)
        got = gpu_check(pa, t, b.context_lens, s)
        assert got == (1, (pa.PA_TABLES_BAD_BLOCK_ID, seq, j, bad))
        assert got == oracle_check(oracle, t, b.context_lens, s)


def test_many_faults_first_one_and_count(pa, oracle):
    """Faults of all kinds sprinkled over a large table: the first in batch order, then block order,
    and the number of offending entries equal the oracle's, whatever order the workgroups ran in."""
    rng = np.random.default_rng(17)
    for trial in range(8):
        B = int(rng.integers(1, 700))
        lens = rng.integers(0, 6000, size=B).astype(np.int32)
        MB = 6000 // 16 + 1
        NB = 5000
        t = rng.integers(0, NB, size=(B, MB)).astype(np.int32)
        n_bad = int(rng.integers(0, 40))
        t[rng.integers(0, B, n_bad), rng.integers(0, MB, n_bad)] = rng.choice([-1, NB, NB + 7, -2 ** 31], n_bad)
        lens[rng.integers(0, B, int(rng.integers(0, 3)))] = rng.choice([-1, 6001, 2 ** 30])
        s = pa.make_shape(B, 8, 2, 128, 16, MB, NB, max_context_len=6000)
        print(f"[case] many faults trial {trial} B={B}", flush=True)
        want = oracle_check(oracle, t, lens, s)
        assert gpu_check(pa, t, lens, s) == want


@pytest.mark.parametrize("Q,window", [(1, 100), (4, 33), (16, 1)])
def test_blocks_a_sliding_window_left_behind_are_not_checked(pa, oracle, Q, window):
    b = W.make_batch("win", 31, [700, 50, 0, 1000, 16, 129], 8, 2, 128, 16, W.KV_BF16, q_len=Q, window=window)
    s = shape_of(pa, b)
    # the generator has set the evicted entries to -1 already
    assert (b.block_tables[0, :10] == -1).all()
    assert gpu_check(pa, b.block_tables, b.context_lens, s) == (0, (0, -1, -1, 0))
    # the block that holds the first visible token of sequence 3 is checked, the one before it is not
    reach = window + Q - 1
    j = (1000 - reach) // 16
    t = b.block_tables.copy()
    t[3, j] = -1
    assert gpu_check(pa, t, b.context_lens, s) == (1, (pa.PA_TABLES_BAD_BLOCK_ID, 3, j, -1))
    assert oracle_check(oracle, t, b.context_lens, s) == (1, (2, 3, j, -1))
    # without the window every block counts
    s0 = shape_of(pa, b, window=0)
    got = gpu_check(pa, b.block_tables, b.context_lens, s0)
    assert got == oracle_check(oracle, b.block_tables, b.context_lens, s0) and got[1][:3] == (2, 0, 0)


def test_shared_prefix_rows_and_lengths_are_checked(pa, oracle):
    b = W.make_batch("pfx", 32, [400, 330, 321, 352], 8, 2, 128, 16, W.KV_BF16, shared_prefix_blocks=20)
    s = shape_of(pa, b)
    assert gpu_check(pa, b.block_tables, b.context_lens, s) == (0, (0, -1, -1, 0))
    t = b.block_tables.copy()
    t[2, 7] = t[2, 20]  # a valid id, but not the one row 0 holds there
    got = gpu_check(pa, t, b.context_lens, s)
    assert got == (1, (pa.PA_TABLES_PREFIX_MISMATCH, 2, 7, int(t[2, 20]))) == oracle_check(oracle, t, b.context_lens, s)
    lens = b.context_lens.copy()
    lens[1] = 319  # shorter than the prefix
    got = gpu_check(pa, t, lens, s)
    assert got == (2, (pa.PA_TABLES_BAD_LENGTH, 1, -1, 319)) == oracle_check(oracle, t, lens, s)


def test_check_tables_arguments(pa):
    import torch

    b = W.make_config(1)
    s = shape_of(pa, b)
    t = torch.from_numpy(b.block_tables).cuda()
    l = torch.from_numpy(b.context_lens).cuda()
    rep = torch.zeros(9, dtype=torch.int32, device="cuda")
    with pytest.raises(pa.PaError) as e:
        pa.pa_check_tables(t, l, shape=s, report=rep[1:])  # misaligned report
    assert e.value.status == pa.PA_ERR_INVALID_ARG
    with pytest.raises(pa.PaError):
        pa.pa_check_tables(t, None, shape=s, report=rep)
    bad = shape_of(pa, b, num_blocks=0)
    with pytest.raises(pa.PaError):
        pa.pa_check_tables(t, l, shape=bad, report=rep)
    empty = shape_of(pa, b, batch=0)
    pa.pa_check_tables(t, l, shape=empty, report=rep)
    torch.cuda.synchronize()
    assert rep[:5].cpu().tolist() == [0, -1, -1, 0, 0]


# ------------------------------------------------------------------ pa_decode_trace and ids outside the pool
def trace_run(pa, b, declared_blocks=None, **kw):
    import torch

    dev = pa.DeviceBatch(b, **kw)
    if declared_blocks is not None:
        dev.shape.num_blocks = declared_blocks
    visited = torch.full((b.batch, b.num_kv_heads, b.max_blocks_per_seq, 3), UNTOUCHED, dtype=torch.int32, device="cuda")
    pa.pa_decode_trace(*dev.args(), shape=dev.shape, workspace=dev.workspace, visited_blocks=visited)
    torch.cuda.synchronize()
    return dev.out.cpu().numpy(), visited.cpu().numpy(), dev


def with_extra_blocks(b, extra):
    """The same batch over a pool with `extra` more blocks at its end, full of NaN patterns, that no
    table entry names."""
    pat = W.BF16_NAN_BITS if b.kv_dtype == W.KV_BF16 else W.FP8_NAN_BYTE
    pad = np.full((extra,) + b.k_cache.shape[1:], pat, dtype=b.k_cache.dtype)
    b.k_cache = np.concatenate([b.k_cache, pad])
    b.v_cache = np.concatenate([b.v_cache, pad])
    b.num_blocks += extra
    return b


@pytest.mark.parametrize("kv,Q,P", [(W.KV_BF16, 1, 0), (W.KV_FP8_E4M3, 1, 5), (W.KV_BF16, 16, 0), (W.KV_BF16, 6, 3)])
def test_id_just_outside_the_declared_pool_is_recorded_and_not_followed(pa, oracle, kv, Q, P):
    """The pool is allocated four blocks larger than the shape declares, and the spoiled entries point
    at those extra blocks, so this test stays inside allocated memory whether or not the check
    works; the extra blocks hold a value pattern of their own that must not show in the output.
    Expected output: the oracle on the same tables with block 0 in place of the refused ids."""
    lens = [700, 33, 300, 1, 257]
    need = sum((L + 15) // 16 for L in lens)
    b = with_extra_blocks(W.make_batch("declared", 40 + Q, lens, 8, 2, 128, 16, kv, q_len=Q, poison=False), 4)
    spoiled = {(0, 5): need, (0, 43): need + 3, (2, 0): need + 1, (4, 16): need + 2}
    for (s, j), bad in spoiled.items():
        b.block_tables[s, j] = bad
    print(f"[case] declared pool {need} of {need + 4} blocks kv={kv} Q={Q} P={P}", flush=True)
    got, visited, dev = trace_run(pa, b, declared_blocks=need, num_partitions=P)
    assert np.isfinite(got).all()
    for s in range(b.batch):
        ids = oracle.visited_blocks(b.block_tables, b.context_lens, 16, s)  # the table as it stands, bad ids included
        for g in range(b.num_kv_heads):
            assert np.array_equal(visited[s, g, :len(ids), 0], ids) and np.array_equal(visited[s, g, :len(ids), 1], ids)
            assert np.all(visited[s, g, len(ids):] == UNTOUCHED)
    for (s, j), bad in spoiled.items():
        assert visited[s, 0, j, 0] == bad and visited[s, 1, j, 1] == bad
    stand_in = W.make_batch("declared", 40 + Q, lens, 8, 2, 128, 16, kv, q_len=Q, poison=False)
    for (s, j) in spoiled:
        stand_in.block_tables[s, j] = 0
    want = oracle.decode_batch(stand_in)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert_parity(flat(got), flat(want), kv, "block 0 read in place of refused ids")
    # and the table check names the first of them
    count, first = gpu_check(pa, b.block_tables, b.context_lens, dev.shape)
    assert (count, first) == (4, (pa.PA_TABLES_BAD_BLOCK_ID, 0, 5, need))


@pytest.mark.parametrize("kv,Q,window", [(W.KV_BF16, 1, 0), (W.KV_FP8_E4M3, 1, 0), (W.KV_BF16, 16, 0), (W.KV_BF16, 1, 100),
                                         (W.KV_BF16, 8, 0)])
def test_wild_ids_at_valid_positions_are_recorded_and_the_call_completes(pa, oracle, kv, Q, window):
    lens = [700, 33, 300, 1, 257]
    b = W.make_batch("wild", 50 + Q + window, lens, 8, 2, 128, 16, kv, q_len=Q, window=window, poison=False)
    first_visible = lambda s: max(0, lens[s] - (window + Q - 1)) // 16 if window > 0 else 0
    spoiled = {(0, 43): -1, (0, 41): 2 ** 30, (2, max(first_visible(2), 3)): -2 ** 31, (4, 16): b.num_blocks, (3, 0): 2 ** 31 - 1}
    for (s, j), bad in spoiled.items():
        b.block_tables[s, j] = bad
    for P in (0, 4):
        print(f"[case] wild ids kv={kv} Q={Q} window={window} P={P}", flush=True)
        got, visited, dev = trace_run(pa, b, num_partitions=P)
        assert np.isfinite(got).all()
        for (s, j), bad in spoiled.items():
            assert visited[s, 0, j, 0] == bad and visited[s, 1, j, 1] == bad and visited[s, 0, j, 2] >= 0
        count, first = gpu_check(pa, b.block_tables, b.context_lens, dev.shape)
        assert (count, first) == oracle_check(oracle, b.block_tables, b.context_lens, dev.shape)
        assert count == len(spoiled) and first[0] == pa.PA_TABLES_BAD_BLOCK_ID
    # sequence 1 has no spoiled entry: its rows are still right
    want = oracle.decode_batch(b, rows=[(1, h) for h in range(8)] if Q == 1 else [(1, i, h) for i in range(Q) for h in range(8)])["out"]
    assert_parity(got[1].reshape(1, -1, 128), want.reshape(1, -1, 128), kv, "untouched sequence")


# ------------------------------------------------------------------ the instrumented shared-prefix pass
def prefix_trace_case(pa, oracle, b, P):
    got, visited, dev = trace_run(pa, b, num_partitions=P)
    pre = 2 * (b.shared_prefix_blocks // 2)  # whole tiles of the prefix go to the prefix pass
    Pr = pa.pa_num_partitions(dev.shape, dev.kv_dtype)
    T, plan = pa.pa_split_plan(dev.shape, dev.kv_dtype, b.context_lens)
    # the per-sequence part of the host plan is the oracle's plan of the contexts with the prefix taken off
    To, own = oracle.block_partition(b.context_lens - pre * 16, b.max_blocks_per_seq, 16, Pr)
    assert T == To
    for s in range(b.batch):
        ids = oracle.visited_blocks(b.block_tables, b.context_lens, 16, s)
        n = len(ids)
        assert np.array_equal(plan[s, pre:n], own[s, :n - pre])
        for g in range(b.num_kv_heads):
            if s == 0:  # the prefix pass reads the prefix through row 0 and records it there
                assert np.array_equal(visited[0, g, :pre, 0], ids[:pre]) and np.array_equal(visited[0, g, :pre, 1], ids[:pre])
                assert np.array_equal(visited[0, g, :pre, 2], plan[0, :pre])
            else:       # no other row's prefix entries are read
                assert np.all(visited[s, g, :pre] == UNTOUCHED)
            assert np.array_equal(visited[s, g, pre:n, 0], ids[pre:]) and np.array_equal(visited[s, g, pre:n, 1], ids[pre:])
            assert np.array_equal(visited[s, g, pre:n, 2], plan[s, pre:n])
            assert np.all(visited[s, g, n:] == UNTOUCHED)
    # the prefix ranges: -2 - r, r = 0 .. Pp-1 in order, both blocks of a tile together, sizes within one tile
    r = -2 - plan[0, :pre]
    assert r[0] == 0 and np.all(np.diff(r) >= 0) and np.all(np.diff(r) <= 1) and np.array_equal(r[0::2], r[1::2])
    sizes = np.bincount(r) // 2
    assert sizes.max() - sizes.min() <= 1
    assert np.array_equal(plan[:, :pre], np.broadcast_to(plan[0, :pre], (b.batch, pre)))
    return got


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("P", [0, 1, 5])
@pytest.mark.parametrize("Hq,Hkv,B,prefix_blocks,Q", [(8, 2, 5, 24, 1), (16, 1, 3, 9, 1), (32, 8, 20, 64, 1), (8, 2, 9, 10, 4)])
def test_prefix_pass_trace_matches_row_zero_and_the_plan(pa, oracle, kv, P, Hq, Hkv, B, prefix_blocks, Q):
    rng = np.random.default_rng(B + prefix_blocks)
    lens = (prefix_blocks * 16 + Q - 1 + rng.integers(0, 300, size=B)).tolist()
    b = W.make_batch("prefix-trace", 600 + B, lens, Hq, Hkv, 128, 16, kv, q_len=Q, shared_prefix_blocks=prefix_blocks)
    print(f"[case] prefix trace kv={kv} P={P} Hq={Hq} Hkv={Hkv} B={B} prefix={prefix_blocks} Q={Q}", flush=True)
    got = prefix_trace_case(pa, oracle, b, P)
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    assert_parity(flat(got), flat(want), kv, "instrumented shared-prefix run")


def test_prefix_pass_trace_on_the_prompt_cache_workload(pa, oracle):
    b = W.make_config(6)
    print("[case] prefix trace, prompt-cache workload", flush=True)
    got = prefix_trace_case(pa, oracle, b, 0)
    rows = [(s, (5 * s) % b.num_q_heads) for s in range(b.batch)]
    want = oracle.decode_batch(b, rows=rows)["out"]
    sel = np.stack([got[s, h] for s, h in rows])
    assert_parity(sel[:, None, :], want[:, None, :], b.kv_dtype, "prompt-cache workload, instrumented")


def test_table_check_in_a_hip_graph(pa, oracle):
    """The check is three launches and no memset, so a serving loop can capture it beside its decode
    step: captured once, replayed over tables that change between replays (clean, spoiled, clean,
    spoiled elsewhere), every replay compared with the oracle's check and with the eager call."""
    import torch

    b = W.make_config(2, length_scale=0.25)
    s = shape_of(pa, b)
    t = torch.from_numpy(b.block_tables).cuda()
    l = torch.from_numpy(b.context_lens).cuda()
    report = torch.full((8,), 777, dtype=torch.int32, device="cuda")
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pa.pa_check_tables(t, l, shape=s, report=report)  # warm-up outside capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            pa.pa_check_tables(t, l, shape=s, report=report)
    torch.cuda.synchronize()
    for i, spoil in enumerate([None, (5, 3, -1), None, (40, 0, b.num_blocks), (2, 1, 2 ** 30)]):
        tables = b.block_tables.copy()
        if spoil is not None:
            tables[spoil[0], spoil[1]] = spoil[2]
        t.copy_(torch.from_numpy(tables))
        report.fill_(777)
        graph.replay()
        torch.cuda.synchronize()
        r = report.cpu().numpy()
        got = (int(r[4]), tuple(int(x) for x in r[:4]))
        print(f"[case] table check, graph replay {i}: {got}", flush=True)
        assert got == oracle_check(oracle, tables, b.context_lens, s) == gpu_check(pa, tables, b.context_lens, s)
        _ = (torch.randn(1 << 16, device="cuda") * 2).sum().item()  # unrelated eager work between replays
