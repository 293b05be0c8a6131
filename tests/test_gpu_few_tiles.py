"""GPU parity of calls with fewer tiles than partitions: some partitions are then empty, also between
two tiles of one sequence, and the merge must still find every sequence that was cut -- by the list of
the partitions' starts (batches of at least P - 1 sequences) as well as by scanning the descriptors."""
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


def sparse_lens(B, seed, long_ones):
    """Mostly empty contexts and a few of two to four tiles."""
    rng = np.random.default_rng(seed)
    lens = np.zeros(B, dtype=np.int64)
    where = rng.choice(B, size=long_ones, replace=False)
    lens[where] = rng.integers(33, 128, size=long_ones)
    return [int(x) for x in lens]


CASES = [
    [0, 38, 0, 27, 0],                 # three tiles; with P = 5 an empty partition lies inside sequence 1
    [0, 70, 0, 0, 0, 0],
    [100, 0, 0, 0, 0, 0, 0, 0],
    sparse_lens(20, 1, 3),
    sparse_lens(64, 2, 5),
    sparse_lens(70, 3, 4),             # more than 64 sequences: the two-pass range search
    sparse_lens(200, 4, 9),
    sparse_lens(600, 5, 2),            # two sequences in 600: their pieces lie a hundred and more partitions apart
    sparse_lens(1500, 6, 3),
]


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv,D", [(1, 2, 1, 64), (1, 8, 2, 128), (4, 8, 1, 128), (16, 4, 1, 128), (16, 8, 1, 64)])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_more_partitions_than_tiles(pa, oracle, kv, Q, Hq, Hkv, D, case):
    import torch

    lens = [L + Q - 1 if L > 0 else 0 for L in CASES[case]]
    B = len(lens)
    b = W.make_batch("few-tiles", 9800 + case + Q + Hq, lens, Hq, Hkv, D, 16, kv, q_len=Q)
    want = oracle.decode_batch(b)["out"]
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    T = sum(-(-L // 32) for L in lens)
    # partition counts above the tile count, on both sides of B + 1 (up to there the merge goes by the list of
    # the partitions' starts, above it scans the descriptors)
    # ... and, for small batches, enough partitions per sequence for the merge kernel of many pieces
    for P in sorted({T + 1, T + 2, (T + B + 1) // 2, B, B + 1, B + 5, 2 * B + 3} | ({8 * B + 1} if B <= 20 else set())):
        if P <= T:
            continue
        print(f"[case] few tiles: {sum(1 for L in lens if L > 0)} of {B} sequences non-empty, {T} tiles, Q={Q} Hq={Hq} "
              f"Hkv={Hkv} D={D} kv={kv} P={P}", flush=True)
        dev = pa.DeviceBatch(b, num_partitions=P)
        assert pa.pa_split_plan(dev.shape, dev.kv_dtype, lens)[0] == T
        out = dev.decode()
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.isfinite(got).all(), "a row nobody wrote (the output starts as NaN)"
        assert_parity(flat(got), flat(want), kv, f"fewer tiles than partitions, P={P}")


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
@pytest.mark.parametrize("Q,Hq,Hkv,B,most", [(1, 8, 2, 24, 900), (4, 8, 1, 24, 900), (1, 8, 2, 600, 130), (4, 8, 1, 1100, 130)])
def test_graph_replay_after_the_lengths_have_shrunk(pa, oracle, kv, Q, Hq, Hkv, B, most):
    """A call captured for full contexts (its partition count follows the host's bound) and replayed
    after most contexts were reset to nothing or to a few tokens, as when finished requests leave a
    serving batch: the replays run with far fewer tiles than partitions.  Small batches (the merge scans
    the descriptors) and batches of more sequences than partitions (it goes by the partitions' starts)."""
    import torch

    rng = np.random.default_rng(9900 + Q)
    full = rng.integers(most // 4, most, size=B).astype(np.int32) + Q - 1
    b = W.make_batch("few-tiles-graph", 9900 + Q + Hq, full.tolist(), Hq, Hkv, 128, 16, kv, poison=False, q_len=Q)
    dev = pa.DeviceBatch(b, max_context_len=int(full.max()))
    P = pa.pa_num_partitions(dev.shape, dev.kv_dtype)

    def enqueue():
        pa.pa_decode(*dev.args(), shape=dev.shape, workspace=dev.workspace)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()  # warm-up outside capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    flat = lambda a: a.reshape(a.shape[0], -1, a.shape[-1])
    for i in range(5):
        lens = full.copy()
        gone = rng.random(B) < 0.6 + 0.08 * i
        # (contexts only ever shrink: the tables hold blocks for the full lengths and -1 behind them)
        lens[gone] = np.where(rng.random(int(gone.sum())) < 0.5, 0,
                              np.minimum(full[gone], Q + rng.integers(0, 70, size=int(gone.sum()))))
        if i == 4:
            lens[:] = 0
            lens[7] = min(int(full[7]), 70 + Q)
            lens[B - 2] = min(int(full[B - 2]), 40 + Q)
        assert np.all(lens <= full)
        b.context_lens = lens.astype(np.int32)
        T = int(sum(-(-int(L) // 32) for L in lens))
        print(f"[case] graph replay {i}: {T} tiles, {P} partitions, {B} sequences, Q={Q} kv={kv}", flush=True)
        dev.context_lens.copy_(torch.from_numpy(b.context_lens))
        dev.out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = dev.out.cpu().numpy()
        assert np.isfinite(got).all()
        assert_parity(flat(got), flat(oracle.decode_batch(b)["out"]), kv, f"graph replay {i} with {T} tiles")
    assert T < P
