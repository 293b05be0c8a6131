"""A compact subset of the oracle pins that can run against any build of the oracle's C file.

Run as ``python -m tests.oracle_core_pins path/to/lib.so`` it swaps that library in and exits
non-zero if a pin fails (used to check that planted mistakes are caught)."""
import ctypes
import sys

import numpy as np

from paper_2605_06068_amd import workloads as W
from tests.dense_reference import dense_attention, dense_window_attention, e4m3_to_f64


def core_pins(oracle):
    """Raises AssertionError if a pin fails."""
    t = oracle.e4m3_table()
    lib = e4m3_to_f64(np.arange(256, dtype=np.uint8))
    ok = ~np.isnan(lib)
    assert np.array_equal(t[ok], lib[ok]) and np.isnan(t[~ok]).all()
    for kv in (W.KV_BF16, W.KV_FP8_E4M3):
        b = W.make_batch("m", 5, [1, 37, 100], 8, 2, 64, 16, kv, num_blocks=20, max_blocks_per_seq=9)
        r = oracle.decode_batch(b, want_f64=True)
        want, _ = dense_attention(b)
        assert np.isfinite(r["out_f64"]).all()
        assert np.max(np.abs(r["out_f64"] - want)) <= 1e-12
        # multi-token window, causal inside the window: library attention with an explicit mask
        w = W.make_batch("w", 6, [2, 37, 100], 8, 2, 64, 16, kv, num_blocks=20, max_blocks_per_seq=9, q_len=3)
        r = oracle.decode_batch(w, want_f64=True)
        assert np.isfinite(r["out_f64"]).all()
        assert np.max(np.abs(r["out_f64"] - dense_window_attention(w))) <= 1e-12
        # sliding window on top (band mask); nothing is evicted here, so a window that is too wide shows
        sw = W.make_batch("s", 7, [2, 37, 100], 8, 2, 64, 16, kv, num_blocks=20, max_blocks_per_seq=9, q_len=3,
                          window=7, poison=False)
        r = oracle.decode_batch(sw, want_f64=True)
        assert np.isfinite(r["out_f64"]).all()
        assert np.max(np.abs(r["out_f64"] - dense_window_attention(sw, sliding=7))) <= 1e-12
    # appending a window of Q tokens and then attending over it: token i of the window must be what
    # query i sees last (one-token windows, so each output is exactly that token's value row)
    rng = np.random.default_rng(3)
    a = W.make_batch("a", 8, [9, 40], 4, 2, 64, 16, W.KV_BF16, num_blocks=8, q_len=3, window=1, poison=False)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((2, 3, 2, 64)).astype(np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((2, 3, 2, 64)).astype(np.float32))
    oracle.kv_append(k_new, v_new, a.k_cache, a.v_cache, a.block_tables, a.context_lens, W.KV_BF16)
    out = oracle.decode_batch(a)["out"]
    for s in range(2):
        for i in range(3):
            for h in range(4):
                assert np.array_equal(out[s, i, h], W.bf16_bits_to_f32(v_new[s, i, h // 2]))
    table_check_pins(oracle)


def table_check_pins(oracle):
    """The table check against cases small enough to read off by hand (expected values are literals)."""
    t = np.array([[3, 1, -1, -1],      # L = 20: blocks 0, 1 are looked at, the -1s are not
                  [0, 2, 4, 5],        # L = 64: all four
                  [7, 7, 7, 7]],       # L = 0: nothing is looked at, whatever the row holds
                 dtype=np.int32)
    lens = np.array([20, 64, 0], dtype=np.int32)
    assert oracle.check_tables(t, lens, 16, 6, 64) == (0, (0, -1, -1, 0))
    assert oracle.check_tables(t, lens, 16, 5, 64) == (1, (2, 1, 3, 5))          # id 5 is outside a pool of 5
    assert oracle.check_tables(t, lens, 16, 4, 64) == (2, (2, 1, 2, 4))          # ids 4 and 5; first in block order
    assert oracle.check_tables(t, lens, 16, 6, 63) == (1, (1, 1, -1, 64))        # a length above the bound
    assert oracle.check_tables(t, lens, 16, 4, 63) == (1, (1, 1, -1, 64))        # ... whose blocks are then not looked at
    lens2 = np.array([33, 64, -2], dtype=np.int32)                               # L = 33 reaches the -1 in block 2
    assert oracle.check_tables(t, lens2, 16, 6, 64) == (2, (2, 0, 2, -1))        # and the negative length counts too
    # sliding window: reach 16 on L = 64 looks at blocks 3 only (token 48 on); on L = 20 at blocks 0 and 1 (token 4 on)
    t3 = t.copy()
    t3[1, :3] = 99
    assert oracle.check_tables(t3, lens, 16, 6, 64, reach=16) == (0, (0, -1, -1, 0))
    assert oracle.check_tables(t3, lens, 16, 6, 64, reach=17) == (1, (2, 1, 2, 99))
    # shared prefix of 2 blocks: rows must repeat row 0 there, and every length must cover it
    tp = np.array([[3, 1, 2], [3, 1, 0], [3, 4, 5]], dtype=np.int32)
    lp = np.array([40, 33, 48], dtype=np.int32)
    assert oracle.check_tables(tp, lp, 16, 6, 48, shared_prefix_blocks=2) == (1, (3, 2, 1, 4))
    assert oracle.check_tables(tp, lp, 16, 6, 48, shared_prefix_blocks=3) == (1, (3, 2, 1, 4))   # whole pairs only
    lp[1] = 31
    assert oracle.check_tables(tp, lp, 16, 6, 48, shared_prefix_blocks=2) == (2, (1, 1, -1, 31))
    lp[1] = 34
    assert oracle.check_tables(tp, lp, 16, 6, 48, shared_prefix_blocks=2, q_len=4)[1] == (1, 1, -1, 34)  # 32 + 4 - 1 = 35
    assert oracle.check_tables(tp, lp, 16, 6, 48, shared_prefix_blocks=2, q_len=3)[1] == (3, 2, 1, 4)


def main(so_path):
    from oracle import pa_oracle

    good = pa_oracle.lib()
    other = ctypes.CDLL(so_path)
    for fn in ("pa_oracle_decode", "pa_oracle_verify", "pa_oracle_window", "pa_oracle_e4m3_table",
               "pa_oracle_kv_append", "pa_oracle_check_tables"):
        getattr(other, fn).restype = getattr(good, fn).restype
        getattr(other, fn).argtypes = getattr(good, fn).argtypes
    pa_oracle._lib = other
    core_pins(pa_oracle)


if __name__ == "__main__":
    main(sys.argv[1])
