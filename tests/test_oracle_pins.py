"""Pins that tie the CPU oracle to things other than itself (all CPU, no GPU).

The paper prints no worked numeric example for attention, so the pins are: closed forms
(one token, equal V rows, zero query, two tokens with sigmoid weights), invariants (weights
sum to one, score-shift invariance, physical-block permutation, poison in dead slots),
dense library softmax on gathered matrices (scipy, torch SDPA in float64), a two-segment
log-sum-exp merge identity, and the e4m3 byte table against the format's corner values and
torch's float8_e4m3fn cast.
"""
import math
import os

import numpy as np
import pytest

from paper_2605_06068_amd import workloads as W
from tests.oracle_core_pins import table_check_pins
from tests.dense_reference import dense_attention, dense_window_attention, e4m3_to_f64, torch_sdpa, widen_bf16

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def tiny(seed, lens, Hq=4, Hkv=2, D=64, kv=W.KV_BF16, **kw):
    return W.make_batch("t", seed, lens, Hq, Hkv, D, 16, kv, **kw)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_single_token_returns_v_exactly(oracle, kv):
    b = tiny(11, [1, 1, 1], Hq=8, Hkv=4, D=64, kv=kv, num_blocks=7)
    out = oracle.decode_batch(b)["out"]
    G = b.group
    for s in range(3):
        phys = b.block_tables[s, 0]
        for h in range(8):
            g = h // G
            raw = b.v_cache[phys, g, 0]
            if kv == W.KV_BF16:
                want = W.bf16_bits_to_f32(raw)
            else:
                want = (e4m3_to_f64(raw) * np.float64(b.v_scale[g])).astype(np.float32)
            assert np.array_equal(out[s, h], want)


def test_single_token_heads_map_to_their_kv_head(oracle):
    # V row of KV head g holds the constant g+1: query head h must return (h // G) + 1.
    b = tiny(12, [1], Hq=8, Hkv=4, D=64, table_kind="identity")
    for g in range(4):
        b.v_cache[:, g] = bf16(np.float32(g + 1))
    out = oracle.decode_batch(b)["out"]
    for h in range(8):
        assert np.all(out[0, h] == h // 2 + 1)


def test_equal_v_rows_return_that_row(oracle):
    b = tiny(13, [53, 16, 17])
    row = bf16(np.linspace(-2, 2, 64))
    b.v_cache[:] = row
    out = oracle.decode_batch(b, want_f64=True)["out_f64"]
    want = widen_bf16(row)
    assert np.max(np.abs(out - want)) <= 1e-14 * 4


def test_zero_query_gives_mean_of_v(oracle):
    b = tiny(14, [45, 7])
    b.q[:] = 0
    out = oracle.decode_batch(b, want_f64=True, want_probs=True)
    for s, L in enumerate(b.context_lens):
        for h in range(4):
            t = np.arange(L)
            v = widen_bf16(b.v_cache[b.block_tables[s, t // 16], h // 2, t % 16])
            assert np.allclose(out["out_f64"][s, h], v.mean(axis=0), rtol=0, atol=1e-13)
            assert np.allclose(out["probs"][s, h, :L], 1.0 / L, rtol=1e-13, atol=0)


def test_equal_k_rows_give_uniform_weights(oracle):
    b = tiny(15, [33])
    b.k_cache[:] = bf16(np.random.default_rng(0).standard_normal(64))
    p = oracle.decode_batch(b, want_probs=True)["probs"]
    assert np.allclose(p[0, :, :33], 1.0 / 33, rtol=1e-13, atol=0)
    assert np.all(p[0, :, 33:] == 0)


def test_two_tokens_sigmoid_weights(oracle):
    # scores s0, s1 -> weights sigmoid(s0-s1), sigmoid(s1-s0); q = e_3 * a, k0 = e_3 * c0, k1 = e_3 * c1.
    b = tiny(16, [2], Hq=2, Hkv=1, D=64, table_kind="identity")
    b.q[:] = 0
    b.k_cache[:] = 0
    a, c0, c1 = 3.0, 1.5, -0.25
    b.q[0, :, 3] = bf16(a)
    b.k_cache[0, 0, 0, 3] = bf16(c0)
    b.k_cache[0, 0, 1, 3] = bf16(c1)
    out = oracle.decode_batch(b, want_f64=True, want_probs=True, want_lse=True)
    scale = float(b.scale)  # 1/8 exactly
    s0, s1 = scale * a * c0, scale * a * c1
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    v0 = widen_bf16(b.v_cache[0, 0, 0])
    v1 = widen_bf16(b.v_cache[0, 0, 1])
    assert abs(out["probs"][0, 0, 0] - w0) <= 1e-15
    assert abs(out["probs"][0, 0, 1] - (1 - w0)) <= 1e-15
    assert np.allclose(out["out_f64"][0, 0], w0 * v0 + (1 - w0) * v1, rtol=0, atol=1e-15)
    assert abs(out["lse"][0, 0] - math.log(math.exp(s0) + math.exp(s1))) <= 1e-15


def test_scale_multiplies_the_scores(oracle):
    # doubling the scale equals doubling q (exact in bf16)
    b = tiny(17, [40, 21])
    r1 = oracle.decode(b.q, b.k_cache, b.v_cache, b.block_tables, b.context_lens, np.float32(0.25), want_f64=True)
    q2 = bf16(W.bf16_bits_to_f32(b.q) * 2)
    r2 = oracle.decode(q2, b.k_cache, b.v_cache, b.block_tables, b.context_lens, np.float32(0.125), want_f64=True)
    assert np.allclose(r1["out_f64"], r2["out_f64"], rtol=0, atol=1e-14)
    r3 = oracle.decode(b.q, b.k_cache, b.v_cache, b.block_tables, b.context_lens, np.float32(0.125), want_f64=True)
    assert np.max(np.abs(r1["out_f64"] - r3["out_f64"])) > 1e-3


# ---------------------------------------------------------------- invariants
def test_weights_sum_to_one_and_vanish_past_the_context(oracle):
    b = W.make_config(1)
    p = oracle.decode_batch(b, want_probs=True)["probs"]
    assert np.max(np.abs(p.sum(-1) - 1.0)) <= 1e-12
    for s, L in enumerate(b.context_lens):
        assert np.all(p[s, :, L:] == 0) and np.all(p[s, :, :L] > 0)


def test_adding_a_vector_to_every_k_row_changes_nothing(oracle):
    # integer-valued K, q and u keep every sum exact in bf16 and float64
    rng = np.random.default_rng(18)
    b = tiny(18, [37, 64])
    b.k_cache[:] = bf16(rng.integers(-8, 9, size=b.k_cache.shape))
    b.q[:] = bf16(rng.integers(-2, 3, size=b.q.shape))
    base = oracle.decode_batch(b, want_f64=True)["out_f64"]
    u = rng.integers(-8, 9, size=64).astype(np.float32)
    b.k_cache[:] = bf16(W.bf16_bits_to_f32(b.k_cache) + u)
    moved = oracle.decode_batch(b, want_f64=True)["out_f64"]
    assert np.max(np.abs(moved - base)) <= 1e-12


def test_permuting_physical_blocks_is_bit_identical(oracle):
    b = W.make_config(1)
    base = oracle.decode_batch(b, want_f64=True)["out_f64"]
    perm = np.random.default_rng(19).permutation(b.num_blocks)  # new id of old block i is perm[i]
    k2 = np.empty_like(b.k_cache)
    v2 = np.empty_like(b.v_cache)
    k2[perm] = b.k_cache
    v2[perm] = b.v_cache
    t2 = np.where(b.block_tables >= 0, perm[np.maximum(b.block_tables, 0)], -1).astype(np.int32)
    moved = oracle.decode(b.q, k2, v2, t2, b.context_lens, b.scale, want_f64=True)["out_f64"]
    assert np.array_equal(moved, base)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_dead_slots_and_unused_table_entries_never_matter(oracle, kv):
    lens = [37, 100, 1, 16]
    clean = tiny(20, lens, kv=kv, num_blocks=24, max_blocks_per_seq=9, poison=False)
    dirty = tiny(20, lens, kv=kv, num_blocks=24, max_blocks_per_seq=9, poison=True)
    nan_pat = W.BF16_NAN_BITS if kv == W.KV_BF16 else W.FP8_NAN_BYTE
    assert (dirty.k_cache == nan_pat).any() and not np.array_equal(dirty.k_cache, clean.k_cache)
    dirty.block_tables[dirty.block_tables < 0] = 2 ** 30  # garbage ids past the valid prefix
    a = oracle.decode_batch(clean)["out"]
    d = oracle.decode_batch(dirty)["out"]
    assert np.isfinite(d).all() and np.array_equal(a, d)


def test_zero_length_sequence_gives_zero_row(oracle):
    b = tiny(21, [0, 5, 0], num_blocks=4, max_blocks_per_seq=2)
    r = oracle.decode_batch(b, want_lse=True)
    assert np.all(r["out"][0] == 0) and np.all(r["out"][2] == 0) and np.isfinite(r["out"]).all()
    assert np.all(np.isneginf(r["lse"][0]))


def test_bad_block_id_inside_the_context_is_an_error(oracle):
    b = tiny(22, [20])
    b.block_tables[0, 1] = b.num_blocks
    with pytest.raises(RuntimeError):
        oracle.decode_batch(b)


# ---------------------------------------------------------------- dense library references
@pytest.mark.parametrize("case", [
    dict(seed=1001, config=1),
    dict(seed=31, lens=[1, 15, 16, 17, 255], Hq=8, Hkv=2, D=128),
    dict(seed=32, lens=[64, 3], Hq=6, Hkv=6, D=64),
    dict(seed=33, lens=[200], Hq=8, Hkv=1, D=128, sigma=2.0),
    dict(seed=34, lens=[77, 130], Hq=16, Hkv=2, D=128, kv=W.KV_FP8_E4M3),
])
def test_matches_dense_softmax_from_scipy_and_torch(oracle, case):
    case = dict(case)
    if "config" in case:
        b = W.make_config(case["config"], seed=case["seed"])
    else:
        b = tiny(case.pop("seed"), case.pop("lens"), **case)
    r = oracle.decode_batch(b, want_f64=True, want_lse=True)
    want, want_lse = dense_attention(b)
    assert np.max(np.abs(r["out_f64"] - want)) <= 1e-12
    assert np.max(np.abs(r["lse"] - want_lse)) <= 1e-12
    assert np.max(np.abs(r["out_f64"] - torch_sdpa(b))) <= 1e-10
    # the float32 result is the float64 one rounded once
    assert np.array_equal(r["out"], r["out_f64"].astype(np.float32))


def test_row_selection_equals_full_run(oracle):
    b = W.make_config(1)
    full = oracle.decode_batch(b)["out"]
    rows = [(1, 3), (0, 0), (1, 0)]
    sel = oracle.decode_batch(b, rows=rows)["out"]
    for i, (s, h) in enumerate(rows):
        assert np.array_equal(sel[i], full[s, h])


def test_two_segment_log_sum_exp_merge_identity(oracle):
    """Attention over [0,L) equals the LSE-weighted merge of attention over [0,m) and [m,L),
    for every m that is a multiple of the block size: the identity split-K relies on."""
    b = tiny(40, [100], Hq=4, Hkv=2, D=64, table_kind="permuted")
    whole = oracle.decode_batch(b, want_f64=True)["out_f64"][0]
    L = 100
    for m in range(16, L, 16):
        left = oracle.decode(b.q, b.k_cache, b.v_cache, b.block_tables, np.array([m], np.int32), b.scale,
                             want_f64=True, want_lse=True)
        t_right = np.full_like(b.block_tables, -1)
        nb = b.block_tables.shape[1] - m // 16
        t_right[0, :nb] = b.block_tables[0, m // 16:]
        right = oracle.decode(b.q, b.k_cache, b.v_cache, t_right, np.array([L - m], np.int32), b.scale,
                              want_f64=True, want_lse=True)
        la, lb = left["lse"][0][:, None], right["lse"][0][:, None]
        mx = np.maximum(la, lb)
        wa, wb = np.exp(la - mx), np.exp(lb - mx)
        merged = (wa * left["out_f64"][0] + wb * right["out_f64"][0]) / (wa + wb)
        assert np.max(np.abs(merged - whole)) <= 1e-12


# ---------------------------------------------------------------- multi-token window (verification)
def test_window_closed_forms_two_tokens(oracle):
    """L = Q = 2: query 0 sees only token 0 and returns its V row exactly; query 1 sees both tokens
    with sigmoid weights of the score difference."""
    D = 64
    b = tiny(50, [2], Hq=2, Hkv=1, D=D, table_kind="identity", q_len=2)
    q = widen_bf16(b.q)[0]                       # [Q, Hq, D]
    K = widen_bf16(b.k_cache[0, 0, :2])          # [2, D]
    V = widen_bf16(b.v_cache[0, 0, :2])
    r = oracle.decode_batch(b, want_f64=True)["out_f64"][0]
    for h in range(2):
        assert np.array_equal(r[0, h], V[0])
        s = (K @ q[1, h]) * np.float64(b.scale)
        w1 = 1.0 / (1.0 + math.exp(s[0] - s[1]))
        assert np.max(np.abs(r[1, h] - ((1 - w1) * V[0] + w1 * V[1]))) <= 1e-14


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_window_row_equals_plain_decode_of_the_truncated_context(oracle, kv):
    """Query token i of a window is ordinary decode attention over the first L - Q + 1 + i tokens."""
    Q = 5
    b = tiny(51, [3, 5, 40, 100], Hq=4, Hkv=2, D=64, kv=kv, q_len=Q)
    win = oracle.decode_batch(b, want_f64=True, want_lse=True)
    for i in range(Q):
        lens = np.maximum(b.context_lens - (Q - 1 - i), 0).astype(np.int32)
        one = oracle.decode(np.ascontiguousarray(b.q[:, i]), b.k_cache, b.v_cache, b.block_tables, lens, b.scale,
                            kv, b.k_scale, b.v_scale, want_f64=True, want_lse=True)
        assert np.array_equal(win["out_f64"][:, i], one["out_f64"])
        assert np.array_equal(win["lse"][:, i], one["lse"])
    # sequence 0 has 3 tokens for a window of 5: the first two query tokens see nothing
    assert np.all(win["out"][0, :2] == 0) and np.any(win["out"][0, 2] != 0)


@pytest.mark.parametrize("case", [
    dict(seed=52, lens=[1, 16, 17, 33, 255], Hq=8, Hkv=2, D=128, q_len=4),
    dict(seed=53, lens=[64, 7], Hq=6, Hkv=6, D=64, q_len=16),
    dict(seed=54, lens=[77, 130], Hq=16, Hkv=2, D=128, kv=W.KV_FP8_E4M3, q_len=3),
])
def test_window_matches_masked_library_attention(oracle, case):
    case = dict(case)
    b = tiny(case.pop("seed"), case.pop("lens"), **case)
    r = oracle.decode_batch(b, want_f64=True)
    assert r["out"].shape == b.q.shape
    assert np.max(np.abs(r["out_f64"] - dense_window_attention(b))) <= 1e-10
    assert np.array_equal(r["out"], r["out_f64"].astype(np.float32))


def test_window_is_causal_later_tokens_never_reach_earlier_queries(oracle):
    Q = 4
    b = tiny(55, [50], Hq=4, Hkv=2, D=64, table_kind="identity", q_len=Q)
    base = oracle.decode_batch(b, want_f64=True, want_probs=True)
    # weights of query i vanish beyond token L - Q + i and sum to one before it
    L = 50
    for i in range(Q):
        p = base["probs"][0, i]
        assert np.all(p[:, L - Q + i + 1:] == 0) and np.all(p[:, L - Q + i] > 0)
        assert np.max(np.abs(p.sum(-1) - 1)) <= 1e-14
    # overwrite K and V of the last window token (position 49 = block 3, slot 1) with other values
    b.k_cache[3, :, 1] = bf16(np.float32(3.0))
    b.v_cache[3, :, 1] = bf16(np.float32(-7.0))
    again = oracle.decode_batch(b, want_f64=True)
    assert np.array_equal(again["out_f64"][0, :Q - 1], base["out_f64"][0, :Q - 1])
    assert not np.array_equal(again["out_f64"][0, Q - 1], base["out_f64"][0, Q - 1])


def test_window_row_selection_and_single_token_window(oracle):
    b = tiny(56, [37, 100], q_len=3)
    full = oracle.decode_batch(b)["out"]
    rows = [(1, 2, 3), (0, 0, 0), (1, 0, 1)]
    sel = oracle.decode_batch(b, rows=rows)["out"]
    for n, (s, i, h) in enumerate(rows):
        assert np.array_equal(sel[n], full[s, i, h])
    # a window of one token is plain decode
    c = W.make_config(1)
    one = oracle.verify(c.q[:, None], c.k_cache, c.v_cache, c.block_tables, c.context_lens, c.scale)["out"]
    assert np.array_equal(one[:, 0], oracle.decode_batch(c)["out"])


# ---------------------------------------------------------------- sliding window
def test_sliding_window_of_one_returns_the_own_value_row(oracle):
    b = tiny(60, [1, 16, 17, 100], Hq=4, Hkv=2, D=64, q_len=3, window=1, poison=False)
    out = oracle.decode_batch(b, want_f64=True)["out_f64"]
    for s, L in enumerate(b.context_lens):
        for i in range(3):
            t = L - 3 + i
            for h in range(4):
                want = widen_bf16(b.v_cache[b.block_tables[s, t // 16], h // 2, t % 16]) if t >= 0 else np.zeros(64)
                assert np.array_equal(out[s, i, h], want)


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_sliding_window_wider_than_the_context_changes_nothing(oracle, kv):
    b = tiny(61, [5, 37, 100], kv=kv, q_len=2)
    free = oracle.decode_batch(b, want_f64=True, want_lse=True)
    b.window = 100  # the latest query sits at position 99 and sees 0 .. 99
    same = oracle.decode_batch(b, want_f64=True, want_lse=True)
    assert np.array_equal(free["out_f64"], same["out_f64"]) and np.array_equal(free["lse"], same["lse"])
    b.window = 99
    cut = oracle.decode_batch(b, want_f64=True)
    assert np.array_equal(cut["out_f64"][:2], free["out_f64"][:2])        # shorter contexts: still everything
    assert np.array_equal(cut["out_f64"][2, 0], free["out_f64"][2, 0])    # position 98 sees 0 .. 98
    assert not np.array_equal(cut["out_f64"][2, 1], free["out_f64"][2, 1])  # position 99 lost token 0


@pytest.mark.parametrize("case", [
    dict(seed=62, lens=[1, 16, 17, 33, 255], Hq=8, Hkv=2, D=128, q_len=1, window=20),
    dict(seed=63, lens=[64, 7, 300], Hq=6, Hkv=6, D=64, q_len=5, window=33),
    dict(seed=64, lens=[77, 130], Hq=16, Hkv=2, D=128, kv=W.KV_FP8_E4M3, q_len=3, window=16),
])
def test_sliding_window_matches_masked_library_attention(oracle, case):
    """The generator evicts what lies before the earliest window (table entries -1, NaN patterns in
    the slots): the result must be finite and equal the library's attention under the band mask."""
    case = dict(case)
    b = tiny(case.pop("seed"), case.pop("lens"), **case)
    r = oracle.decode_batch(b, want_f64=True, want_probs=True)
    assert np.isfinite(r["out_f64"]).all()
    q4 = b.q if b.q.ndim == 4 else b.q[:, None]
    view = type("V", (), dict(vars(b), q=q4))()
    want = dense_window_attention(view, sliding=b.window)
    got = r["out_f64"] if b.q.ndim == 4 else r["out_f64"][:, None]
    assert np.max(np.abs(got - want)) <= 1e-10
    probs = r["probs"] if b.q.ndim == 4 else r["probs"][:, None]
    for s, L in enumerate(b.context_lens):
        for i in range(b.q_len):
            pos = L - b.q_len + i
            lo = max(0, pos - b.window + 1)
            if pos >= 0:
                assert np.all(probs[s, i][:, :lo] == 0) and np.all(probs[s, i][:, pos + 1:] == 0)
                assert np.all(probs[s, i][:, lo:pos + 1] > 0)


def test_sliding_window_blocks_and_plan(oracle):
    lens = np.array([100, 40, 3, 0, 1000, 31, 32, 33], np.int32)
    tables = np.arange(8 * 64, dtype=np.int32).reshape(8, 64)
    for reach in (1, 16, 17, 50, 2000):
        for s, L in enumerate(lens):
            first, ids = oracle.window_blocks(tables, lens, 16, s, reach)
            t_first = max(0, int(L) - reach)
            want = [tables[s, j] for j in range(64) if j * 16 < L and (j + 1) * 16 > t_first]
            assert list(ids) == want and (not want or first == t_first // 16)
        for P in (1, 3, 8):
            T, owner = oracle.block_partition(lens, 64, 16, P, reach=reach)
            tiles = [sum(1 for i in range(0, int(L), 32) if i + 32 > max(0, int(L) - reach)) for L in lens]
            assert T == sum(tiles)
            flat = []
            for s, L in enumerate(lens):
                t_first = max(0, int(L) - reach)
                for j in range(64):
                    live = j * 16 < L and (j + 1) * 16 > t_first
                    assert (owner[s, j] >= 0) == live
                    if live:
                        flat.append(owner[s, j])
            assert all(a <= b for a, b in zip(flat, flat[1:]))
            counts = np.bincount([owner[s, 2 * i] if owner[s, 2 * i] >= 0 else owner[s, 2 * i + 1]
                                  for s, L in enumerate(lens) for i in range(32)
                                  if max(owner[s, 2 * i], owner[s, 2 * i + 1]) >= 0], minlength=P)
            assert counts.max() - counts.min() <= 1
    T0, owner0 = oracle.block_partition(lens, 64, 16, 5)
    T1, owner1 = oracle.block_partition(lens, 64, 16, 5, reach=10 ** 6)
    assert T0 == T1 and np.array_equal(owner0, owner1)


# ---------------------------------------------------------------- fp8 table
def test_e4m3_table_corner_values_and_torch_cast(oracle):
    t = oracle.e4m3_table()
    assert t[0x00] == 0.0 and t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9
    assert t[0x08] == 2.0 ** -6 and t[0x38] == 1.0 and t[0x40] == 2.0 and t[0x7E] == 448.0
    assert math.isnan(t[0x7F]) and math.isnan(t[0xFF])
    assert np.array_equal(t[0x80:0xFF], -t[0x00:0x7F]) and np.signbit(t[0x80])
    lib = e4m3_to_f64(np.arange(256, dtype=np.uint8))
    ok = ~np.isnan(lib)
    assert ok.sum() == 254 and np.array_equal(t[ok], lib[ok]) and np.isnan(t[~ok]).all()


def test_fp8_scales_belong_to_their_kv_head(oracle):
    # identical bytes in every head, distinct scales: outputs must scale with v_scale[h // G]
    b = tiny(41, [1], Hq=4, Hkv=2, D=64, kv=W.KV_FP8_E4M3, table_kind="identity")
    b.v_cache[:, 1] = b.v_cache[:, 0]
    b.v_scale[:] = [0.5, 3.0]
    out = oracle.decode_batch(b)["out"]
    assert np.array_equal(out[0, 2], out[0, 0] * 6) and np.array_equal(out[0, 3], out[0, 1] * 6)
    # k_scale scales the scores: a huge K scale on head 1 turns its softmax into an argmax
    b = tiny(42, [30], Hq=4, Hkv=2, D=64, kv=W.KV_FP8_E4M3)
    b.k_scale[:] = [1e-6, 50.0]
    p = oracle.decode_batch(b, want_probs=True)["probs"][0]
    assert np.allclose(p[0, :30], 1 / 30, rtol=1e-3) and p[2, :30].max() > 0.99


# ---------------------------------------------------------------- KV append
def test_e4m3_encoder_matches_torch_cast_and_the_format_rules(oracle):
    import torch

    rng = np.random.default_rng(50)
    xs = np.concatenate([
        rng.standard_normal(2000).astype(np.float32) * np.float32(3.0),
        (rng.standard_normal(500) * 100).astype(np.float32),
        (rng.standard_normal(500) * 2.0 ** -7).astype(np.float32),
        np.array([0.0, -0.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 5 * 2.0 ** -10, 1.0625, 1.1875, 447.9, 448.0, -448.0,
                  463.9], dtype=np.float32),
    ])
    inside = np.abs(xs) < 464  # torch's cast has no saturation: beyond this it returns NaN
    want = torch.from_numpy(xs[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(x) for x in xs[inside]], dtype=np.uint8)
    assert np.array_equal(got, want)
    # saturation and sign, by the rule itself
    assert oracle.e4m3_encode(464.0) == 0x7E and oracle.e4m3_encode(1e30) == 0x7E and oracle.e4m3_encode(-1e30) == 0xFE
    # decode(encode(v)) == v for every finite code value
    t = oracle.e4m3_table()
    for code in range(256):
        if not math.isnan(t[code]):
            assert oracle.e4m3_encode(t[code]) == code


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_kv_append_writes_exactly_the_last_slot(oracle, kv):
    rng = np.random.default_rng(51)
    b = tiny(51, [17, 0, 32, 1, 100], Hq=4, Hkv=2, D=64, kv=kv, poison=False)
    k0, v0 = b.k_cache.copy(), b.v_cache.copy()
    k_new = bf16(rng.standard_normal((5, 2, 64)))
    v_new = bf16(rng.standard_normal((5, 2, 64)))
    oracle.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.context_lens, kv, b.k_scale, b.v_scale)
    changed = np.zeros(b.k_cache.shape[:3], dtype=bool)
    for s, L in enumerate(b.context_lens):
        if L <= 0:
            continue
        phys, slot = b.block_tables[s, (L - 1) // 16], (L - 1) % 16
        changed[phys, :, slot] = True
        for g in range(2):
            if kv == W.KV_BF16:
                assert np.array_equal(b.k_cache[phys, g, slot], k_new[s, g])
                assert np.array_equal(b.v_cache[phys, g, slot], v_new[s, g])
            else:
                kq = W.bf16_bits_to_f32(k_new[s, g]) / np.float32(b.k_scale[g])
                vq = W.bf16_bits_to_f32(v_new[s, g]) / np.float32(b.v_scale[g])
                assert np.array_equal(b.k_cache[phys, g, slot], W.f32_to_e4m3_bytes(kq))
                assert np.array_equal(b.v_cache[phys, g, slot], W.f32_to_e4m3_bytes(vq))
    assert np.array_equal(b.k_cache[~changed], k0[~changed]) and np.array_equal(b.v_cache[~changed], v0[~changed])
    # appended rows are what the attention oracle then sees at position L-1
    out = oracle.decode_batch(b, want_probs=True)
    assert np.isfinite(out["out"]).all()


@pytest.mark.parametrize("kv", [W.KV_BF16, W.KV_FP8_E4M3])
def test_kv_append_of_a_window_equals_token_by_token_appends(oracle, kv):
    """Appending Q tokens at once writes exactly what Q single-token appends write while the context
    grows to the same length; tokens that would land before position 0 are dropped."""
    rng = np.random.default_rng(52)
    Q = 5
    lens = np.array([17, 0, 32, 3, 100, 5], dtype=np.int32)  # one context shorter than the window
    b = tiny(52, lens.tolist(), Hq=4, Hkv=2, D=64, kv=kv, poison=False)
    k_new = bf16(rng.standard_normal((6, Q, 2, 64)))
    v_new = bf16(rng.standard_normal((6, Q, 2, 64)))
    k0, v0 = b.k_cache.copy(), b.v_cache.copy()
    oracle.kv_append(k_new, v_new, b.k_cache, b.v_cache, b.block_tables, b.context_lens, kv, b.k_scale, b.v_scale)
    k1, v1 = k0.copy(), v0.copy()
    for i in range(Q):
        step_lens = lens - (Q - 1 - i)            # the context after token i of the window
        oracle.kv_append(np.ascontiguousarray(k_new[:, i]), np.ascontiguousarray(v_new[:, i]), k1, v1, b.block_tables,
                         np.maximum(step_lens, 0).astype(np.int32), kv, b.k_scale, b.v_scale)
    assert np.array_equal(b.k_cache, k1) and np.array_equal(b.v_cache, v1)
    # sequence 3 (3 tokens, window of 5): only the last 3 window tokens exist, at positions 0..2
    phys = b.block_tables[3, 0]
    if kv == W.KV_BF16:
        assert np.array_equal(b.k_cache[phys, :, :3], np.swapaxes(k_new[3, 2:], 0, 1))
    assert np.array_equal(b.k_cache[phys, :, 3:], k0[phys, :, 3:])
    # the empty sequence got nothing
    assert (b.k_cache != k0).any() and np.array_equal(b.block_tables[1], np.full_like(b.block_tables[1], -1))


# ---------------------------------------------------------------- indexing helpers
def test_visited_blocks_follow_the_table(oracle):
    b = W.make_config(1)
    assert oracle.visited_blocks(b.block_tables, b.context_lens, 16, 0).tolist() == b.block_tables[0, :3].tolist()
    assert oracle.visited_blocks(b.block_tables, b.context_lens, 16, 1).tolist() == b.block_tables[1, :7].tolist()


def test_check_tables_hand_cases(oracle):
    table_check_pins(oracle)


def test_check_tables_finds_planted_faults(oracle):
    """A clean generated table passes; one entry spoiled at a place the test chooses is reported at
    exactly that place; entries the attention never looks at may hold anything."""
    rng = np.random.default_rng(11)
    b = W.make_config(4, length_scale=1 / 8)
    t, lens, NB = b.block_tables, b.context_lens, b.num_blocks
    top = int(lens.max())
    assert oracle.check_tables(t, lens, 16, NB, top) == (0, (0, -1, -1, 0))
    for bad in (-1, NB, 2 ** 30, -2 ** 31):
        s = int(rng.integers(0, b.batch))
        j = int(rng.integers(0, (int(lens[s]) + 15) // 16))
        spoiled = t.copy()
        spoiled[s, j] = bad
        assert oracle.check_tables(spoiled, lens, 16, NB, top) == (1, (2, s, j, bad))
        spoiled[s, (int(lens[s]) + 15) // 16:] = bad   # behind the context: never looked at
        assert oracle.check_tables(spoiled, lens, 16, NB, top)[0] == 1
    two = t.copy()
    two[5, 0] = NB
    two[2, 0] = -5
    assert oracle.check_tables(two, lens, 16, NB, top) == (2, (2, 2, 0, -5))


def test_block_partition_is_a_balanced_contiguous_cut(oracle):
    """Properties the split plan's definition fixes, checked without re-using its formula: every
    valid block has exactly one owner, owners never decrease along the batch's token order, both
    blocks of a 32-token tile share an owner, and the tile counts of the partitions differ by at
    most one (floor(k*T/P) cuts)."""
    rng = np.random.default_rng(5)
    for lens in ([37, 100], [0, 5, 0, 700, 16, 1], rng.integers(1, 3000, size=40).tolist(), [5000], [0, 0]):
        lens = np.asarray(lens, dtype=np.int32)
        MB = int(max(1, -(-int(lens.max()) // 16))) + 2
        for P in (1, 2, 3, 7, 64, 1000):
            T, owner = oracle.block_partition(lens, MB, 16, P)
            assert T == sum(-(-int(L) // 32) for L in lens if L > 0)
            seq = []
            for bi, L in enumerate(lens):
                nblk = -(-int(L) // 16) if L > 0 else 0
                assert np.all(owner[bi, nblk:] == -1) and np.all(owner[bi, :nblk] >= 0)
                row = owner[bi, :nblk]
                assert np.all(row[0::2][:len(row[1::2])] == row[1::2])  # tile = two blocks, one owner
                seq.extend(row[0::2].tolist())  # one entry per tile
            assert len(seq) == T and all(x <= y for x, y in zip(seq, seq[1:])) and all(0 <= x < P for x in seq)
            counts = np.bincount(np.asarray(seq, dtype=np.int64), minlength=P) if T else np.zeros(P, int)
            assert counts.max() - counts.min() <= 1 and counts.sum() == T
            if T:
                # closed form of the first and last cut
                assert counts[P - 1] == T - (P - 1) * T // P and counts[0] == T // P


# ---------------------------------------------------------------- stored regression values
def test_config1_golden_values(oracle):
    """Values written by tests/golden/make_golden.py (which calls only the oracle)."""
    want = np.loadtxt(os.path.join(GOLDEN, "config1_seed1001_out.txt"))
    b = W.make_config(1)
    got = oracle.decode_batch(b, want_f64=True)["out_f64"].reshape(-1, 64)
    assert np.max(np.abs(got - want)) <= 1e-15
