"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, plans splits as the definition says, and rejects bad arguments before any
launch."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_06068_amd import binding as pa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def shape(**kw):
    base = dict(batch=4, num_q_heads=32, num_kv_heads=8, head_dim=128, block_size=16, max_blocks_per_seq=256,
                num_blocks=1024, max_context_len=0, num_partitions=0, q_len=0, shared_prefix_blocks=0, window=0, out_dtype=0,
                precise_weights=0)
    base.update(kw)
    return pa.make_shape(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pa_decode.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pa_[a-z_0-9]+)\s*\(", header))
    assert declared == set(pa.EXPORTS), declared ^ set(pa.EXPORTS)
    L = pa.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    assert pa.status_string(pa.PA_OK) == "PA_OK"
    assert pa.status_string(pa.PA_ERR_WORKSPACE_TOO_SMALL) == "PA_ERR_WORKSPACE_TOO_SMALL"
    assert pa.status_string(77) == "PA_ERR_UNKNOWN"


def test_shape_struct_matches_header_field_order():
    header = open(os.path.join(ROOT, "include", "pa_decode.h")).read()
    body = re.search(r"typedef struct pa_shape \{(.*?)\} pa_shape;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"int32_t\s+([a-z_]+);", body)
    assert fields == [f[0] for f in pa.pa_shape._fields_]
    assert ctypes.sizeof(pa.pa_shape) == 4 * len(fields)


@pytest.mark.parametrize("kv", [pa.PA_KV_BF16, pa.PA_KV_FP8_E4M3])
def test_split_plan_is_the_definition(oracle, kv):
    rng = np.random.default_rng(3)
    for B, lens in ((4, [0, 1, 4096, 33]), (4, [4096] * 4), (4, [31, 32, 33, 64]), (64, rng.integers(1, 4097, 64)),
                    (3, [0, 0, 0])):
        for forced in [0, 1, 2, 3, 7, 64, 1000]:
            s = shape(batch=B, num_partitions=forced)
            P = pa.pa_num_partitions(s, kv)
            assert P >= 1 and (forced == 0 or P == forced)
            T, plan = pa.pa_split_plan(s, kv, lens)
            To, want = oracle.block_partition(np.asarray(lens, np.int32), 256, 16, P)
            assert T == To and np.array_equal(plan, want)


def test_partition_count_depends_on_host_shape_only():
    a = pa.pa_num_partitions(shape(max_context_len=4096), pa.PA_KV_BF16)
    b = pa.pa_num_partitions(shape(max_context_len=4096), pa.PA_KV_BF16)
    assert a == b and a >= 1
    # never more partitions than there can be tiles; a single partition needs no workspace
    s1 = shape(batch=1, max_context_len=32)
    assert pa.pa_num_partitions(s1, pa.PA_KV_BF16) == 1 and pa.pa_decode_workspace_size(s1, pa.PA_KV_BF16) == 0
    assert pa.pa_num_partitions(shape(batch=2, max_context_len=96), pa.PA_KV_BF16) <= 6


def test_workspace_size_covers_partials():
    s = shape(num_partitions=16)
    need = 2 * 16 * 32 * (128 + 1) * 4 + 4 * 16 + 16 * 4  # partials + 16 bytes per sequence and 4 per partition for the merge
    got = pa.pa_decode_workspace_size(s, pa.PA_KV_BF16)
    assert need <= got <= need + 4 * 256


def test_query_window_scales_the_workspace_and_leaves_the_plan_alone():
    one = shape(num_partitions=16)
    # 128 columns per KV head: the stage-split workgroup at head_dim 128, unless the weights keep their low part
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=16), pa.PA_KV_FP8_E4M3) == "mfma-staged"
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=16), pa.PA_KV_BF16) == "mfma-wide"  # bf16: up to 64 columns
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=8), pa.PA_KV_BF16) == "mfma-staged"
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=16, precise_weights=1), pa.PA_KV_BF16) == "mfma-wide"
    # head_dim 64: bf16 up to 128 columns (its tiles are half as large), fp8 up to 64
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=16, head_dim=64), pa.PA_KV_BF16) == "mfma-staged"
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=16, head_dim=64), pa.PA_KV_FP8_E4M3) == "mfma-wide"
    assert pa.pa_kernel_variant(shape(num_q_heads=64, q_len=8, head_dim=64), pa.PA_KV_FP8_E4M3) == "mfma-staged"
    for Q in (2, 4, 16):
        win = shape(num_partitions=16, q_len=Q)
        assert pa.pa_kernel_variant(win, pa.PA_KV_BF16) == ("mfma" if Q * 4 <= 32 else "mfma-staged")  # 512 tiles, 16 partitions
        need = 2 * 16 * Q * 32 * (128 + 1) * 4 + 4 * 16 + 16 * 4
        assert need <= pa.pa_decode_workspace_size(win, pa.PA_KV_BF16) <= need + 4 * 256
        lens = [100, 4096, 1, 33]
        assert pa.pa_split_plan(win, pa.PA_KV_BF16, lens)[0] == pa.pa_split_plan(one, pa.PA_KV_BF16, lens)[0]
        assert np.array_equal(pa.pa_split_plan(win, pa.PA_KV_BF16, lens)[1], pa.pa_split_plan(one, pa.PA_KV_BF16, lens)[1])
    # q_len 0 and 1 are the same call
    assert pa.pa_decode_workspace_size(shape(q_len=1), pa.PA_KV_BF16) == pa.pa_decode_workspace_size(shape(), pa.PA_KV_BF16)
    # up to 32 columns per KV head: one wave per (partition, KV head), narrow groups and head_dim 64 included
    assert pa.pa_kernel_variant(shape(num_q_heads=8, q_len=2), pa.PA_KV_BF16) == "mfma"
    assert pa.pa_kernel_variant(shape(num_q_heads=8), pa.PA_KV_BF16) == "mfma"
    assert pa.pa_kernel_variant(shape(num_q_heads=16, head_dim=64), pa.PA_KV_BF16) == "mfma"
    # 17 .. 32 columns: two column tiles in one wave when every partition has a long run of tiles (here: at
    # most 128 tiles per sequence and 256 partitions of the full device), else two score and two value waves
    big = dict(batch=64, num_q_heads=16, head_dim=64, q_len=16)
    assert pa.pa_kernel_variant(shape(**big), pa.PA_KV_FP8_E4M3) == "mfma"
    assert pa.pa_kernel_variant(shape(**dict(big, batch=4)), pa.PA_KV_FP8_E4M3) == "mfma-staged"
    assert pa.pa_kernel_variant(shape(**dict(big, batch=4, num_partitions=8)), pa.PA_KV_FP8_E4M3) == "mfma"
    assert pa.pa_kernel_variant(shape(**dict(big, head_dim=128)), pa.PA_KV_FP8_E4M3) == "mfma-staged"  # fp8 at head_dim 128: two score and two value waves
    assert pa.pa_kernel_variant(shape(**dict(big, head_dim=128)), pa.PA_KV_BF16) == "mfma"
    assert pa.pa_kernel_variant(shape(num_q_heads=24, head_dim=64, q_len=16), pa.PA_KV_FP8_E4M3) == "mfma-staged"  # 48


@pytest.mark.parametrize("Q,window", [(1, 1), (1, 16), (1, 100), (4, 33), (16, 5), (1, 10 ** 6)])
def test_sliding_window_split_plan_is_the_definition(oracle, Q, window):
    rng = np.random.default_rng(window + Q)
    for lens in ([0, 1, 4096, 33], [31, 32, 33, 64], rng.integers(1, 4097, 64).tolist()):
        for forced in (0, 1, 3, 64):
            s = shape(batch=len(lens), num_partitions=forced, q_len=Q, window=window)
            P = pa.pa_num_partitions(s, pa.PA_KV_BF16)
            T, plan = pa.pa_split_plan(s, pa.PA_KV_BF16, lens)
            To, want = oracle.block_partition(np.asarray(lens, np.int32), 256, 16, P, reach=window + Q - 1)
            assert T == To and np.array_equal(plan, want)
    # a window bounds the tiles a sequence can contribute, hence the partition count
    few = pa.pa_num_partitions(shape(batch=2, window=40), pa.PA_KV_BF16)
    assert few <= 2 * 3


def test_shared_prefix_plan_and_workspace():
    B, Hq, D, prefix_blocks = 4, 32, 128, 9          # 9 blocks: 4 whole tiles are shared, the 9th block is not
    lens = [144, 145, 400, 1000]
    for forced in (0, 1, 3, 5):
        s = shape(batch=B, shared_prefix_blocks=prefix_blocks, num_partitions=forced)
        P = pa.pa_num_partitions(s, pa.PA_KV_BF16)
        T, plan = pa.pa_split_plan(s, pa.PA_KV_BF16, lens)
        tiles = [-(-L // 32) - 4 for L in lens]
        assert T == sum(tiles)
        # the prefix blocks: the same range id in every row, ranges balanced over the 4 prefix tiles
        assert np.all(plan[:, :8] <= -2) and np.all(plan[:, :8] == plan[0, :8])
        ranges = -2 - plan[0, :8:2]
        assert np.array_equal(plan[0, :8:2], plan[0, 1:8:2]) and ranges[0] == 0 and np.all(np.diff(ranges) >= 0)
        Pp = ranges[-1] + 1
        assert 1 <= Pp <= 4 and sorted(set(ranges)) == list(range(Pp))
        # the rest: a balanced cut of the remaining tiles in batch order
        t = 0
        for b, L in enumerate(lens):
            nblk = -(-L // 16)
            for lt in range(4, 4 + tiles[b]):
                k = plan[b, 2 * lt]
                assert (k * T) // P <= t < ((k + 1) * T) // P
                if 2 * lt + 1 < nblk:
                    assert plan[b, 2 * lt + 1] == k
                t += 1
            assert np.all(plan[b, nblk:] == -1)
        # partials of the rest (+ 16 bytes per sequence for the merge) + one result per row from the
        # per-sequence pass + Pp partial results over the prefix
        need = (0 if P == 1 else 2 * P * Hq * (D + 1) * 4 + B * 16 + P * 4) + B * Hq * (D + 1) * 4 + Pp * B * Hq * (D + 1) * 4
        got = pa.pa_decode_workspace_size(s, pa.PA_KV_BF16)
        assert need <= got <= need + 8 * 256
    with pytest.raises(pa.PaError):  # a context that ends inside the shared prefix
        pa.pa_split_plan(shape(batch=B, shared_prefix_blocks=prefix_blocks), pa.PA_KV_BF16, [144, 100, 400, 1000])
    # one shared block is less than a tile: the call is the plain one
    s1 = shape(batch=B, shared_prefix_blocks=1)
    assert pa.pa_decode_workspace_size(s1, pa.PA_KV_BF16) == pa.pa_decode_workspace_size(shape(batch=B), pa.PA_KV_BF16)
    # under a sliding window the promise goes unused: plan, partitions and workspace of the windowed call
    # without it, and none of its conditions (a context may end inside the prefix, any column count)
    for extra in (dict(), dict(q_len=4), dict(q_len=64)):
        sw = shape(batch=B, window=100, shared_prefix_blocks=prefix_blocks, **extra)
        s0 = shape(batch=B, window=100, **extra)
        for kv in (pa.PA_KV_BF16, pa.PA_KV_FP8_E4M3):
            assert pa.pa_num_partitions(sw, kv) == pa.pa_num_partitions(s0, kv)
            assert pa.pa_decode_workspace_size(sw, kv) == pa.pa_decode_workspace_size(s0, kv)
            assert pa.pa_kernel_variant(sw, kv) == pa.pa_kernel_variant(s0, kv)
        Tw, planw = pa.pa_split_plan(sw, pa.PA_KV_BF16, [144, 100, 400, 1000])
        T0, plan0 = pa.pa_split_plan(s0, pa.PA_KV_BF16, [144, 100, 400, 1000])
        assert Tw == T0 and np.array_equal(planw, plan0) and np.all(planw > -2)


def test_split_plan_rejects_lengths_above_the_bound():
    s = shape(max_context_len=100)
    with pytest.raises(pa.PaError):
        pa.pa_split_plan(s, pa.PA_KV_BF16, [1, 2, 101, 4])


@pytest.mark.parametrize("bad,code", [
    (dict(num_q_heads=30), pa.PA_ERR_INVALID_ARG),
    (dict(batch=-1), pa.PA_ERR_INVALID_ARG),
    (dict(max_context_len=256 * 16 + 1), pa.PA_ERR_INVALID_ARG),
    (dict(num_partitions=-3), pa.PA_ERR_INVALID_ARG),
    (dict(num_partitions=70000), pa.PA_ERR_UNSUPPORTED),
    (dict(batch=70000, max_context_len=64), pa.PA_ERR_UNSUPPORTED),
    (dict(head_dim=96), pa.PA_ERR_UNSUPPORTED),
    (dict(block_size=32), pa.PA_ERR_UNSUPPORTED),
    (dict(num_q_heads=8 * 513), pa.PA_ERR_UNSUPPORTED),                  # more than 512 query heads per KV head
    (dict(q_len=-1), pa.PA_ERR_INVALID_ARG),
    (dict(q_len=513, num_q_heads=8), pa.PA_ERR_UNSUPPORTED),
    (dict(q_len=129), pa.PA_ERR_UNSUPPORTED),                            # 129 tokens x 4 heads > 512 columns
    (dict(q_len=16, num_q_heads=8 * 33), pa.PA_ERR_UNSUPPORTED),        # 16 tokens x 33 heads > 512 columns per KV head
    (dict(q_len=2, num_q_heads=8 * 257), pa.PA_ERR_UNSUPPORTED),
    (dict(shared_prefix_blocks=-2), pa.PA_ERR_INVALID_ARG),
    (dict(shared_prefix_blocks=257), pa.PA_ERR_INVALID_ARG),              # more than a table row holds
    (dict(shared_prefix_blocks=8, max_context_len=100), pa.PA_ERR_INVALID_ARG),  # contexts shorter than the prefix
    (dict(shared_prefix_blocks=8, q_len=33), pa.PA_ERR_UNSUPPORTED),             # more than 128 columns
    (dict(shared_prefix_blocks=8, q_len=4, max_context_len=130), pa.PA_ERR_INVALID_ARG),  # a query token inside the prefix
    (dict(shared_prefix_blocks=8, num_q_heads=8 * 129), pa.PA_ERR_UNSUPPORTED),  # groups wider than 128
    (dict(window=-1), pa.PA_ERR_INVALID_ARG),
    (dict(out_dtype=2), pa.PA_ERR_INVALID_ARG),
    (dict(out_dtype=-1), pa.PA_ERR_INVALID_ARG),
    (dict(precise_weights=2), pa.PA_ERR_INVALID_ARG),
    (dict(num_kv_heads=2 ** 17, num_q_heads=2 ** 17), pa.PA_ERR_UNSUPPORTED),
])
def test_bad_shapes_are_rejected(bad, code):
    s = shape(**bad)
    with pytest.raises(pa.PaError) as e:
        pa.pa_num_partitions(s, pa.PA_KV_BF16)
    assert e.value.status == code
    assert pa.pa_decode_workspace_size(s, pa.PA_KV_BF16) == 0
    assert pa.pa_kernel_variant(s, pa.PA_KV_BF16) is None


def _raw_decode(s, kv=pa.PA_KV_BF16, q=0x1000, k=0x2000, v=0x3000, bt=0x4000, cl=0x5000, out=0x6000, ks=None, vs=None,
                ws=None, ws_bytes=0, scale=0.1):
    """Calls pa_decode with fake device addresses: only paths that return before a launch."""
    vp = ctypes.c_void_p
    return pa.lib().pa_decode(vp(q), vp(k), vp(v), vp(bt), vp(cl), ctypes.c_float(scale), kv, vp(out), vp(ks), vp(vs),
                              ctypes.byref(s), vp(ws), ctypes.c_size_t(ws_bytes), None)


def test_pointer_and_workspace_checks_return_before_any_launch():
    s = shape()
    assert _raw_decode(s, q=None) == pa.PA_ERR_INVALID_ARG
    assert _raw_decode(s, out=None) == pa.PA_ERR_INVALID_ARG
    assert _raw_decode(s, k=0x2004) == pa.PA_ERR_INVALID_ARG  # misaligned
    assert _raw_decode(s, kv=7) == pa.PA_ERR_INVALID_ARG
    assert _raw_decode(s, kv=pa.PA_KV_FP8_E4M3) == pa.PA_ERR_INVALID_ARG  # fp8 without scales
    assert _raw_decode(s, scale=float("nan")) == pa.PA_ERR_INVALID_ARG
    need = pa.pa_decode_workspace_size(s, pa.PA_KV_BF16)
    assert need > 0
    assert _raw_decode(s, ws=None) == pa.PA_ERR_INVALID_ARG
    assert _raw_decode(s, ws=0x10000, ws_bytes=need - 1) == pa.PA_ERR_WORKSPACE_TOO_SMALL
    assert _raw_decode(s, ws=0x10010, ws_bytes=need) == pa.PA_ERR_INVALID_ARG  # workspace not 256-aligned
    # an empty batch is a successful no-op
    assert _raw_decode(shape(batch=0)) == pa.PA_OK


def test_binding_refuses_host_tensors():
    import torch

    s = shape(batch=1, max_context_len=16)
    t = torch.zeros(16)
    with pytest.raises(ValueError):
        pa.pa_decode(t, t, t, t, t, 0.1, pa.PA_KV_BF16, t, shape=s)


@pytest.mark.parametrize("extra", [dict(q_len=4, num_q_heads=16), dict(shared_prefix_blocks=8, num_q_heads=64),
                                   dict(window=64, num_q_heads=64), dict(q_len=16, num_q_heads=64)])
@pytest.mark.parametrize("kv", [pa.PA_KV_BF16, pa.PA_KV_FP8_E4M3])
def test_head_dim_64_takes_every_kind_of_call(extra, kv):
    s = shape(head_dim=64, **extra)
    assert pa.pa_num_partitions(s, kv) >= 1
    assert pa.pa_kernel_variant(s, kv) in ("mfma", "mfma-wide", "mfma-staged")


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""        # no result line for a run that did not happen


def test_missing_library_is_an_error_not_a_fallback(tmp_path, monkeypatch):
    """With no loadable library the binding raises: there is no other path to fall back to."""
    bogus = tmp_path / "libpa_decode.so"
    bogus.write_bytes(b"not a shared object")
    monkeypatch.setattr(pa, "_lib", None)
    monkeypatch.setattr(pa, "LIB_PATH", str(bogus))
    with pytest.raises(OSError):
        pa.lib()
    with pytest.raises(OSError):
        pa.pa_num_partitions(shape(), pa.PA_KV_BF16)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and as C++11, with nothing else included."""
    import shutil
    import subprocess

    if shutil.which("gcc") is None or shutil.which("g++") is None:
        pytest.skip("no host compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "pa_decode.h"\nint main(void) { pa_shape s; (void)s; return (int)sizeof(s) == 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", "-x", "c++", str(src)],
                   check=True)


def test_bench_reads_counters_only_for_the_workload_it_ran():
    """The recorded HBM traffic belongs to one kernel on one workload: a run with other query
    lengths, windows or head shapes must not pick up the plain run's figure."""
    import sys

    sys.path.insert(0, ROOT)
    import bench

    base = "llama3_8b_b64_ctx512-4096_bf16"
    assert bench.recorded_traffic(base + "_qlen7")[0] is None
    assert bench.recorded_traffic(base + "_window5")[0] is None
    assert bench.recorded_traffic("no_such_workload")[0] is None
    got, where = bench.recorded_traffic(base)
    assert got is None or got > 577_638_400  # when the summary is current: at least the KV bytes of that batch
    assert isinstance(where, str) and where  # ... and the line always says where the figure comes from, or why there is none


def test_check_tables_rejects_bad_arguments_before_any_launch():
    vp = ctypes.c_void_p
    s = shape()
    L = pa.lib()
    assert L.pa_check_tables(None, vp(0x5000), ctypes.byref(s), vp(0x6000), None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), None, ctypes.byref(s), vp(0x6000), None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), vp(0x5000), ctypes.byref(s), None, None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), vp(0x5000), ctypes.byref(s), vp(0x6004), None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), vp(0x5000), None, vp(0x6000), None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), vp(0x5000), ctypes.byref(shape(num_blocks=0)), vp(0x6000), None) == pa.PA_ERR_INVALID_ARG
    assert L.pa_check_tables(vp(0x4000), vp(0x5000), ctypes.byref(shape(block_size=8)), vp(0x6000), None) == pa.PA_ERR_UNSUPPORTED


def test_built_library_carries_the_digest_of_the_sources_beside_it():
    from paper_2605_06068_amd import build

    pa.lib()
    assert build.built_digest() == build.source_digest()
    assert pa.lib().pa_source_digest().decode() == build.source_digest()


def test_device_code_has_no_packed_fp32_arithmetic():
    """The device pass is compiled with the packed-fp32 target feature switched off; the generated
    gfx950 assembly of every kernel must hold none of those instructions (the same sources compiled
    without the switch do hold them, so the switch reaches the device back end)."""
    from paper_2605_06068_amd import build

    asm = build.device_asm()
    assert asm.count("global_load_lds_dwordx4") > 100  # it is the kernels' assembly
    assert re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", asm) == []
