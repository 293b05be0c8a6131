"""Seeded synthetic decode batches over a paged KV cache.

This module only *draws inputs*: lengths, block tables, random q/K/V values and
their storage encodings (bf16 bit patterns, fp8 bytes with per-head scales).  It
contains none of the attention arithmetic (no scores, no softmax, no
dequantisation) and imports neither the CPU oracle nor the HIP library, so both
can be fed the very same bytes.

Workload shapes follow the serving scenario the paper describes for its
standard-LLM case (Appendix A, Scenario A: grouped-query attention with 32
query heads over 8 KV heads, head size 128, a 128k-token window, batches that
arise from tens to ~100 requests/s with 128 output tokens, paged KV cache with
continuous batching) and its long-shared-prefix case (Scenario C: 32k-token
prefixes).  The paper's prompt pool is not public, so the values are N(0,1)
draws and the lengths are drawn from the ranges listed per config below.

Layouts (row-major, contiguous):
  q             [B, Hq, D]        bf16 bit patterns (uint16); [B, Q, Hq, D] for a multi-token
                                  verification window of Q query tokens (q_len > 1)
  k_cache       [NB, Hkv, BS, D]  bf16 bit patterns (uint16) or e4m3 bytes (uint8)
  v_cache       [NB, Hkv, BS, D]  same encoding as k_cache
  block_tables  [B, MB]           int32, unused entries = -1
  context_lens  [B]               int32 (the token appended this step included)
  k_scale/v_scale [Hkv]           float32, fp8 only
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

KV_BF16 = 0
KV_FP8_E4M3 = 1

BF16_NAN_BITS = 0x7FC0
FP8_NAN_BYTE = 0x7F
E4M3_MAX = 448.0


@dataclass
class DecodeBatch:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    max_blocks_per_seq: int
    num_blocks: int
    kv_dtype: int
    scale: np.float32
    q: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    block_tables: np.ndarray
    context_lens: np.ndarray
    k_scale: Optional[np.ndarray] = None
    v_scale: Optional[np.ndarray] = None
    seed: int = 0
    meta: dict = field(default_factory=dict)
    q_len: int = 1  # query tokens per sequence; > 1: q is [B, Q, Hq, D], the last Q tokens are the window
    shared_prefix_blocks: int = 0  # leading table entries that are the same physical blocks for every sequence
    window: int = 0  # sliding window: a query at position t sees tokens t-window+1 .. t (0 = its whole past)

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def kv_elem_bytes(self) -> int:
        return 2 if self.kv_dtype == KV_BF16 else 1

    @property
    def total_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self) -> int:
        """Bytes of K and V belonging to valid tokens (what one decode step must read when every
        sequence reads its own context)."""
        return self.total_tokens * self.num_kv_heads * self.head_dim * 2 * self.kv_elem_bytes

    @property
    def kv_bytes_unique(self) -> int:
        """The same with the shared prefix counted once: bytes of the distinct valid slots."""
        shared = self.shared_prefix_blocks * self.block_size
        tokens = self.total_tokens - (self.batch - 1) * shared if self.batch > 0 else 0
        return tokens * self.num_kv_heads * self.head_dim * 2 * self.kv_elem_bytes

    @property
    def kv_bytes_visible(self) -> int:
        """Bytes of K and V some query of the step can see: with a sliding window only the last
        window + q_len - 1 tokens of every context."""
        if self.window <= 0:
            return self.kv_bytes
        reach = self.window + self.q_len - 1
        tokens = int(np.minimum(self.context_lens.astype(np.int64), reach).sum())
        return tokens * self.num_kv_heads * self.head_dim * 2 * self.kv_elem_bytes


# --------------------------------------------------------------------------------------
# encodings
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns the uint16 bit patterns."""
    a = np.asarray(x, dtype=np.float32)
    u = np.ascontiguousarray(a).reshape(-1).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    a = np.asarray(b, dtype=np.uint16)
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(a.shape)


def f32_to_e4m3_bytes(x: np.ndarray) -> np.ndarray:
    """Saturating round-to-nearest-even cast of float32 to OCP e4m3 bytes.

    Uses the library cast of ``torch.float8_e4m3fn`` on the CPU (a storage
    conversion of generated inputs; decoding is the consumers' business).
    """
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp_(-E4M3_MAX, E4M3_MAX)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


# --------------------------------------------------------------------------------------
# block tables
# --------------------------------------------------------------------------------------
def blocks_needed(context_lens: np.ndarray, block_size: int) -> np.ndarray:
    return (context_lens.astype(np.int64) + block_size - 1) // block_size


def permuted_block_tables(rng: np.random.Generator, context_lens: np.ndarray, block_size: int,
                          num_blocks: int, max_blocks_per_seq: int) -> np.ndarray:
    """Sequence b takes the next ceil(L_b/BS) entries of one random permutation of the pool."""
    nblk = blocks_needed(context_lens, block_size)
    assert int(nblk.sum()) <= num_blocks and int(nblk.max(initial=0)) <= max_blocks_per_seq
    perm = rng.permutation(num_blocks).astype(np.int32)
    tables = np.full((len(context_lens), max_blocks_per_seq), -1, dtype=np.int32)
    pos = 0
    for b, n in enumerate(nblk):
        tables[b, :n] = perm[pos:pos + n]
        pos += int(n)
    return tables


def interleaved_block_tables(rng: np.random.Generator, context_lens: np.ndarray, block_size: int,
                             num_blocks: int, max_blocks_per_seq: int) -> np.ndarray:
    """Continuous-batching growth: sequences claim the next free id 0,1,2,... in random turns,
    so ids increase inside a sequence while sequences interleave through the pool."""
    nblk = blocks_needed(context_lens, block_size)
    assert int(nblk.sum()) <= num_blocks and int(nblk.max(initial=0)) <= max_blocks_per_seq
    turns = rng.permutation(np.repeat(np.arange(len(context_lens), dtype=np.int64), nblk))
    order = np.argsort(turns, kind="stable")  # ids claimed by seq 0, then by seq 1, ...
    tables = np.full((len(context_lens), max_blocks_per_seq), -1, dtype=np.int32)
    pos = 0
    for b, n in enumerate(nblk):
        tables[b, :n] = order[pos:pos + n].astype(np.int32)
        pos += int(n)
    return tables


def shared_prefix_block_tables(rng: np.random.Generator, context_lens: np.ndarray, block_size: int,
                               num_blocks: int, max_blocks_per_seq: int, prefix_blocks: int) -> np.ndarray:
    """A prompt prefix cached once: the first ``prefix_blocks`` entries of every row are the same
    physical blocks; the rest of each sequence takes its own blocks from one random permutation."""
    nblk = blocks_needed(context_lens, block_size)
    assert int(nblk.min(initial=prefix_blocks)) >= prefix_blocks, "every context must cover the shared prefix"
    own = nblk - prefix_blocks
    assert prefix_blocks + int(own.sum()) <= num_blocks and int(nblk.max(initial=0)) <= max_blocks_per_seq
    perm = rng.permutation(num_blocks).astype(np.int32)
    tables = np.full((len(context_lens), max_blocks_per_seq), -1, dtype=np.int32)
    tables[:, :prefix_blocks] = perm[:prefix_blocks]
    pos = prefix_blocks
    for b, n in enumerate(own):
        tables[b, prefix_blocks:prefix_blocks + n] = perm[pos:pos + n]
        pos += int(n)
    return tables


# --------------------------------------------------------------------------------------
# value generation (chunked so that multi-GB pools never need a float32 copy of the whole)
# --------------------------------------------------------------------------------------
_CHUNK_ELEMS = 1 << 24


def _normal_chunks(seed_seq: np.random.SeedSequence, n_elems: int, sigma: float, encode, out_flat: np.ndarray,
                   pre_scale: Optional[np.ndarray] = None, period: int = 0, inner: int = 0):
    """Fill out_flat[i] = encode(sigma * N(0,1) [/ pre_scale[head(i)]]) chunk by chunk.

    Each chunk has its own child seed, so the result does not depend on the thread count.
    ``pre_scale`` (per KV head) with ``period`` = Hkv*inner and ``inner`` = BS*D divides values
    by the head's scale before encoding (fp8 storage).
    """
    n_chunks = (n_elems + _CHUNK_ELEMS - 1) // _CHUNK_ELEMS
    children = seed_seq.spawn(n_chunks)

    def work(c):
        lo = c * _CHUNK_ELEMS
        hi = min(n_elems, lo + _CHUNK_ELEMS)
        x = np.random.default_rng(children[c]).standard_normal(hi - lo, dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        if pre_scale is not None:
            assert lo % inner == 0 and (hi - lo) % inner == 0
            rows = x.reshape(-1, inner)
            head = (lo // inner + np.arange(rows.shape[0], dtype=np.int64)) % (period // inner)
            rows /= pre_scale[head][:, None]
        out_flat[lo:hi] = encode(x)

    workers = max(1, min(8, (os.cpu_count() or 1), n_chunks))
    if workers == 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(work, range(n_chunks)))


def _valid_slot_mask(tables: np.ndarray, context_lens: np.ndarray, block_size: int, num_blocks: int,
                     reach: int = 0) -> np.ndarray:
    """[NB, BS] bool: slot holds a token of some sequence (with ``reach`` > 0: one of its last
    ``reach`` tokens, the only ones a sliding-window call may look at)."""
    valid = np.zeros((num_blocks, block_size), dtype=bool)
    for b, L in enumerate(context_lens):
        L = int(L)
        t = np.arange(max(0, L - reach) if reach > 0 else 0, L)
        valid[tables[b, t // block_size], t % block_size] = True
    return valid


def make_batch(name: str, seed: int, context_lens: Sequence[int], num_q_heads: int, num_kv_heads: int,
               head_dim: int, block_size: int = 16, kv_dtype: int = KV_BF16, sigma: float = 1.0,
               num_blocks: Optional[int] = None, max_blocks_per_seq: Optional[int] = None,
               table_kind: str = "permuted", poison: bool = True, q_len: int = 1,
               shared_prefix_blocks: int = 0, window: int = 0) -> DecodeBatch:
    """Draw one decode batch.  ``poison`` fills every slot no valid token owns with NaN patterns
    (parity runs); with ``poison=False`` those slots are zero (timing runs).  ``q_len`` > 1 draws a
    window of that many query tokens per sequence (q becomes [B, Q, Hq, D]); the cache contents do not
    depend on it.  ``shared_prefix_blocks`` > 0 makes that many leading blocks common to all sequences
    (``table_kind`` is then ignored).  ``window`` > 0 marks the batch for sliding-window attention:
    everything before the earliest window of a sequence counts as evicted, i.e. its slots are
    poisoned like other dead slots and its table entries are set to -1."""
    rng = np.random.default_rng(seed)
    lens = np.asarray(context_lens, dtype=np.int32)
    B = len(lens)
    nblk = blocks_needed(lens, block_size)
    NB_needed = int(nblk.sum()) - (B - 1) * shared_prefix_blocks if shared_prefix_blocks > 0 else int(nblk.sum())
    NB = NB_needed if num_blocks is None else int(num_blocks)
    NB = max(NB, 1)
    MB = int(max(1, nblk.max(initial=1))) if max_blocks_per_seq is None else int(max_blocks_per_seq)
    if shared_prefix_blocks > 0:
        tables = shared_prefix_block_tables(rng, lens, block_size, NB, MB, shared_prefix_blocks)
    elif table_kind == "permuted":
        tables = permuted_block_tables(rng, lens, block_size, NB, MB)
    elif table_kind == "interleaved":
        tables = interleaved_block_tables(rng, lens, block_size, NB, MB)
    elif table_kind == "identity":
        tables = np.full((B, MB), -1, dtype=np.int32)
        pos = 0
        for b, n in enumerate(nblk):
            tables[b, :n] = np.arange(pos, pos + int(n), dtype=np.int32)
            pos += int(n)
    else:
        raise ValueError(table_kind)

    ss_q, ss_k, ss_v = np.random.SeedSequence(seed).spawn(3)
    q = np.empty(B * q_len * num_q_heads * head_dim, dtype=np.uint16)
    _normal_chunks(ss_q, q.size, sigma, f32_to_bf16_bits, q)
    q = q.reshape((B, num_q_heads, head_dim) if q_len == 1 else (B, q_len, num_q_heads, head_dim))

    n_kv = NB * num_kv_heads * block_size * head_dim
    inner = block_size * head_dim
    k_scale = v_scale = None
    if kv_dtype == KV_BF16:
        k_cache = np.empty(n_kv, dtype=np.uint16)
        v_cache = np.empty(n_kv, dtype=np.uint16)
        _normal_chunks(ss_k, n_kv, sigma, f32_to_bf16_bits, k_cache)
        _normal_chunks(ss_v, n_kv, sigma, f32_to_bf16_bits, v_cache)
        nan_pat = np.uint16(BF16_NAN_BITS)
    elif kv_dtype == KV_FP8_E4M3:
        # Per-KV-head scale = amax/448.  The draws are i.i.d., so amax is estimated from the
        # normal tail at the pool size and then made safe by the saturating cast.
        n_per_head = max(2, NB * inner)
        amax = sigma * math.sqrt(2.0 * math.log(n_per_head))
        jitter = 1.0 + 0.05 * rng.random((2, num_kv_heads))
        k_scale = (amax * jitter[0] / E4M3_MAX).astype(np.float32)
        v_scale = (amax * jitter[1] / E4M3_MAX).astype(np.float32)
        k_cache = np.empty(n_kv, dtype=np.uint8)
        v_cache = np.empty(n_kv, dtype=np.uint8)
        period = num_kv_heads * inner
        _normal_chunks(ss_k, n_kv, sigma, f32_to_e4m3_bytes, k_cache, k_scale, period, inner)
        _normal_chunks(ss_v, n_kv, sigma, f32_to_e4m3_bytes, v_cache, v_scale, period, inner)
        nan_pat = np.uint8(FP8_NAN_BYTE)
    else:
        raise ValueError(kv_dtype)
    k_cache = k_cache.reshape(NB, num_kv_heads, block_size, head_dim)
    v_cache = v_cache.reshape(NB, num_kv_heads, block_size, head_dim)

    reach = window + q_len - 1 if window > 0 else 0
    valid = _valid_slot_mask(tables, lens, block_size, NB, reach)
    if reach > 0 and poison:
        for b, L in enumerate(lens):
            tables[b, :max(0, int(L) - reach) // block_size] = -1  # evicted blocks
    fill = nan_pat if poison else nan_pat.dtype.type(0)
    dead_blk, dead_slot = np.nonzero(~valid)
    if dead_blk.size:
        k_cache[dead_blk, :, dead_slot, :] = fill
        v_cache[dead_blk, :, dead_slot, :] = fill

    scale = np.float32(1.0 / math.sqrt(float(head_dim)))
    return DecodeBatch(name=name, batch=B, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, head_dim=head_dim,
                       block_size=block_size, max_blocks_per_seq=MB, num_blocks=NB, kv_dtype=kv_dtype, scale=scale,
                       q=q, k_cache=k_cache, v_cache=v_cache, block_tables=tables, context_lens=lens,
                       k_scale=k_scale, v_scale=v_scale, seed=seed, q_len=q_len,
                       shared_prefix_blocks=shared_prefix_blocks, window=window,
                       meta={"sigma": sigma, "table_kind": table_kind, "poison": poison})


# --------------------------------------------------------------------------------------
# the named configurations
# --------------------------------------------------------------------------------------
CONFIG_NAMES = {
    1: "tiny_b2_gqa2_d64",
    2: "llama3_8b_b64_ctx512-4096_bf16",
    3: "long_b8_ctx32k-128k_bf16",
    4: "ragged_b256_ctx16-16k_bf16",
    5: "llama3_70b_heads_b128_ctx8192_fp8",
    6: "prompt_cache_b20_prefix32k_suffix128-255_bf16",
}


def config_context_lens(config: int, seed: int, length_scale: float = 1.0) -> np.ndarray:
    """Context lengths of a named config.  ``length_scale`` < 1 shrinks the length range (and
    only that) so the CPU oracle can cover a whole batch of the same structure in seconds."""
    rng = np.random.default_rng([seed, 7])

    def s(x):
        return max(1, int(round(x * length_scale)))

    if config == 1:
        return np.array([37, 100], dtype=np.int32)
    if config == 2:
        return rng.integers(s(512), s(4096) + 1, size=64).astype(np.int32)
    if config == 3:
        return rng.integers(s(32768), s(131072) + 1, size=8).astype(np.int32)
    if config == 4:
        u = rng.uniform(math.log(16.0), math.log(max(17.0, 16384.0 * length_scale)), size=256)
        return np.maximum(1, np.round(np.exp(u))).astype(np.int32)
    if config == 5:
        return np.full(128, s(8192), dtype=np.int32)
    if config == 6:
        # 20 concurrent requests over one cached 32k-token prefix, each with a suffix of 128 tokens and up to
        # 127 tokens generated so far
        prefix = (s(32768) // 32) * 32
        return (prefix + 128 + rng.integers(0, 128, size=20)).astype(np.int32)
    raise ValueError(f"unknown config {config}")


# head shape, KV type and value scale of the named configs: (num_q_heads, num_kv_heads, head_dim, kv_dtype, sigma)
CONFIG_SHAPES = {
    1: (4, 2, 64, KV_BF16, 1.0),
    2: (32, 8, 128, KV_BF16, 0.5),
    3: (32, 8, 128, KV_BF16, 0.5),
    4: (32, 8, 128, KV_BF16, 0.5),
    5: (64, 8, 128, KV_FP8_E4M3, 1.0),
    6: (32, 8, 128, KV_BF16, 0.5),
}


def make_config(config: int, seed: Optional[int] = None, poison: bool = True, length_scale: float = 1.0,
                batch_limit: Optional[int] = None, q_len: int = 1, window: int = 0,
                num_q_heads: Optional[int] = None, num_kv_heads: Optional[int] = None,
                head_dim: Optional[int] = None, kv_dtype: Optional[int] = None) -> DecodeBatch:
    """Build named config 1..6.  Default seed is 1000+config.  ``batch_limit`` keeps only the first
    sequences (same lengths they would have in the full batch).  ``q_len`` > 1 turns the batch into a
    verification step over windows of that many tokens (same cache, more query rows).  The head
    shape and KV type can be overridden (same lengths and tables, another model shape); the name of
    the batch then says so."""
    seed = 1000 + config if seed is None else seed
    lens = config_context_lens(config, seed, length_scale)
    if batch_limit is not None:
        lens = lens[:batch_limit]
    Hq, Hkv, D, kv, sigma = CONFIG_SHAPES[config]
    name = CONFIG_NAMES[config]
    if (num_q_heads, num_kv_heads, head_dim, kv_dtype) != (None, None, None, None):
        Hq = Hq if num_q_heads is None else num_q_heads
        Hkv = Hkv if num_kv_heads is None else num_kv_heads
        D = D if head_dim is None else head_dim
        kv = kv if kv_dtype is None else kv_dtype
        name += f"_hq{Hq}_hkv{Hkv}_d{D}_{'bf16' if kv == KV_BF16 else 'fp8'}"
    if length_scale != 1.0:
        name += f"_lenx{length_scale:g}"
    if config == 1:
        return make_batch(name, seed, lens, Hq, Hkv, D, 16, kv, sigma, num_blocks=16, poison=poison, q_len=q_len, window=window)
    if config == 4:
        return make_batch(name, seed, lens, Hq, Hkv, D, 16, kv, sigma, table_kind="interleaved", poison=poison,
                          q_len=q_len, window=window)
    if config == 6:
        prefix_tokens = (max(1, int(round(32768 * length_scale))) // 32) * 32
        return make_batch(name, seed, lens, Hq, Hkv, D, 16, kv, sigma, poison=poison, q_len=q_len,
                          shared_prefix_blocks=prefix_tokens // 16)
    if config in (2, 3, 5):
        return make_batch(name, seed, lens, Hq, Hkv, D, 16, kv, sigma, poison=poison, q_len=q_len, window=window)
    raise ValueError(config)
