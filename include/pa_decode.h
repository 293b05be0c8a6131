/*
 * pa_decode — batched single-token decode attention over a paged (block-table) KV cache
 * with grouped-query heads, for AMD MI355X (gfx950).  C ABI of libpa_decode.so.
 *
 * The operation is the attention step of autoregressive decoding in the serving stack the
 * paper describes for its standard LLM scenario (Appendix A, Scenario A: a dense decoder
 * with grouped-query attention, 32 query heads sharing 8 key/value heads, served with a
 * paged KV cache and continuous batching).  For every sequence b and query head h, with
 * G = num_q_heads / num_kv_heads and KV head g = h / G:
 *
 *     out[b][h][:] = sum_t softmax_t( scale * <q[b][h], K_t> ) * V_t,   t in [0, context_lens[b])
 *     K_t = deq(k_cache[ block_tables[b][t / block_size] ][g][t % block_size][:]),  V_t likewise
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers owned by the caller, contiguous in the layouts
 *     below and 16-byte aligned.  The shape struct and the split-plan arrays are HOST memory.
 *   - The library allocates no device memory, never reads device memory on the host, and (except
 *     pa_decode_profile) never synchronises: work is enqueued on the given HIP stream (hipStream_t
 *     passed as void*, NULL = the default stream) and the call returns at once.  Calls that share
 *     a workspace must be ordered by the caller.  Between calls it keeps nothing about the data;
 *     what it does keep, per process, is the compute-unit count of the device that was current at
 *     the first call (the number of partitions, hence the workspace size and the cut points,
 *     follow from it: a process is assumed to drive GPUs of one kind).
 *   - Errors are return codes (pa_status).  Everything the host can check (null pointers, shape,
 *     alignment, workspace size) is rejected BEFORE any launch; the contents of block_tables and
 *     context_lens are trusted by pa_decode and pa_kv_append: ids of tokens a query can see must
 *     lie in [0, num_blocks) and 0 <= context_lens[b] <= max_context_len.  pa_check_tables checks
 *     exactly that on the device without following any id, and pa_decode_trace refuses to follow
 *     an id outside the pool.
 *   - A launch failure is detected with hipGetLastError() after the launches of a call: that
 *     clears, and may report, an error left by another HIP call of the same host thread.
 *   - Table entries past ceil(context_lens[b] / block_size), token slots past context_lens[b] in
 *     a sequence's last block, and blocks no sequence owns are never dereferenced / never
 *     influence the result (they may hold garbage ids and NaN patterns).
 *   - context_lens[b] counts the token appended in this step.  context_lens[b] == 0 yields a zero
 *     output row.
 *
 * Layouts (row-major)
 *     q             [batch, num_q_heads, head_dim]                        bf16
 *     k_cache       [num_blocks, num_kv_heads, block_size, head_dim]      bf16, or e4m3 bytes
 *     v_cache       [num_blocks, num_kv_heads, block_size, head_dim]      same type as k_cache
 *     block_tables  [batch, max_blocks_per_seq]                           int32
 *     context_lens  [batch]                                               int32
 *     k_scale, v_scale [num_kv_heads]                                     float32 (fp8 KV only)
 *     out           [batch, num_q_heads, head_dim]                        float32 (bf16 if shape.out_dtype says so)
 *
 * Multi-token verification (shape.q_len = Q >= 2 with Q * G <= 512; the single forward pass over a window of
 * K proposed tokens in the paper's predicted-output speculative decoding, Appendix A, Scenario B):
 * the Q window tokens are already in the cache as the LAST Q tokens of every context
 * (context_lens counts them), q and out gain a query-token axis,
 *     q   [batch, Q, num_q_heads, head_dim]      out [batch, Q, num_q_heads, head_dim]
 * and query token i attends causally, to t in [0, context_lens[b] - Q + i]; a query token with no
 * visible token yields a zero row.  The KV cache is read once for all Q tokens up to Q * G = 128
 * (query token, head) pairs per KV head, once per 128 of them above that (Q * G <= 512).
 *
 * Shared prefix (shape.shared_prefix_blocks > 0; the long common prompt prefix of the paper's
 * prompt-caching workload, Appendix A, Scenario C: many concurrent requests over one cached
 * prefix of tens of thousands of tokens plus short individual suffixes): the result is the same
 * attention as above, but the blocks of the prefix (rounded down to whole tiles of two blocks)
 * are read once for the whole batch, with the (sequence, head) pairs as matrix columns, instead
 * of once per sequence; the rest of every context is processed per sequence as usual and a merge
 * kernel joins the two by their log-sum-exps.  The promise is not checked on the device: block
 * ids of the prefix are taken from row 0 of block_tables.  Supported for Q * G <= 128; in a
 * multi-token call every query token must lie after the prefix (context_lens[b] >= prefix tokens
 * + Q - 1).
 *
 * Sliding window (shape.window = W > 0; attention over the last W positions only, as in the
 * streaming encoder of the paper's Appendix A, Scenario D, whose per-stream cache is evicted in
 * step with the window): the sum above runs over t in [max(0, p - W + 1), p], p being the query's
 * position (context_lens[b] - 1 for plain decode, context_lens[b] - Q + i for query token i of a
 * multi-token call).  Blocks that lie entirely before the earliest window of a sequence
 * (before token context_lens[b] - Q - W + 1) are never dereferenced: their table entries may be
 * stale.  Together with a shared prefix the promise is accepted and goes unused (no prefix pass, none
 * of its conditions): every sequence reads its own last W + Q - 1 tokens, whichever blocks hold them,
 * and no block before them.
 *
 * Supported: batch <= 65535; head_dim in {64, 128}; block_size == 16; num_q_heads a multiple of num_kv_heads with
 * Q * G <= 512; PA_KV_FP8_E4M3 is the OCP e4m3 format (bias 7, no
 * infinities, 0x7F/0xFF NaN) with one float32 scale per KV head for K and one for V.
 */
#ifndef PA_DECODE_H
#define PA_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pa_status {
    PA_OK = 0,
    PA_ERR_INVALID_ARG = 1,         /* null pointer, misaligned pointer, inconsistent shape */
    PA_ERR_UNSUPPORTED = 2,         /* well-formed but outside the supported set above */
    PA_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes < pa_decode_workspace_size() */
    PA_ERR_HIP = 4                  /* a HIP runtime call (launch, event) failed */
} pa_status;

typedef enum pa_kv_dtype { PA_KV_BF16 = 0, PA_KV_FP8_E4M3 = 1 } pa_kv_dtype;

/* element type of `out` (pa_shape.out_dtype) */
typedef enum pa_out_dtype { PA_OUT_F32 = 0, PA_OUT_BF16 = 1 } pa_out_dtype;

/* Host-side description of one call.  Everything the launch plan depends on is here, so the
 * plan never needs the device-resident context_lens. */
typedef struct pa_shape {
    int32_t batch;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t block_size;
    int32_t max_blocks_per_seq; /* row stride of block_tables */
    int32_t num_blocks;         /* blocks in the pool (k_cache.shape[0]) */
    int32_t max_context_len;    /* host-known upper bound on context_lens; 0 = max_blocks_per_seq * block_size */
    int32_t num_partitions;     /* 0 = library heuristic; otherwise the number P of partitions of the
                                   split plan below (1 .. 65535; tests force values) */
    int32_t q_len;              /* query tokens per sequence: 0 or 1 = plain decode; 2 .. 512 = multi-token
                                   verification (see pa_decode; q_len * G <= 512) */
    int32_t shared_prefix_blocks; /* 0, or the caller's promise that the first shared_prefix_blocks entries of
                                   every row of block_tables are the same physical blocks (a prompt prefix
                                   cached once for the whole batch) and every context is at least that long:
                                   those blocks are then read once for all sequences (see pa_decode) */
    int32_t out_dtype;          /* PA_OUT_F32 (0), or PA_OUT_BF16: out holds bf16, every element the float32 result
                                   rounded to nearest even */
    int32_t window;             /* 0 = every query sees its whole past; W > 0 = sliding window: the query at
                                   position t sees tokens t-W+1 .. t only (see pa_decode) */
    int32_t precise_weights;    /* 0 = the library chooses how many bits of the softmax weights enter the PV
                                   product (see "Arithmetic" at pa_decode); 1 = 16 significant bits on every path */
} pa_shape;

/*
 * The split plan (flash-decoding style split-K over the context, balanced over the whole batch).
 * The context of sequence b is cut into tiles of 32 tokens: tiles_b = ceil(context_lens[b] / 32)
 * (0 for an empty context); the tiles of all sequences, in batch order, form one global tile
 * sequence of length T.  It is cut into P contiguous ranges, partition k owning global tiles
 * [floor(k*T/P), floor((k+1)*T/P)).  One wavefront per (partition, KV head) processes a range;
 * a sequence that lies inside one range is finished there, a sequence that a range boundary
 * cuts gets one partial result per range it touches and the merge kernel combines them by
 * their log-sum-exps.  P is a pure function of the shape and of the device's compute-unit count
 * (never of device data); the boundaries follow from the context lengths on the device.
 *
 * pa_num_partitions: P for this shape, or a negative pa_status on an invalid / unsupported shape.
 */
int32_t pa_num_partitions(const pa_shape *shape, pa_kv_dtype kv_dtype);

/*
 * The plan as the kernels apply it, computed on the host from a HOST copy of the context
 * lengths: block_partition (HOST, [batch, max_blocks_per_seq]) receives, for every KV block
 * that holds a valid token, the index of the partition that processes it, and -1 elsewhere.
 * With a sliding window only the tiles from the one holding the first visible token on are
 * counted and assigned, and blocks entirely before that token stay -1.
 * With a shared prefix T counts the tiles after the prefix only, a length below the prefix is an
 * error, and the entries of the prefix blocks hold -2 - r, r being the range of the prefix tiles
 * (cut into balanced ranges in the same way) whose workgroups read the block.
 * Returns T, or a negative pa_status (bad shape, null pointer, a length above max_context_len).
 */
int32_t pa_split_plan(const pa_shape *shape, pa_kv_dtype kv_dtype, const int32_t *context_lens,
                      int32_t *block_partition);

/* Bytes of device workspace pa_decode needs for this shape: two partial results (normalised
 * output row + log-sum-exp per query head and query token) per partition, and 16 bytes per
 * sequence plus 4 per partition that tell the merge kernel whether and where a sequence was cut; with a shared prefix in
 * addition one partial result per range of the prefix and one more per output row.  0 when P == 1.  Returns 0 as well for
 * an invalid shape (pa_decode then reports the error). */
size_t pa_decode_workspace_size(const pa_shape *shape, pa_kv_dtype kv_dtype);

/*
 * The decode attention step.  Enqueues a partition kernel (block-table walk, K/V tile loads,
 * scores, online softmax, PV; final rows for sequences inside one partition, partials for the
 * others) and, when P > 1, a merge kernel that combines the partials by their log-sum-exps.
 *
 *   q, k_cache, v_cache, block_tables, context_lens, out   device, layouts above
 *   scale            softmax scale applied to q.K (e.g. 1/sqrt(head_dim))
 *   k_scale, v_scale device float32[num_kv_heads]; required for PA_KV_FP8_E4M3, ignored (may be
 *                    NULL) for PA_KV_BF16
 *   workspace        device, 256-byte aligned, >= pa_decode_workspace_size() bytes; may be NULL
 *                    when that size is 0.  Contents on entry are irrelevant; only entries written
 *                    by this call are read back.
 *   stream           hipStream_t
 *
 * The result is deterministic run to run (no floating-point atomics).
 * Arithmetic: scores, softmax and accumulation in float32; the softmax weights are the operand of a
 * bf16 matrix product with the values.  With shape.precise_weights = 0 they enter it with 16
 * significant bits (a bf16 number plus its rounding remainder) for PA_KV_BF16 calls with
 * q_len * G <= 16 and no shared prefix: result within ~1e-5 of the exact one for values of unit
 * size; and with 8 bits (one bf16 number, relative rounding error <= 2^-9 per weight, unbiased) for
 * every other call (fp8 KV, more than 16 columns, a shared prefix): result within 2^-9 * max|v| of
 * the exact one for the dequantised values, a few 1e-3 in practice for values of unit size, and
 * proportionally more for larger ones.  With shape.precise_weights = 1 every call uses 16 bits
 * (result within ~1e-5 * max|v|) at the price of one more matrix instruction per operand: nothing
 * for plain bf16 decode, 5-25 % more time for the calls listed above.  The paper's accuracy
 * gates compare generated text with a reference implementation's (Appendix A, Scenario B: greedy
 * outputs must match); a caller held to such a gate, or one whose values are not of unit size,
 * sets it.  Range of the scores: the 8-bit paths fold the scale into the exponent (one fused
 * multiply-add per score), which leaves every exponent off by up to 2^-24 |score * scale|: nothing
 * for scores of ordinary size (below 2^-12 up to 2^12), a loss of accuracy beyond, and overflowing
 * weights (a non-finite result) from about 2^26.  The 16-bit paths scale first and subtract the
 * maximum from the products: the largest weight is exactly 1 whatever the size of the scores.
 */
pa_status pa_decode(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                    const int32_t *context_lens, float scale, pa_kv_dtype kv_dtype, void *out,
                    const float *k_scale, const float *v_scale, const pa_shape *shape, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * pa_decode for callers that cannot allocate device memory or hold a workspace of their own: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  The same step
 * with the same arguments minus the workspace: the partials and merge notes live in a static
 * device array of PA_STATIC_SCRATCH_BYTES inside the library (one copy per GPU the library runs
 * on, held until the process ends), whose address is looked up once per device, at the first call
 * made with that device current.  The call itself allocates nothing and synchronises nothing.
 *   - A shape whose pa_decode_workspace_size() exceeds PA_STATIC_SCRATCH_BYTES is refused with
 *     PA_ERR_WORKSPACE_TOO_SMALL before any launch (16 MiB hold the one-token step of every
 *     workload this library was measured on; multi-token calls on wide models need pa_decode).
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 *     host threads) race; order them.  Nothing in the array needs clearing between calls: a call
 *     reads back only what it wrote itself.
 *   - The result is bit-identical to pa_decode's for the same arguments.
 */
#define PA_STATIC_SCRATCH_BYTES (16u << 20)
pa_status pa_decode_static(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                           const int32_t *context_lens, float scale, pa_kv_dtype kv_dtype, void *out,
                           const float *k_scale, const float *v_scale, const pa_shape *shape, void *stream);

/*
 * The write that precedes the decode step in a serving loop (the paper's scenarios keep the
 * KV cache paged and append to it token by token: Appendix A, Scenarios A and C): stores the key
 * and value rows of the token generated in this step into the cache, at logical position
 * context_lens[b] - 1 of sequence b (the lengths already count the new token; sequences with
 * context_lens[b] <= 0 are skipped), i.e. into block block_tables[b][(L-1) / block_size], slot
 * (L-1) % block_size.  With shape.q_len = Q > 1 (the window of proposed tokens a verification
 * call is about to look at, Appendix A, Scenario B) it stores Q rows per sequence, token i at
 * position context_lens[b] - Q + i (tokens whose position would be negative are skipped).
 *
 *   k_new, v_new   device bf16 [batch, num_kv_heads, head_dim] ([batch, Q, num_kv_heads, head_dim]
 *                  for Q > 1), 16-byte aligned
 *   k_cache, v_cache, block_tables, context_lens   device, layouts above (caches are written)
 *   kv_dtype       PA_KV_BF16: rows are copied.  PA_KV_FP8_E4M3: every element is divided by its
 *                  KV head's scale (k_scale / v_scale, float32 division) and rounded to the nearest
 *                  e4m3 value, ties to even, saturating at +-448.  Inputs must be finite.
 *
 * Only batch, num_kv_heads, head_dim, block_size, max_blocks_per_seq and q_len of the shape matter
 * here (the shape must be valid as a whole).  One kernel on `stream`; no workspace; can be
 * captured into a HIP graph together with pa_decode.
 */
pa_status pa_kv_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                       const int32_t *block_tables, const int32_t *context_lens, pa_kv_dtype kv_dtype,
                       const float *k_scale, const float *v_scale, const pa_shape *shape, void *stream);

/*
 * The debug path of the boundary: the same computation with the production indexing code
 * instrumented and every block id held against the pool before it becomes an address (slow; for
 * tests and for finding a bad table).  In addition to out it records, for checking the
 * block-table walk and the split boundaries bit for bit:
 *   visited_blocks [batch, num_kv_heads, max_blocks_per_seq, 3] int32 device: for logical block j
 *                  of sequence b and KV head g, the id the table gave the kernel for its K loads
 *                  ([..,0]) and for its V loads ([..,1]) and the partition that processed it
 *                  ([..,2]).  Entries of blocks the kernel never touched keep the caller's initial
 *                  contents.
 * An id outside [0, shape.num_blocks) is recorded as it stands and NOT followed: block 0 is read
 * in its place, the call completes normally, and `out` is then meaningless for that sequence.
 * With a shared prefix the prefix pass reads the prefix blocks through row 0 of block_tables for
 * the whole batch: their records appear under sequence 0 only, with -2 - r in place of the
 * partition, r being the range of the prefix tiles as in pa_split_plan.
 */
pa_status pa_decode_trace(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                          const int32_t *context_lens, float scale, pa_kv_dtype kv_dtype, void *out,
                          const float *k_scale, const float *v_scale, const pa_shape *shape, void *workspace,
                          size_t workspace_bytes, void *stream, int32_t *visited_blocks);

/* What pa_check_tables found (report[0]) */
typedef enum pa_tables_status {
    PA_TABLES_OK = 0,
    PA_TABLES_BAD_LENGTH = 1,      /* context_lens[b] < 0, > max_context_len, or shorter than a shared prefix allows */
    PA_TABLES_BAD_BLOCK_ID = 2,    /* an id outside [0, num_blocks) where a query can see a token */
    PA_TABLES_PREFIX_MISMATCH = 3  /* an entry of the shared prefix that differs from row 0 */
} pa_tables_status;

/*
 * Checks, on the device and without following a single id, what pa_decode trusts about a paged
 * KV cache's tables (the paper's serving stack addresses every cached token through such a block
 * table: Appendix A, Scenario A), for the call `shape` describes:
 *   - 0 <= context_lens[b] <= max_context_len (the resolved bound), and with a shared prefix
 *     context_lens[b] >= prefix tokens + q_len - 1;
 *   - for every sequence whose length passed, every block that holds a token some query of the
 *     call can see (all blocks up to the context's last; with a sliding window those from the
 *     block of token max(0, context_lens[b] - window - q_len + 1) on) has an id in [0, num_blocks);
 *   - inside a shared prefix (whole pairs of blocks) every row repeats row 0.
 * Entries behind a context, and blocks a sliding window has left behind, may hold anything.  A shared
 * prefix declared together with a sliding window goes unused by pa_decode and is not checked here
 * (neither the lengths against it nor the rows against row 0).
 *
 *   block_tables, context_lens   device, layouts above; only these two are read
 *   report   device int32[8], 16-byte aligned, written by this call: [0] a pa_tables_status,
 *            [1] sequence b, [2] logical block j (-1: the length itself) and [3] the offending value
 *            of the FIRST offending entry in batch order, then block order ([1] = [2] = -1 and
 *            [3] = 0 when there is none), [4] the number of offending entries; [5..7] scratch.
 * Three small launches on `stream`; no workspace, no synchronisation (the caller reads `report`
 * after synchronising the stream); can be captured into a HIP graph.
 */
pa_status pa_check_tables(const int32_t *block_tables, const int32_t *context_lens, const pa_shape *shape,
                          int32_t *report, void *stream);

/*
 * Measurement helper: runs pa_decode `steps` times on `stream` with HIP events around each
 * kernel, SYNCHRONISES the stream, and returns the mean duration in milliseconds of the
 * partition kernel and of the merge kernel (0 when no merge is launched).  HOST output pointers.
 */
pa_status pa_decode_profile(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                            const int32_t *context_lens, float scale, pa_kv_dtype kv_dtype, void *out,
                            const float *k_scale, const float *v_scale, const pa_shape *shape, void *workspace,
                            size_t workspace_bytes, void *stream, int32_t steps, float *partition_ms,
                            float *merge_ms);

/* Name of the partition kernel variant pa_decode picks for this shape ("mfma": one wavefront per
 * (partition, KV head), up to 32 query rows (Q * G) per KV head (16 for fp8 at head_dim 128); "mfma-wide":
 * a workgroup of 2, 4 or 8 wavefronts, up to 128; "mfma-staged": a workgroup of 4 or 8 wavefronts, half of
 * them computing scores and softmax weights and half the product with V, for the query-row counts above
 * "mfma"'s: up to 64, and up to 128 with fp8 KV at head_dim 128 and with bf16 KV at head_dim 64 (17 .. 32
 * rows with long runs of tiles per partition stay on "mfma"), unless shape.precise_weights is set); NULL for
 * an invalid or unsupported shape.
 * Static storage. */
const char *pa_kernel_variant(const pa_shape *shape, pa_kv_dtype kv_dtype);

/* SHA-256 (hex) over the library's sources as the build recorded it, "" when the build recorded
 * none: lets a loader refuse a library that was not built from the sources beside it.  Static storage. */
const char *pa_source_digest(void);

/* Human-readable name of a status code.  Static storage. */
const char *pa_status_string(pa_status status);

#ifdef __cplusplus
}
#endif
#endif /* PA_DECODE_H */
