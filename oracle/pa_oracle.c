/*
 * CPU oracle for batched single-token decode attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE, not a product path: only the tests, the smoke check and the
 * benchmark's CPU-baseline leg may build or call this file.  It shares no code with
 * the HIP library.  The attention functions know nothing about tiles, splits or online
 * softmax.  Next to them sit the helpers that the indexing checks compare the kernels with: the
 * block-table walk, the check of a table against the pool, and the split plan.  The paper
 * defines no split, so that last helper restates the definition the product publishes in its
 * header (tiles of 32 tokens in batch order, cut into P balanced ranges) by brute force; its
 * pins are property checks (balanced, monotone, tile-aligned), not a second copy of the formula.
 *
 * What it computes is the plain definition of grouped-query attention for one new
 * query token per sequence (the paper's Appendix A, Scenario A, describes the model
 * family: grouped-query attention in which 32 query heads share 8 key/value heads,
 * served from a paged KV cache).  For sequence b, query head h, KV head g = h / G
 * with G = Hq / Hkv, and logical token t in [0, L_b):
 *
 *     phys  = block_tables[b][t / BS],   slot = t % BS
 *     k_t   = deq(k_cache[phys][g][slot][:]),   v_t = deq(v_cache[phys][g][slot][:])
 *     s_t   = scale * sum_d q[b][h][d] * k_t[d]
 *     p_t   = exp(s_t - max_u s_u) / sum_u exp(s_u - max_u s_u)
 *     out[b][h][:] = sum_t p_t * v_t[:]
 *
 * everything in float64, two passes over the scores, one final rounding of out to
 * float32.  deq widens bf16 bit patterns exactly, or maps an OCP e4m3 byte through a
 * 256-entry table (built here from the format's closed form) times the KV head's
 * scale (k_scale for K, v_scale for V).  L_b = 0 gives a zero row.
 *
 * pa_oracle_verify is the same definition for a window of Q query tokens per sequence with a
 * causal mask inside the window (query i sees tokens 0 .. L_b - Q + i).
 *
 * Every pin that ties this file to something other than itself lives in
 * tests/test_oracle_pins.py (closed forms, invariants, dense library softmax, brute
 * force); no function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PA_ORACLE_KV_BF16 0
#define PA_ORACLE_KV_FP8_E4M3 1

/* OCP 8-bit floating point, E4M3 variant: 1 sign, 4 exponent (bias 7), 3 mantissa bits;
 * no infinities; S.1111.111 is NaN; exponent field 0 is subnormal: (m/8) * 2^-6. */
static double e4m3_value(unsigned byte)
{
    unsigned sign = (byte >> 7) & 1u;
    unsigned expo = (byte >> 3) & 0xFu;
    unsigned mant = byte & 0x7u;
    double mag;
    if (expo == 0xFu && mant == 0x7u)
        return NAN;
    if (expo == 0)
        mag = ldexp((double)mant / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)mant / 8.0, (int)expo - 7);
    return sign ? -mag : mag;
}

void pa_oracle_e4m3_table(double *table256)
{
    for (unsigned i = 0; i < 256; ++i)
        table256[i] = e4m3_value(i);
}

static double bf16_value(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

typedef struct {
    const uint16_t *q;
    const void *k_cache, *v_cache;
    const int32_t *block_tables, *context_lens;
    double scale;
    int kv_dtype;
    const float *k_scale, *v_scale;
    int32_t B, Hq, Hkv, D, BS, MB, NB;
    double e4m3[256];
} problem;

static double load_kv(const problem *p, const void *cache, const float *head_scale, int64_t phys, int g,
                      int slot, int d)
{
    int64_t idx = ((phys * p->Hkv + g) * p->BS + slot) * (int64_t)p->D + d;
    if (p->kv_dtype == PA_ORACLE_KV_BF16)
        return bf16_value(((const uint16_t *)cache)[idx]);
    return p->e4m3[((const uint8_t *)cache)[idx]] * (double)head_scale[g];
}

/* One output row: query vector qrow (head h) of sequence b against that sequence's logical
 * tokens t_first .. L-1 (t_first = 0 unless a sliding window cuts the past off).  scores has room
 * for L doubles.  Returns 0, or -2 on a block id outside the pool for a visible token. */
static int attend_row(const problem *p, int b, int h, const uint16_t *qrow, int t_first, int L, double *scores,
                      double *out_row, double *lse_out, double *probs_row)
{
    const int G = p->Hq / p->Hkv;
    const int g = h / G;

    for (int d = 0; d < p->D; ++d)
        out_row[d] = 0.0;
    if (L <= 0) {
        if (lse_out)
            *lse_out = -INFINITY;
        return 0;
    }
    double smax = -INFINITY;
    for (int t = t_first; t < L; ++t) {
        int64_t phys = p->block_tables[(int64_t)b * p->MB + t / p->BS];
        if (phys < 0 || phys >= p->NB)
            return -2;
        double acc = 0.0;
        for (int d = 0; d < p->D; ++d)
            acc += bf16_value(qrow[d]) * load_kv(p, p->k_cache, p->k_scale, phys, g, t % p->BS, d);
        scores[t] = p->scale * acc;
        if (scores[t] > smax)
            smax = scores[t];
    }
    double denom = 0.0;
    for (int t = t_first; t < L; ++t) {
        scores[t] = exp(scores[t] - smax);
        denom += scores[t];
    }
    for (int t = t_first; t < L; ++t) {
        int64_t phys = p->block_tables[(int64_t)b * p->MB + t / p->BS];
        double w = scores[t] / denom;
        if (probs_row)
            probs_row[t] = w;
        for (int d = 0; d < p->D; ++d)
            out_row[d] += w * load_kv(p, p->v_cache, p->v_scale, phys, g, t % p->BS, d);
    }
    if (lse_out)
        *lse_out = smax + log(denom);
    return 0;
}

/*
 * Shared driver: Q query tokens per sequence (q is [B, Q, Hq, D]); query token i of sequence b
 * sees the logical tokens 0 .. L_b - Q + i, i.e. the window's own tokens are the LAST Q tokens
 * of the context and each sees itself and everything before it.  Q == 1 is plain decode.
 * window > 0 is a sliding window: the query at position pos sees tokens pos-window+1 .. pos only.
 * Rows: row_b == NULL -> all B*Q*Hq rows in layout order, else the (row_b, row_i, row_h) triples
 * (row_i == NULL means token 0).
 */
static int run_rows(const uint16_t *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                    const int32_t *context_lens, float scale, int kv_dtype, const float *k_scale,
                    const float *v_scale, int32_t B, int32_t Q, int32_t window, int32_t Hq, int32_t Hkv, int32_t D,
                    int32_t BS, int32_t MB, int32_t NB, int64_t n_rows, const int32_t *row_b, const int32_t *row_i,
                    const int32_t *row_h, float *out_f32, double *out_f64, double *lse, double *probs,
                    int64_t probs_stride)
{
    if (window < 0)
        return -1;
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !out_f32)
        return -1;
    if (B < 0 || Q <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || BS <= 0 || MB <= 0 || NB <= 0 || Hq % Hkv != 0)
        return -1;
    if (kv_dtype != PA_ORACLE_KV_BF16 && kv_dtype != PA_ORACLE_KV_FP8_E4M3)
        return -1;
    if (kv_dtype == PA_ORACLE_KV_FP8_E4M3 && (!k_scale || !v_scale))
        return -1;
    if (!row_b != !row_h)
        return -1;
    if (!row_b && n_rows != (int64_t)B * Q * Hq)
        return -1;

    problem p;
    p.q = q; p.k_cache = k_cache; p.v_cache = v_cache;
    p.block_tables = block_tables; p.context_lens = context_lens;
    p.scale = (double)scale; p.kv_dtype = kv_dtype; p.k_scale = k_scale; p.v_scale = v_scale;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.BS = BS; p.MB = MB; p.NB = NB;
    pa_oracle_e4m3_table(p.e4m3);

    int64_t max_len = 1;
    for (int64_t r = 0; r < n_rows; ++r) {
        int b = row_b ? row_b[r] : (int)(r / ((int64_t)Q * Hq));
        int i = row_b ? (row_i ? row_i[r] : 0) : (int)((r / Hq) % Q);
        int h = row_h ? row_h[r] : (int)(r % Hq);
        if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= Q)
            return -1;
        int L = context_lens[b];
        if ((int64_t)L > (int64_t)MB * BS)
            return -1;
        if (probs && L > probs_stride)
            return -1;
        if (L > max_len)
            max_len = L;
    }

    int status = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_len);
        double *row = (double *)malloc(sizeof(double) * (size_t)D);
        if (!scores || !row) {
#pragma omp atomic write
            status = -3;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < n_rows; ++r) {
                int b = row_b ? row_b[r] : (int)(r / ((int64_t)Q * Hq));
                int i = row_b ? (row_i ? row_i[r] : 0) : (int)((r / Hq) % Q);
                int h = row_h ? row_h[r] : (int)(r % Hq);
                const uint16_t *qrow = q + (((int64_t)b * Q + i) * Hq + h) * D;
                int visible = context_lens[b] - Q + 1 + i; /* tokens 0 .. L_b - Q + i */
                int t_first = (window > 0 && visible > window) ? visible - window : 0;
                int rc = attend_row(&p, b, h, qrow, t_first, visible, scores, row, lse ? &lse[r] : NULL,
                                    probs ? probs + r * probs_stride : NULL);
                if (rc != 0) {
#pragma omp atomic write
                    status = rc;
                }
                for (int d = 0; d < D; ++d) {
                    out_f32[r * D + d] = (float)row[d];
                    if (out_f64)
                        out_f64[r * D + d] = row[d];
                }
            }
        }
        free(scores);
        free(row);
    }
    return status;
}

/*
 * Attention rows for the whole batch (row_b == NULL: n_rows must be B*Hq, row r is
 * b = r / Hq, h = r % Hq) or for a selection of (row_b[r], row_h[r]) pairs.
 *
 *   out_f32   [n_rows, D] float32, required
 *   out_f64   [n_rows, D] float64, optional (NULL to skip)
 *   lse       [n_rows]    float64 log-sum-exp of the scaled scores, optional
 *   probs     [n_rows, probs_stride] float64 softmax weights per logical token, optional
 *
 * Returns 0; -1 bad shape/argument; -2 a valid token's block id is outside [0, NB);
 * -3 out of memory.
 */
int pa_oracle_decode(const uint16_t *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                     const int32_t *context_lens, float scale, int kv_dtype, const float *k_scale,
                     const float *v_scale, int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t BS, int32_t MB,
                     int32_t NB, int64_t n_rows, const int32_t *row_b, const int32_t *row_h, float *out_f32,
                     double *out_f64, double *lse, double *probs, int64_t probs_stride)
{
    return run_rows(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, k_scale, v_scale, B, 1, 0, Hq,
                    Hkv, D, BS, MB, NB, n_rows, row_b, NULL, row_h, out_f32, out_f64, lse, probs, probs_stride);
}

/*
 * Multi-token verification (the single forward pass over a window of K proposed tokens in the
 * paper's predicted-output speculative decoding: Appendix A, Scenario B): the K = Q
 * window tokens are already in the cache as the last Q tokens of each context (context_lens
 * counts them), q is [B, Q, Hq, D], and query token i attends causally: to logical tokens
 * 0 .. L_b - Q + i.  A query with no visible token (L_b - Q + i < 0) gives a zero row.
 * Outputs as pa_oracle_decode with rows [B, Q, Hq] (or the selected (b, i, h) triples).
 */
int pa_oracle_verify(const uint16_t *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                     const int32_t *context_lens, float scale, int kv_dtype, const float *k_scale,
                     const float *v_scale, int32_t B, int32_t Q, int32_t Hq, int32_t Hkv, int32_t D, int32_t BS,
                     int32_t MB, int32_t NB, int64_t n_rows, const int32_t *row_b, const int32_t *row_i,
                     const int32_t *row_h, float *out_f32, double *out_f64, double *lse, double *probs,
                     int64_t probs_stride)
{
    if (row_b && !row_i)
        return -1;
    return run_rows(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, k_scale, v_scale, B, Q, 0, Hq,
                    Hkv, D, BS, MB, NB, n_rows, row_b, row_i, row_h, out_f32, out_f64, lse, probs, probs_stride);
}

/*
 * Sliding-window attention (the attention pattern of the streaming encoder in the paper's
 * Appendix A, Scenario D, here over the paged cache): as pa_oracle_verify (Q >= 1 query tokens per
 * sequence, the last Q tokens of each context), but the query at position pos = L_b - Q + i
 * attends to the window tokens max(0, pos - window + 1) .. pos only.  Table entries and cache
 * contents before the earliest window of a sequence are never read.
 */
int pa_oracle_window(const uint16_t *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                     const int32_t *context_lens, float scale, int kv_dtype, const float *k_scale,
                     const float *v_scale, int32_t B, int32_t Q, int32_t window, int32_t Hq, int32_t Hkv, int32_t D,
                     int32_t BS, int32_t MB, int32_t NB, int64_t n_rows, const int32_t *row_b, const int32_t *row_i,
                     const int32_t *row_h, float *out_f32, double *out_f64, double *lse, double *probs,
                     int64_t probs_stride)
{
    if (row_b && !row_i)
        return -1;
    if (window <= 0)
        return -1;
    return run_rows(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, k_scale, v_scale, B, Q, window,
                    Hq, Hkv, D, BS, MB, NB, n_rows, row_b, row_i, row_h, out_f32, out_f64, lse, probs, probs_stride);
}

/*
 * Where the walk goes, for the indexing checks: the physical block ids that sequence b's
 * valid tokens live in, in logical order (block_tables[b][0 .. ceil(L_b/BS))).  Writes at
 * most cap ids and returns how many the sequence has.
 */
int32_t pa_oracle_visited_blocks(const int32_t *block_tables, const int32_t *context_lens, int32_t MB, int32_t BS,
                                 int32_t b, int32_t *ids, int32_t cap)
{
    int32_t L = context_lens[b];
    int32_t n = L <= 0 ? 0 : (L + BS - 1) / BS;
    for (int32_t i = 0; i < n && i < cap; ++i)
        ids[i] = block_tables[(int64_t)b * MB + i];
    return n;
}

/*
 * The same under a sliding window: with `reach` = window + Q - 1 the earliest token any query of
 * sequence b sees is max(0, L_b - reach); the blocks from the one holding that token to the end of
 * the context are the ones a correct walk touches.  Writes their ids in logical order and returns
 * their number; *first_block receives the logical index of the first of them.
 */
int32_t pa_oracle_window_blocks(const int32_t *block_tables, const int32_t *context_lens, int32_t MB, int32_t BS,
                                int32_t b, int32_t reach, int32_t *first_block, int32_t *ids, int32_t cap)
{
    int32_t L = context_lens[b];
    if (L <= 0) {
        *first_block = 0;
        return 0;
    }
    int32_t t_first = L > reach ? L - reach : 0;
    int32_t jb = t_first / BS, je = (L - 1) / BS;
    *first_block = jb;
    for (int32_t j = jb; j <= je && j - jb < cap; ++j)
        ids[j - jb] = block_tables[(int64_t)b * MB + j];
    return je - jb + 1;
}

/*
 * What a caller of the paged attention step promises about its block tables and lengths, checked
 * entry by entry in batch order, then block order (the paged KV cache of the paper's Appendix A,
 * Scenario A, addresses every token through such a table):
 *   - 0 <= L_b <= max_ctx, and with a shared prefix of prefix_blocks blocks (only whole pairs of
 *     blocks count: 2 * (prefix_blocks / 2)) also L_b >= prefix tokens + Q - 1          (kind 1)
 *   - every block that holds a token some query can see (all of them, or with reach =
 *     window + Q - 1 > 0 those from the block of token max(0, L_b - reach) on) has an id in
 *     [0, NB)                                                                             (kind 2)
 *   - inside the shared prefix the id equals the one in row 0 of the table                (kind 3)
 * A sequence whose length is refused has none of its blocks looked at.  Returns the number of
 * offending entries; first[0..3] receive {kind, b, j, value} of the first one in that order
 * (j = -1 and value = L_b for a length), or {0, -1, -1, 0} when there is none.
 */
int64_t pa_oracle_check_tables(const int32_t *block_tables, const int32_t *context_lens, int32_t B, int32_t MB,
                               int32_t BS, int32_t NB, int32_t max_ctx, int32_t reach, int32_t prefix_blocks,
                               int32_t Q, int32_t *first)
{
    int64_t bad = 0;
    int32_t shared = 2 * (prefix_blocks / 2);
    first[0] = 0;
    first[1] = -1;
    first[2] = -1;
    first[3] = 0;
    for (int32_t b = 0; b < B; ++b) {
        int32_t L = context_lens[b];
        int length_ok = L >= 0 && L <= max_ctx && !(shared > 0 && L < shared * BS + Q - 1);
        if (!length_ok) {
            if (bad++ == 0) {
                first[0] = 1;
                first[1] = b;
                first[2] = -1;
                first[3] = L;
            }
            continue;
        }
        int32_t t_first = (reach > 0 && L > reach) ? L - reach : 0;
        for (int32_t t = t_first - t_first % BS; t < L; t += BS) {
            int32_t j = t / BS;
            int32_t id = block_tables[(int64_t)b * MB + j];
            int kind = 0;
            if (id < 0 || id >= NB)
                kind = 2;
            else if (j < shared && id != block_tables[j])
                kind = 3;
            if (kind != 0 && bad++ == 0) {
                first[0] = kind;
                first[1] = b;
                first[2] = j;
                first[3] = id;
            }
        }
    }
    return bad;
}

/*
 * The split plan written from its definition (the product states it in its public header):
 * every sequence is cut into tiles of 32 tokens, tiles_b = ceil(L_b / 32); the tiles of all
 * sequences in batch order are numbered 0 .. T-1; partition k of P owns the global tiles t with
 * floor(k*T/P) <= t < floor((k+1)*T/P).  For every KV block (16 tokens, so two per tile) that
 * holds a valid token this writes the owning partition into block_partition[b*MB + j], and -1
 * for every other entry.  Done the slow way: each tile searches all partitions.  Returns T.
 */
int64_t pa_oracle_block_partition_window(const int32_t *context_lens, int32_t B, int32_t MB, int32_t BS, int32_t P,
                                         int32_t reach, int32_t *block_partition);

int64_t pa_oracle_block_partition(const int32_t *context_lens, int32_t B, int32_t MB, int32_t BS, int32_t P,
                                  int32_t *block_partition)
{
    return pa_oracle_block_partition_window(context_lens, B, MB, BS, P, 0, block_partition);
}

/*
 * The same plan under a sliding window (reach = window + Q - 1 > 0; 0 = no window): tiles keep
 * their place in the sequence (tile i = tokens 32 i .. 32 i + 31), but only those that hold a token
 * at or after t_first = max(0, L_b - reach) are numbered and assigned, and a block that lies
 * entirely before t_first stays -1 even when its tile is assigned.
 */
int64_t pa_oracle_block_partition_window(const int32_t *context_lens, int32_t B, int32_t MB, int32_t BS, int32_t P,
                                         int32_t reach, int32_t *block_partition)
{
    const int tile_tokens = 32;
    int64_t T = 0;
    for (int32_t b = 0; b < B; ++b) {
        int32_t L = context_lens[b];
        int32_t t_first = (reach > 0 && L > reach) ? L - reach : 0;
        for (int32_t first = 0; first < L; first += tile_tokens)
            if (first + tile_tokens > t_first)
                ++T;
    }
    for (int64_t i = 0; i < (int64_t)B * MB; ++i)
        block_partition[i] = -1;
    int64_t t = 0;
    for (int32_t b = 0; b < B; ++b) {
        int32_t L = context_lens[b];
        int32_t t_first = (reach > 0 && L > reach) ? L - reach : 0;
        for (int32_t first = 0; first < L; first += tile_tokens) {
            if (first + tile_tokens <= t_first)
                continue;
            int32_t owner = -1;
            for (int32_t k = 0; k < P; ++k) {
                int64_t lo = ((int64_t)k * T) / P, hi = ((int64_t)(k + 1) * T) / P;
                if (lo <= t && t < hi)
                    owner = k;
            }
            for (int32_t tok = first; tok < L && tok < first + tile_tokens; tok += BS)
                if (tok + BS > t_first)
                    block_partition[(int64_t)b * MB + tok / BS] = owner;
            ++t;
        }
    }
    return T;
}

/*
 * Nearest e4m3 code of a finite float: round to nearest, ties to the code with an even mantissa
 * (codes are consecutive, so "even code"), saturating at +-448; the sign bit is copied.  Found the
 * slow way: compare against every non-negative finite code value.
 */
unsigned pa_oracle_e4m3_encode(float x)
{
    unsigned sign = signbit(x) ? 0x80u : 0u;
    double mag = fabs((double)x);
    unsigned best = 0;
    double best_err = INFINITY;
    for (unsigned code = 0; code <= 0x7Eu; ++code) {
        double err = fabs(e4m3_value(code) - mag);
        if (err < best_err || (err == best_err && (code & 1u) == 0)) {
            best = code;
            best_err = err;
        }
    }
    return sign | best;
}

/*
 * KV append by its definition: the key and value rows of the Q tokens added in this step (bf16,
 * [B, Q, Hkv, D]; Q = 1 is the ordinary decode step) go to the last Q logical positions of each
 * context, token i to position t = L_b - Q + i (skipped when t < 0), i.e. block
 * block_tables[b][t/BS], slot t % BS.  bf16 caches receive the bit patterns unchanged; e4m3 caches receive
 * encode(float(x) / scale[g]) with the division in float32 (the precision the product states for
 * this decision).  Returns 0, -1 bad argument, -2 block id outside the pool.
 */
int pa_oracle_kv_append(const uint16_t *k_new, const uint16_t *v_new, void *k_cache, void *v_cache,
                        const int32_t *block_tables, const int32_t *context_lens, int kv_dtype, const float *k_scale,
                        const float *v_scale, int32_t B, int32_t Q, int32_t Hkv, int32_t D, int32_t BS, int32_t MB,
                        int32_t NB)
{
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !context_lens || Q < 1)
        return -1;
    if (kv_dtype == PA_ORACLE_KV_FP8_E4M3 && (!k_scale || !v_scale))
        return -1;
    for (int64_t bi = 0; bi < (int64_t)B * Q; ++bi) {
        int32_t b = (int32_t)(bi / Q), i = (int32_t)(bi % Q);
        int32_t t = context_lens[b] - Q + i;
        if (t < 0)
            continue;
        int64_t phys = block_tables[(int64_t)b * MB + t / BS];
        if (phys < 0 || phys >= NB)
            return -2;
        for (int32_t g = 0; g < Hkv; ++g)
            for (int32_t d = 0; d < D; ++d) {
                int64_t src = (((int64_t)b * Q + i) * Hkv + g) * D + d;
                int64_t dst = ((phys * Hkv + g) * BS + t % BS) * (int64_t)D + d;
                if (kv_dtype == PA_ORACLE_KV_BF16) {
                    ((uint16_t *)k_cache)[dst] = k_new[src];
                    ((uint16_t *)v_cache)[dst] = v_new[src];
                } else {
                    float kq = (float)bf16_value(k_new[src]) / k_scale[g];
                    float vq = (float)bf16_value(v_new[src]) / v_scale[g];
                    ((uint8_t *)k_cache)[dst] = (uint8_t)pa_oracle_e4m3_encode(kq);
                    ((uint8_t *)v_cache)[dst] = (uint8_t)pa_oracle_e4m3_encode(vq);
                }
            }
    }
    return 0;
}

/* How many threads the row loops may use from now on (the benchmark's one-thread leg); the
 * arithmetic of a row does not depend on it. */
void pa_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int pa_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
