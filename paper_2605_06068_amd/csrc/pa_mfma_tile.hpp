// Pieces shared by the two matrix-core partition kernels (pa_partition_mfma.hpp: one wavefront per
// (partition, KV head), up to 32 columns; pa_partition_mfma_wide.hpp: a workgroup of wavefronts,
// 16 or 32 columns each): the geometry of a tile in LDS, the LDS-DMA load, the cursor over the
// global tile sequence, and what one wavefront does with one tile of 32 tokens and one or two
// tiles of 16 columns -- which blocks and rows to load, scores, online softmax, PV.  D = head_dim
// is 128 or 64.
//
// LDS tile layout: row t (one token, 2 D bytes bf16 / D bytes fp8) at byte t*rowbytes; the 16-byte
// piece holding dims [8c, 8c+8) (fp8: [16c, 16c+16)) sits at piece position c ^ (t mod pieces).
// The XOR swizzle is applied on the *global* side of the LDS-DMA load (the LDS side of such a
// load is always lane-linear), which keeps every 16-lane group on one contiguous row and spreads
// the operand reads (16 different rows per 16 lanes) and the transposing reads over the banks.
// Measured with the SQ counters on the decode workload (head_dim 128): LDS busy 4.0 cycles per LDS
// instruction against 2.7 for conflict-free 1 KB / 512 B reads (rows of 128 B or less repeat their
// banks every few rows: twice the minimum and more); waves wait on LDS for under 1 % of their
// time either way, so this was left alone.
//
// The P^T operand needs no data movement: the score tile comes out of the MFMA with lane l
// holding column l%16 and tokens 4*(l/16)+{0..3}; declaring MFMA k-index 8*(l/16)+e to mean
// token 4*(l/16)+e of the first block (e<4) or of the second block (e>=4) makes the score
// registers, once exponentiated and packed to bf16, the B operand of the PV product as they
// stand.  The V^T operand is read with the same k-index convention.
#pragma once
#include <type_traits>

#include "pa_device.hpp"
#include "pa_plan.hpp"

namespace pa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// One query row (always bf16) and how the 1 KB wave-wide LDS-DMA load covers such rows.
template <int D>
struct QGeom {
    static constexpr int kRow = 2 * D;                     // bytes
    static constexpr int kPieces = kRow / 16;              // 16-byte pieces per row
    static constexpr int kRowsPerDma = kWave / kPieces;    // 4 (head_dim 128) or 8 (64)
};

// Storage geometry of one (block, head) slab of the KV cache.
template <int D, int KV>
struct KvGeom {
    static_assert(D == 64 || D == 128, "head_dim");
    static constexpr int kRow = KV == KV_BF16 ? 2 * D : D;  // bytes per token row
    static constexpr int kSlab = kBlockSize * kRow;          // 16 rows
    static constexpr int kPieces = kRow / 16;                // 16-byte pieces per row
    static constexpr int kRowsPerDma = kWave / kPieces;      // rows one 1 KB wave-wide load covers
    static constexpr int kDmaPerSlab = kSlab / 1024;
    static constexpr int kStage = 4 * kSlab;                 // K block 0, K block 1, V block 0, V block 1
    static constexpr int kDmaPerTile = 4 * kDmaPerSlab;
};

// eight e4m3 bytes -> eight bf16 (exact), in byte order
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t lo, uint32_t hi)
{
    const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)lo, 1.0f, false);
    const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)lo, 1.0f, true);
    const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)hi, 1.0f, false);
    const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)hi, 1.0f, true);
    return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// 16-byte-per-lane load from global memory straight into LDS.  LDS destination is
// lds_addr + lane*16 (wave-uniform lds_addr travels in M0); the global source is
// base (wave-uniform) + voff (per lane).  Completion is tracked by vmcnt.
// STREAM marks the load non-temporal: the KV cache is read once per call and is far larger than
// the L2, so its lines should not displace what is re-read (block tables, lengths, query rows,
// partial results).  Measured on the 8B-shaped batch: 108 -> 95 us per step.
template <bool STREAM>
__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const void* base)
{
    // M0 is an operand the compiler sets (and so knows about); the wait state a write of M0 needs
    // before an instruction that reads it is inside the statement, where the compiler cannot see
    if constexpr (STREAM)
        asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" :: "v"(voff), "s"(base), "{m0}"(lds_addr) : "memory");
    else
        asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(base), "{m0}"(lds_addr) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Position inside the global tile sequence: sequence b, its length, the first tile of it that the
// plan covers, the number of tiles it covers, and the local tile (tile ft + lt of the sequence).
struct Cursor {
    int b, lt, nt, L, ft;
};

__device__ __forceinline__ void advance(Cursor& c, const int32_t* context_lens, int B, Span sp = Span{0, 0})
{
    if (++c.lt < c.nt) return;
    c.lt = 0;
    do {
        ++c.b;
        c.L = c.b < B ? uniform_load(context_lens, c.b) : 0;
        c.nt = tiles_of(c.L, sp);
    } while (c.nt == 0 && c.b < B);
    c.ft = first_tile(c.L, sp);
}

// Output rows of empty contexts are zero.  The sequences are dealt out over the partitions (slice k of
// P); the calling wave looks at its slice 64 sequences at a time and zero-fills, all lanes together,
// the rows of KV head g's group for every empty one (the wave of KV head 0 also notes that there
// is nothing to merge).  All 64 lanes must call.
__device__ __forceinline__ void zero_rows_of_empty_contexts(const Params& p, int k, int g, int B, int Q, int D, int lane)
{
    const int per = (B + p.P - 1) / p.P;
    const int b_end = min(B, (k + 1) * per);
    for (int b0 = k * per; b0 < b_end; b0 += kWave) {
        const int b = b0 + lane;
        unsigned long long empty = __ballot(b < b_end && p.context_lens[b] <= 0);
        while (empty != 0ull) {
            const int bb = b0 + __ffsll((long long)empty) - 1;
            empty &= empty - 1ull;
            for (int i = 0; i < Q; ++i) {
                const int64_t row = ((int64_t)bb * p.QH + (int64_t)i * p.Hq + g * p.G) * D;
                for (int e = 4 * lane; e < p.G * D; e += 4 * kWave) store_out4(p, row + e, 0.f, 0.f, 0.f, 0.f);
            }
            if (g == 0 && p.merge_desc != nullptr && lane == 0) write_seq_desc(p.merge_desc, bb, 0, 0, 0, 0);
        }
    }
}

// ---- one tile (two KV blocks) of a sequence: what to load ---------------------------------------
// Per block of the tile: its physical id and the rows [lo, hi) that hold tokens some query can
// see.  Every other row (past the context, before the earliest sliding window) may hold anything,
// NaN patterns included, and is replaced on the way in by row lo of the same block; the softmax
// masks those positions.  A first block that lies entirely before the window may be gone: its
// table entry is not read, and the first visible row of the second block (which exists: it
// holds that token) stands in.  Without a second block, rows of the first one stand in.
struct TileBlocks {
    int j0;         // logical index of the tile's first block
    int phys[2];
    int lo[2], hi[2];
    bool first_gone, second;
};

// `reach` > 0: sliding window, nothing further back than `reach` tokens from the end is visible.
__device__ __forceinline__ TileBlocks tile_blocks(const int32_t* block_tables, int MB, const Cursor& c, int reach)
{
    TileBlocks t;
    const int nblk = (c.L + kBlockSize - 1) / kBlockSize;
    const int32_t* table = block_tables + (int64_t)c.b * MB;
    t.j0 = 2 * (c.lt + c.ft);
    const int t_first = (reach > 0 && c.L > reach) ? c.L - reach : 0;  // first token any query sees
    t.lo[0] = min(max(t_first - t.j0 * kBlockSize, 0), kBlockSize);
    t.hi[0] = min(c.L - t.j0 * kBlockSize, kBlockSize);
    t.first_gone = t.lo[0] >= kBlockSize;
    t.second = t.j0 + 1 < nblk;
    if (t.second) {
        t.phys[1] = uniform_load(table, t.j0 + 1);
        t.lo[1] = max(t_first - (t.j0 + 1) * kBlockSize, 0);
        t.hi[1] = min(c.L - (t.j0 + 1) * kBlockSize, kBlockSize);
    }
    if (!t.first_gone) {
        t.phys[0] = uniform_load(table, t.j0);
    } else {
        t.phys[0] = t.phys[1];
        t.lo[0] = t.hi[0] = t.lo[1];
    }
    if (!t.second) {
        t.phys[1] = t.phys[0];
        t.lo[1] = t.hi[1] = t.lo[0];
    }
    return t;
}

// A tile whose 32 rows are all visible (it ends inside the context and starts inside every
// window) needs none of the above: two table entries, two slab addresses.
__device__ __forceinline__ bool interior_tile(const Cursor& c, int reach)
{
    const int first = 2 * (c.lt + c.ft) * kBlockSize;
    return first + kTileTokens <= c.L && (reach == 0 || first >= c.L - reach);
}

// The two block ids of such a tile, asked for one tile ahead: the issue side requests the ids of
// the tile it will load NEXT as soon as it has sent the loads of the current one, so the scalar
// loads travel while the wave computes and the next round of LDS-DMA loads starts without a
// round trip to the table.  Returns whether id0 / id1 now hold the ids of the tile `c` stands on;
// false when that tile is not interior (or there is none): the general path then reads its ids
// itself.  (Plain scalars, not a struct: everything here has to stay in scalar registers.)
__device__ __forceinline__ bool ask_next_ids(const int32_t* block_tables, int MB, const Cursor& c, int B, int reach, int& id0,
                                             int& id1)
{
    const bool valid = c.b < B && c.lt < c.nt && interior_tile(c, reach);
    if (valid) {
        const int32_t* table = block_tables + (int64_t)c.b * MB;
        const int j0 = 2 * (c.lt + c.ft);
        id0 = uniform_load(table, j0);
        id1 = uniform_load(table, j0 + 1);
    }
    return valid;
}

// Instrumented runs only.  Before any id becomes an address it is held against the pool: an id
// outside [0, num_blocks) is kept as it stands for the record (`raw`) and block 0 is read in its
// place, so a table with a bad entry at a valid position shows up in the trace instead of as a
// memory fault.  All lanes must call (the ids are wave-uniform).
struct RawIds {
    int id0, id1;  // (plain scalars: an array indexed at run time would live in scratch memory)
};

__device__ __forceinline__ RawIds check_tile_blocks(TileBlocks& t, int num_blocks)
{
    const RawIds raw{t.phys[0], t.phys[1]};
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
        if ((unsigned)t.phys[sub] >= (unsigned)num_blocks) t.phys[sub] = 0;
    return raw;
}

// ... and the record: for logical block j0 + sub of (sequence b, KV head g), slot `which` (0: the
// id the K loads of that block were addressed with, 1: the V loads) and, with the K loads, the
// partition `k` that did it.  Blocks the tile does not read (gone from a sliding window, past the
// context) leave no record.  One lane calls.
__device__ __forceinline__ void trace_block_use(int32_t* trace, const TileBlocks& t, const RawIds& raw, int sub, int which,
                                                int b, int g, int k, int Hkv, int MB)
{
    if (sub == 0 ? t.first_gone : !t.second) return;
    int32_t* v = trace + (((int64_t)b * Hkv + g) * MB + t.j0 + sub) * 3;
    v[which] = sub ? raw.id1 : raw.id0;
    if (which == 0) v[2] = k;
}

// this lane's global byte offset for LDS-DMA instruction r of a slab (rows r*kRowsPerDma ..)
template <int D, int KV>
__device__ __forceinline__ uint32_t slab_dma_offset(int r, int lane)
{
    using Geo = KvGeom<D, KV>;
    const int t = r * Geo::kRowsPerDma + lane / Geo::kPieces;
    return t * Geo::kRow + (((lane % Geo::kPieces) ^ (t & (Geo::kPieces - 1))) << 4);
}

// the same with the stand-in rule applied: rows outside [lo, hi) load row lo instead
template <int D, int KV>
__device__ __forceinline__ uint32_t live_or_stand_in(uint32_t off, int row, int lo, int hi)
{
    using Geo = KvGeom<D, KV>;
    return (row >= lo && row < hi) ? off : lo * Geo::kRow + (off & (Geo::kRow - 1));
}

// ---- one tile: what a wavefront computes on it ---------------------------------------------------
// Per-lane LDS read offsets of the MFMA operands (lane = 16*q4 + n).
template <int D, int KV>
struct OperandOffsets {
    uint32_t kread[D / 32];  // inside a K slab: this lane's operand piece for k-step kk (token n, dims 32kk + 8q4 + [0,8))
    uint32_t vread[D / 16];  // inside the V half of a stage: this lane's transposing-read source for dim tile dt

    __device__ __forceinline__ void init(int n, int q4)
    {
        using Geo = KvGeom<D, KV>;
        constexpr int kMask = Geo::kPieces - 1;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            if (KV == KV_BF16)  // 16 bytes
                kread[kk] = n * Geo::kRow + (((4 * kk + q4) ^ (n & kMask)) << 4);
            else                // 8 bytes: half of 16-byte piece 2kk + q4/2
                kread[kk] = n * Geo::kRow + (((2 * kk + (q4 >> 1)) ^ (n & kMask)) << 4) + ((q4 & 1) << 3);
        }
        // bf16: one read per block, rows = tokens 4q4 + n/4, 8 bytes = 4 dims.  fp8: one read for both blocks,
        // rows n/2 = 0..3 -> tokens 4q4.. of block 0, rows 4..7 -> the same tokens of block 1, 8 bytes = 8 dims.
        if (KV == KV_BF16) {
            const int row = 4 * q4 + (n >> 2);
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt)
                vread[dt] = row * Geo::kRow + ((n & 1) << 3) + (((2 * dt + ((n >> 1) & 1)) ^ (row & kMask)) << 4);
        } else {
            const int r = n >> 1;
            const int tok = 4 * q4 + (r & 3);
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt)
                vread[dt] = (r >> 2) * Geo::kSlab + tok * Geo::kRow + ((dt ^ (tok & kMask)) << 4) + ((n & 1) << 3);
        }
    }
};

// The 16 columns' query rows from an LDS slot (row c at c * 2 D bytes, swizzled like a bf16 K row)
// into MFMA B-operand registers; a padding column gets zeros.
template <int D>
__device__ __forceinline__ void load_query_operand(const char* slot, int n, int q4, bool col_ok, bf16x8 (&qreg)[D / 32])
{
    using QG = QGeom<D>;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        uint4 w = *reinterpret_cast<const uint4*>(slot + (col_ok ? n : 0) * QG::kRow +
                                                  (((4 * kk + q4) ^ (n & (QG::kPieces - 1))) << 4));
        if (!col_ok) w = make_uint4(0, 0, 0, 0);
        qreg[kk] = as_bf16x8(w);
    }
}

// The K operand of k-step kk for the two blocks of the tile (token n, dims 32 kk + 8 q4 + [0, 8))
template <int D, int KV>
__device__ __forceinline__ void load_k_operand(const char* kbuf, const OperandOffsets<D, KV>& of, int kk, bf16x8& a0, bf16x8& a1)
{
    constexpr int kSlabBytes = KvGeom<D, KV>::kSlab;
    if (KV == KV_BF16) {
        a0 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + of.kread[kk]));
        a1 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + kSlabBytes + of.kread[kk]));
    } else {
        const uint2 w0 = *reinterpret_cast<const uint2*>(kbuf + of.kread[kk]);
        const uint2 w1 = *reinterpret_cast<const uint2*>(kbuf + kSlabBytes + of.kread[kk]);
        a0 = fp8x8_to_bf16x8(w0.x, w0.y);
        a1 = fp8x8_to_bf16x8(w1.x, w1.y);
    }
}

// S^T[token, column] = K . Q^T for the two blocks of the tile and NCT tiles of 16 columns; the K
// operand is read (and, fp8, converted) once for all of them
template <int D, int KV, int NCT>
__device__ __forceinline__ void qk_scores(const char* kbuf, const OperandOffsets<D, KV>& of,
                                          const bf16x8 (&qreg)[NCT][D / 32], f32x4 (&s0)[NCT], f32x4 (&s1)[NCT])
{
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        s0[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
        s1[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        bf16x8 a0, a1;
        load_k_operand<D, KV>(kbuf, of, kk, a0, a1);
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            s0[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qreg[ct][kk], s0[ct], 0, 0, 0);
            s1[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qreg[ct][kk], s1[ct], 0, 0, 0);
        }
    }
}

// Do the softmax weights enter the PV product with their rounding remainder (two bf16 numbers per
// weight) or as one bf16 number?  By default the remainder is kept where it is free: bf16 KV in a
// wave with one 16-column tile, which waits for memory either way (plain decode above all).  It is
// dropped where the second matrix instruction per operand costs time: fp8 KV (the weights keep 8
// significant bits against the 4 of the values they multiply; 70B-head-shaped batch 365 -> 343 us),
// waves with two column tiles and the multi-wave kernel (16 query tokens on long contexts
// 450 -> 407 us, the shared-prefix pass 53 -> 48 us per step).  The error this leaves is at most
// 2^-9 max|v| and in practice a few 1e-3 for values of unit size.  A caller that needs more (values
// of larger magnitude, an accuracy gate on generated text) sets pa_shape.precise_weights, which
// keeps the remainder on every path (the kernels' PRECISE parameter).
constexpr bool p_has_low_part(int kv, int nct, bool multi_wave) { return kv == KV_BF16 && nct == 1 && !multi_wave; }

// Online softmax state of one column (replicated over the four lanes that hold its tokens) and
// the unnormalised output accumulators out^T[dim, column].  The running sum of the weights is an
// accumulator of the matrix pipe as well: the PV step multiplies the weights by a row of ones
// next to the value rows, so the sum costs no vector instructions, needs no reduction over the
// four lanes at the end (every element of lacc is the column's total), and is the sum of exactly
// the rounded weights that multiplied the values.
template <int D>
struct ColumnState {
    float m;
    f32x4 lacc;
    f32x4 acc[D / 16];

    // once, before a wave's first tile
    __device__ __forceinline__ void clear()
    {
        m = kNegBig;
        lacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // A new segment begins.  Only the maximum is reset: the column's first visible score will find
    // m == kNegBig and wipe the accumulators with a rescale factor of zero (online_softmax), so no
    // accumulator is written here, on a path every tile's control flow would have to merge with.
    // Until then they hold the (finite) left-overs of the previous segment: seen() says whether
    // the column has anything of its own.
    __device__ __forceinline__ void reset() { m = kNegBig; }

    __device__ __forceinline__ bool seen() const { return m > kNegBig; }
    __device__ __forceinline__ float weight_sum() const { return lacc[0]; }
};

// The running maximum is raised only when a score exceeds it by more than this (log2 domain):
// weights then reach 2^6 at most, which float32 sums and bf16 operands hold as well as values
// below 1, and the cross-lane maximum, the rescale factor and the rescaling of the accumulators
// leave the common path (after a sequence's first tiles the maximum rarely moves that far).
constexpr float kLazyMax = 6.f;

// Largest / smallest of a lane's eight scores in four instructions (v_maximum3_f32 / v_minimum3_f32).
// Written with fmaxf the compiler first passes every matrix-instruction result through a
// v_max_f32 x, x, x of its own, the quieting of signalling NaNs that the C function promises:
// seven more instructions per column tile and step.  These propagate a NaN instead of skipping
// it; a column with a NaN score ends as a NaN row either way, through its weights.
__device__ __forceinline__ float max8_f32(const f32x4& a, const f32x4& b)
{
    const float x = __builtin_elementwise_maximum(__builtin_elementwise_maximum(a[0], a[1]), a[2]);
    const float y = __builtin_elementwise_maximum(__builtin_elementwise_maximum(a[3], b[0]), b[1]);
    const float z = __builtin_elementwise_maximum(__builtin_elementwise_maximum(b[2], b[3]), x);
    return __builtin_elementwise_maximum(y, z);
}
__device__ __forceinline__ float min8_f32(const f32x4& a, const f32x4& b)
{
    const float x = __builtin_elementwise_minimum(__builtin_elementwise_minimum(a[0], a[1]), a[2]);
    const float y = __builtin_elementwise_minimum(__builtin_elementwise_minimum(a[3], b[0]), b[1]);
    const float z = __builtin_elementwise_minimum(__builtin_elementwise_minimum(b[2], b[3]), x);
    return __builtin_elementwise_minimum(y, z);
}

// Online softmax step (log2 domain) on the tile's scores.  The lane's tokens are t0 + {0..3} and
// t0 + 16 + {0..3}; with MASKED the column sees only tokens low <= t < lim (the end of the context,
// the causal limit of a multi-token call, the start of a sliding window); without it the whole tile.
// qs (softmax scale * log2 e, times the K scale for fp8) is folded into the exponent:
// weight = 2^(s * qs - m).  Leaves the P^T operand in bf16.  With P_LO it is a pair, high part +
// rounding remainder (16 significant bits: the weights lose nothing that matters against the fp32
// accumulation) and the PV product costs two matrix instructions per operand; without, the weights
// enter at bf16 precision (relative rounding error <= 2^-9 each, unbiased) and pb_lo is left alone.
// See p_has_low_part().
template <bool MASKED, int D, bool P_LO>
__device__ __forceinline__ void online_softmax(const f32x4& s0, const f32x4& s1, float qs, int t0, int lim, int low,
                                               ColumnState<D>& st, bf16x8& pb, bf16x8& pb_lo)
{
    // Two ways to the same exponents.  PRODUCTS: every score is scaled first and the maximum is taken
    // over the products, so the largest one meets itself in the subtraction and its weight is exactly
    // 1 (a context of one token returns its value row bit for bit even when the weights carry their
    // low part); used where instructions are free (P_LO) and on masked tiles.  Otherwise the maximum
    // is taken over the raw scores and scale and subtraction are one fused multiply-add per score.
    constexpr bool PRODUCTS = MASKED || P_LO;
    float v[8];
    bool ok[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        v[r] = s0[r];
        v[4 + r] = s1[r];
        ok[r] = !MASKED || (t0 + r < lim && t0 + r >= low);
        ok[4 + r] = !MASKED || (t0 + kBlockSize + r < lim && t0 + kBlockSize + r >= low);
    }
    // the largest exponent among this lane's visible tokens
    float mx;
    if (PRODUCTS) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = ok[r] ? v[r] * qs : kNegBig;
        mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    } else if (qs >= 0.f) {  // the same for every lane
        mx = max8_f32(s0, s1) * qs;
    } else {
        mx = min8_f32(s0, s1) * qs;
    }
    if (__any(mx > st.m + kLazyMax)) {
        const float m_new = fmaxf(st.m, rows_max(mx));
        // nothing seen so far: the accumulators hold the previous segment's values, drop them
        const float alpha = st.seen() ? fast_exp2(st.m - m_new) : 0.f;
        st.m = m_new;
        st.lacc *= alpha;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) st.acc[dt] *= alpha;
    }
    const float neg_m = -st.m;
    float x[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (PRODUCTS)
            x[r] = ok[r] ? fast_exp2(v[r] - st.m) : 0.f;  // a column may see nothing of a tile
        else
            x[r] = fast_exp2(fmaf(v[r], qs, neg_m));
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        pb[r] = (__bf16)x[r];
        if (P_LO) pb_lo[r] = (__bf16)(x[r] - (float)pb[r]);
    }
}

// out^T[dim, column] += V^T . P^T for NCT tiles of 16 columns; the V^T operand is read (and, fp8,
// converted) once for all of them.  A row of ones joins the value rows: its product is the sum of
// the column's weights (ColumnState::lacc).
template <int D, int KV, int NCT, bool P_LO>
__device__ __forceinline__ void pv_accumulate(const char* vbuf, const OperandOffsets<D, KV>& of, const bf16x8 (&pb)[NCT],
                                              const bf16x8 (&pb_lo)[NCT], ColumnState<D> (&st)[NCT])
{
    constexpr int kSlabBytes = KvGeom<D, KV>::kSlab;
    const __bf16 one = (__bf16)1.0f;
    const bf16x8 ones{one, one, one, one, one, one, one, one};
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        st[ct].lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[ct], st[ct].lacc, 0, 0, 0);
        if (P_LO) st[ct].lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb_lo[ct], st[ct].lacc, 0, 0, 0);
    }
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
        bf16x8 va;
        if (KV == KV_BF16) {
            const i16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + of.vread[dt]));
            const i16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + kSlabBytes + of.vread[dt]));
            va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            const i32x2 v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)(vbuf + of.vread[dt]));
            va = fp8x8_to_bf16x8((uint32_t)v[0], (uint32_t)v[1]);
        }
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            st[ct].acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[ct], st[ct].acc[dt], 0, 0, 0);
            if (P_LO)
                st[ct].acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb_lo[ct], st[ct].acc[dt], 0, 0, 0);
        }
    }
}

// One column's D output values times `inv`, as float32 to `dst` (a partial row in the workspace)
template <int D>
__device__ __forceinline__ void store_partial_row(float* dst, const ColumnState<D>& st, float inv, int q4)
{
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        *reinterpret_cast<float4*>(dst + 16 * dt + 4 * q4) =
            make_float4(st.acc[dt][0] * inv, st.acc[dt][1] * inv, st.acc[dt][2] * inv, st.acc[dt][3] * inv);
}

// ... or as a final row of `out` (element index `row`), in the output's type
template <int D>
__device__ __forceinline__ void store_final_row(const Params& p, int64_t row, const ColumnState<D>& st, float inv, int q4)
{
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        store_out4(p, row + 16 * dt + 4 * q4, st.acc[dt][0] * inv, st.acc[dt][1] * inv, st.acc[dt][2] * inv,
                   st.acc[dt][3] * inv);
}

}  // namespace pa
