// Partition kernel, matrix-core variant (head_dim 128 or 64, bf16 or fp8 KV) for up to 32 columns.
// The columns of its matrix tile are the (query token, query head) pairs that share one KV
// head: q_len * G of them (plain decode: the G heads of the group), padded to CPAD = 4, 8 or
// 16 inside one 16-column MFMA tile, or to 32 = two such tiles that share every K and V operand
// read.  One wavefront per (partition, KV head) walks its balanced range of the batch's global
// tile sequence (see pa_plan.hpp); no workgroup barriers, no atomics.  More columns than 32 go
// to the multi-wave kernel in pa_partition_mfma_wide.hpp.
//
// Data path per 32-token tile (two KV blocks; layouts and the per-tile arithmetic are in
// pa_mfma_tile.hpp):
//   HBM --global_load_lds (16 B/lane, 1 KB per instruction)--> LDS ring of NSTAGE tiles
//   K:  ds_read_b128 in MFMA operand layout -> S^T[token, column] = K . Q^T  (mfma 16x16x32 bf16)
//   online softmax on S^T in registers (lane = column, 8 tokens per lane per tile)
//   V:  ds_read_b64_tr_b16 (transposing LDS read) -> out^T[dim, column] += V^T . P^T
// The ring keeps running across sequence boundaries inside the range; the query rows of each new
// sequence travel through a small LDS ring of their own, ahead of its first tile.
//
// Multi-token calls (q_len > 1) are causal inside the new tokens: query i of a sequence of L
// tokens sits at position L - q_len + i and sees tokens 0 .. L - q_len + i.
//
// Wait-count discipline: the LDS-DMA loads are issued and awaited by hand (s_waitcnt vmcnt(N)
// with N = number of *newer DMA loads* allowed to stay in flight).  Loads complete in order,
// so "at most N operations outstanding" implies every load older than the newest N has landed,
// whatever else (stores, extra loads) is in flight: other traffic only makes a wait stricter.
// Everything else the loop needs from memory comes through the scalar cache (block ids,
// context lengths), which the vector-memory counter does not see.  The LDS-DMA destination
// travels in M0, which the inline asm takes as an input operand, so the compiler sets it and
// knows that it did.
#pragma once
#include "pa_device.hpp"
#include "pa_mfma_tile.hpp"
#include "pa_plan.hpp"

namespace pa {

// bytes of one tile (K block 0, K block 1, V block 0, V block 1) in LDS
constexpr int mfma_stage_bytes(int d, int kv)
{
    return d == 128 ? (kv == KV_BF16 ? KvGeom<128, KV_BF16>::kStage : KvGeom<128, KV_FP8>::kStage)
                    : (kv == KV_BF16 ? KvGeom<64, KV_BF16>::kStage : KvGeom<64, KV_FP8>::kStage);
}

// LDS-DMA loads that bring in the query rows of `cpad` columns, 1 KB each
constexpr int mfma_q_loads(int d, int cpad)
{
    return (cpad * 2 * d + 1023) / 1024;
}

// Two column tiles keep ONE slot of query rows and refill it with the rows of the next segment
// as soon as the current ones are in registers (as the multi-wave kernel does); one column tile
// keeps a ring of NSTAGE slots filled just ahead of each segment's first tile.
constexpr bool mfma_one_q_slot(int cpad) { return cpad > 16; }

// LDS bytes one workgroup (one wave) of the kernel uses: tile ring + query-row slots.
constexpr int mfma_lds_bytes(int d, int nstage, int cpad, int kv)
{
    return nstage * mfma_stage_bytes(d, kv) + (mfma_one_q_slot(cpad) ? 1 : nstage) * mfma_q_loads(d, cpad) * 1024;
}

// wait until at most `later_tiles` whole tiles (PER_TILE loads each, at most MAXT tiles) plus EXTRA
// loads are still in flight
template <int EXTRA, int PER_TILE, int MAXT>
__device__ __forceinline__ void wait_tile(int later_tiles)
{
    static_assert(MAXT * PER_TILE + EXTRA <= 63, "vmcnt is a 6-bit counter");
    if constexpr (MAXT == 0) {
        wait_vmcnt<EXTRA>();
    } else {
        if (later_tiles >= MAXT) wait_vmcnt<MAXT * PER_TILE + EXTRA>();
        else wait_tile<EXTRA, PER_TILE, MAXT - 1>(later_tiles);
    }
}

// PRECISE: the softmax weights keep their low part on every path (see p_has_low_part).
template <int D, int NSTAGE, int CPAD, int KV, bool TRACE, bool PRECISE>
__global__ __launch_bounds__(64) void partition_mfma_kernel(const Params p)
{
    static_assert(NSTAGE >= 2 && NSTAGE <= 8, "ring depth");
    static_assert(CPAD == 4 || CPAD == 8 || CPAD == 16 || CPAD == 32, "padded column count");
    constexpr int NCT = CPAD > 16 ? CPAD / 16 : 1;  // MFMA column tiles
    constexpr bool P_LO = PRECISE || p_has_low_part(KV, NCT, false);
    using Geo = KvGeom<D, KV>;
    using QG = QGeom<D>;
    constexpr int kSlabBytes = Geo::kSlab;
    constexpr int kStageBytes = Geo::kStage;
    constexpr int kDmaPerTile = Geo::kDmaPerTile;
    constexpr int kQLoads = mfma_q_loads(D, CPAD);
    constexpr int kQSlot = kQLoads * 1024;
    constexpr bool ONE_SLOT = mfma_one_q_slot(CPAD);
    static_assert(mfma_lds_bytes(D, NSTAGE, CPAD, KV) <= 65536, "static LDS limit");
    __shared__ __attribute__((aligned(1024))) char smem[mfma_lds_bytes(D, NSTAGE, CPAD, KV)];

    const int lane = threadIdx.x;
    // partition index fastest: workgroups go to the chip's eight dies round-robin, so (with P a
    // multiple of 8) the waves of all KV heads of one partition share a die and read the
    // contiguous slabs of each physical block from there (measured 0.5-1.4 % faster than head-fastest)
    const int g = blockIdx.x / p.P;
    const int k = blockIdx.x % p.P;
    const int G = p.G;
    const int B = p.B;
    const int Q = p.Q;
    const int ncols = Q * G;   // real columns: (query token i, head h of the group) -> column i*G + h
    const int n = lane & 15;   // column of the tile / row-in-block, depending on the operand
    const int q4 = lane >> 4;  // 0..3
    // Tiles the plan leaves out at the head of every sequence.  Shared-prefix calls: the first
    // skip tiles belong to the prefix pass, and no row this kernel writes is final (the merge adds
    // the prefix part).  Sliding window: nothing further back than window + Q - 1 tokens from the
    // end of a context is visible to any query, and blocks before that are never touched.
    const int skip = p.skip_tiles;
    const int reach = p.window > 0 ? p.window + Q - 1 : 0;
    const Span sp{skip, reach};

    // ---- this wave's range of the global tile sequence
    const RangeStart rs = find_range(p.context_lens, B, k, p.P, lane, sp);
    if (skip == 0) zero_rows_of_empty_contexts(p, k, g, B, Q, D, lane);  // (behind a shared prefix no context is empty)
    const bool describes = g == 0 && p.merge_desc != nullptr;  // this wave tells the merge about its sequences
    if (describes && p.cut_list != nullptr && lane == 0)  // does my range start inside a sequence, and which
        p.cut_list[k] = (rs.t_lo < rs.T && rs.t_lo > rs.cum) ? rs.b : -1;
    if (rs.t_lo >= rs.t_hi) return;
    const int ntiles = rs.t_hi - rs.t_lo;
    const int first_b = rs.b;
    Cursor ic;  // issue side
    ic.b = first_b;
    ic.lt = rs.t_lo - rs.cum;
    ic.L = rs.L;
    ic.nt = tiles_of(ic.L, sp);
    ic.ft = first_tile(ic.L, sp);
    Cursor cc = ic;  // compute side

    // ---- per-lane address pieces
    uint32_t dma_off[Geo::kDmaPerSlab];  // LDS-DMA of a KV slab, instruction r
    int dma_row[Geo::kDmaPerSlab];       // the token row of the block it loads
#pragma unroll
    for (int r = 0; r < Geo::kDmaPerSlab; ++r) {
        dma_off[r] = slab_dma_offset<D, KV>(r, lane);
        dma_row[r] = r * Geo::kRowsPerDma + lane / Geo::kPieces;
    }
    // LDS-DMA of the query rows (always bf16: 1 KB, i.e. 4 or 8 rows, per instruction).  LDS row c
    // holds column c, i.e. query token c / G, head c % G of this group; padding rows re-read column 0.
    uint32_t qdma_off[kQLoads];
#pragma unroll
    for (int r = 0; r < kQLoads; ++r) {
        const int c = r * QG::kRowsPerDma + lane / QG::kPieces;
        const int src = c < ncols ? ((c / G) * p.Hq + (c % G)) * QG::kRow : 0;
        qdma_off[r] = src + (((lane % QG::kPieces) ^ (c & (QG::kPieces - 1))) << 4);
    }
    OperandOffsets<D, KV> of;
    of.init(n, q4);
    // this lane's columns: 16 ct + n of column tile ct
    bool col_ok[NCT];   // a real column
    int col_back[NCT];  // tokens at the end of the context its query must not see
    int col_row[NCT];   // its output row inside its sequence
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int c = 16 * ct + n;
        col_ok[ct] = c < ncols;
        const int col_i = col_ok[ct] ? c / G : 0, col_h = col_ok[ct] ? c % G : 0;
        col_back[ct] = col_ok[ct] ? Q - 1 - col_i : (1 << 30);
        col_row[ct] = col_i * p.Hq + g * G + col_h;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t ldsq = lds0 + NSTAGE * kStageBytes;
    const char* qslots = smem + NSTAGE * kStageBytes;

    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;  // bytes between physical blocks
    const uint32_t head_stride32 = (uint32_t)p.Hkv * (uint32_t)kSlabBytes;  // the same; the host keeps it below 2^32
    const char* kc = static_cast<const char*>(p.k_cache) + (int64_t)g * kSlabBytes;
    const char* vc = static_cast<const char*>(p.v_cache) + (int64_t)g * kSlabBytes;

    int q_issue = 0;  // query slot the issue side fills next
    auto issue_q = [&](int b) __attribute__((always_inline)) {
        const char* qb = reinterpret_cast<const char*>(p.q) + ((int64_t)b * p.QH + g * G) * QG::kRow;
#pragma unroll
        for (int r = 0; r < kQLoads; ++r) dma16<false>(ldsq + q_issue * kQSlot + r * 1024, qdma_off[r], qb);
        if (!ONE_SLOT) q_issue = (q_issue + 1 == NSTAGE) ? 0 : q_issue + 1;
    };
    int nx_id0 = 0, nx_id1 = 0;  // ids of the tile `ic` stands on ...
    bool nx_valid = false;       // ... if they were asked for ahead
    auto issue = [&](int i, int stage) __attribute__((always_inline)) {
        // ring of slots: a new segment starts, send its query rows ahead of its first tile
        if (!ONE_SLOT && (i == 0 || ic.lt == 0)) issue_q(ic.b);
        const uint32_t ldst = lds0 + stage * kStageBytes;
        if (!TRACE && nx_valid) {
            // interior tile, ids already here: every row is visible
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const char* kb = kc + (uint64_t)(uint32_t)(sub ? nx_id1 : nx_id0) * head_stride32;
#pragma unroll
                for (int r = 0; r < Geo::kDmaPerSlab; ++r) dma16<true>(ldst + sub * kSlabBytes + r * 1024, dma_off[r], kb);
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const char* vb = vc + (uint64_t)(uint32_t)(sub ? nx_id1 : nx_id0) * head_stride32;
#pragma unroll
                for (int r = 0; r < Geo::kDmaPerSlab; ++r)
                    dma16<true>(ldst + 2 * kSlabBytes + sub * kSlabBytes + r * 1024, dma_off[r], vb);
            }
        } else {
            TileBlocks tb = tile_blocks(p.block_tables, p.MB, ic, reach);
            RawIds raw{};
            if (TRACE) raw = check_tile_blocks(tb, p.num_blocks);
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const char* kb = kc + tb.phys[sub] * head_stride;
                if (TRACE && lane == 0) trace_block_use(p.trace_blocks, tb, raw, sub, 0, ic.b, g, k, p.Hkv, p.MB);
#pragma unroll
                for (int r = 0; r < Geo::kDmaPerSlab; ++r)
                    dma16<true>(ldst + sub * kSlabBytes + r * 1024,
                          live_or_stand_in<D, KV>(dma_off[r], dma_row[r], tb.lo[sub], tb.hi[sub]), kb);
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const char* vb = vc + tb.phys[sub] * head_stride;
                if (TRACE && lane == 0) trace_block_use(p.trace_blocks, tb, raw, sub, 1, ic.b, g, k, p.Hkv, p.MB);
#pragma unroll
                for (int r = 0; r < Geo::kDmaPerSlab; ++r)
                    dma16<true>(ldst + 2 * kSlabBytes + sub * kSlabBytes + r * 1024,
                          live_or_stand_in<D, KV>(dma_off[r], dma_row[r], tb.lo[sub], tb.hi[sub]), vb);
            }
        }
        advance(ic, p.context_lens, B, sp);
        nx_valid = ask_next_ids(p.block_tables, p.MB, ic, B, reach, nx_id0, nx_id1);
    };

    // ---- online softmax state: lane = column n, tokens 4*q4+{0..3} of each block
    const float qs = KV == KV_FP8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;  // K scale folded in
    const float vs = KV == KV_FP8 ? p.v_scale[g] : 1.f;
    ColumnState<D> st[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) st[ct].clear();
    bf16x8 qreg[NCT][D / 32];
    int q_comp = 0;       // query slot of the segment being computed
    int seg_first_lt = 0;

    // ---- prologue: (one slot: the first segment's query rows,) fill the ring
    if (ONE_SLOT) issue_q(first_b);
    int q_age = 0;  // one slot: tiles issued since the slot was last refilled
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t)
        if (t < ntiles) {
            issue(t, t);
            ++q_age;
        }

    int stage = 0;
    for (int tile = 0; tile < ntiles; ++tile) {
        // refill the buffer consumed in the previous iteration (its LDS reads have all returned)
        const int ahead = tile + NSTAGE - 1;
        if (ahead < ntiles) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            int stg = stage + NSTAGE - 1;
            if (stg >= NSTAGE) stg -= NSTAGE;
            issue(ahead, stg);
            ++q_age;
        }
        const int later = min(NSTAGE - 1, ntiles - 1 - tile);
        const char* kbuf = smem + stage * kStageBytes;
        const char* vbuf = kbuf + 2 * kSlabBytes;

        // K of this tile and its segment's query rows have landed.  Ring of slots: the rows were
        // issued just before the K loads.  One slot: they were issued q_age tiles ago, which after a
        // segment shorter than the ring is later than this tile's loads; then nothing but the tiles
        // issued after the rows may still be in flight.
        if (ONE_SLOT && (tile == 0 || cc.lt == 0) && q_age <= later)
            wait_tile<0, kDmaPerTile, NSTAGE - 1>(q_age);
        else
            wait_tile<kDmaPerTile / 2, kDmaPerTile, NSTAGE - 1>(later);
        bool refilled = false;  // one slot: query rows of the next segment were issued in this iteration
        const bool seg_start = tile == 0 || cc.lt == 0;
        if (seg_start) {
            seg_first_lt = cc.lt;
            if (describes && cc.lt == 0 && lane == 0) {  // the sequence's first tile is mine
                const int cum = rs.t_lo + tile, end = cum + cc.nt;
                write_seq_desc(p.merge_desc, cc.b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
            }
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                st[ct].reset();
                load_query_operand<D>(qslots + q_comp * kQSlot + ct * 16 * QG::kRow, n, q4, col_ok[ct], qreg[ct]);
            }
            if (!ONE_SLOT) {
                q_comp = (q_comp + 1 == NSTAGE) ? 0 : q_comp + 1;
            } else if (tile + (cc.nt - cc.lt) < ntiles) {
                // refill the slot with the rows of the next segment of this range
                int nb = cc.b;
                do {
                    ++nb;
                } while (nb < B - 1 && tiles_of(uniform_load(p.context_lens, nb), sp) == 0);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slot has been read
                issue_q(nb);
                q_age = 0;
                refilled = true;
            }
        }

        f32x4 s0[NCT], s1[NCT];
        qk_scores<D, KV, NCT>(kbuf, of, qreg, s0, s1);

        // The column sees tokens low <= t < lim.  Only the last tiles of a sequence (the end of the
        // context, the causal limits of a multi-token call) and the tiles where sliding windows begin
        // need the mask: everywhere else every column sees the whole tile.
        const int tile_first = (cc.lt + cc.ft) * kTileTokens;
        const int t0 = tile_first + 4 * q4;
        const bool unmasked = tile_first + kTileTokens <= cc.L - (Q - 1) && (reach == 0 || tile_first >= cc.L - p.window);
        bf16x8 pb[NCT], pb_lo[NCT];
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            const int lim = cc.L - col_back[ct];
            const int low = p.window > 0 ? lim - p.window : INT32_MIN;  // first token the column's window holds
            if (unmasked)
                online_softmax<false, D, P_LO>(s0[ct], s1[ct], qs, t0, lim, low, st[ct], pb[ct], pb_lo[ct]);
            else
                online_softmax<true, D, P_LO>(s0[ct], s1[ct], qs, t0, lim, low, st[ct], pb[ct], pb_lo[ct]);
        }

        // V of this tile landed (query rows just issued are newer and may stay in flight)
        if (ONE_SLOT && refilled)
            wait_tile<kQLoads, kDmaPerTile, NSTAGE - 1>(later);
        else
            wait_tile<0, kDmaPerTile, NSTAGE - 1>(later);
        pv_accumulate<D, KV, NCT, P_LO>(vbuf, of, pb, pb_lo, st);

        // ---- segment end: normalise, write
        if (cc.lt == cc.nt - 1 || tile == ntiles - 1) {
            const bool whole = seg_first_lt == 0 && cc.lt == cc.nt - 1;  // the entire sequence: final result
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const float l = st[ct].weight_sum();
                if (col_ok[ct]) {
                    // a column that saw no token (its query sits before this segment) leaves a zero
                    // row with an "empty" log-sum-exp
                    const bool seen = st[ct].seen();
                    const float inv = seen ? vs / l : 0.f;
                    const float lse = seen ? st[ct].m + fast_log2(l) : kNegBig;
                    if (whole && skip > 0) {  // final but for the prefix part: to the workspace, for the prefix merge
                        const int64_t row = (int64_t)cc.b * p.QH + col_row[ct];
                        if (q4 == 0) p.seq_lse[row] = lse;
                        store_partial_row(p.seq_o + row * D, st[ct], inv, q4);
                    } else if (whole) {
                        store_final_row(p, ((int64_t)cc.b * p.QH + col_row[ct]) * D, st[ct], inv, q4);
                    } else {
                        const int64_t slot = ((int64_t)2 * k + (cc.b != first_b ? 1 : 0)) * p.QH + col_row[ct];
                        if (q4 == 0) p.part_lse[slot] = lse;
                        store_partial_row(p.part_o + slot * D, st[ct], inv, q4);
                    }
                }
            }
        }
        advance(cc, p.context_lens, B, sp);
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }
}

}  // namespace pa
