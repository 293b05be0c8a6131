// Partition kernel, matrix-core variant for many columns per KV head (multi-token verification,
// wide groups: up to 128 (query token, query head) pairs per workgroup, further workgroups side by
// side beyond that).  A workgroup of NW
// wavefronts serves one (partition, KV head): the waves share ONE ring of K/V tiles in LDS, so
// the cache is read from HBM once for all columns, and each wave computes its own NCT = 1 or 2
// tiles of 16 columns (columns 16 NCT w .. 16 NCT (w + 1) - 1) exactly as the single-wave kernel
// does: same operand layouts, same swizzle, same online softmax (pa_mfma_tile.hpp; wait-count
// discipline as described in pa_partition_mfma.hpp).  Two tiles share every K and V operand read
// and every fp8 conversion.
//
// Per tile, every wave loads 1/NW of the tile's LDS-DMA instructions and the workgroup meets at
// one barrier:
//     wait for my own loads of tile t          (s_waitcnt vmcnt, counted by hand)
//     s_barrier                                (all parts of tile t are in LDS; everyone is done
//                                               reading tile t-1, whose buffer is refilled next)
//     issue my part of tile t + NSTAGE - 1
//     scores, online softmax, PV for my columns on tile t
// All waves of a workgroup walk the same range, so they execute the same number of barriers.
//
// Query rows: every wave keeps ONE private LDS slot (16 rows) for the rows of its own
// columns.  At the start of a segment it moves the slot into registers and at once refills the
// slot with the rows of the next segment in its range, so the rows are there long before that
// segment's first tile; after a short segment (fewer tiles than the ring is deep) the wait at
// the segment start is tightened to cover those loads (q_age below).
//
// PREFIX mode is the pass over a prefix that every sequence of a decode batch shares (the same
// physical blocks at the head of every block table).  The columns are then the (sequence, head)
// pairs: to this kernel the batch is ONE sequence, the prefix, with one "query token" per real
// sequence (or Q of them in a multi-token call: every query token lies after the prefix and sees
// all of it) and no causal mask.  The prefix tiles are cut into Pp ranges, workgroup
// (column group, KV head, range) leaves one partial result per column, and the prefix merge
// kernel adds them to what the per-sequence pass computed over the rest of each context.
#pragma once
#include <type_traits>

#include "pa_device.hpp"
#include "pa_mfma_tile.hpp"
#include "pa_plan.hpp"

namespace pa {

// one wave's query rows: nct tiles of 16 columns
constexpr int wide_q_slot_bytes(int d, int nct) { return nct * 16 * 2 * d; }

constexpr int mfma_wide_lds_bytes(int d, int nw, int nct, int nstage, int kv)
{
    return nstage * mfma_stage_bytes(d, kv) + nw * wide_q_slot_bytes(d, nct);
}

// wait until at most `tiles` * PER_TILE of this wave's loads are still in flight (tiles clamped to MAXT)
template <int PER_TILE, int MAXT>
__device__ __forceinline__ void wait_loads(int tiles)
{
    static_assert(MAXT * PER_TILE <= 63, "vmcnt is a 6-bit counter");
    if constexpr (MAXT == 0) {
        wait_vmcnt<0>();
    } else {
        if (tiles >= MAXT) wait_vmcnt<MAXT * PER_TILE>();
        else wait_loads<PER_TILE, MAXT - 1>(tiles);
    }
}

// The second launch bound (two waves per SIMD, where the workgroup's LDS lets that happen at all)
// caps the register budget at 256, which makes the compiler keep the MFMA accumulators in ordinary
// VGPRs: with more it parks them in AGPRs and moves all 32 to VGPRs and back in every tile around
// the rarely taken rescale branch.
template <int D, int NW, int NCT, int NSTAGE, int KV, bool TRACE, bool PREFIX, bool PRECISE>
__global__ __launch_bounds__(NW * 64, NW >= 4 ? 2 : 1) void partition_mfma_wide_kernel(const Params p)
{
    static_assert(NW == 2 || NW == 4 || NW == 8, "waves per workgroup");
    static_assert(NCT == 1 || NCT == 2, "MFMA column tiles per wave");
    constexpr int kWaveCols = 16 * NCT;  // columns one wave computes
    constexpr bool P_LO = PRECISE || p_has_low_part(KV, NCT, true);
    static_assert(NSTAGE >= 3, "the ring holds the tile in use, the one being refilled and at least one in flight");
    using Geo = KvGeom<D, KV>;
    using QG = QGeom<D>;
    constexpr int kSlabBytes = Geo::kSlab;
    constexpr int kStageBytes = Geo::kStage;
    // LDS-DMA instructions per tile and loading wave: the tile's loads divide evenly over the
    // waves, or (small tiles) over the first of them and the others load only their query rows
    constexpr int PT = Geo::kDmaPerTile >= NW ? Geo::kDmaPerTile / NW : 1;
    static_assert(Geo::kDmaPerTile % PT == 0 && (Geo::kDmaPerTile >= NW ? PT * NW == Geo::kDmaPerTile : true),
                  "shares of a tile's loads");
    constexpr int kMaxLater = NSTAGE - 2;      // tiles in flight behind the one a wave waits for
    constexpr int kQSlotBytes = wide_q_slot_bytes(D, NCT);
    constexpr int kQLoads = kQSlotBytes / 1024;
    static_assert(mfma_wide_lds_bytes(D, NW, NCT, NSTAGE, KV) <= 160 * 1024, "LDS of one compute unit");
    __shared__ __attribute__((aligned(1024))) char smem[mfma_wide_lds_bytes(D, NW, NCT, NSTAGE, KV)];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // partition index fastest, as in the single-wave kernel; then the KV head, then (prefix pass
    // with more than 16*NW columns) the column group
    const int nparts = PREFIX ? p.Pp : p.P;
    const int k = blockIdx.x % nparts;
    const int g = (blockIdx.x / nparts) % p.Hkv;
    const int col0 = (blockIdx.x / nparts / p.Hkv) * (kWaveCols * NW);
    const int G = p.G;
    const int B = PREFIX ? 1 : p.B;      // sequences as this kernel sees them
    const int Q = PREFIX ? p.B * p.Q : p.Q;  // query tokens per such sequence (prefix pass: those of all real sequences)
    const int ncols = Q * G;
    const int n = lane & 15;
    const int q4 = lane >> 4;

    // sliding window (never together with a shared prefix): see the single-wave kernel.  In the
    // per-sequence pass of a shared-prefix call the first skip tiles of every sequence belong to the
    // prefix pass, and no row this pass writes is final (the prefix merge adds the prefix part).
    const int reach = (!PREFIX && p.window > 0) ? p.window + Q - 1 : 0;
    const int skip = PREFIX ? 0 : p.skip_tiles;
    const Span sp{skip, reach};
    RangeStart rs;
    if (PREFIX) {
        rs.T = p.skip_tiles;
        rs.t_lo = part_begin(k, rs.T, nparts);
        rs.t_hi = part_begin(k + 1, rs.T, nparts);
        rs.b = 0;
        rs.cum = 0;
        rs.L = rs.T * kTileTokens;
    } else {
        rs = find_range(p.context_lens, B, k, p.P, lane, sp);
    }
    if (!PREFIX && skip == 0 && w == 0 && col0 == 0) zero_rows_of_empty_contexts(p, k, g, B, Q, D, lane);  // (behind a shared prefix no context is empty)
    const bool describes = !PREFIX && g == 0 && w == 0 && col0 == 0 && p.merge_desc != nullptr;  // tells the merge about its sequences
    if (describes && p.cut_list != nullptr && lane == 0)  // does my range start inside a sequence, and which
        p.cut_list[k] = (rs.t_lo < rs.T && rs.t_lo > rs.cum) ? rs.b : -1;
    if (rs.t_lo >= rs.t_hi) return;  // the same for every wave of the workgroup
    const int ntiles = rs.t_hi - rs.t_lo;
    const int first_b = rs.b;
    Cursor ic;
    ic.b = first_b;
    ic.lt = rs.t_lo - rs.cum;
    ic.L = rs.L;
    ic.nt = tiles_of(ic.L, sp);
    ic.ft = first_tile(ic.L, sp);
    Cursor cc = ic;

    // ---- this wave's share of a tile's loads: instructions w*PT .. w*PT+PT-1 of the tile's
    // kDmaPerTile, numbered slab by slab (K block 0, K block 1, V block 0, V block 1)
    int my_slab[PT];       // 0..3
    uint32_t my_dst[PT];   // LDS byte offset inside a stage
    uint32_t my_off[PT];   // this lane's global byte offset inside the slab (swizzled piece)
    int my_tok[PT];        // token row of the block this lane loads
    const bool loader = w * PT < Geo::kDmaPerTile;
#pragma unroll
    for (int j = 0; j < PT; ++j) {
        const int d = loader ? w * PT + j : 0;
        my_slab[j] = d / Geo::kDmaPerSlab;
        const int r = d % Geo::kDmaPerSlab;
        my_dst[j] = my_slab[j] * kSlabBytes + r * 1024;
        my_tok[j] = r * Geo::kRowsPerDma + lane / Geo::kPieces;
        my_off[j] = slab_dma_offset<D, KV>(r, lane);
    }
    // query rows of this wave's columns: LDS row lc holds column c = kWaveCols w + lc
    uint32_t qdma_off[kQLoads];
#pragma unroll
    for (int r = 0; r < kQLoads; ++r) {
        const int lc = r * QG::kRowsPerDma + lane / QG::kPieces;
        const int c = col0 + kWaveCols * w + lc;
        const int src = c < ncols ? ((c / G) * p.Hq + (c % G)) * QG::kRow : 0;
        qdma_off[r] = src + (((lane % QG::kPieces) ^ (lc & (QG::kPieces - 1))) << 4);
    }
    OperandOffsets<D, KV> of;
    of.init(n, q4);
    // this lane's columns: kWaveCols w + 16 ct + n of column tile ct
    const bool wave_active = col0 + kWaveCols * w < ncols;  // a wave without real columns only loads its share of the tiles
    bool col_ok[NCT];
    int col_back[NCT];  // tokens at the end of the context the column must not see (prefix pass: every column sees all of it)
    int col_row[NCT];   // output row inside its sequence
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int col = col0 + kWaveCols * w + 16 * ct + n;
        col_ok[ct] = col < ncols;
        const int col_i = col_ok[ct] ? col / G : 0, col_h = col_ok[ct] ? col % G : 0;
        col_back[ct] = col_ok[ct] ? (PREFIX ? 0 : Q - 1 - col_i) : (1 << 30);
        col_row[ct] = col_i * p.Hq + g * G + col_h;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t ldsq = lds0 + NSTAGE * kStageBytes + w * kQSlotBytes;
    const char* qslot = smem + NSTAGE * kStageBytes + w * kQSlotBytes;

    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;
    const uint32_t head_stride32 = (uint32_t)p.Hkv * (uint32_t)kSlabBytes;  // the same; the host keeps it below 2^32
    const char* kc = static_cast<const char*>(p.k_cache) + (int64_t)g * kSlabBytes;
    const char* vc = static_cast<const char*>(p.v_cache) + (int64_t)g * kSlabBytes;

    auto issue_q = [&](int b) __attribute__((always_inline)) {
        const char* qb = reinterpret_cast<const char*>(p.q) + ((int64_t)b * (Q * p.Hq) + g * G) * QG::kRow;
#pragma unroll
        for (int r = 0; r < kQLoads; ++r) dma16<false>(ldsq + r * 1024, qdma_off[r], qb);
    };
    // returns whether this wave put loads in flight
    int nx_id0 = 0, nx_id1 = 0;  // ids of the tile `ic` stands on ...
    bool nx_valid = false;       // ... if they were asked for ahead
    auto issue = [&](int stage) __attribute__((always_inline)) {
        const uint32_t ldst = lds0 + stage * kStageBytes;
        if (!TRACE && nx_valid) {
            // interior tile, ids already here: every row is visible
            if (loader) {
#pragma unroll
                for (int j = 0; j < PT; ++j) {
                    const uint32_t id = (uint32_t)((my_slab[j] & 1) ? nx_id1 : nx_id0);
                    const char* base = (my_slab[j] >> 1 ? vc : kc) + (uint64_t)id * head_stride32;
                    dma16<!PREFIX>(ldst + my_dst[j], my_off[j], base);  // the prefix pass measured 3 % faster with ordinary loads
                }
            }
        } else {
            TileBlocks tb = tile_blocks(p.block_tables, p.MB, ic, reach);
            if (TRACE) {
                const RawIds raw = check_tile_blocks(tb, p.num_blocks);
                // the waves of a workgroup load different slabs of the tile from the same two ids: each loading
                // wave records the (block, K or V) pairs of its own instructions, for the first column group.
                // The prefix pass reads row 0 of the table for the whole batch and records its range as -2 - k.
                if (loader && lane == 0 && col0 == 0) {
#pragma unroll
                    for (int j = 0; j < PT; ++j)
                        trace_block_use(p.trace_blocks, tb, raw, my_slab[j] & 1, my_slab[j] >> 1, ic.b, g, PREFIX ? -2 - k : k,
                                        p.Hkv, p.MB);
                }
            }
            if (loader) {
#pragma unroll
                for (int j = 0; j < PT; ++j) {
                    const int sub = my_slab[j] & 1;
                    const char* base = (my_slab[j] >> 1 ? vc : kc) + (sub ? tb.phys[1] : tb.phys[0]) * head_stride;
                    dma16<!PREFIX>(ldst + my_dst[j],
                          live_or_stand_in<D, KV>(my_off[j], my_tok[j], sub ? tb.lo[1] : tb.lo[0], sub ? tb.hi[1] : tb.hi[0]),
                          base);
                }
            }
        }
        advance(ic, p.context_lens, B, sp);
        nx_valid = ask_next_ids(p.block_tables, p.MB, ic, B, reach, nx_id0, nx_id1);
        return loader;
    };

    const float qs = KV == KV_FP8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;
    const float vs = KV == KV_FP8 ? p.v_scale[g] : 1.f;
    ColumnState<D> st[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) st[ct].clear();
    bf16x8 qreg[NCT][D / 32];
    int seg_first_lt = 0;

    // ---- prologue: the first segment's query rows, then the ring
    issue_q(first_b);
    int q_age = 0;  // tiles this wave has put loads in flight for since it last issued query rows
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t)
        if (t < ntiles && issue(t)) ++q_age;

    // what a wave does when tile `tile` (the compute cursor stands on it) begins a segment
    auto begin_segment = [&](int tile) __attribute__((always_inline)) {
        seg_first_lt = cc.lt;
        if (describes && cc.lt == 0 && lane == 0) {  // the sequence's first tile is this workgroup's
            const int cum = rs.t_lo + tile, end = cum + cc.nt;
            write_seq_desc(p.merge_desc, cc.b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
        }
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            st[ct].reset();
            load_query_operand<D>(qslot + ct * 16 * QG::kRow, n, q4, col_ok[ct], qreg[ct]);
        }
        // refill the slot with the rows of the next segment of this range, if there is one
        if (tile + (cc.nt - cc.lt) < ntiles) {
            int nb = cc.b;
            do {
                ++nb;
            } while (nb < B - 1 && tiles_of(uniform_load(p.context_lens, nb), sp) == 0);  // (none of its own behind a shared prefix counts as empty)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slot has been read
            issue_q(nb);
            q_age = 0;
        }
    };
    // softmax, PV and, at the end of a segment, the result of tile `tile` from its scores
    auto finish_tile = [&](int tile, const char* vbuf, const f32x4 (&s0)[NCT], const f32x4 (&s1)[NCT]) __attribute__((always_inline)) {
        // The column sees tokens low <= t < lim.  Only the last tiles of a sequence (where the causal
        // limits lie) and the tiles where the columns' sliding windows begin need the mask:
        // everywhere else every column sees the whole tile.
        const int tile_first = (cc.lt + cc.ft) * kTileTokens;
        const int t0 = tile_first + 4 * q4;
        const bool unmasked = PREFIX || (tile_first + kTileTokens <= cc.L - (Q - 1) &&
                                         (reach == 0 || tile_first >= cc.L - p.window));
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

        pv_accumulate<D, KV, NCT, P_LO>(vbuf, of, pb, pb_lo, st);

        // ---- segment end: normalise, write
        if (cc.lt == cc.nt - 1 || tile == ntiles - 1) {
            const bool whole = seg_first_lt == 0 && cc.lt == cc.nt - 1;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const float l = st[ct].weight_sum();
                if (col_ok[ct]) {
                    // a column that saw no token (its query sits before this segment) leaves a zero row
                    // with an "empty" log-sum-exp
                    const bool seen = st[ct].seen();
                    const float inv = seen ? vs / l : 0.f;
                    const float lse = seen ? st[ct].m + fast_log2(l) : kNegBig;
                    if (PREFIX) {
                        const int64_t slot = (int64_t)k * ((int64_t)p.B * p.QH) + col_row[ct];
                        if (q4 == 0) p.prefix_lse[slot] = lse;
                        store_partial_row(p.prefix_o + slot * D, st[ct], inv, q4);
                    } else if (whole && skip > 0) {  // final but for the prefix part: to the workspace, for the prefix merge
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
    };

    int stage = 0;
    for (int tile = 0; tile < ntiles; ++tile) {
        const bool seg_start = tile == 0 || cc.lt == 0;
        // my loads of this tile have landed once at most the tiles issued after it are in flight; at
        // a segment start the query rows (issued q_age tiles ago) must have landed as well
        int later = min(kMaxLater, ntiles - 1 - tile);
        if (seg_start && q_age < later) later = q_age;
        wait_loads<PT, kMaxLater>(later);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // my LDS reads of the previous tile have returned
        __builtin_amdgcn_s_barrier();
        const int ahead = tile + NSTAGE - 1;
        if (ahead < ntiles) {
            int stg = stage + NSTAGE - 1;
            if (stg >= NSTAGE) stg -= NSTAGE;
            if (issue(stg)) ++q_age;
        }
        const char* kbuf = smem + stage * kStageBytes;
        if (wave_active) {  // a wave without columns keeps loading and meeting the others at the barrier
            if (seg_start) begin_segment(tile);
            f32x4 s0[NCT], s1[NCT];
            qk_scores<D, KV, NCT>(kbuf, of, qreg, s0, s1);
            finish_tile(tile, kbuf + 2 * kSlabBytes, s0, s1);
        }
        advance(cc, p.context_lens, B, sp);
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }
}

}  // namespace pa
