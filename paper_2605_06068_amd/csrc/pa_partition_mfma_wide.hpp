// Partition kernel, matrix-core variant for more than 16 columns per KV head (multi-token
// verification: q_len * G = 17 .. 128 (query token, query head) pairs).  A workgroup of NW
// wavefronts serves one (partition, KV head): the waves share ONE ring of K/V tiles in LDS, so
// the cache is read from HBM once for all columns, and each wave computes its own tile of 16
// columns (columns 16w .. 16w+15) exactly as the single-wave kernel does: same operand
// layouts, same swizzle, same online softmax (see pa_partition_mfma.hpp).
//
// Per tile, every wave loads 1/NW of the tile's LDS-DMA instructions and the workgroup meets at
// one barrier:
//     wait for my own loads of tile t          (s_waitcnt vmcnt, counted by hand)
//     s_barrier                                (all parts of tile t are in LDS; everyone is done
//                                               reading tile t-1, whose buffer is refilled next)
//     issue my part of tile t + NSTAGE - 1
//     scores, online softmax, PV for my 16 columns on tile t
// All waves of a workgroup walk the same range, so they execute the same number of barriers.
//
// Query rows: every wave keeps ONE private LDS slot (16 rows of 256 B) for the rows of its own
// columns.  At the start of a segment it moves the slot into registers and at once refills the
// slot with the rows of the next segment in its range, so the rows are there long before that
// segment's first tile; after a short segment (fewer tiles than the ring is deep) the wait at
// the segment start is tightened to cover those loads (q_age below).
//
// PREFIX mode is the pass over a prefix that every sequence of a decode batch shares (the same
// physical blocks at the head of every block table).  The columns are then the (sequence, head)
// pairs: to this kernel the batch is ONE sequence, the prefix, with one "query token" per real
// sequence and no causal mask.  The prefix tiles are cut into Pp ranges, workgroup
// (column group, KV head, range) leaves one partial result per column, and the prefix merge
// kernel adds them to what the per-sequence pass computed over the rest of each context.
#pragma once
#include <type_traits>

#include "pa_device.hpp"
#include "pa_partition_mfma.hpp"
#include "pa_plan.hpp"

namespace pa {

constexpr int kQSlotBytesWide = 16 * kQRowBytes;  // one wave's query rows

constexpr int mfma_wide_lds_bytes(int nw, int nstage, int kv)
{
    return nstage * (kv == KV_BF16 ? KvGeom<KV_BF16>::kStage : KvGeom<KV_FP8>::kStage) + nw * kQSlotBytesWide;
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
template <int NW, int NSTAGE, int KV, bool TRACE, bool PREFIX>
__global__ __launch_bounds__(NW * 64, NW >= 4 ? 2 : 1) void partition_mfma_wide_kernel(const Params p)
{
    constexpr int D = 128;
    static_assert(NW == 2 || NW == 4 || NW == 8, "waves per workgroup");
    static_assert(NSTAGE >= 3, "the ring holds the tile in use, the one being refilled and at least one in flight");
    using Geo = KvGeom<KV>;
    constexpr int kSlabBytes = Geo::kSlab;
    constexpr int kStageBytes = Geo::kStage;
    constexpr int PT = Geo::kDmaPerTile / NW;  // LDS-DMA instructions per tile and wave
    static_assert(PT >= 1 && PT * NW == Geo::kDmaPerTile, "the tile's loads divide evenly over the waves");
    constexpr int kMaxLater = NSTAGE - 2;      // tiles in flight behind the one a wave waits for
    static_assert(mfma_wide_lds_bytes(NW, NSTAGE, KV) <= 160 * 1024, "LDS of one compute unit");
    __shared__ __attribute__((aligned(1024))) char smem[mfma_wide_lds_bytes(NW, NSTAGE, KV)];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    static_assert(!(PREFIX && TRACE), "the prefix pass has no instrumented variant");
    // partition index fastest, as in the single-wave kernel; then the KV head, then (prefix pass
    // with more than 16*NW columns) the column group
    const int nparts = PREFIX ? p.Pp : p.P;
    const int k = blockIdx.x % nparts;
    const int g = (blockIdx.x / nparts) % p.Hkv;
    const int col0 = (blockIdx.x / nparts / p.Hkv) * (16 * NW);
    const int G = p.G;
    const int B = PREFIX ? 1 : p.B;      // sequences as this kernel sees them
    const int Q = PREFIX ? p.B : p.Q;    // query tokens per such sequence
    const int ncols = Q * G;
    const int n = lane & 15;
    const int q4 = lane >> 4;

    // sliding window (never together with a shared prefix): see the single-wave kernel
    const int reach = (!PREFIX && p.window > 0) ? p.window + Q - 1 : 0;
    const Span sp{0, reach};
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
    if (!PREFIX && k == 0 && w == 0) {  // empty contexts: their output rows are zero
        for (int b0 = 0; b0 < B; b0 += kWave) {
            const int b = b0 + lane;
            if (b < B && p.context_lens[b] <= 0) {
                for (int i = 0; i < Q; ++i) {
                    const int64_t row = ((int64_t)b * p.QH + (int64_t)i * p.Hq + g * G) * D;
                    for (int e = 0; e < G * D; ++e) store_out1(p, row + e, 0.f);
                }
                if (g == 0 && p.merge_desc != nullptr) write_seq_desc(p.merge_desc, b, 0, 0, 0, 0);
            }
        }
    }
    const bool describes = !PREFIX && g == 0 && w == 0 && p.merge_desc != nullptr;  // tells the merge about its sequences
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
#pragma unroll
    for (int j = 0; j < PT; ++j) {
        const int d = w * PT + j;
        my_slab[j] = d / Geo::kDmaPerSlab;
        const int r = d % Geo::kDmaPerSlab;
        my_dst[j] = my_slab[j] * kSlabBytes + r * 1024;
        my_tok[j] = r * Geo::kRowsPerDma + lane / Geo::kPieces;
        my_off[j] = my_tok[j] * Geo::kRow + (((lane % Geo::kPieces) ^ (my_tok[j] & (Geo::kPieces - 1))) << 4);
    }
    // query rows of this wave's columns: LDS row r4*4 + q4 holds column c = 16w + that row
    uint32_t qdma_off[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int lc = 4 * r + q4;
        const int c = col0 + 16 * w + lc;
        const int src = c < ncols ? ((c / G) * p.Hq + (c % G)) * kQRowBytes : 0;
        qdma_off[r] = src + ((n ^ lc) << 4);
    }
    uint32_t kread[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        if (KV == KV_BF16)
            kread[kk] = n * Geo::kRow + (((4 * kk + q4) ^ n) << 4);
        else
            kread[kk] = n * Geo::kRow + (((2 * kk + (q4 >> 1)) ^ (n & 7)) << 4) + ((q4 & 1) << 3);
    }
    // this lane's column
    const int col = col0 + 16 * w + n;
    const bool col_ok = col < ncols;
    const bool wave_active = col0 + 16 * w < ncols;  // a wave without real columns only loads its share of the tiles
    const int col_i = col_ok ? col / G : 0, col_h = col_ok ? col % G : 0;
    // tokens at the end of the context the column must not see (prefix pass: every column sees all of it)
    const int col_back = col_ok ? (PREFIX ? 0 : Q - 1 - col_i) : (1 << 30);
    const int col_row = col_i * p.Hq + g * G + col_h;          // output row inside its sequence
    uint32_t qpiece[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qpiece[kk] = n * kQRowBytes + (((4 * kk + q4) ^ n) << 4);
    uint32_t vread[8];
    if (KV == KV_BF16) {
        const int row = 4 * q4 + (n >> 2);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            vread[dt] = row * Geo::kRow + ((n & 1) << 3) + (((2 * dt + ((n >> 1) & 1)) ^ row) << 4);
    } else {
        const int r = n >> 1;
        const int tok = 4 * q4 + (r & 3);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            vread[dt] = (r >> 2) * kSlabBytes + tok * Geo::kRow + ((dt ^ (tok & 7)) << 4) + ((n & 1) << 3);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t ldsq = lds0 + NSTAGE * kStageBytes + w * kQSlotBytesWide;
    const char* qslot = smem + NSTAGE * kStageBytes + w * kQSlotBytesWide;

    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;
    const char* kc = static_cast<const char*>(p.k_cache) + (int64_t)g * kSlabBytes;
    const char* vc = static_cast<const char*>(p.v_cache) + (int64_t)g * kSlabBytes;

    auto issue_q = [&](int b) {
        const char* qb = reinterpret_cast<const char*>(p.q) + ((int64_t)b * (Q * p.Hq) + g * G) * kQRowBytes;
#pragma unroll
        for (int r = 0; r < 4; ++r) dma16(ldsq + r * 1024, qdma_off[r], qb);
    };
    auto issue = [&](int stage) {
        const int nblk = (ic.L + kBlockSize - 1) / kBlockSize;
        const int32_t* table = p.block_tables + (int64_t)ic.b * p.MB;
        const int j0 = 2 * (ic.lt + ic.ft);
        // Per block of the tile: its physical id and the rows [lo, hi) that hold tokens some query can
        // see.  Every other row (past the context, before the earliest window) may hold anything,
        // NaN patterns included, and is replaced on the way in by row lo of the same block; the
        // softmax masks those positions.
        int phys[2], lo[2], hi[2];
        const int t_first = (reach > 0 && ic.L > reach) ? ic.L - reach : 0;  // first token any query sees
        lo[0] = min(max(t_first - j0 * kBlockSize, 0), kBlockSize);
        hi[0] = min(ic.L - j0 * kBlockSize, kBlockSize);
        // a first block that lies entirely before the window may be gone: its table entry is not read
        const bool first_gone = lo[0] >= kBlockSize;
        const bool second = j0 + 1 < nblk;
        if (second) {
            phys[1] = uniform_load(table, j0 + 1);
            lo[1] = max(t_first - (j0 + 1) * kBlockSize, 0);
            hi[1] = min(ic.L - (j0 + 1) * kBlockSize, kBlockSize);
        }
        if (!first_gone) {
            phys[0] = uniform_load(table, j0);
        } else {  // stand-in: the first visible row of the second block (which exists: it holds that token)
            phys[0] = phys[1];
            lo[0] = hi[0] = lo[1];
        }
        if (!second) {  // no second block: stand-in rows from the first one
            phys[1] = phys[0];
            lo[1] = hi[1] = lo[0];
        }
        if (TRACE && w == 0 && lane == 0) {
            int32_t* v = p.trace_blocks + (((int64_t)ic.b * p.Hkv + g) * p.MB + j0) * 3;
            if (!first_gone) { v[0] = phys[0]; v[1] = phys[0]; v[2] = k; }
            if (second) { v[3] = phys[1]; v[4] = phys[1]; v[5] = k; }
        }
        const uint32_t ldst = lds0 + stage * kStageBytes;
#pragma unroll
        for (int j = 0; j < PT; ++j) {
            const int sub = my_slab[j] & 1;
            const char* base = (my_slab[j] >> 1 ? vc : kc) + (sub ? phys[1] : phys[0]) * head_stride;
            const int rlo = sub ? lo[1] : lo[0], rhi = sub ? hi[1] : hi[0];
            const bool live = my_tok[j] >= rlo && my_tok[j] < rhi;
            dma16(ldst + my_dst[j], live ? my_off[j] : rlo * Geo::kRow + (my_off[j] & (Geo::kRow - 1)), base);
        }
        advance(ic, p.context_lens, B, sp);
    };

    const float qs = KV == KV_FP8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;
    const float vs = KV == KV_FP8 ? p.v_scale[g] : 1.f;
    float m = kNegBig, lsum = 0.f;
    f32x4 acc[8];
    bf16x8 qreg[4];
    int seg_first_lt = 0;

    // ---- prologue: the first segment's query rows, then the ring
    issue_q(first_b);
    int q_age = 0;  // tiles this wave has issued since it last issued query rows
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t)
        if (t < ntiles) {
            issue(t);
            ++q_age;
        }

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
            int st = stage + NSTAGE - 1;
            if (st >= NSTAGE) st -= NSTAGE;
            issue(st);
            ++q_age;
        }
        const char* kbuf = smem + stage * kStageBytes;
        const char* vbuf = kbuf + 2 * kSlabBytes;
        if (!wave_active) {  // keeps loading and meeting the others at the barrier; nothing to compute
            advance(cc, p.context_lens, B, sp);
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            continue;
        }

        if (seg_start) {
            seg_first_lt = cc.lt;
            if (describes && cc.lt == 0 && lane == 0) {  // the sequence's first tile is this workgroup's
                const int cum = rs.t_lo + tile, end = cum + cc.nt;
                write_seq_desc(p.merge_desc, cc.b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
            }
            m = kNegBig;
            lsum = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                uint4 v = *reinterpret_cast<const uint4*>(qslot + qpiece[kk]);
                if (!col_ok) v = make_uint4(0, 0, 0, 0);
                qreg[kk] = as_bf16x8(v);
            }
            // refill the slot with the rows of the next segment of this range, if there is one
            if (tile + (cc.nt - cc.lt) < ntiles) {
                int nb = cc.b;
                do {
                    ++nb;
                } while (nb < B - 1 && uniform_load(p.context_lens, nb) <= 0);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slot has been read
                issue_q(nb);
                q_age = 0;
            }
        }

        // ---- scores: S^T[token, column] for the two blocks of the tile
        f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 a0, a1;
            if (KV == KV_BF16) {
                a0 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + kread[kk]));
                a1 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + kSlabBytes + kread[kk]));
            } else {
                const uint2 w0 = *reinterpret_cast<const uint2*>(kbuf + kread[kk]);
                const uint2 w1 = *reinterpret_cast<const uint2*>(kbuf + kSlabBytes + kread[kk]);
                a0 = fp8x8_to_bf16x8(w0.x, w0.y);
                a1 = fp8x8_to_bf16x8(w1.x, w1.y);
            }
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qreg[kk], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qreg[kk], s1, 0, 0, 0);
        }

        // ---- online softmax (log2 domain); the column sees tokens t < L - col_back.  Only the last
        // tiles of a sequence need the mask: everywhere else every column sees the whole tile.
        bf16x8 pb, pb_lo;
        auto softmax = [&](auto masked_tag) {
            constexpr bool MASKED = decltype(masked_tag)::value;
            const int t0 = (cc.lt + cc.ft) * kTileTokens + 4 * q4;
            const int lim = cc.L - col_back;
            const int low = p.window > 0 ? lim - p.window : INT32_MIN;  // first token the column's window holds
            float x[8];
            bool ok[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ok[r] = !MASKED || (t0 + r < lim && t0 + r >= low);
                ok[4 + r] = !MASKED || (t0 + kBlockSize + r < lim && t0 + kBlockSize + r >= low);
                x[r] = ok[r] ? s0[r] * qs : kNegBig;
                x[4 + r] = ok[4 + r] ? s1[r] * qs : kNegBig;
            }
            float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            mx = rows_max(mx);
            const float m_new = fmaxf(m, mx);
            const float alpha = fast_exp2(m - m_new);
            float ps = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                x[r] = ok[r] ? fast_exp2(x[r] - m_new) : 0.f;  // a column may see nothing of a tile
                ps += x[r];
            }
            lsum = lsum * alpha + ps;
            m = m_new;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;
            }
            // P^T operand as a bf16 pair (high part + rounding remainder)
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                pb[r] = (__bf16)x[r];
                pb_lo[r] = (__bf16)(x[r] - (float)pb[r]);
            }
        };
        // no mask needed: every column sees the whole tile (not at the end of a context, where the
        // causal limits lie, nor in the tiles where the windows of the columns begin)
        const int tile_first = (cc.lt + cc.ft) * kTileTokens;
        const bool unmasked = PREFIX || (tile_first + kTileTokens <= cc.L - (Q - 1) &&
                                         (reach == 0 || tile_first >= cc.L - p.window));
        if (unmasked)
            softmax(std::false_type{});
        else
            softmax(std::true_type{});

        // ---- out^T[dim, column] += V^T . P^T
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            bf16x8 va;
            if (KV == KV_BF16) {
                const i16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + vread[dt]));
                const i16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + kSlabBytes + vread[dt]));
                va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
            } else {
                const i32x2 v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)(vbuf + vread[dt]));
                va = fp8x8_to_bf16x8((uint32_t)v[0], (uint32_t)v[1]);
            }
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb, acc[dt], 0, 0, 0);
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb_lo, acc[dt], 0, 0, 0);
        }

        // ---- segment end: finish the row sums, normalise, write
        if (cc.lt == cc.nt - 1 || tile == ntiles - 1) {
            const bool whole = seg_first_lt == 0 && cc.lt == cc.nt - 1;
            const float l = rows_sum(lsum);
            if (col_ok) {
                // a column that saw no token (its query sits before this segment) leaves a zero row
                // with an "empty" log-sum-exp
                const float inv = l > 0.f ? vs / l : 0.f;
                if (!PREFIX && whole) {
                    const int64_t row = ((int64_t)cc.b * p.QH + col_row) * D;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
                        store_out4(p, row + 16 * dt + 4 * q4, acc[dt][0] * inv, acc[dt][1] * inv, acc[dt][2] * inv,
                                   acc[dt][3] * inv);
                } else {
                    float* dst;
                    if (PREFIX) {
                        const int64_t slot = (int64_t)k * ((int64_t)p.B * p.Hq) + col_row;
                        dst = p.prefix_o + slot * D;
                        if (q4 == 0) p.prefix_lse[slot] = m + fast_log2(l);
                    } else {
                        const int64_t slot = ((int64_t)2 * k + (cc.b != first_b ? 1 : 0)) * p.QH + col_row;
                        dst = p.part_o + slot * D;
                        if (q4 == 0) p.part_lse[slot] = l > 0.f ? m + fast_log2(l) : kNegBig;
                    }
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
                        *reinterpret_cast<float4*>(dst + 16 * dt + 4 * q4) =
                            make_float4(acc[dt][0] * inv, acc[dt][1] * inv, acc[dt][2] * inv, acc[dt][3] * inv);
                }
            }
        }
        advance(cc, p.context_lens, B, sp);
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }
}

}  // namespace pa
