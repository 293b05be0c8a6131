// Partition kernel, matrix-core variant (head_dim 128, bf16 or fp8 KV) for up to 16 columns.
// The columns of its matrix tile are the (query token, query head) pairs that share one KV
// head: q_len * G of them (plain decode: the G heads of the group), padded to CPAD = 4, 8 or
// 16 inside one 16-column MFMA tile.  One wavefront per (partition, KV head) walks its balanced
// range of the batch's global tile sequence (see pa_plan.hpp); no workgroup barriers, no
// atomics.  More columns than 16 go to the multi-wave kernel in pa_partition_mfma_wide.hpp.
//
// Data path per 32-token tile (two KV blocks):
//   HBM --global_load_lds (16 B/lane, 1 KB per instruction)--> LDS ring of NSTAGE tiles
//   K:  ds_read_b128 in MFMA operand layout -> S^T[token, column] = K . Q^T  (mfma 16x16x32 bf16)
//   online softmax on S^T in registers (lane = column, 8 tokens per lane per tile)
//   V:  ds_read_b64_tr_b16 (transposing LDS read) -> out^T[dim, column] += V^T . P^T
// The ring keeps running across sequence boundaries inside the range; the query rows of each new sequence
// travel through a small LDS ring of their own, ahead of its first tile.
//
// Multi-token calls (q_len > 1) are causal inside the new tokens: query i of a sequence of L
// tokens sits at position L - q_len + i and sees tokens 0 .. L - q_len + i.
//
// LDS tile layout: row t (one token, 256 B) at byte t*256; the 16-byte piece holding dims
// [8c, 8c+8) sits at piece position c ^ (t & 15).  The XOR swizzle is applied on the *global*
// side of the LDS-DMA load (the LDS side of such a load is always lane-linear), which keeps
// every 16-lane group on one contiguous 256-byte row, and makes both the operand reads (16
// different rows per 16 lanes) and the transposing reads bank-conflict free.
//
// The P^T operand needs no data movement: the score tile comes out of the MFMA with lane l
// holding column l%16 and tokens 4*(l/16)+{0..3}; declaring MFMA k-index 8*(l/16)+e to mean
// token 4*(l/16)+e of the first block (e<4) or of the second block (e>=4) makes the score
// registers, once exponentiated and packed to bf16, the B operand of the PV product as they
// stand.  The V^T operand is read with the same k-index convention.
//
// Wait-count discipline: the LDS-DMA loads are issued and awaited by hand (s_waitcnt vmcnt(N)
// with N = number of *newer DMA loads* allowed to stay in flight).  Loads complete in order,
// so "at most N operations outstanding" implies every load older than the newest N has landed,
// whatever else (stores, extra loads) is in flight: other traffic only makes a wait stricter.
// Everything else the loop needs from memory comes through the scalar cache (block ids,
// context lengths), which the vector-memory counter does not see.  The inline asm writes M0
// (the LDS-DMA destination register); nothing else in these kernels uses M0.
#pragma once
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

constexpr int kQRowBytes = 256;  // one query row: 128 bf16

// Storage geometry of one (block, head) slab of the KV cache, head_dim 128.
template <int KV>
struct KvGeom {
    static constexpr int kRow = KV == KV_BF16 ? 256 : 128;  // bytes per token row
    static constexpr int kSlab = kBlockSize * kRow;          // 16 rows
    static constexpr int kPieces = kRow / 16;                // 16-byte pieces per row
    static constexpr int kRowsPerDma = kWave / kPieces;      // rows one 1 KB wave-wide load covers
    static constexpr int kDmaPerSlab = kSlab / 1024;
    static constexpr int kStage = 4 * kSlab;                 // K block 0, K block 1, V block 0, V block 1
    static constexpr int kDmaPerTile = 4 * kDmaPerSlab;
};

// LDS bytes one workgroup (one wave) of the kernel uses: tile ring + query-row ring.
constexpr int mfma_lds_bytes(int nstage, int cpad, int kv)
{
    return nstage * ((kv == KV_BF16 ? KvGeom<KV_BF16>::kStage : KvGeom<KV_FP8>::kStage) + cpad * kQRowBytes);
}

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
// lds_addr + lane*16 (wave-uniform lds_addr goes through M0); the global source is
// base (wave-uniform) + voff (per lane).  Completion is tracked by vmcnt.
__device__ __forceinline__ void dma16(uint32_t lds_addr, uint32_t voff, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(base) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// wait until at most `later_tiles` whole tiles (PER_TILE loads each) plus EXTRA loads are still in flight
template <int EXTRA, int NSTAGE, int PER_TILE>
__device__ __forceinline__ void wait_tile(int later_tiles)
{
    static_assert(3 * PER_TILE + EXTRA <= 63, "vmcnt is a 6-bit counter");
    if (NSTAGE >= 4 && later_tiles >= 3) wait_vmcnt<3 * PER_TILE + EXTRA>();
    else if (NSTAGE >= 3 && later_tiles == 2) wait_vmcnt<2 * PER_TILE + EXTRA>();
    else if (later_tiles == 1) wait_vmcnt<1 * PER_TILE + EXTRA>();
    else wait_vmcnt<EXTRA>();
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

template <int NSTAGE, int CPAD, int KV, bool TRACE>
__global__ __launch_bounds__(64) void partition_mfma_kernel(const Params p)
{
    constexpr int D = 128;
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring depth");
    static_assert(CPAD == 4 || CPAD == 8 || CPAD == 16, "padded column count");
    using Geo = KvGeom<KV>;
    constexpr int kSlabBytes = Geo::kSlab;
    constexpr int kStageBytes = Geo::kStage;
    constexpr int kDmaPerTile = Geo::kDmaPerTile;
    constexpr int kQSlot = CPAD * kQRowBytes;
    static_assert(mfma_lds_bytes(NSTAGE, CPAD, KV) <= 65536, "static LDS limit");
    __shared__ __attribute__((aligned(1024))) char smem[mfma_lds_bytes(NSTAGE, CPAD, KV)];

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
    if (k == 0 && skip == 0) {  // empty contexts: their output rows are zero
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
    const bool describes = g == 0 && skip == 0 && p.merge_desc != nullptr;  // this wave tells the merge about its sequences
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
    // LDS-DMA of a KV slab: instruction r covers rows r*kRowsPerDma ..; this lane's global byte offset
    uint32_t dma_off[Geo::kDmaPerSlab];
#pragma unroll
    for (int r = 0; r < Geo::kDmaPerSlab; ++r) {
        const int t = r * Geo::kRowsPerDma + lane / Geo::kPieces;
        dma_off[r] = t * Geo::kRow + (((lane % Geo::kPieces) ^ (t & (Geo::kPieces - 1))) << 4);
    }
    // LDS-DMA of the query rows (always bf16: 4 rows of 256 B per instruction).  LDS row c holds
    // column c, i.e. query token c / G, head c % G of this group; padding rows re-read column 0.
    uint32_t qdma_off[CPAD / 4];
#pragma unroll
    for (int r = 0; r < CPAD / 4; ++r) {
        const int c = 4 * r + q4;
        const int src = c < ncols ? ((c / G) * p.Hq + (c % G)) * kQRowBytes : 0;
        qdma_off[r] = src + ((n ^ (c & 15)) << 4);
    }
    uint32_t kread[4];  // LDS byte offset inside a slab of this lane's K operand piece for k-step kk
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        if (KV == KV_BF16)  // 16 bytes: dims 32kk + 8q4 + [0,8) of token n
            kread[kk] = n * Geo::kRow + (((4 * kk + q4) ^ n) << 4);
        else                // 8 bytes: the same dims, half of 16-byte piece 2kk + q4/2
            kread[kk] = n * Geo::kRow + (((2 * kk + (q4 >> 1)) ^ (n & 7)) << 4) + ((q4 & 1) << 3);
    }
    // this lane's column n
    const bool col_ok = n < ncols;                                 // a real column
    const int col_i = col_ok ? n / G : 0, col_h = col_ok ? n % G : 0;
    const int col_back = col_ok ? Q - 1 - col_i : (1 << 30);       // tokens at the end of the context its query must not see
    const int col_row = col_i * p.Hq + g * G + col_h;              // its output row inside its sequence
    const uint32_t qread = (col_ok ? n : 0) * kQRowBytes;          // LDS byte offset of its query row
    uint32_t qpiece[4];  // swizzled position of dims 32kk + 8q4 + [0,8) in a query row of this lane's columns
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qpiece[kk] = ((4 * kk + q4) ^ n) << 4;
    // LDS byte offset (inside the V half of a stage) of this lane's transposing-read source for dim tile dt.
    // bf16: one read per block, rows = tokens 4q4 + n/4, 8 bytes = 4 dims.  fp8: one read for both blocks,
    // rows n/2 = 0..3 -> tokens 4q4.. of block 0, rows 4..7 -> the same tokens of block 1, 8 bytes = 8 dims.
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
    const uint32_t ldsq = lds0 + NSTAGE * kStageBytes;
    const char* qslots = smem + NSTAGE * kStageBytes;

    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;  // bytes between physical blocks
    const char* kc = static_cast<const char*>(p.k_cache) + (int64_t)g * kSlabBytes;
    const char* vc = static_cast<const char*>(p.v_cache) + (int64_t)g * kSlabBytes;

    int q_issue = 0;  // query slot the issue side fills next
    auto issue = [&](int i, int stage) {
        if (i == 0 || ic.lt == 0) {  // a new segment starts: send its query rows ahead of its first tile
            const char* qb = reinterpret_cast<const char*>(p.q) + ((int64_t)ic.b * p.QH + g * G) * kQRowBytes;
#pragma unroll
            for (int r = 0; r < CPAD / 4; ++r) dma16(ldsq + q_issue * kQSlot + r * 1024, qdma_off[r], qb);
            q_issue = (q_issue + 1 == NSTAGE) ? 0 : q_issue + 1;
        }
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
        if (TRACE && lane == 0) {
            int32_t* v = p.trace_blocks + (((int64_t)ic.b * p.Hkv + g) * p.MB + j0) * 3;
            if (!first_gone) { v[0] = phys[0]; v[1] = phys[0]; v[2] = k; }
            if (second) { v[3] = phys[1]; v[4] = phys[1]; v[5] = k; }
        }
        const uint32_t ldst = lds0 + stage * kStageBytes;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const char* kb = kc + phys[sub] * head_stride;
#pragma unroll
            for (int r = 0; r < Geo::kDmaPerSlab; ++r) {
                const int row = r * Geo::kRowsPerDma + lane / Geo::kPieces;
                const bool live = row >= lo[sub] && row < hi[sub];
                dma16(ldst + sub * kSlabBytes + r * 1024,
                      live ? dma_off[r] : lo[sub] * Geo::kRow + (dma_off[r] & (Geo::kRow - 1)), kb);
            }
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const char* vb = vc + phys[sub] * head_stride;
#pragma unroll
            for (int r = 0; r < Geo::kDmaPerSlab; ++r) {
                const int row = r * Geo::kRowsPerDma + lane / Geo::kPieces;
                const bool live = row >= lo[sub] && row < hi[sub];
                dma16(ldst + 2 * kSlabBytes + sub * kSlabBytes + r * 1024,
                      live ? dma_off[r] : lo[sub] * Geo::kRow + (dma_off[r] & (Geo::kRow - 1)), vb);
            }
        }
        advance(ic, p.context_lens, B, sp);
    };

    // ---- online softmax state: lane = column n, tokens 4*q4+{0..3} of each block
    const float qs = KV == KV_FP8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;  // K scale folded in
    const float vs = KV == KV_FP8 ? p.v_scale[g] : 1.f;
    float m = kNegBig, lsum = 0.f;
    f32x4 acc[8];
    bf16x8 qreg[4];
    int q_comp = 0;       // query slot of the segment being computed
    int seg_first_lt = 0;

    // ---- prologue: fill the ring
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t)
        if (t < ntiles) issue(t, t);

    int stage = 0;
    for (int tile = 0; tile < ntiles; ++tile) {
        // refill the buffer consumed in the previous iteration (its LDS reads have all returned)
        const int ahead = tile + NSTAGE - 1;
        if (ahead < ntiles) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            int st = stage + NSTAGE - 1;
            if (st >= NSTAGE) st -= NSTAGE;
            issue(ahead, st);
        }
        const int later = min(NSTAGE - 1, ntiles - 1 - tile);
        const char* kbuf = smem + stage * kStageBytes;
        const char* vbuf = kbuf + 2 * kSlabBytes;

        wait_tile<kDmaPerTile / 2, NSTAGE, kDmaPerTile>(later);  // K of this tile (and its segment's query rows) landed
        if (tile == 0 || cc.lt == 0) {  // segment start
            seg_first_lt = cc.lt;
            if (describes && cc.lt == 0 && lane == 0) {  // the sequence's first tile is mine
                const int cum = rs.t_lo + tile, end = cum + cc.nt;
                write_seq_desc(p.merge_desc, cc.b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
            }
            const char* qsl = qslots + q_comp * kQSlot;
            m = kNegBig;
            lsum = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                uint4 w = *reinterpret_cast<const uint4*>(qsl + qread + qpiece[kk]);
                if (!col_ok) w = make_uint4(0, 0, 0, 0);
                qreg[kk] = as_bf16x8(w);
            }
            q_comp = (q_comp + 1 == NSTAGE) ? 0 : q_comp + 1;
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

        // ---- online softmax (log2 domain); the column sees tokens t < L - col_back
        const int t0 = (cc.lt + cc.ft) * kTileTokens + 4 * q4;
        const int lim = cc.L - col_back;
        const int low = p.window > 0 ? lim - p.window : INT32_MIN;  // first token the column's window holds
        float x[8];
        bool ok[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            ok[r] = t0 + r < lim && t0 + r >= low;
            ok[4 + r] = t0 + kBlockSize + r < lim && t0 + kBlockSize + r >= low;
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
        // P^T operand as a bf16 pair (high part + rounding remainder): 16 significant bits, so
        // the weights lose nothing that matters against the fp32 accumulation
        bf16x8 pb, pb_lo;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            pb[r] = (__bf16)x[r];
            pb_lo[r] = (__bf16)(x[r] - (float)pb[r]);
        }

        // ---- out^T[dim, column] += V^T . P^T
        wait_tile<0, NSTAGE, kDmaPerTile>(later);
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
            const bool whole = seg_first_lt == 0 && cc.lt == cc.nt - 1;  // the entire sequence: final result
            const float l = rows_sum(lsum);
            if (col_ok) {
                // a column that saw no token (its query sits before this segment) leaves a zero
                // row with an "empty" log-sum-exp
                const float inv = l > 0.f ? vs / l : 0.f;
                if (whole) {
                    const int64_t row = ((int64_t)cc.b * p.QH + col_row) * D;
                    if (skip > 0 && q4 == 0)
                        p.seq_lse[(int64_t)cc.b * p.QH + col_row] = l > 0.f ? m + fast_log2(l) : kNegBig;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
                        store_out4(p, row + 16 * dt + 4 * q4, acc[dt][0] * inv, acc[dt][1] * inv, acc[dt][2] * inv,
                                   acc[dt][3] * inv);
                } else {
                    const int64_t slot = ((int64_t)2 * k + (cc.b != first_b ? 1 : 0)) * p.QH + col_row;
                    float* dst = p.part_o + slot * D;
                    if (q4 == 0) p.part_lse[slot] = l > 0.f ? m + fast_log2(l) : kNegBig;
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
