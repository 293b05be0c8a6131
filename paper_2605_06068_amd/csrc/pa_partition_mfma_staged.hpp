// Partition kernel, matrix-core variant for 17 .. 128 columns per KV head in which the waves of a
// workgroup split a tile's work by STAGE as well as by column.
//
// The multi-wave kernel of pa_partition_mfma_wide.hpp gives every wave the whole chain of a tile
// -- K reads, scores, softmax, V reads, PV -- for its own columns, holds the query operand AND the
// output accumulators in every wave, and so fits two waves per SIMD, which do not cover each
// other's dependent waits.  Here a workgroup has 2 NS waves (NS = 2 up to 64 columns, 4 above):
// waves 0 .. NS-1 ("score waves") hold the query operand and compute scores and softmax weights of
// tile i, waves NS .. 2 NS - 1 ("value waves") hold the accumulators and add the PV product of
// tile i-1, at the same time.  Wave w and wave w + NS serve the same NCT = 1 or 2 tiles of 16
// columns.  The weights travel through LDS (one 16-byte write and read per lane and column tile,
// in the register layout both matrix products use, so nothing is shuffled), together with each
// column's running maximum and rescale factor.  Every wave needs half the registers, four waves
// fit a SIMD, and a tile's chain is cut in two halves that overlap.
//
// Per step i = 0 .. ntiles (one more than there are tiles: the value waves run one behind), every
// wave of the workgroup meets at ONE barrier:
//     score waves                                   value waves
//     wait for my loads of K(i)                     wait for my loads of V(i-1)
//     ------------------------------ s_barrier -----------------------------------
//     issue my part of K(i+2)                       issue my part of V(i+1)
//     scores, softmax of tile i                     read weights(i-1), rescale, PV of tile i-1,
//     write weights(i), {alpha, m}(i)               at a segment's end: normalise, write
// K and V have rings of their own (three half-stages each: the one in use and two in flight).
// The barrier of step i says: K(i) and V(i-1) are complete, weights(i-1) are written, and nobody
// reads K(i-1), V(i-2) or weights(i-2) any more (their buffers are the ones refilled next).  All
// waves execute ntiles + 1 barriers.
//
// Layouts, swizzle, block and row selection, the arithmetic of softmax and PV, the wait-count
// discipline and the handling of query rows are those of the other two kernels
// (pa_mfma_tile.hpp, pa_partition_mfma.hpp).  fp8 KV at head_dim 128 differs in one step: the
// scores come from the fp8 matrix instruction (qk_scores_fp8 below), not from K converted to bf16.
// Every wave of a role takes an equal share of a tile's 1 KB load instructions, which is what
// bounds NS: a tile of K (or V) is 8 of them with bf16 at head_dim 128, 4 with fp8 at 128 or bf16
// at 64, 2 with fp8 at head_dim 64 (so no four score waves there).
//
// Most steps lie in the middle of a sequence, and for those the loops below skip the cursor
// arithmetic of the general step (a "run", see the score waves' loop): with sixteen waves per
// compute unit every scalar instruction per step and wave counts.  Measured, 70B-head-shaped fp8
// batch, 16 query tokens = 128 columns: 850-900 us on the multi-wave kernel, 800 us split by
// stage, 735 us with the fp8 score instruction, 685-730 us with runs; 4 query tokens = 32 columns
// (two score and two value waves): 453 -> 369 us per step.  head_dim 64, 8B-shaped batch, 16 query
// tokens: 64 bf16 columns 71.8 -> 66.3 us, 128 bf16 columns 99.3 -> 95.8, 64 fp8 columns 63.7 -> 59.5
// against the multi-wave kernel; long contexts, 64 fp8 columns: 208.7 -> 172.3 us.
#pragma once
#include <type_traits>

#include "pa_device.hpp"
#include "pa_mfma_tile.hpp"
#include "pa_partition_mfma_wide.hpp"
#include "pa_plan.hpp"

namespace pa {

constexpr int kStagedRing = 3;  // half-stages (the K or the V blocks of one tile) per ring

// LDS of a workgroup with ns score waves (and as many value waves) of nct column tiles each: the two
// rings, the score waves' query-row slots, and two sets of hand-over buffers
constexpr int staged_half_bytes(int d, int kv) { return mfma_stage_bytes(d, kv) / 2; }
constexpr int staged_weight_bytes(int ns, int nct) { return ns * nct * 1024; }    // one tile's weights
constexpr int staged_column_bytes(int ns, int nct) { return ns * nct * 16 * 8; }  // one tile's {alpha, m}

constexpr int staged_lds_bytes(int d, int ns, int nct, int kv)
{
    return 2 * kStagedRing * staged_half_bytes(d, kv) + ns * wide_q_slot_bytes(d, nct) + 2 * staged_weight_bytes(ns, nct) +
           2 * staged_column_bytes(ns, nct);
}

// The softmax step of online_softmax() for a wave that does not hold the accumulators: the same
// weights, and instead of rescaling in place the factor `alpha` the holder has to apply (1 where
// the maximum stayed, 0 for a column that had seen nothing: whatever its accumulators hold is
// dropped).  Weights at bf16 precision.
// `qs` is the wave-uniform scale (its sign picks the extreme to look for), `qsl` the scale this
// lane's column multiplies by: qs times a positive factor of the column's own (1 unless the query
// rows were rescaled, see split_query_fp8).
// The two halves of softmax_weights<false> for a caller that has matrix instructions to issue in
// between: the running maximum (and alpha) first, the weights second.
__device__ __forceinline__ void softmax_maximum(const f32x4& s0, const f32x4& s1, float qs, float qsl, float& m, float& alpha)
{
    float mx;
    if (qs >= 0.f)  // the same for every lane
        mx = max8_f32(s0, s1) * qsl;
    else
        mx = min8_f32(s0, s1) * qsl;
    alpha = 1.f;
    if (__any(mx > m + kLazyMax)) {
        const float m_new = fmaxf(m, rows_max(mx));
        alpha = m > kNegBig ? fast_exp2(m - m_new) : 0.f;
        m = m_new;
    }
}

__device__ __forceinline__ void softmax_exponentials(const f32x4& s0, const f32x4& s1, float qsl, float m, bf16x8& pb)
{
    const float neg_m = -m;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        pb[r] = (__bf16)fast_exp2(fmaf(s0[r], qsl, neg_m));
        pb[4 + r] = (__bf16)fast_exp2(fmaf(s1[r], qsl, neg_m));
    }
}

template <bool MASKED>
__device__ __forceinline__ void softmax_weights(const f32x4& s0, const f32x4& s1, float qs, float qsl, int t0, int lim, int low,
                                                float& m, float& alpha, bf16x8& pb)
{
    float v[8];
    bool ok[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        v[r] = s0[r];
        v[4 + r] = s1[r];
        ok[r] = !MASKED || (t0 + r < lim && t0 + r >= low);
        ok[4 + r] = !MASKED || (t0 + kBlockSize + r < lim && t0 + kBlockSize + r >= low);
    }
    float mx;
    if (MASKED) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = ok[r] ? v[r] * qsl : kNegBig;
        mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
    } else if (qs >= 0.f) {  // the same for every lane
        mx = max8_f32(s0, s1) * qsl;
    } else {
        mx = min8_f32(s0, s1) * qsl;
    }
    alpha = 1.f;
    if (__any(mx > m + kLazyMax)) {
        const float m_new = fmaxf(m, rows_max(mx));
        alpha = m > kNegBig ? fast_exp2(m - m_new) : 0.f;
        m = m_new;
    }
    const float neg_m = -m;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const float x = MASKED ? (ok[r] ? fast_exp2(v[r] - m) : 0.f) : fast_exp2(fmaf(v[r], qsl, neg_m));
        pb[r] = (__bf16)x;
    }
}

// ---- fp8 KV: scores on the fp8 matrix instruction, no conversion of K --------------------------
// v_mfma_f32_16x16x128_f8f6f4 contracts the whole head_dim of 128 in one instruction; lane
// l = 16 q4 + n holds 32 consecutive bytes of row n of its operand, dims 32 q4 .. 32 q4 + 31 (any
// assignment of dims to byte positions does, as long as both operands use the same one).  The K
// bytes go in as they lie in the cache.  The query rows, bf16, are split once per segment into
// two e4m3 numbers each: with x = q * 2^s (s chosen per row so that the largest |x| lies in
// [128, 256)), hi = e4m3(x) keeps the upper four significant bits and x - hi, which has at most
// four more, is an e4m3 number again whenever |x| >= 1/4; below that (elements 2^10 times smaller
// than the row's largest) the remainder is rounded to a multiple of 2^-9.  K . hi + K . lo is then
// K . q 2^s up to float32 summation order, and 2^-s joins the column's softmax scale.  Two fp8
// instructions of depth 128 take the matrix pipe as long as the four bf16 ones of depth 32 they
// replace, and the 32 conversions per wave and tile are gone.
typedef int i32x8 __attribute__((ext_vector_type(8)));

// The 16 columns' query rows from an LDS slot into the two fp8 operands; returns 2^-s of this
// lane's column.  A padding column gets zeros.
__device__ __forceinline__ float split_query_fp8(const char* slot, int n, int q4, bool col_ok, i32x8& hi, i32x8& lo)
{
    using QG = QGeom<128>;
    float x[32];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        uint4 w = *reinterpret_cast<const uint4*>(slot + (col_ok ? n : 0) * QG::kRow + (((4 * q4 + h) ^ (n & (QG::kPieces - 1))) << 4));
        if (!col_ok) w = make_uint4(0, 0, 0, 0);
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[8 * h + 2 * e] = bf16_lo(u[e]);
            x[8 * h + 2 * e + 1] = bf16_hi(u[e]);
        }
    }
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 32; ++e) amax = fmaxf(amax, fabsf(x[e]));
    amax = rows_max(amax);  // over the four lanes that hold the row
    // amax = f 2^ex with f in [0.5, 1): x 2^(8 - ex) has its largest element in [128, 256).  (Rows whose
    // largest element lies below 2^-100 keep the factor of 2^-100: the powers of two stay finite.)
    const int ex = amax > 0.f ? max(__builtin_amdgcn_frexp_expf(amax), -100) : 8;
    const float up = __builtin_amdgcn_ldexpf(1.f, 8 - ex), down = __builtin_amdgcn_ldexpf(1.f, ex - 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float a = x[4 * e] * up, b = x[4 * e + 1] * up, c = x[4 * e + 2] * up, d = x[4 * e + 3] * up;
        int wh = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
        wh = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, wh, true);
        const float ra = a - __builtin_amdgcn_cvt_f32_fp8(wh, 0), rb = b - __builtin_amdgcn_cvt_f32_fp8(wh, 1),
                    rc = c - __builtin_amdgcn_cvt_f32_fp8(wh, 2), rd = d - __builtin_amdgcn_cvt_f32_fp8(wh, 3);
        int wl = __builtin_amdgcn_cvt_pk_fp8_f32(ra, rb, 0, false);
        wl = __builtin_amdgcn_cvt_pk_fp8_f32(rc, rd, wl, true);
        hi[e] = wh;
        lo[e] = wl;
    }
    return down;
}

// S^T[token, column] for the two blocks of an fp8 tile and NCT tiles of 16 columns
template <int NCT>
__device__ __forceinline__ void qk_scores_fp8(const char* kbuf, const uint32_t (&kread)[2], const i32x8 (&qhi)[NCT],
                                              const i32x8 (&qlo)[NCT], f32x4 (&s0)[NCT], f32x4 (&s1)[NCT])
{
    constexpr int kSlabBytes = KvGeom<128, KV_FP8>::kSlab;
    i32x8 a[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
        const uint4 p0 = *reinterpret_cast<const uint4*>(kbuf + sub * kSlabBytes + kread[0]);
        const uint4 p1 = *reinterpret_cast<const uint4*>(kbuf + sub * kSlabBytes + kread[1]);
        a[sub] = i32x8{(int)p0.x, (int)p0.y, (int)p0.z, (int)p0.w, (int)p1.x, (int)p1.y, (int)p1.z, (int)p1.w};
    }
    const f32x4 zero{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        s0[ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[0], qhi[ct], zero, 0, 0, 0, 0, 0, 0);
        s1[ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[1], qhi[ct], zero, 0, 0, 0, 0, 0, 0);
    }
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        s0[ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[0], qlo[ct], s0[ct], 0, 0, 0, 0, 0, 0);
        s1[ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[1], qlo[ct], s1[ct], 0, 0, 0, 0, 0, 0);
    }
}

// ... the same in two steps, for interleaving: the K operand of a tile, then one column tile's scores
__device__ __forceinline__ void read_k_fp8(const char* kbuf, const uint32_t (&kread)[2], i32x8 (&a)[2])
{
    constexpr int kSlabBytes = KvGeom<128, KV_FP8>::kSlab;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
        const uint4 p0 = *reinterpret_cast<const uint4*>(kbuf + sub * kSlabBytes + kread[0]);
        const uint4 p1 = *reinterpret_cast<const uint4*>(kbuf + sub * kSlabBytes + kread[1]);
        a[sub] = i32x8{(int)p0.x, (int)p0.y, (int)p0.z, (int)p0.w, (int)p1.x, (int)p1.y, (int)p1.z, (int)p1.w};
    }
}
__device__ __forceinline__ void qk_scores_fp8_one(const i32x8 (&a)[2], const i32x8& qhi, const i32x8& qlo, f32x4& s0, f32x4& s1)
{
    const f32x4 zero{0.f, 0.f, 0.f, 0.f};
    s0 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[0], qhi, zero, 0, 0, 0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[1], qhi, zero, 0, 0, 0, 0, 0, 0);
    s0 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[0], qlo, s0, 0, 0, 0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[1], qlo, s1, 0, 0, 0, 0, 0, 0);
}

// Waves per SIMD the register budget is cut for (the second launch bound): as many as the LDS lets
// a compute unit hold, four at most (128 registers each); the instrumented variants, whose records
// need a few more, settle for two.
constexpr int staged_waves_per_simd(int d, int ns, int nct, int kv, bool trace)
{
    const int by_lds = (160 * 1024 / staged_lds_bytes(d, ns, nct, kv)) * 2 * ns / 4;
    const int most = trace ? 2 : 4;
    return by_lds < most ? by_lds : most;
}

template <int D, int NS, int NCT, int KV, bool TRACE>
__global__ __launch_bounds__(2 * NS * 64, staged_waves_per_simd(D, NS, NCT, KV, TRACE)) void partition_mfma_staged_kernel(const Params p)
{
    static_assert(D == 128 || D == 64, "head_dim");
    constexpr bool QK_F8 = KV == KV_FP8 && D == 128;  // scores on the fp8 matrix instruction (whose depth is 128)
    static_assert(NS == 2 || NS == 4, "score waves per workgroup");
    static_assert(NCT == 1 || NCT == 2, "MFMA column tiles per wave");
    constexpr int kWaveCols = 16 * NCT;
    using Geo = KvGeom<D, KV>;
    using QG = QGeom<D>;
    constexpr int kSlabBytes = Geo::kSlab;
    constexpr int kHalf = 2 * kSlabBytes;               // the K (or V) blocks 0 and 1 of a tile
    constexpr int kDmaPerHalf = 2 * Geo::kDmaPerSlab;
    constexpr int PT = kDmaPerHalf / NS;                // LDS-DMA instructions per wave and tile
    static_assert(PT >= 1 && PT * NS == kDmaPerHalf, "shares of a tile's loads");
    constexpr int kQSlotBytes = wide_q_slot_bytes(D, NCT);
    constexpr int kQLoads = kQSlotBytes / 1024;
    constexpr int kQBase = 2 * kStagedRing * kHalf;
    constexpr int kWBase = kQBase + NS * kQSlotBytes;
    constexpr int kCBase = kWBase + 2 * staged_weight_bytes(NS, NCT);
    static_assert(staged_lds_bytes(D, NS, NCT, KV) == kCBase + 2 * staged_column_bytes(NS, NCT), "layout");
    static_assert(staged_lds_bytes(D, NS, NCT, KV) <= 160 * 1024, "LDS of one compute unit");
    __shared__ __attribute__((aligned(1024))) char smem[staged_lds_bytes(D, NS, NCT, KV)];

    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool score = w < NS;   // the wave's role
    const int wl = w & (NS - 1); // its column slice, and its share of the role's loads
    const int k = blockIdx.x % p.P;
    const int g = (blockIdx.x / p.P) % p.Hkv;
    const int col0 = (blockIdx.x / p.P / p.Hkv) * (kWaveCols * NS);
    const int G = p.G;
    const int B = p.B;
    const int Q = p.Q;
    const int ncols = Q * G;
    const int n = lane & 15;
    const int q4 = lane >> 4;

    const int reach = p.window > 0 ? p.window + Q - 1 : 0;
    const int skip = p.skip_tiles;
    const Span sp{skip, reach};
    const RangeStart rs = find_range(p.context_lens, B, k, p.P, lane, sp);
    if (skip == 0 && w == 0 && col0 == 0) zero_rows_of_empty_contexts(p, k, g, B, Q, D, lane);
    const bool describes = g == 0 && w == 0 && col0 == 0 && p.merge_desc != nullptr;
    if (describes && p.cut_list != nullptr && lane == 0)
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

    // ---- this wave's share of its role's loads: instructions wl*PT .. wl*PT+PT-1 of the half tile
    // (block 0, then block 1)
    int my_sub[PT];        // block of the tile
    uint32_t my_dst[PT];   // LDS byte offset inside a half-stage
    uint32_t my_off[PT];   // this lane's global byte offset inside the slab (swizzled piece)
    int my_tok[PT];        // token row of the block this lane loads
#pragma unroll
    for (int j = 0; j < PT; ++j) {
        const int d = wl * PT + j;
        my_sub[j] = d / Geo::kDmaPerSlab;
        const int r = d % Geo::kDmaPerSlab;
        my_dst[j] = my_sub[j] * kSlabBytes + r * 1024;
        my_tok[j] = r * Geo::kRowsPerDma + lane / Geo::kPieces;
        my_off[j] = slab_dma_offset<D, KV>(r, lane);
    }
    OperandOffsets<D, KV> of;
    of.init(n, q4);
    const bool wave_active = col0 + kWaveCols * wl < ncols;  // a wave without real columns only loads and meets the others
    bool col_ok[NCT];
    int col_back[NCT];
    int col_row[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int col = col0 + kWaveCols * wl + 16 * ct + n;
        col_ok[ct] = col < ncols;
        const int col_i = col_ok[ct] ? col / G : 0, col_h = col_ok[ct] ? col % G : 0;
        col_back[ct] = col_ok[ct] ? Q - 1 - col_i : (1 << 30);
        col_row[ct] = col_i * p.Hq + g * G + col_h;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t ring0 = lds0 + (score ? 0 : kStagedRing * kHalf);  // my role's ring
    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;
    const uint32_t head_stride32 = (uint32_t)p.Hkv * (uint32_t)kSlabBytes;  // the same; the host keeps it below 2^32
    const char* cache = static_cast<const char*>(score ? p.k_cache : p.v_cache) + (int64_t)g * kSlabBytes;
    // what the two waves of a column slice hand over, per step parity: weights and {alpha, m}
    char* const wbuf = smem + kWBase + wl * NCT * 1024 + lane * 16;
    char* const cbuf = smem + kCBase + wl * NCT * 128 + n * 8;

    int nx_id0 = 0, nx_id1 = 0;  // ids of the tile `ic` stands on ...
    bool nx_valid = false;       // ... if they were asked for ahead
    auto issue = [&](int stage) __attribute__((always_inline)) {
        const uint32_t ldst = ring0 + stage * kHalf;
        if (!TRACE && nx_valid) {
            // interior tile, ids already here: every row is visible
#pragma unroll
            for (int j = 0; j < PT; ++j) {
                const uint32_t id = (uint32_t)(my_sub[j] ? nx_id1 : nx_id0);
                dma16<true>(ldst + my_dst[j], my_off[j], cache + (uint64_t)id * head_stride32);
            }
        } else {
            TileBlocks tb = tile_blocks(p.block_tables, p.MB, ic, reach);
            if (TRACE) {
                // every wave records the (block, K or V) pairs of its own instructions, for the first column group
                const RawIds raw = check_tile_blocks(tb, p.num_blocks);
                if (lane == 0 && col0 == 0) {
#pragma unroll
                    for (int j = 0; j < PT; ++j)
                        trace_block_use(p.trace_blocks, tb, raw, my_sub[j], score ? 0 : 1, ic.b, g, k, p.Hkv, p.MB);
                }
            }
#pragma unroll
            for (int j = 0; j < PT; ++j) {
                const int sub = my_sub[j];
                dma16<true>(ldst + my_dst[j],
                            live_or_stand_in<D, KV>(my_off[j], my_tok[j], sub ? tb.lo[1] : tb.lo[0], sub ? tb.hi[1] : tb.hi[0]),
                            cache + (sub ? tb.phys[1] : tb.phys[0]) * head_stride);
            }
        }
        advance(ic, p.context_lens, B, sp);
        nx_valid = ask_next_ids(p.block_tables, p.MB, ic, B, reach, nx_id0, nx_id1);
    };

    if (score) {
        // ================================ score waves ================================
        const uint32_t ldsq = lds0 + kQBase + wl * kQSlotBytes;
        const char* qslot = smem + kQBase + wl * kQSlotBytes;
        // query rows of this wave's columns: LDS row lc holds column c = kWaveCols wl + lc (the per-lane source
        // offsets are worked out at every use, once per segment, rather than held in registers)
        auto issue_q = [&](int b) __attribute__((always_inline)) {
            const char* qb = reinterpret_cast<const char*>(p.q) + ((int64_t)b * (Q * p.Hq) + g * G) * QG::kRow;
#pragma unroll
            for (int r = 0; r < kQLoads; ++r) {
                const int lc = r * QG::kRowsPerDma + lane / QG::kPieces;
                const int c = col0 + kWaveCols * wl + lc;
                const int src = c < ncols ? ((c / G) * p.Hq + (c % G)) * QG::kRow : 0;
                dma16<false>(ldsq + r * 1024, src + (((lane % QG::kPieces) ^ (lc & (QG::kPieces - 1))) << 4), qb);
            }
        };
        const float qs = KV == KV_FP8 ? p.scale_log2 * p.k_scale[g] : p.scale_log2;
        float m[NCT];
        float qsl[NCT];            // the column's scale: qs, times 2^-s of its query row for fp8 KV
        bf16x8 qreg[NCT][D / 32];  // bf16 KV: the query operand
        i32x8 qhi[NCT], qlo[NCT];  // fp8 KV: the same as two fp8 operands
        // fp8 KV: this lane's two 16-byte pieces of K row n (dims 32 q4 .. 32 q4 + 31) inside a slab
        const uint32_t kread8[2] = {(uint32_t)(n * Geo::kRow + (((2 * q4) ^ (n & (Geo::kPieces - 1))) << 4)),
                                    (uint32_t)(n * Geo::kRow + (((2 * q4 + 1) ^ (n & (Geo::kPieces - 1))) << 4))};

        // scores, weights and their hand-over for the tile in K stage `stage`; unmasked: every column sees
        // the whole tile (all but the last tiles of a sequence and the tiles where sliding windows begin)
        auto score_tile = [&](int stage, int par, bool unmasked) __attribute__((always_inline)) {
            f32x4 s0[NCT], s1[NCT];
            float alpha[NCT];
            bf16x8 pb[NCT];
            if constexpr (QK_F8 && NCT == 2) {
                if (unmasked) {
                    // the second column tile's matrix instructions run while the first one's exponentials issue
                    i32x8 a[2];
                    read_k_fp8(smem + stage * kHalf, kread8, a);
                    qk_scores_fp8_one(a, qhi[0], qlo[0], s0[0], s1[0]);
                    softmax_maximum(s0[0], s1[0], qs, qsl[0], m[0], alpha[0]);
                    qk_scores_fp8_one(a, qhi[1], qlo[1], s0[1], s1[1]);
                    softmax_exponentials(s0[0], s1[0], qsl[0], m[0], pb[0]);
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
                        __builtin_amdgcn_sched_group_barrier(0x002 | 0x400, 5, 0);  // five vector / transcendental ones
                    }
                    {  // keeps the first tile's weights on this side of the second tile's branch
                        typedef int i32x4 __attribute__((ext_vector_type(4)));
                        i32x4 w = __builtin_bit_cast(i32x4, pb[0]);
                        asm volatile("" : "+v"(w));
                        pb[0] = __builtin_bit_cast(bf16x8, w);
                    }
                    softmax_maximum(s0[1], s1[1], qs, qsl[1], m[1], alpha[1]);
                    softmax_exponentials(s0[1], s1[1], qsl[1], m[1], pb[1]);
                } else {
                    qk_scores_fp8<NCT>(smem + stage * kHalf, kread8, qhi, qlo, s0, s1);
                }
            } else if constexpr (QK_F8) {
                qk_scores_fp8<NCT>(smem + stage * kHalf, kread8, qhi, qlo, s0, s1);
            } else {
                qk_scores<D, KV, NCT>(smem + stage * kHalf, of, qreg, s0, s1);
            }
            const int tile_first = (cc.lt + cc.ft) * kTileTokens;
            if (QK_F8 && NCT == 2 && unmasked) {
                // done above
            } else if (unmasked) {
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
                    softmax_weights<false>(s0[ct], s1[ct], qs, qsl[ct], 0, 0, 0, m[ct], alpha[ct], pb[ct]);
            } else {
                const int t0 = tile_first + 4 * q4;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const int lim = cc.L - col_back[ct];
                    const int low = p.window > 0 ? lim - p.window : INT32_MIN;
                    softmax_weights<true>(s0[ct], s1[ct], qs, qsl[ct], t0, lim, low, m[ct], alpha[ct], pb[ct]);
                }
            }
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                *reinterpret_cast<bf16x8*>(wbuf + par * staged_weight_bytes(NS, NCT) + ct * 1024) = pb[ct];
                if (q4 == 0)
                    *reinterpret_cast<float2*>(cbuf + par * staged_column_bytes(NS, NCT) + ct * 128) = make_float2(alpha[ct], m[ct]);
            }
        };

        // prologue: the first segment's query rows, then K of the first two tiles
        issue_q(first_b);
        int q_age = 0;  // tiles this wave has put loads in flight for since it last issued query rows
        for (int t = 0; t < 2; ++t)
            if (t < ntiles) {
                issue(t);
                ++q_age;
            }

        // A run of steps in the middle of things: the tiles to score are no segment's first and need
        // no mask, the tiles to load are interior tiles of one sequence, and neither is its sequence's
        // last.  Such steps take none of the cursor arithmetic of the general step: the table is walked
        // with a pointer, two entries per tile, asked for one step ahead, and the cursors are counted
        // up.  (With eight waves per workgroup and sixteen per compute unit, the scalar instructions of
        // that arithmetic, every wave's own copy of it, cost more time than the matrix instructions.)
        int run = 0;                 // steps of the current run still to go
        const int32_t* tp = nullptr; // table entries of the tile to load next, while a run lasts
        int id0 = 0, id1 = 0;        // ... and their values

        int stage = 0;
        for (int i = 0; i < ntiles; ++i) {
            const bool fast = run > 0;
            const bool seg_start = !fast && (i == 0 || cc.lt == 0);
            // K(i) has landed once at most the tile issued after it is in flight; at a segment start the
            // query rows (issued q_age tiles ago) must have landed as well
            if (fast || (i + 1 < ntiles && !(seg_start && q_age == 0)))
                wait_vmcnt<PT>();
            else
                wait_vmcnt<0>();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // my reads of K(i-1) have returned, my weights(i-1) are written
            __builtin_amdgcn_s_barrier();
            int stg = stage + 2;
            if (stg >= kStagedRing) stg -= kStagedRing;
            if (fast) {
#pragma unroll
                for (int j = 0; j < PT; ++j)
                    dma16<true>(ring0 + stg * kHalf + my_dst[j], my_off[j],
                                cache + (uint64_t)(uint32_t)(my_sub[j] ? id1 : id0) * head_stride32);
                ++ic.lt;
                ++q_age;
            } else if (i + 2 < ntiles) {
                issue(stg);
                ++q_age;
            }
            if (wave_active) {
                if (seg_start) {
                    if (describes && cc.lt == 0 && lane == 0) {  // the sequence's first tile is this workgroup's
                        const int cum = rs.t_lo + i, end = cum + cc.nt;
                        write_seq_desc(p.merge_desc, cc.b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
                    }
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        m[ct] = kNegBig;
                        if constexpr (QK_F8) {
                            qsl[ct] = qs * split_query_fp8(qslot + ct * 16 * QG::kRow, n, q4, col_ok[ct], qhi[ct], qlo[ct]);
                        } else {
                            qsl[ct] = qs;
                            load_query_operand<D>(qslot + ct * 16 * QG::kRow, n, q4, col_ok[ct], qreg[ct]);
                        }
                    }
                    // refill the slot with the rows of the next segment of this range, if there is one
                    if (i + (cc.nt - cc.lt) < ntiles) {
                        int nb = cc.b;
                        do {
                            ++nb;
                        } while (nb < B - 1 && tiles_of(uniform_load(p.context_lens, nb), sp) == 0);
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slot has been read
                        issue_q(nb);
                        q_age = 0;
                    }
                }
                const int tile_first = (cc.lt + cc.ft) * kTileTokens;
                score_tile(stage, i & 1,
                           fast || (tile_first + kTileTokens <= cc.L - (Q - 1) && (reach == 0 || tile_first >= cc.L - p.window)));
            }
            if (fast) {
                ++cc.lt;
                --run;
                asm volatile("" ::: "memory");  // the next ids are asked for behind this tile's LDS traffic
                tp += 2;
                if (run > 0) {  // (the entries behind the run's last tile may not exist)
                    id0 = uniform_load(tp, 0);
                    id1 = uniform_load(tp, 1);
                }
            } else {
                advance(cc, p.context_lens, B, sp);
                // does a run begin with the next step?
                if (!TRACE && reach == 0 && cc.lt > 0 && ic.b < B) {
                    const int n_c = min((cc.L - (Q - 1)) / kTileTokens - cc.ft, cc.nt - 1) - cc.lt;
                    const int n_i = min(ic.L / kTileTokens - ic.ft, ic.nt - 1) - ic.lt;
                    run = max(min(min(n_c, n_i), ntiles - 3 - i), 0);
                    if (run > 0) {
                        tp = p.block_tables + (int64_t)ic.b * p.MB + 2 * (ic.lt + ic.ft);
                        id0 = nx_valid ? nx_id0 : uniform_load(tp, 0);
                        id1 = nx_valid ? nx_id1 : uniform_load(tp, 1);
                        nx_valid = false;
                    }
                }
            }
            stage = (stage + 1 == kStagedRing) ? 0 : stage + 1;
        }
        // step ntiles, the value waves' last: the weights of the last tile are written
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    } else {
        // ================================ value waves ================================
        // The value waves issue ahead of the score waves they share a SIMD with: their step is mostly
        // matrix instructions, which then start as soon as their operands are there and run while the
        // score waves' vector instructions fill the issue slots in between (fp8 KV, 32 / 64 / 128
        // columns: 365 -> 352, 529 -> 515, 717 -> 694 us per step; bf16 KV unchanged).
        __builtin_amdgcn_s_setprio(1);
        const float vs = KV == KV_FP8 ? p.v_scale[g] : 1.f;
        ColumnState<D> st[NCT];
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) st[ct].clear();
        int seg_first_lt = 0;

        // weights of the tile in V stage `stage` from the hand-over buffers, rescale, PV
        auto value_tile = [&](int stage, int par) __attribute__((always_inline)) {
            bf16x8 pb[NCT], pb_lo[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                pb[ct] = *reinterpret_cast<const bf16x8*>(wbuf + par * staged_weight_bytes(NS, NCT) + ct * 1024);
                const float2 am = *reinterpret_cast<const float2*>(cbuf + par * staged_column_bytes(NS, NCT) + ct * 128);
                if (__any(am.x != 1.f)) {
                    st[ct].lacc *= am.x;
#pragma unroll
                    for (int dt = 0; dt < D / 16; ++dt) st[ct].acc[dt] *= am.x;
                }
                st[ct].m = am.y;
            }
            pv_accumulate<D, KV, NCT, false>(smem + (kStagedRing + stage) * kHalf, of, pb, pb_lo, st);
        };

        issue(0);  // V of the first tile

        // step 0, the score waves' first: nothing to compute yet
        __builtin_amdgcn_s_barrier();
        if (1 < ntiles) issue(1);

        // a run of steps in the middle of things (see the score waves): the tiles to multiply are neither
        // first nor last of their segment, the tiles to load are interior tiles of one sequence
        int run = 0;
        const int32_t* tp = nullptr;
        int id0 = 0, id1 = 0;

        int stage = 0;  // of V(i-1)
        for (int i = 1; i <= ntiles; ++i) {
            const bool fast = run > 0;
            // V(i-1) has landed once at most V(i), issued after it, is in flight
            if (i < ntiles)
                wait_vmcnt<PT>();
            else
                wait_vmcnt<0>();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // my reads of V(i-2) and weights(i-2) have returned
            __builtin_amdgcn_s_barrier();
            int stg = stage + 2;
            if (stg >= kStagedRing) stg -= kStagedRing;
            if (fast) {
#pragma unroll
                for (int j = 0; j < PT; ++j)
                    dma16<true>(ring0 + stg * kHalf + my_dst[j], my_off[j],
                                cache + (uint64_t)(uint32_t)(my_sub[j] ? id1 : id0) * head_stride32);
                ++ic.lt;
            } else if (i + 1 < ntiles) {
                issue(stg);
            }
            const int tile = i - 1;
            if (wave_active) {
                if (!fast && (tile == 0 || cc.lt == 0)) seg_first_lt = cc.lt;
                value_tile(stage, tile & 1);

                // ---- segment end: normalise, write
                if (!fast && (cc.lt == cc.nt - 1 || tile == ntiles - 1)) {
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
            }
            if (fast) {
                ++cc.lt;
                --run;
                asm volatile("" ::: "memory");
                tp += 2;
                if (run > 0) {
                    id0 = uniform_load(tp, 0);
                    id1 = uniform_load(tp, 1);
                }
            } else {
                advance(cc, p.context_lens, B, sp);
                // does a run begin with the next step?
                if (!TRACE && reach == 0 && cc.lt > 0 && ic.b < B) {
                    const int n_c = cc.nt - 1 - cc.lt;
                    const int n_i = min(ic.L / kTileTokens - ic.ft, ic.nt - 1) - ic.lt;
                    run = max(min(min(n_c, n_i), ntiles - 2 - i), 0);
                    if (run > 0) {
                        tp = p.block_tables + (int64_t)ic.b * p.MB + 2 * (ic.lt + ic.ft);
                        id0 = nx_valid ? nx_id0 : uniform_load(tp, 0);
                        id1 = nx_valid ? nx_id1 : uniform_load(tp, 1);
                        nx_valid = false;
                    }
                }
            }
            stage = (stage + 1 == kStagedRing) ? 0 : stage + 1;
        }
    }
}

}  // namespace pa
