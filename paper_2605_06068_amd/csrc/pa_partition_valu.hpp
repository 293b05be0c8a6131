// Partition kernel, vector-ALU variant: for query-head groups too narrow to form a matrix
// tile, for head_dim 64 and for fp8 KV.  One wavefront per (partition, KV head) walks its range
// of the batch's global tile sequence (see pa_plan.hpp), one KV block at a time.
//
// A wave-wide 16-byte load covers 64 consecutive 16-byte pieces of a (block, head) slab, i.e.
// 64/CH whole token rows (CH = pieces per row).  Lane l owns piece l % CH of token row l / CH,
// so a dot product is 8 FMAs per head in-lane plus a DPP sum over the CH lanes of the row.
// Each lane row keeps its own online-softmax state (running max, sum, accumulator slice) for
// the tokens it has seen; the rows are combined once at the end of the split.
#pragma once
#include "pa_device.hpp"
#include "pa_plan.hpp"

namespace pa {

template <int D, int KV>
struct RowPiece {  // 8 consecutive elements of one token row, widened to fp32
    float e[8];
    __device__ __forceinline__ void load(const void* cache, int64_t elem_off)
    {
        if (KV == KV_BF16) {
            const uint4 w = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(cache) + elem_off);
            e[0] = bf16_lo(w.x); e[1] = bf16_hi(w.x); e[2] = bf16_lo(w.y); e[3] = bf16_hi(w.y);
            e[4] = bf16_lo(w.z); e[5] = bf16_hi(w.z); e[6] = bf16_lo(w.w); e[7] = bf16_hi(w.w);
        } else {
            const uint2 w = *reinterpret_cast<const uint2*>(static_cast<const uint8_t*>(cache) + elem_off);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                e[i] = e4m3_to_f32((w.x >> (8 * i)) & 0xffu);
                e[4 + i] = e4m3_to_f32((w.y >> (8 * i)) & 0xffu);
            }
        }
    }
};

template <int D, int GMAX, int KV, bool TRACE>
__global__ __launch_bounds__(64) void partition_valu_kernel(const Params p)
{
    constexpr int CH = D / 8;         // 16-byte (bf16) / 8-byte (fp8) pieces per token row
    constexpr int ROWS = kWave / CH;  // token rows covered by one wave-wide load
    constexpr int STEPS = kBlockSize / ROWS;

    const int lane = threadIdx.x;
    const int g = blockIdx.x / p.P;  // partition index fastest, as in the matrix-core kernel
    const int k = blockIdx.x % p.P;
    const int G = p.G;
    const int B = p.B;
    const int c = lane % CH;
    const int row = lane / CH;

    // ---- this wave's range of the global tile sequence
    const RangeStart rs = find_range(p.context_lens, B, k, p.P, lane);
    if (k == 0) {  // empty contexts: their output rows are zero
        for (int b0 = 0; b0 < B; b0 += kWave) {
            const int b = b0 + lane;
            if (b < B && p.context_lens[b] <= 0) {
                const int64_t orow = ((int64_t)b * p.Hq + g * G) * D;
                for (int i = 0; i < G * D; ++i) store_out1(p, orow + i, 0.f);
                if (g == 0 && p.merge_desc != nullptr) write_seq_desc(p.merge_desc, b, 0, 0, 0, 0);
            }
        }
    }
    const bool describes = g == 0 && p.merge_desc != nullptr;  // this wave tells the merge about its sequences
    if (rs.t_lo >= rs.t_hi) return;
    const int ntiles = rs.t_hi - rs.t_lo;
    const int first_b = rs.b;
    int b = first_b;
    int lt = rs.t_lo - rs.cum;
    int L = rs.L;
    int nt = tiles_of(L);
    int seg_first_lt = lt;

    const float vs = (KV == KV_FP8) ? p.v_scale[g] : 1.f;
    float qs = p.scale_log2;  // scale*log2(e), with the K scale folded in
    if (KV == KV_FP8) qs *= p.k_scale[g];
    float qf[GMAX][8];
    float m[GMAX], l[GMAX], acc[GMAX][8];

    for (int tile = 0; tile < ntiles; ++tile) {
        if (tile == 0 || lt == 0) {  // segment start: this lane's slice of the G query rows, fresh state
            seg_first_lt = lt;
            if (describes && lt == 0 && lane == 0) {  // the sequence's first tile is mine
                const int cum = rs.t_lo + tile, end = cum + nt;
                write_seq_desc(p.merge_desc, b, end > rs.t_hi ? k + 1 : 0, cum, end, rs.T);
            }
#pragma unroll
            for (int h = 0; h < GMAX; ++h) {
                m[h] = kNegBig;
                l[h] = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
                if (h < G) {
                    const uint4 w = *reinterpret_cast<const uint4*>(p.q + ((int64_t)b * p.Hq + g * G + h) * D + c * 8);
                    qf[h][0] = bf16_lo(w.x) * qs; qf[h][1] = bf16_hi(w.x) * qs; qf[h][2] = bf16_lo(w.y) * qs;
                    qf[h][3] = bf16_hi(w.y) * qs; qf[h][4] = bf16_lo(w.z) * qs; qf[h][5] = bf16_hi(w.z) * qs;
                    qf[h][6] = bf16_lo(w.w) * qs; qf[h][7] = bf16_hi(w.w) * qs;
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) qf[h][i] = 0.f;
                }
            }
        }
        const int32_t* table = p.block_tables + (int64_t)b * p.MB;
        const int nblk = (L + kBlockSize - 1) / kBlockSize;
        for (int j = 2 * lt; j < min(2 * lt + 2, nblk); ++j) {
            const int phys = __builtin_amdgcn_readfirstlane(table[j]);
            if (TRACE && lane == 0) {
                int32_t* v = p.trace_blocks + (((int64_t)b * p.Hkv + g) * p.MB + j) * 3;
                v[0] = phys;
                v[1] = phys;
                v[2] = k;
            }
            const int64_t slab = ((int64_t)phys * p.Hkv + g) * (kBlockSize * D);
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
                const int slot = st * ROWS + row;
                const bool valid = j * kBlockSize + slot < L;
                RowPiece<D, KV> kp, vp;
                // slots past the context are dead: read slot 0 of the block instead (always valid)
                const int64_t off = slab + (valid ? slot : 0) * D + c * 8;
                kp.load(p.k_cache, off);
                vp.load(p.v_cache, off);
#pragma unroll
                for (int h = 0; h < GMAX; ++h) {
                    if (h < G) {
                        float part = 0.f;
#pragma unroll
                        for (int i = 0; i < 8; ++i) part = fmaf(qf[h][i], kp.e[i], part);
                        float sc = group_sum<CH>(part);
                        sc = valid ? sc : kNegBig;
                        const float m_new = fmaxf(m[h], sc);
                        const float alpha = fast_exp2(m[h] - m_new);
                        const float pr = valid ? fast_exp2(sc - m_new) : 0.f;
                        m[h] = m_new;
                        l[h] = l[h] * alpha + pr;
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[h][i] = fmaf(pr, vp.e[i], acc[h][i] * alpha);
                    }
                }
            }
        }

        if (lt == nt - 1 || tile == ntiles - 1) {
            // segment end: combine the ROWS lane rows (lanes with equal c), then lane row 0 writes
            const bool whole = seg_first_lt == 0 && lt == nt - 1;
#pragma unroll
            for (int h = 0; h < GMAX; ++h) {
                if (h < G) {
                    float mt = m[h];
#pragma unroll
                    for (int o = CH; o < kWave; o <<= 1) mt = fmaxf(mt, __shfl_xor(mt, o, kWave));
                    const float f = fast_exp2(m[h] - mt);
                    float lt_sum = l[h] * f;
#pragma unroll
                    for (int o = CH; o < kWave; o <<= 1) lt_sum += __shfl_xor(lt_sum, o, kWave);
                    float o8[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        float a = acc[h][i] * f;
#pragma unroll
                        for (int o = CH; o < kWave; o <<= 1) a += __shfl_xor(a, o, kWave);
                        o8[i] = a * (vs / lt_sum);
                    }
                    if (row == 0) {
                        const int hq = g * G + h;
                        if (whole) {
                            const int64_t e0 = ((int64_t)b * p.Hq + hq) * D + c * 8;
                            store_out4(p, e0, o8[0], o8[1], o8[2], o8[3]);
                            store_out4(p, e0 + 4, o8[4], o8[5], o8[6], o8[7]);
                        } else {
                            const int64_t slot = ((int64_t)2 * k + (b != first_b ? 1 : 0)) * p.Hq + hq;
                            float* dst = p.part_o + slot * D + c * 8;
                            if (c == 0) p.part_lse[slot] = mt + fast_log2(lt_sum);
                            *reinterpret_cast<float4*>(dst) = make_float4(o8[0], o8[1], o8[2], o8[3]);
                            *reinterpret_cast<float4*>(dst + 4) = make_float4(o8[4], o8[5], o8[6], o8[7]);
                        }
                    }
                }
            }
        }
        // next tile of the range
        if (++lt == nt) {
            lt = 0;
            do {
                ++b;
                L = b < B ? __builtin_amdgcn_readfirstlane(p.context_lens[b]) : 0;
                nt = tiles_of(L);
            } while (nt == 0 && b < B);
        }
    }
}

}  // namespace pa
