// Partition kernel, vector-ALU variant: for query-head groups too narrow to form a matrix
// tile (G < 4).  One wavefront per (sequence, KV head, split).
//
// A wave-wide 16-byte load covers 64 consecutive 16-byte pieces of a (block, head) slab, i.e.
// 64/CH whole token rows (CH = pieces per row).  Lane l owns piece l % CH of token row l / CH,
// so a dot product is 8 FMAs per head in-lane plus a DPP sum over the CH lanes of the row.
// Each lane row keeps its own online-softmax state (running max, sum, accumulator slice) for
// the tokens it has seen; the rows are combined once at the end of the split.
#pragma once
#include "pa_device.hpp"

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

    const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int L = p.context_lens[b];
    const int start = s * p.C;
    const int lane = threadIdx.x;
    if (L <= 0 && s == 0) {  // empty context: the output rows of this group are zero
        for (int i = lane; i < p.G * D; i += kWave) p.out[((int64_t)b * p.Hq + g * p.G) * D + i] = 0.f;
    }
    if (start >= L) return;
    const int end = min(start + p.C, L);
    const int c = lane % CH;
    const int row = lane / CH;
    const int G = p.G;

    if (TRACE && lane == 0) {
        int32_t* r = p.trace_ranges + (((int64_t)b * p.Hkv + g) * p.S + s) * 2;
        r[0] = start;
        r[1] = end;
    }

    // this lane's slice of the G query rows, pre-multiplied by scale*log2(e) (K scale folded in)
    float qs = p.scale_log2;
    if (KV == KV_FP8) qs *= p.k_scale[g];
    float qf[GMAX][8];
#pragma unroll
    for (int h = 0; h < GMAX; ++h) {
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

    float m[GMAX], l[GMAX], acc[GMAX][8];
#pragma unroll
    for (int h = 0; h < GMAX; ++h) {
        m[h] = kNegBig;
        l[h] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
    }

    const int32_t* table = p.block_tables + (int64_t)b * p.MB;
    const int jb = start / kBlockSize, je = (end + kBlockSize - 1) / kBlockSize;
    for (int j = jb; j < je; ++j) {
        const int phys = __builtin_amdgcn_readfirstlane(table[j]);
        if (TRACE && lane == 0) {
            int32_t* v = p.trace_blocks + (((int64_t)b * p.Hkv + g) * p.MB + j) * 2;
            v[0] = phys;
            v[1] = phys;
        }
        const int64_t slab = ((int64_t)phys * p.Hkv + g) * (kBlockSize * D);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int slot = st * ROWS + row;
            const bool valid = j * kBlockSize + slot < end;
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

    // combine the ROWS lane rows (lanes with equal c), then lane row 0 writes
    const float vs = (KV == KV_FP8) ? p.v_scale[g] : 1.f;
#pragma unroll
    for (int h = 0; h < GMAX; ++h) {
        if (h < G) {
            float mt = m[h];
#pragma unroll
            for (int o = CH; o < kWave; o <<= 1) mt = fmaxf(mt, __shfl_xor(mt, o, kWave));
            const float f = fast_exp2(m[h] - mt);
            float lt = l[h] * f;
#pragma unroll
            for (int o = CH; o < kWave; o <<= 1) lt += __shfl_xor(lt, o, kWave);
            float o8[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float a = acc[h][i] * f;
#pragma unroll
                for (int o = CH; o < kWave; o <<= 1) a += __shfl_xor(a, o, kWave);
                o8[i] = a * (vs / lt);
            }
            if (row == 0) {
                const int hq = g * G + h;
                float* dst;
                if (p.S == 1 || L <= p.C) {
                    dst = p.out + ((int64_t)b * p.Hq + hq) * D + c * 8;
                } else {
                    dst = p.part_o + (((int64_t)b * p.Hq + hq) * p.S + s) * D + c * 8;
                    if (c == 0) p.part_lse[((int64_t)b * p.Hq + hq) * p.S + s] = mt + fast_log2(lt);
                }
                *reinterpret_cast<float4*>(dst) = make_float4(o8[0], o8[1], o8[2], o8[3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(o8[4], o8[5], o8[6], o8[7]);
            }
        }
    }
}

}  // namespace pa
