// Merge kernel: combines the per-split partial outputs of one (sequence, query head) row by
// their log-sum-exps.  With lse_s = log2(sum_t 2^(score_t)) over split s and o_s the split's
// normalised output, out = sum_s w_s o_s / sum_s w_s with w_s = 2^(lse_s - max_s lse_s).
// Rows whose sequence has a single split were written to `out` by the partition kernel and
// are skipped here; only entries of splits s < ceil(L/C), which the partition kernel of the
// same call wrote, are read.
#pragma once
#include "pa_device.hpp"

namespace pa {

template <int D>
__global__ __launch_bounds__(64) void merge_kernel(const Params p)
{
    constexpr int V = D / kWave;  // floats per lane (1 or 2)
    const int h = blockIdx.x, b = blockIdx.y;
    const int L = p.context_lens[b];
    if (L <= p.C) return;
    const int n = (L + p.C - 1) / p.C;
    const int lane = threadIdx.x;
    const int64_t row = (int64_t)b * p.Hq + h;
    const float* lse = p.part_lse + row * p.S;
    const float* po = p.part_o + row * p.S * D;

    float mx = kNegBig;
    for (int s = lane; s < n; s += kWave) mx = fmaxf(mx, lse[s]);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));

    float acc[V], wsum = 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    for (int s = 0; s < n; ++s) {
        const float w = fast_exp2(lse[s] - mx);
        wsum += w;
        if (V == 2) {
            const float2 x = *reinterpret_cast<const float2*>(po + (int64_t)s * D + lane * 2);
            acc[0] = fmaf(w, x.x, acc[0]);
            acc[V - 1] = fmaf(w, x.y, acc[V - 1]);
        } else {
            acc[0] = fmaf(w, po[(int64_t)s * D + lane], acc[0]);
        }
    }
    const float inv = 1.f / wsum;
    float* dst = p.out + row * D;
    if (V == 2) {
        *reinterpret_cast<float2*>(dst + lane * 2) = make_float2(acc[0] * inv, acc[V - 1] * inv);
    } else {
        dst[lane] = acc[0] * inv;
    }
}

}  // namespace pa
