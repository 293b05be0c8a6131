// Merge kernel: combines the partial results of every sequence that a partition boundary cuts
// (see pa_plan.hpp).  With lse_s = log2(sum_t 2^(score_t)) over segment s and o_s the segment's
// normalised output, out = sum_s w_s o_s / sum_s w_s with w_s = 2^(lse_s - max_s lse_s).
//
// One wavefront per (cut sequence b, output row h of a sequence: query head, or (query token,
// query head) pair of a multi-token call).  The descriptor the partition kernel wrote for b (see
// write_seq_desc) says whether b was cut and, if so, names the first boundary j strictly inside
// it (the start of partition j) and b's place in the tile sequence.  The grid has room for
// min(B, P - 1) cut sequences; slot y takes the y-th sequence that was cut, the rest exit.  The partials of b come from the partitions
// k = j-1, j, j+1, ... whose ranges intersect b: slot 2k when b holds partition k's first tile,
// slot 2k+1 otherwise (only possible for k = j-1).  Only slots written by the partition kernel
// of the same call are read.
#pragma once
#include "pa_device.hpp"
#include "pa_plan.hpp"

namespace pa {

// The y-th sequence (in batch order) whose descriptor says it was cut, or -1 if there are fewer:
// the merge grids have one slot per sequence that CAN be cut (at most P - 1 of them are), and
// slot y takes the y-th one that was.  All 64 lanes must call; the result is wave-uniform.
__device__ __forceinline__ int nth_cut_sequence(const int32_t* desc, int B, int y, int lane)
{
    int seen = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        const bool cut = b < B && desc[4 * (int64_t)b] != 0;
        const unsigned long long mask = __ballot(cut);
        const int c = __popcll(mask);
        if (y < seen + c) {
            const bool hit = cut && (int)__popcll(mask & ((1ull << lane) - 1ull)) == y - seen;
            return b0 + __ffsll((long long)__ballot(hit)) - 1;
        }
        seen += c;
    }
    return -1;
}

// The sequence merge slot y works on, or -1.  Large batches come with a list of the sequences that
// the partitions' starts cut (cut_list[k] for boundary k = y + 1): the slot takes the sequence its
// boundary cuts if that is the first boundary inside it (a sequence cut several times is merged
// once; an empty partition that lies between two tiles of a sequence counts as a boundary there, or
// a sequence whose first boundary it is would be merged by nobody).  Small batches (one or two 64-lane scans) look for the y-th cut sequence instead.  All
// 64 lanes must call; the result is wave-uniform.
__device__ __forceinline__ int slot_sequence(const Params& p, int y, int lane)
{
    if (p.cut_list == nullptr) return nth_cut_sequence(p.merge_desc, p.B, y, lane);
    const int k = y + 1;
    const int b = uniform_load(p.cut_list, k);
    if (b < 0) return -1;
    return uniform_load(p.merge_desc, 4 * (int64_t)b) == k ? b : -1;
}

template <int D>
__global__ __launch_bounds__(64) void merge_kernel(const Params p)
{
    constexpr int V = D / kWave;  // floats per lane (1 or 2)
    __shared__ int s_slot[kWave];
    __shared__ float s_w[kWave];
    const int h = blockIdx.x;
    const int lane = threadIdx.x;
    const int P = p.P;

    // what the partition kernel left about the sequences: see write_seq_desc
    const int b = slot_sequence(p, blockIdx.y, lane);
    if (b < 0) return;  // fewer sequences were cut than the grid has room for
    const int j = uniform_load(p.merge_desc, 4 * (int64_t)b);
    const int cum = uniform_load(p.merge_desc, 4 * (int64_t)b + 1), end_b = uniform_load(p.merge_desc, 4 * (int64_t)b + 2),
              T = uniform_load(p.merge_desc, 4 * (int64_t)b + 3);

    float acc[V], wsum = 0.f, mrun = kNegBig;
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;

    for (int base = j - 1; base < P; base += kWave) {
        const int kk = base + lane;
        bool valid = false;
        int slot = 0;
        if (kk < P) {
            const int lo = part_begin(kk, T, P), hi = part_begin(kk + 1, T, P);
            valid = hi > lo && lo < end_b && hi > cum;
            slot = 2 * kk + ((kk == j - 1 && lo != cum) ? 1 : 0);
        }
        const unsigned long long vmask = __ballot(valid);
        if (vmask == 0ull) {
            // 64 partitions without a piece: behind the sequence, or empty partitions inside it (a call
            // with far fewer tiles than partitions spreads a sequence's pieces that far apart)
            if (part_begin(base, T, P) >= end_b) break;
            continue;
        }
        const float lse = valid ? p.part_lse[(int64_t)slot * p.QH + h] : kNegBig;
        float cm = lse;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) cm = fmaxf(cm, __shfl_xor(cm, o, kWave));
        const float m_new = fmaxf(mrun, cm);
        const float rescale = fast_exp2(mrun - m_new);
        const float w = valid ? fast_exp2(lse - m_new) : 0.f;
        float ws = w;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) ws += __shfl_xor(ws, o, kWave);
        wsum = wsum * rescale + ws;
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] *= rescale;
        mrun = m_new;

        // compact the valid (slot, weight) pairs, then stream the partial rows 8 at a time
        const int pos = __popcll(vmask & ((1ull << lane) - 1ull));
        const int cnt = __popcll(vmask);
        if (valid) {
            s_slot[pos] = slot;
            s_w[pos] = w;
        }
        __syncthreads();
        for (int i0 = 0; i0 < cnt; i0 += 8) {
            float wv[8];
            float2 xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = min(i0 + u, cnt - 1);
                wv[u] = (i0 + u < cnt) ? s_w[idx] : 0.f;
                const float* row = p.part_o + ((int64_t)s_slot[idx] * p.QH + h) * D;
                if (V == 2) {
                    xv[u] = *reinterpret_cast<const float2*>(row + lane * 2);
                } else {
                    xv[u].x = row[lane];
                    xv[u].y = 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc[0] = fmaf(wv[u], xv[u].x, acc[0]);
                if (V == 2) acc[V - 1] = fmaf(wv[u], xv[u].y, acc[V - 1]);
            }
        }
        __syncthreads();
    }
    const float inv = 1.f / wsum;
    const int64_t row = ((int64_t)b * p.QH + h) * D;
    if (V == 2)
        store_out2(p, row + lane * 2, acc[0] * inv, acc[V - 1] * inv);
    else
        store_out1(p, row + lane, acc[0] * inv);
}

// ---------------------------------------------------------------------------------------------
// The same merge for calls with many output rows per sequence (multi-token calls, wide models):
// one wavefront merges FOUR rows of one cut sequence, 16 lanes per row, D / 16 floats per lane.
// The rows of a sequence share its pieces, so control flow stays wave-uniform; every lane walks
// the pieces itself (no cross-lane traffic), four pieces at a time with all their loads in
// flight together.  Against one wave per row this cuts the number of waves, and with it the
// rounds of dependent round trips the grid needs, by four (8B-shaped batch, 16 query tokens =
// 512 rows x 63 cut sequences: 16.9 -> 12.3 us); with few rows per sequence one wave per row is
// as fast or faster, and the host keeps it there.
constexpr int kMergeRowsPerWave = 4;

template <int D>
__global__ __launch_bounds__(64) void merge_rows_kernel(const Params p)
{
    constexpr int kLanesPerRow = kWave / kMergeRowsPerWave;  // 16
    constexpr int V4 = D / kLanesPerRow / 4;                  // float4s per lane: 2 (head_dim 128) or 1 (64)
    const int lane = threadIdx.x;
    const int P = p.P;
    const int b = slot_sequence(p, blockIdx.y, lane);
    if (b < 0) return;  // fewer sequences were cut than the grid has room for
    const int j = uniform_load(p.merge_desc, 4 * (int64_t)b);
    const int cum = uniform_load(p.merge_desc, 4 * (int64_t)b + 1), end_b = uniform_load(p.merge_desc, 4 * (int64_t)b + 2),
              T = uniform_load(p.merge_desc, 4 * (int64_t)b + 3);

    const int h = blockIdx.x * kMergeRowsPerWave + lane / kLanesPerRow;
    const bool row_ok = h < p.QH;
    const int hr = row_ok ? h : p.QH - 1;  // lanes past the last row follow along on the last one and store nothing
    const int sub = lane % kLanesPerRow;

    // partition j-1 holds the tile before the boundary, a tile of b: its piece exists and stands
    // in (with weight 0) for partitions of the walk that have no tiles
    const int lo_first = part_begin(j - 1, T, P);
    const int64_t safe = (int64_t)(2 * (j - 1) + (lo_first != cum ? 1 : 0)) * p.QH + hr;

    float4 acc[V4];
#pragma unroll
    for (int i = 0; i < V4; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float wsum = 0.f, m = kNegBig;
    for (int kk0 = j - 1; kk0 < P; kk0 += 4) {
        if (part_begin(kk0, T, P) >= end_b) break;  // past the sequence's last tile
        float lse[4];
        float4 x[4][V4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int kk = kk0 + u;
            ok[u] = false;
            int64_t r = safe;
            if (kk < P) {
                const int lo = part_begin(kk, T, P), hi = part_begin(kk + 1, T, P);
                ok[u] = hi > lo && lo < end_b && hi > cum;
                if (ok[u]) r = (int64_t)(2 * kk + ((kk == j - 1 && lo != cum) ? 1 : 0)) * p.QH + hr;
            }
            lse[u] = p.part_lse[r];
            const float4* src = reinterpret_cast<const float4*>(p.part_o + r * D) + sub * V4;
#pragma unroll
            for (int i = 0; i < V4; ++i) x[u][i] = src[i];
        }
        float cm = kNegBig;
#pragma unroll
        for (int u = 0; u < 4; ++u) cm = ok[u] ? fmaxf(cm, lse[u]) : cm;
        const float m_new = fmaxf(m, cm);
        const float rescale = fast_exp2(m - m_new);
        wsum *= rescale;
#pragma unroll
        for (int i = 0; i < V4; ++i) {
            acc[i].x *= rescale;
            acc[i].y *= rescale;
            acc[i].z *= rescale;
            acc[i].w *= rescale;
        }
        m = m_new;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = ok[u] ? fast_exp2(lse[u] - m_new) : 0.f;
            wsum += w;
#pragma unroll
            for (int i = 0; i < V4; ++i) {
                acc[i].x = fmaf(w, x[u][i].x, acc[i].x);
                acc[i].y = fmaf(w, x[u][i].y, acc[i].y);
                acc[i].z = fmaf(w, x[u][i].z, acc[i].z);
                acc[i].w = fmaf(w, x[u][i].w, acc[i].w);
            }
        }
    }
    if (!row_ok) return;
    const float inv = 1.f / wsum;
    const int64_t row = ((int64_t)b * p.QH + h) * D + sub * (4 * V4);
#pragma unroll
    for (int i = 0; i < V4; ++i)
        store_out4(p, row + 4 * i, acc[i].x * inv, acc[i].y * inv, acc[i].z * inv, acc[i].w * inv);
}

// ---------------------------------------------------------------------------------------------
// Rows with many pieces: a workgroup of kMergeWaves wavefronts per output row.
//
// combine_pieces() combines, by their log-sum-exps, `nsrc` pieces of one output row and stores
// the row.  piece(s, row_ptr, lse) describes piece s (false: it does not exist).  The pieces are
// taken 256 at a time: thread t looks at piece t (address, log-sum-exp), the workgroup agrees on
// the maximum and the weights, then wave w sums pieces w, w+4, ... with eight row loads in
// flight, and the four sums are added through LDS.  `safe_row` is any row that is certainly
// written (it stands in, with weight 0, for pieces that do not exist).
constexpr int kMergeWaves = 4;

template <int D, class Piece>
__device__ __forceinline__ void combine_pieces(const Params& p, int64_t out_elem, int nsrc, const float* safe_row,
                                               Piece piece)
{
    constexpr int V = D / kWave;
    constexpr int NT = kMergeWaves * kWave;
    __shared__ const float* s_row[NT];
    __shared__ float s_w[NT];
    __shared__ float s_red[2][kMergeWaves];
    __shared__ float s_acc[kMergeWaves][D];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid >> 6;

    float acc[V], wsum = 0.f, mrun = kNegBig;
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;

    for (int base = 0; base < nsrc; base += NT) {
        const int s = base + tid;
        const float* src = safe_row;
        float lse = kNegBig;
        const bool valid = s < nsrc && piece(s, src, lse);
        if (!valid) {
            src = safe_row;
            lse = kNegBig;
        }
        // workgroup-wide maximum of the log-sum-exps
        float cm = lse;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) cm = fmaxf(cm, __shfl_xor(cm, o, kWave));
        if (lane == 0) s_red[0][w] = cm;
        __syncthreads();
        cm = fmaxf(fmaxf(s_red[0][0], s_red[0][1]), fmaxf(s_red[0][2], s_red[0][3]));
        const float m_new = fmaxf(mrun, cm);
        const float rescale = fast_exp2(mrun - m_new);
        const float wt = valid ? fast_exp2(lse - m_new) : 0.f;
        float ws = wt;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) ws += __shfl_xor(ws, o, kWave);
        if (lane == 0) s_red[1][w] = ws;
        s_row[tid] = src;
        s_w[tid] = wt;
        __syncthreads();
        wsum = wsum * rescale + (s_red[1][0] + s_red[1][1]) + (s_red[1][2] + s_red[1][3]);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] *= rescale;
        mrun = m_new;

        // wave w sums pieces w, w + 4, ... of this batch, eight row loads in flight
        const int cnt = min(NT, nsrc - base);
        const int mine = cnt > w ? (cnt - w + kMergeWaves - 1) / kMergeWaves : 0;
        for (int i0 = 0; i0 < mine; i0 += 8) {
            float wv[8];
            float2 xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = w + kMergeWaves * min(i0 + u, mine - 1);
                wv[u] = (i0 + u < mine) ? s_w[idx] : 0.f;
                const float* r = s_row[idx];
                if (V == 2) {
                    xv[u] = *reinterpret_cast<const float2*>(r + lane * 2);
                } else {
                    xv[u].x = r[lane];
                    xv[u].y = 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc[0] = fmaf(wv[u], xv[u].x, acc[0]);
                if (V == 2) acc[V - 1] = fmaf(wv[u], xv[u].y, acc[V - 1]);
            }
        }
        __syncthreads();  // s_row / s_w / s_red are reused by the next batch
    }
    // add the four waves' sums
#pragma unroll
    for (int i = 0; i < V; ++i) s_acc[w][lane * V + i] = acc[i];
    __syncthreads();
    if (w == 0) {
        const float inv = 1.f / wsum;
        float o[V];
#pragma unroll
        for (int i = 0; i < V; ++i)
            o[i] = ((s_acc[0][lane * V + i] + s_acc[1][lane * V + i]) + (s_acc[2][lane * V + i] + s_acc[3][lane * V + i])) * inv;
        if (V == 2)
            store_out2(p, out_elem + lane * 2, o[0], o[V - 1]);
        else
            store_out1(p, out_elem + lane, o[0]);
    }
}

// The merge of merge_kernel above for calls whose sequences are cut many times (few sequences,
// many partitions: a single long context is cut by every partition): same descriptors, same
// slots, but a workgroup per (sequence, output row) that splits the pieces over its waves.
template <int D>
__global__ __launch_bounds__(kMergeWaves * kWave) void merge_many_kernel(const Params p)
{
    const int h = blockIdx.x;
    const int P = p.P;
    const int b = slot_sequence(p, blockIdx.y, threadIdx.x & (kWave - 1));
    if (b < 0) return;  // fewer sequences were cut than the grid has room for (the same for every thread)
    const int j = uniform_load(p.merge_desc, 4 * (int64_t)b);
    const int cum = uniform_load(p.merge_desc, 4 * (int64_t)b + 1), end_b = uniform_load(p.merge_desc, 4 * (int64_t)b + 2),
              T = uniform_load(p.merge_desc, 4 * (int64_t)b + 3);
    const int k_last = part_of(end_b - 1, T, P);
    const int nsrc = k_last - (j - 1) + 1;
    // partition j-1 holds the tile before the boundary, a tile of b: its piece exists
    const int lo_first = part_begin(j - 1, T, P);
    const float* safe_row = p.part_o + ((int64_t)(2 * (j - 1) + (lo_first != cum ? 1 : 0)) * p.QH + h) * D;
    combine_pieces<D>(p, ((int64_t)b * p.QH + h) * D, nsrc, safe_row, [&](int s, const float*& src, float& lse) {
        const int kk = j - 1 + s;
        const int lo = part_begin(kk, T, P), hi = part_begin(kk + 1, T, P);
        if (hi <= lo) return false;  // partitions without tiles wrote nothing
        const int64_t slot = (int64_t)(2 * kk + ((kk == j - 1 && lo != cum) ? 1 : 0)) * p.QH + h;
        src = p.part_o + slot * D;
        lse = p.part_lse[slot];
        return true;
    });
}

// Merge kernel of shared-prefix calls.  One workgroup per (output row h of a sequence, sequence b) combines
// every piece of that output row:
//   - the Pp partials of the prefix pass (slot kp of prefix_o / prefix_lse), and
//   - what the per-sequence pass produced over the rest of the context: nothing (the context ends
//     with the prefix), or the row in seq_o with its log-sum-exp in seq_lse (the rest lies
//     inside one partition), or the partials of the partitions that cut it (slots as above).
template <int D>
__global__ __launch_bounds__(kMergeWaves * kWave) void merge_prefix_kernel(const Params p)
{
    const int h = blockIdx.x;
    const int b = blockIdx.y;
    const Span sp{p.skip_tiles, 0};
    const int P = p.P;
    const int64_t rows = (int64_t)p.B * p.QH;
    const int64_t row = (int64_t)b * p.QH + h;

    // The sequence's own tiles (those after the prefix): none (the context ends with the prefix), or
    // what the per-sequence pass noted about them (write_seq_desc: j = 0, they lie inside one
    // partition and the row waits in seq_o; else j is the first boundary inside them, cum and end
    // their place in the global sequence of own tiles).  With a single partition nothing is noted
    // and nothing is cut.
    const int nb = tiles_of(uniform_load(p.context_lens, b), sp);
    int k_first = 0, nrest = 0, cum = 0, T = 0;
    bool inside_one = false;
    if (nb > 0) {
        const int j = p.merge_desc != nullptr ? uniform_load(p.merge_desc, 4 * (int64_t)b) : 0;
        inside_one = j == 0;
        nrest = 1;
        if (!inside_one) {
            cum = uniform_load(p.merge_desc, 4 * (int64_t)b + 1);
            const int end_b = uniform_load(p.merge_desc, 4 * (int64_t)b + 2);
            T = uniform_load(p.merge_desc, 4 * (int64_t)b + 3);
            k_first = j - 1;
            nrest = part_of(end_b - 1, T, P) - k_first + 1;
        }
    }
    // prefix range 0 of this row is always written and finite
    combine_pieces<D>(p, row * D, p.Pp + nrest, p.prefix_o + row * D, [&](int s, const float*& src, float& lse) {
        if (s < p.Pp) {
            src = p.prefix_o + ((int64_t)s * rows + row) * D;
            lse = p.prefix_lse[(int64_t)s * rows + row];
            return true;
        }
        if (inside_one) {
            src = p.seq_o + row * D;
            lse = p.seq_lse[row];
            return true;
        }
        const int kk = k_first + (s - p.Pp);
        const int lo = part_begin(kk, T, P), hi = part_begin(kk + 1, T, P);
        if (hi <= lo) return false;  // partitions without tiles wrote nothing
        const int64_t slot = (int64_t)(2 * kk + ((kk == k_first && lo != cum) ? 1 : 0)) * p.QH + h;
        src = p.part_o + slot * D;
        lse = p.part_lse[slot];
        return true;
    });
}

}  // namespace pa
