// The work partition of one decode call ("split plan"), shared by the partition and merge
// kernels and by the host-side pa_split_plan().
//
// The context of sequence b is cut into tiles of 32 tokens (two KV blocks):
//     tiles_b = ceil(L_b / 32)  (0 for L_b <= 0),   T = sum_b tiles_b,   cum_b = sum_{b' < b} tiles_b'.
// Concatenating the sequences' tiles in batch order gives one global tile sequence [0, T).
// It is cut into P contiguous, balanced ranges: partition k owns global tiles
//     [ floor(k*T/P), floor((k+1)*T/P) ).
// P depends on the host-known shape and the device only; the cut points depend on the
// device-resident context lengths and are therefore computed on the device by every wave.
// One wavefront per (partition, KV head) walks its range; each maximal run of tiles of one
// sequence inside a range is a *segment*.  A segment that covers its whole sequence is written
// straight to `out`; otherwise it leaves a partial (normalised output + log-sum-exp) that the
// merge kernel combines.  A partition has at most two such partials: slot 2k for the segment
// of the sequence that contains the partition's first tile, slot 2k+1 for any other (which can
// only be its last one).
#pragma once
#include "pa_device.hpp"

namespace pa {

constexpr int kTileTokens = 32;

__host__ __device__ __forceinline__ int tiles_of(int L) { return L > 0 ? (L + kTileTokens - 1) / kTileTokens : 0; }

// first global tile of partition k
__host__ __device__ __forceinline__ int part_begin(int k, int T, int P) { return (int)(((int64_t)k * T) / P); }

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(v, o, kWave);
        if (lane >= o) v += u;
    }
    return v;
}

// Total number of tiles of the batch.  All 64 lanes must call.
__device__ __forceinline__ int total_tiles(const int32_t* context_lens, int B, int lane)
{
    int sum = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        sum += b < B ? tiles_of(context_lens[b]) : 0;
    }
    return wave_sum(sum);
}

// The sequence that contains global tile t (0 <= t < T) and the number of tiles before it.
// All 64 lanes must call; results are wave-uniform.
__device__ __forceinline__ void locate_tile(const int32_t* context_lens, int B, int t, int lane, int& b_out, int& cum_out)
{
    int carry = 0;
    b_out = B - 1;
    cum_out = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        const int n = b < B ? tiles_of(context_lens[b]) : 0;
        const int incl = wave_inclusive_scan(n, lane) + carry;
        const unsigned long long hit = __ballot(incl > t);
        if (hit != 0ull) {
            const int l = __ffsll((long long)hit) - 1;
            b_out = b0 + l;
            cum_out = __shfl(incl - n, l, kWave);
            return;
        }
        carry = __shfl(incl, kWave - 1, kWave);
    }
}

// Uniform (scalar-cache) load of a 32-bit word: keeps table and length lookups off the
// vector-memory counter that the hand-scheduled LDS-DMA ring relies on.
__device__ __forceinline__ int32_t uniform_load(const int32_t* p, int64_t idx)
{
    typedef __attribute__((address_space(4))) const int32_t cint;
    cint* cp = (cint*)(p);
    return cp[idx];
}

}  // namespace pa
