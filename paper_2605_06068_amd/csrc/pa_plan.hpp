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

// Which tiles of a sequence the plan covers.  `skip` leading tiles belong to someone else (a prefix
// shared by the whole batch, handled by a pass of its own).  `reach` > 0 bounds how far back from
// the end of the context any query of the call can see (sliding window: window + q_len - 1
// tokens); tiles that lie entirely before that are left out as well, and their blocks may be gone.
struct Span {
    int skip;
    int reach;
};

// first tile of a context of L tokens that the plan covers
__host__ __device__ __forceinline__ int first_tile(int L, Span sp)
{
    const int w = (sp.reach > 0 && L > sp.reach) ? (L - sp.reach) / kTileTokens : 0;
    return w > sp.skip ? w : sp.skip;
}

// number of tiles it covers
__host__ __device__ __forceinline__ int tiles_of(int L, Span sp = Span{0, 0})
{
    const int n = L > 0 ? (L + kTileTokens - 1) / kTileTokens : 0;
    const int f = first_tile(L, sp);
    return n > f ? n - f : 0;
}

// first global tile of partition k
__host__ __device__ __forceinline__ int part_begin(int k, int T, int P) { return (int)(((int64_t)k * T) / P); }

// the partition that owns global tile t: the largest k with part_begin(k) <= t
__host__ __device__ __forceinline__ int part_of(int t, int T, int P) { return (int)((((int64_t)t + 1) * P - 1) / T); }

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
__device__ __forceinline__ int total_tiles(const int32_t* context_lens, int B, int lane, Span sp = Span{0, 0})
{
    int sum = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        sum += b < B ? tiles_of(context_lens[b], sp) : 0;
    }
    return wave_sum(sum);
}

// The sequence that contains global tile t (0 <= t < T) and the number of tiles before it.
// All 64 lanes must call; results are wave-uniform.
__device__ __forceinline__ void locate_tile(const int32_t* context_lens, int B, int t, int lane, int& b_out, int& cum_out,
                                            Span sp = Span{0, 0})
{
    int carry = 0;
    b_out = B - 1;
    cum_out = 0;
    for (int b0 = 0; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        const int n = b < B ? tiles_of(context_lens[b], sp) : 0;
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

// Where partition k of P starts: total tile count T, the partition's global tile range
// [t_lo, t_hi), and whenever t_lo < T (every non-empty range, and the empty ones that lie between
// two tiles: there are some as soon as the call has fewer tiles than partitions) the sequence b
// that holds tile t_lo, the number of tiles before b and b's context length.  All 64 lanes must
// call; results are wave-uniform.
// A batch of up to 64 sequences needs a single load of the context lengths.
struct RangeStart {
    int T, t_lo, t_hi, b, cum, L;
};

__device__ __forceinline__ RangeStart find_range(const int32_t* context_lens, int B, int k, int P, int lane, Span sp = Span{0, 0})
{
    RangeStart r;
    r.b = 0;
    r.cum = 0;
    r.L = 0;
    if (B <= kWave) {
        const int L = lane < B ? context_lens[lane] : 0;
        const int n = tiles_of(L, sp);
        const int incl = wave_inclusive_scan(n, lane);
        r.T = __builtin_amdgcn_readlane(incl, kWave - 1);
        r.t_lo = part_begin(k, r.T, P);
        r.t_hi = part_begin(k + 1, r.T, P);
        if (r.t_lo < r.T) {
            const unsigned long long hit = __ballot(incl > r.t_lo);
            const int l = __ffsll((long long)hit) - 1;
            r.b = l;
            r.cum = __builtin_amdgcn_readlane(incl - n, l);
            r.L = __builtin_amdgcn_readlane(L, l);
        }
        return r;
    }
    // First pass: the total, and on the way the running total at the end of every group of 16 chunks
    // (1024 sequences), kept by lane `group` (a batch has at most 64 groups).  Second pass: only the
    // group that holds tile t_lo is searched chunk by chunk.
    constexpr int kGroupChunks = 16;
    int sum = 0, running = 0, group_end = 0;
    const int nchunks = (B + kWave - 1) / kWave;
    for (int c0 = 0; c0 < nchunks; c0 += kGroupChunks) {
        const int c1 = min(c0 + kGroupChunks, nchunks);
#pragma unroll 4
        for (int c = c0; c < c1; ++c) {  // independent loads: several in flight
            const int b = c * kWave + lane;
            sum += b < B ? tiles_of(context_lens[b], sp) : 0;
        }
        running += wave_sum(sum);
        sum = 0;
        if (lane == c0 / kGroupChunks) group_end = running;
    }
    r.T = __builtin_amdgcn_readfirstlane(running);
    r.t_lo = part_begin(k, r.T, P);
    r.t_hi = part_begin(k + 1, r.T, P);
    if (r.t_lo >= r.T) return r;
    const int ngroups = (nchunks + kGroupChunks - 1) / kGroupChunks;
    const unsigned long long in_group = __ballot(lane < ngroups && group_end > r.t_lo);
    const int group = __ffsll((long long)in_group) - 1;  // exists: t_lo < T
    int carry = group > 0 ? __shfl(group_end, group - 1, kWave) : 0;
    for (int b0 = group * kGroupChunks * kWave; b0 < B; b0 += kWave) {
        const int b = b0 + lane;
        const int L = b < B ? context_lens[b] : 0;
        const int n = tiles_of(L, sp);
        const int incl = wave_inclusive_scan(n, lane) + carry;
        const unsigned long long hit = __ballot(incl > r.t_lo);
        if (hit != 0ull) {
            const int l = __ffsll((long long)hit) - 1;
            r.b = b0 + l;
            r.cum = __builtin_amdgcn_readlane(incl - n, l);
            r.L = __builtin_amdgcn_readlane(L, l);
            break;
        }
        carry = __builtin_amdgcn_readlane(incl, kWave - 1);
    }
    return r;
}

// What the merge kernel needs to know about sequence b, written by the partition kernel so that
// the merge neither scans the context lengths nor searches for boundaries: {j, cum, end, T}.
// j = 0: nothing to merge (the sequence is empty, or lies inside one partition).  Otherwise j is
// the first partition boundary strictly inside the sequence (the start of partition j), cum and
// end are the sequence's first tile and last tile + 1 in the global tile sequence, T the total.
// The writer is the wave (KV head 0) that processes the sequence's FIRST tile: it is the one that
// sees whether the sequence runs past the end of its own range.  Empty sequences are covered by
// the wave that zero-fills their output rows.
__device__ __forceinline__ void write_seq_desc(int32_t* desc, int b, int j, int cum, int end, int T)
{
    int4 d;
    d.x = j;
    d.y = cum;
    d.z = end;
    d.w = T;
    *reinterpret_cast<int4*>(desc + 4 * (int64_t)b) = d;
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
