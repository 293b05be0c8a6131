// Device-side helpers shared by the partition and merge kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pa {

constexpr int kWave = 64;
constexpr int kBlockSize = 16;          // tokens per KV block (the only block size supported)
constexpr float kNegBig = -1.0e30f;     // "minus infinity" that stays finite under subtraction
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

enum : int { KV_BF16 = 0, KV_FP8 = 1 };

// Everything a launch needs.  Pointers are device memory.
struct Params {
    const uint16_t* q;            // [B, Hq, D] bf16
    const void* k_cache;          // [NB, Hkv, 16, D]
    const void* v_cache;
    const int32_t* block_tables;  // [B, MB]
    const int32_t* context_lens;  // [B]
    const float* k_scale;         // [Hkv] or null
    const float* v_scale;
    float* out;                   // [B, Hq, D] float32, or the same shape in bf16 when out_bf16 is set
    float* part_o;                // [2P, Hq, D] normalised partial outputs (null when P == 1)
    float* part_lse;              // [2P, Hq]    log2-domain log-sum-exp of each partial
    int32_t* merge_desc;          // [B, 4] what the merge kernel needs to know per sequence (null when P == 1)
    int32_t* cut_list;            // [P] the sequence inside which partition k starts (empty partitions included), or -1 (null: the merge scans merge_desc instead)
    int32_t* trace_blocks;        // [B, Hkv, MB, 3] or null
    float scale_log2;             // softmax scale * log2(e)
    int32_t B, Hq, Hkv, G, MB;
    int32_t num_blocks;           // blocks in the pool: instrumented runs hold every id against it
    int32_t Q;                    // query tokens per sequence (1 = plain decode)
    int32_t QH;                   // Q * Hq: output rows per sequence (q, out and the partials are [.., Q, Hq, D])
    int32_t P;                    // number of partitions of the global tile sequence
    int32_t out_bf16;             // final rows are stored as bf16 (round to nearest even) instead of float32
    int32_t window;               // sliding window: a query at position t sees tokens t-window+1 .. t (0: everything before it)
    // shared-prefix calls only (skip_tiles > 0): the first skip_tiles tiles of every sequence are one
    // and the same physical blocks; a pass of its own reads them once for all sequences
    int32_t skip_tiles;           // tiles of the shared prefix (0: no shared prefix)
    int32_t Pp;                   // partitions of the prefix tiles
    float* seq_o;                 // [B, QH, D] rows the per-sequence pass finished inside one partition: they still lack the prefix part
    float* seq_lse;               // [B, QH]    their log-sum-exps
    float* prefix_o;              // [Pp, B*QH, D] normalised partial outputs over the prefix
    float* prefix_lse;            // [Pp, B*QH]
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// OCP e4m3 byte -> float, by bit manipulation (exact; NaN bytes are never read from valid slots).
__device__ __forceinline__ float e4m3_to_f32(uint32_t byte)
{
    const uint32_t sign = (byte & 0x80u) << 24;
    const uint32_t mag = byte & 0x7fu;
    // normal numbers: move exponent/mantissa into place and rebias (127 - 7 = 120)
    float r = __uint_as_float((mag << 20) + (120u << 23));
    // subnormals (exponent field 0): value = mant * 2^-9
    if (mag < 8u) r = (float)mag * 0.001953125f;
    return __uint_as_float(__float_as_uint(r) | sign);
}

// DPP moves inside rows of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16

// Sum over aligned groups of LANES lanes (8 or 16); every lane of the group gets the total.
template <int LANES>
__device__ __forceinline__ float group_sum(float v)
{
    v += dpp_f<kDppXor1>(v);
    v += dpp_f<kDppXor2>(v);
    v += dpp_f<kDppHalfMirror>(v);
    if (LANES == 16) v += dpp_f<kDppMirror>(v);
    return v;
}

// Reductions over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48) with gfx950's
// row-swapping permutes: permlane16_swap(x, x) returns {rows 0,0,2,2 ; rows 1,1,3,3} of x and
// permlane32_swap(x, x) returns {rows 0,1,0,1 ; rows 2,3,2,3}, so each step is one swap and
// one VALU op instead of a round trip through the LDS crossbar.  Every lane gets the result.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float rows_max(float v)
{
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float rows_sum(float v)
{
    u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Stores of FINAL output rows (partials in the workspace are always float32).  `elem` is the
// element index inside `out`, whatever its type.
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void store_out4(const Params& p, int64_t elem, float a, float b, float c, float d)
{
    if (p.out_bf16)
        *reinterpret_cast<bf16x4_t*>(reinterpret_cast<uint16_t*>(p.out) + elem) =
            bf16x4_t{(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    else
        *reinterpret_cast<float4*>(p.out + elem) = make_float4(a, b, c, d);
}

__device__ __forceinline__ void store_out2(const Params& p, int64_t elem, float a, float b)
{
    if (p.out_bf16)
        *reinterpret_cast<bf16x2_t*>(reinterpret_cast<uint16_t*>(p.out) + elem) = bf16x2_t{(__bf16)a, (__bf16)b};
    else
        *reinterpret_cast<float2*>(p.out + elem) = make_float2(a, b);
}

__device__ __forceinline__ void store_out1(const Params& p, int64_t elem, float a)
{
    if (p.out_bf16)
        reinterpret_cast<__bf16*>(p.out)[elem] = (__bf16)a;
    else
        p.out[elem] = a;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

}  // namespace pa
