// KV append: stores the key and value rows of the Q tokens added in this step (Q = 1: the token
// just generated; Q > 1: a window of proposed tokens about to be verified) into the paged cache,
// at logical positions context_lens[b] - Q .. context_lens[b] - 1 of every sequence (the lengths
// already count the new tokens), quantising to e4m3 with the KV head's scale when the cache is
// fp8.  One thread per 8 consecutive elements of one (sequence, token, KV head) row.
#pragma once
#include "pa_device.hpp"

namespace pa {

// two floats -> two e4m3 bytes (round to nearest even, saturating at +-448), packed in the low 16 bits
__device__ __forceinline__ uint32_t e4m3_pair(float a, float b)
{
    a = a > 448.f ? 448.f : (a < -448.f ? -448.f : a);
    b = b > 448.f ? 448.f : (b < -448.f ? -448.f : b);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

template <int D, int KV>
__global__ __launch_bounds__(256) void kv_append_kernel(const uint16_t* __restrict__ k_new,
                                                         const uint16_t* __restrict__ v_new, void* k_cache,
                                                         void* v_cache, const int32_t* __restrict__ block_tables,
                                                         const int32_t* __restrict__ context_lens,
                                                         const float* __restrict__ k_scale,
                                                         const float* __restrict__ v_scale, int B, int Q, int Hkv,
                                                         int MB)
{
    constexpr int CH = D / 8;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)B * Q * Hkv * CH) return;
    const int c = (int)(i % CH);
    const int g = (int)((i / CH) % Hkv);
    const int tok = (int)((i / ((int64_t)CH * Hkv)) % Q);
    const int b = (int)(i / ((int64_t)CH * Hkv * Q));
    const int t = context_lens[b] - Q + tok;
    if (t < 0) return;  // an empty sequence, or a window that starts before the sequence does
    const int64_t phys = block_tables[(int64_t)b * MB + t / kBlockSize];
    const int64_t dst = ((phys * Hkv + g) * kBlockSize + t % kBlockSize) * D + c * 8;
    const int64_t src = (((int64_t)b * Q + tok) * Hkv + g) * D + c * 8;
    const uint4 kw = *reinterpret_cast<const uint4*>(k_new + src);
    const uint4 vw = *reinterpret_cast<const uint4*>(v_new + src);
    if (KV == KV_BF16) {
        *reinterpret_cast<uint4*>(static_cast<uint16_t*>(k_cache) + dst) = kw;
        *reinterpret_cast<uint4*>(static_cast<uint16_t*>(v_cache) + dst) = vw;
    } else {
        const float ks = k_scale[g], vs = v_scale[g];
        uint2 ko, vo;
        ko.x = e4m3_pair(bf16_lo(kw.x) / ks, bf16_hi(kw.x) / ks) | (e4m3_pair(bf16_lo(kw.y) / ks, bf16_hi(kw.y) / ks) << 16);
        ko.y = e4m3_pair(bf16_lo(kw.z) / ks, bf16_hi(kw.z) / ks) | (e4m3_pair(bf16_lo(kw.w) / ks, bf16_hi(kw.w) / ks) << 16);
        vo.x = e4m3_pair(bf16_lo(vw.x) / vs, bf16_hi(vw.x) / vs) | (e4m3_pair(bf16_lo(vw.y) / vs, bf16_hi(vw.y) / vs) << 16);
        vo.y = e4m3_pair(bf16_lo(vw.z) / vs, bf16_hi(vw.z) / vs) | (e4m3_pair(bf16_lo(vw.w) / vs, bf16_hi(vw.w) / vs) << 16);
        *reinterpret_cast<uint2*>(static_cast<uint8_t*>(k_cache) + dst) = ko;
        *reinterpret_cast<uint2*>(static_cast<uint8_t*>(v_cache) + dst) = vo;
    }
}

}  // namespace pa
