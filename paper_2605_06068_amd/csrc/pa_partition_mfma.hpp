// Partition kernel, matrix-core variant (head_dim 128): for query-head groups wide enough to
// form a matrix tile (4 <= G <= 16; the group is padded to the 16 columns of an MFMA tile).
// One wavefront per (sequence, KV head, split); no workgroup barriers.
//
// Data path per 32-token tile (two KV blocks):
//   HBM --global_load_lds (16 B/lane, 1 KB per instruction)--> LDS ring of NSTAGE tiles
//   K:  ds_read_b128 in MFMA operand layout -> S^T[token, head] = K . Q^T   (mfma 16x16x32 bf16)
//   online softmax on S^T in registers (lane = head column, 8 tokens per lane per tile)
//   V:  ds_read_b64_tr_b16 (transposing LDS read) -> out^T[dim, head] += V^T . P^T
//
// LDS tile layout: row t (one token, 256 B) at byte t*256; the 16-byte piece holding dims
// [8c, 8c+8) sits at piece position c ^ (t & 15).  The XOR swizzle is applied on the *global*
// side of the LDS-DMA load (the LDS side of such a load is always lane-linear), which keeps
// every 16-lane group on one contiguous 256-byte row, and makes both the operand reads (16
// different rows per 16 lanes) and the transposing reads bank-conflict free.
//
// The P^T operand needs no data movement: the score tile comes out of the MFMA with lane l
// holding head l%16 and tokens 4*(l/16)+{0..3}; declaring MFMA k-index 8*(l/16)+e to mean token
// 4*(l/16)+e of the first block (e<4) or of the second block (e>=4) makes the score registers,
// once exponentiated and packed to bf16, the B operand of the PV product as they stand.  The
// V^T operand is read with the same k-index convention.
#pragma once
#include "pa_device.hpp"

namespace pa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

constexpr int kTileTokens = 32;
constexpr int kRowBytes = 256;    // 128 bf16
constexpr int kSlabBytes = 4096;  // one (block, head): 16 rows
constexpr int kStageBytes = 4 * kSlabBytes;  // K block 0, K block 1, V block 0, V block 1
constexpr int kDmaPerTile = 16;   // 1 KB each

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

// wait until at most `later_tiles` whole tiles plus EXTRA loads are still in flight
template <int EXTRA, int NSTAGE>
__device__ __forceinline__ void wait_tile(int later_tiles)
{
    if (NSTAGE >= 4 && later_tiles >= 3) wait_vmcnt<3 * kDmaPerTile + EXTRA>();
    else if (NSTAGE >= 3 && later_tiles == 2) wait_vmcnt<2 * kDmaPerTile + EXTRA>();
    else if (later_tiles == 1) wait_vmcnt<1 * kDmaPerTile + EXTRA>();
    else wait_vmcnt<EXTRA>();
}

// The LDS-DMA loads above are issued and awaited by hand, invisibly to the compiler's own
// wait-count bookkeeping.  An ordinary load whose result is first used inside the tile loop
// would make the compiler wait there for *all* outstanding vector-memory operations, i.e.
// drain the ring every iteration.  Passing the loaded register through an empty asm makes the
// compiler complete the load at this point instead.
template <typename T>
__device__ __forceinline__ void settle(T& v)
{
    asm volatile("" : "+v"(v));
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int NSTAGE, bool TRACE>
__global__ __launch_bounds__(64) void partition_mfma_kernel(const Params p)
{
    constexpr int D = 128;
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring depth");
    __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * kStageBytes];

    const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int L = p.context_lens[b];
    const int start = s * p.C;
    const int lane = threadIdx.x;
    const int G = p.G;
    if (L <= 0 && s == 0) {  // empty context: the output rows of this group are zero
        for (int i = lane; i < G * D; i += kWave) p.out[((int64_t)b * p.Hq + g * G) * D + i] = 0.f;
    }
    if (start >= L) return;
    const int end = min(start + p.C, L);
    const int n = lane & 15;   // head column / row-in-block, depending on the operand
    const int q4 = lane >> 4;  // 0..3

    if (TRACE && lane == 0) {
        int32_t* r = p.trace_ranges + (((int64_t)b * p.Hkv + g) * p.S + s) * 2;
        r[0] = start;
        r[1] = end;
    }

    // ---- per-lane address pieces
    uint32_t dma_off[4];  // global byte offset inside a slab for DMA instruction i (rows 4i..4i+3)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = 4 * i + q4;
        dma_off[i] = t * kRowBytes + ((n ^ t) << 4);
    }
    uint32_t kread[4];  // LDS byte offset inside a slab of this lane's K operand piece for k-step kk
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kread[kk] = n * kRowBytes + (((4 * kk + q4) ^ n) << 4);
    uint32_t vread[8];  // LDS byte offset inside a slab of this lane's transposing-read source for dim tile dt
    {
        const int row = 4 * q4 + (n >> 2);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            vread[dt] = row * kRowBytes + ((n & 1) << 3) + (((2 * dt + ((n >> 1) & 1)) ^ row) << 4);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    // ---- Q^T operand: head n of the group (zero for padding columns), dims 32kk + 8*q4 + [0,8)
    bf16x8 qreg[4];
    {
        const uint16_t* qrow = p.q + ((int64_t)b * p.Hq + g * G + (n < G ? n : 0)) * D + 8 * q4;
        uint4 w[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) w[kk] = *reinterpret_cast<const uint4*>(qrow + 32 * kk);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (n >= G) w[kk] = make_uint4(0, 0, 0, 0);
            settle(w[kk].x); settle(w[kk].y); settle(w[kk].z); settle(w[kk].w);
            qreg[kk] = as_bf16x8(w[kk]);
        }
    }

    // ---- block table of this split, 64 entries at a time, one per lane
    const int32_t* table = p.block_tables + (int64_t)b * p.MB;
    const int jb = start / kBlockSize;
    const int nblk = (end + kBlockSize - 1) / kBlockSize - jb;
    const int ntiles = (nblk + 1) / 2;
    int tbl = (lane < nblk) ? table[jb + lane] : 0;
    settle(tbl);
    int phys0 = 0;

    const int64_t head_stride = (int64_t)p.Hkv * kSlabBytes;  // bytes between physical blocks
    const char* kc = static_cast<const char*>(p.k_cache) + (int64_t)g * kSlabBytes;
    const char* vc = static_cast<const char*>(p.v_cache) + (int64_t)g * kSlabBytes;

    auto issue = [&](int tile, int stage) {
        if (tile > 0 && (tile & 31) == 0) {  // next 64 table entries
            const int base = 2 * tile;
            tbl = (base + lane < nblk) ? table[jb + base + lane] : 0;
            settle(tbl);
        }
        const uint32_t ldst = lds0 + stage * kStageBytes;
        const char* kb[2];
        const char* vb[2];
        int nvalid[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int jj = 2 * tile + sub;
            int phys;
            if (jj < nblk) {
                phys = __builtin_amdgcn_readlane(tbl, jj & 63);
                nvalid[sub] = min(kBlockSize, end - (jb + jj) * kBlockSize);
                if (sub == 0) phys0 = phys;
                if (TRACE && lane == 0) {
                    int32_t* v = p.trace_blocks + (((int64_t)b * p.Hkv + g) * p.MB + jb + jj) * 2;
                    v[0] = phys;
                    v[1] = phys;
                }
            } else {  // block beyond the split: re-read row 0 of the tile's first block, masked later
                phys = phys0;
                nvalid[sub] = 1;
            }
            kb[sub] = kc + phys * head_stride;
            vb[sub] = vc + phys * head_stride;
        }
        // rows past the context hold garbage (possibly NaN patterns): load row 0 of the block instead
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t off = (4 * i + q4 < nvalid[sub]) ? dma_off[i] : (dma_off[i] & 255u);
                dma16(ldst + sub * kSlabBytes + i * 1024, off, kb[sub]);
            }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t off = (4 * i + q4 < nvalid[sub]) ? dma_off[i] : (dma_off[i] & 255u);
                dma16(ldst + 2 * kSlabBytes + sub * kSlabBytes + i * 1024, off, vb[sub]);
            }
    };

    // ---- online softmax state: lane = head n, tokens 4*q4+{0..3} of each block
    float qs = p.scale_log2;
    float m = kNegBig, lsum = 0.f;
    f32x4 acc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

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

        // ---- scores: S^T[token, head] for the two blocks of the tile
        wait_tile<kDmaPerTile / 2, NSTAGE>(later);
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 a0 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + kread[kk]));
            const bf16x8 a1 = as_bf16x8(*reinterpret_cast<const uint4*>(kbuf + kSlabBytes + kread[kk]));
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qreg[kk], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qreg[kk], s1, 0, 0, 0);
        }

        // ---- online softmax (log2 domain)
        const int t0 = start + tile * kTileTokens + 4 * q4;
        float x[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            x[r] = (t0 + r < end) ? s0[r] * qs : kNegBig;
            x[4 + r] = (t0 + kBlockSize + r < end) ? s1[r] * qs : kNegBig;
        }
        float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2(m - m_new);
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            x[r] = fast_exp2(x[r] - m_new);
            ps += x[r];
        }
        lsum = lsum * alpha + ps;
        m = m_new;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;
        }
        bf16x8 pb;
#pragma unroll
        for (int r = 0; r < 8; ++r) pb[r] = (__bf16)x[r];

        // ---- out^T[dim, head] += V^T . P^T
        wait_tile<0, NSTAGE>(later);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const i16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + vread[dt]));
            const i16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(vbuf + kSlabBytes + vread[dt]));
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb, acc[dt], 0, 0, 0);
        }
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }

    // ---- epilogue: finish the row sums, normalise, write
    lsum += __shfl_xor(lsum, 16, kWave);
    lsum += __shfl_xor(lsum, 32, kWave);
    if (n < G) {
        const float inv = 1.f / lsum;
        const int hq = g * G + n;
        float* dst;
        if (p.S == 1 || L <= p.C) {
            dst = p.out + ((int64_t)b * p.Hq + hq) * D;
        } else {
            dst = p.part_o + (((int64_t)b * p.Hq + hq) * p.S + s) * D;
            if (q4 == 0) p.part_lse[((int64_t)b * p.Hq + hq) * p.S + s] = m + fast_log2(lsum);
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            *reinterpret_cast<float4*>(dst + 16 * dt + 4 * q4) =
                make_float4(acc[dt][0] * inv, acc[dt][1] * inv, acc[dt][2] * inv, acc[dt][3] * inv);
    }
}

}  // namespace pa
