// Host side of libpa_decode.so: argument checks, the launch plan (a pure function of the
// host-known shape and the device's compute-unit count) and the kernel launches behind the C ABI
// declared in include/pa_decode.h.
#include "pa_decode.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>
#include <vector>

#include "pa_check_tables.hpp"
#include "pa_device.hpp"
#include "pa_kv_append.hpp"
#include "pa_merge.hpp"
#include "pa_partition_mfma.hpp"
#include "pa_partition_mfma_staged.hpp"
#include "pa_partition_mfma_wide.hpp"
#include "pa_plan.hpp"

// Scratch memory of pa_decode_static, the entry point for callers that cannot allocate: one array
// per GPU the library runs on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels get the device address that call returns.
#define PA_STATIC_SCRATCH_BYTES_IMPL (16u << 20)
static_assert(PA_STATIC_SCRATCH_BYTES_IMPL == PA_STATIC_SCRATCH_BYTES, "as the header states");
static __device__ __align__(256) unsigned char scratch[PA_STATIC_SCRATCH_BYTES_IMPL];

namespace {

using pa::Params;

// Up to here one wave per (partition, KV head), with one or two MFMA column tiles; above, a
// workgroup of waves.  Two column tiles per wave beat two waves with one tile each (8B-shaped
// batch, 5 / 8 query tokens: 118 / 125 us against 130 / 137 us; long-context batch, 8 tokens: 380
// against 427 us) except for fp8 at head_dim 128, where the second tile's arithmetic no longer
// hides behind the loads (70B-head-shaped batch, 4 tokens: 540 against 523 us).
constexpr int max_cols_one_wave(int d, int kv) { return (kv == PA_KV_FP8_E4M3 && d == 128) ? 16 : 32; }
constexpr int kMaxColsMfma = 128;  // columns of the widest workgroup: eight 16-column MFMA tiles
constexpr int kMaxColGroups = 4;   // workgroups side by side on one (partition, KV head), each reading the tiles for its own columns
constexpr int kMaxCols = kMaxColsMfma * kMaxColGroups;
constexpr int kMaxQueryLen = kMaxCols;  // with one query head per KV head; in general q_len * G <= kMaxCols
// Depth of the LDS tile ring of the one-wave kernel: two tiles for every head_dim and KV type.
// What pays is resident waves (head_dim 128: one per SIMD; head_dim 64, whose tiles are half the
// size: two), not deeper rings.  Measured: head_dim 64 fp8, 64 sequences of 1k-8k tokens: 2 tiles
// and 8 waves per compute unit 67 us, 8 tiles and 4 waves 85 us; head_dim 128 fp8 with 16 padded
// columns, where 4 tiles leave room for 3 waves only: 477 us against 381 us with 2 tiles.
constexpr int mfma_stages(int, int) { return 2; }
constexpr int mfma_waves_per_cu(int d) { return d == 128 ? 4 : 8; }
// ring depth of the multi-wave kernel (the ring is shared by the workgroup's waves), by KV type
// and the workgroup's columns (32, 64 or 128): with 128 columns 3 stages leave room for two
// workgroups per CU
constexpr int kWideStagesBf16[3] = {4, 4, 3};
constexpr int kWideStagesFp8[3] = {4, 4, 4};
constexpr int kWideStages64Bf16 = 4;  // head_dim 64: half the bytes per tile
constexpr int kWideStages64Fp8 = 6;
// resident waves per compute unit the multi-wave plan aims at, LDS permitting: two workgroups of
// up to 4 waves for bf16 (two of 8 waves in the prefix pass); three for fp8, whose smaller tiles
// leave the LDS for it (64 columns on the 70B-head-shaped fp8 batch: 710 -> 669 us per step)
constexpr int wide_waves_per_cu(int kv, int nw) { return kv == PA_KV_BF16 ? (nw == 8 ? 16 : 8) : 12; }
constexpr int kLdsPerCu = 160 * 1024;
constexpr int kDefaultCus = 256;   // MI355X; used when no device can be queried
constexpr int kMaxPartitions = 65535;
constexpr int kMaxBatch = 65535;
constexpr int kMinTilesOneWave = 2;  // tiles a partition should at least have: one-wave kernels
// ... and should have while that leaves every compute unit a wave (one request of 8k tokens, 32 / 64 query
// and 8 KV heads, 1 and 2 tokens: 15.8 / 16.6 / 16.8 / 19.4 us with 128 partitions, 14.4 / 14.7 / 14.8 / 16.2 with 64)
constexpr int kWantTilesOneWave = 4;
constexpr int kMinTilesWide = 4;     // multi-wave kernel
// stage-split kernel, while that leaves a workgroup for every compute unit (one request, 64 query / 8 KV
// heads, fp8 KV, 4 tokens: 16k tokens 28.6 -> 22.5 us with 32 instead of 128 partitions, 64k tokens
// 43.6 -> 40.4 us with 64; batches have more tiles than that either way)
constexpr int kMinTilesStaged = 32;
// tiles per partition from which one wave takes two column tiles: where the alternative is the
// two-wave multi-wave workgroup (head_dim 64), and where it is the stage-split workgroup of two
// score and two value waves (head_dim 128, bf16), which stays ahead for longer (one sequence, 64
// query / 8 KV heads, 4 tokens: 64k tokens = 16 tiles per partition 59.7 against 53.9 us; at 36
// tiles per partition, 8B-shaped batch, the two tie; at 156, long-context batch, 365.9 against 372.6)
constexpr int kMinTilesTwoColumnTiles = 16;
constexpr int kMinTilesTwoColumnTilesStaged = 48;
constexpr int kMergeManyPerSeq = 8;  // partitions per sequence from which the multi-wave merge kernel is used
// output rows per sequence from which a merge wave takes four rows (8B-shaped batch: 32 rows 6.7
// against 7.0 us, 128 rows 9.2 against 8.5 us, 256 rows 12.8 against 11.1 us, 512 rows 16.9 against 12.3 us)
constexpr int kMergeRowsFrom = 128;

struct Plan {
    int32_t P;          // partitions of the global tile sequence
    bool one_wave;      // the per-sequence pass runs on the one-wave kernel
    bool staged;        // ... on the stage-split kernel
    int32_t max_ctx;    // resolved max context length
    size_t lse_offset;  // byte offset of the lse array inside the workspace
    size_t desc_offset; // byte offset of the merge descriptors
    size_t cut_offset;  // byte offset of the list of sequences the partitions' starts cut
    size_t ws_bytes;
    // shared-prefix calls
    int32_t skip_tiles;       // tiles of the shared prefix (0: none)
    int32_t Pp;               // partitions of the prefix tiles
    int32_t prefix_waves;     // waves per workgroup of the prefix pass
    int32_t prefix_groups;    // column groups of the prefix pass (16 * prefix_waves columns each)
    size_t seq_o_offset, seq_lse_offset, prefix_o_offset, prefix_lse_offset;
};

int query_len(const pa_shape* s) { return s->q_len > 0 ? s->q_len : 1; }

// tiles (pairs of blocks) at the head of every block table that the whole batch shares and the prefix
// pass reads once.  Under a sliding window the promise goes unused: every sequence reads its own last
// window + Q - 1 tokens and nothing before them, so there is nothing left to share.
int shared_tiles(const pa_shape* s) { return s->window > 0 ? 0 : s->shared_prefix_blocks / 2; }

// columns of the score matrix per KV head: (query token, query head of the group) pairs
int columns(const pa_shape* s) { return query_len(s) * (s->num_q_heads / s->num_kv_heads); }

// Padded column count of the one-wave kernel for `cols` (query tokens x heads of a group) columns.
// Narrow groups are padded inside the 16-column tile: the kernel is bound by the KV traffic, and
// runs at the same speed for 1 column as for 16; 17..32 columns are two such tiles.
int mfma_col_pad(int cols) { return cols <= 4 ? 4 : (cols <= 8 ? 8 : (cols <= 16 ? 16 : 32)); }

// Shape of a workgroup of the multi-wave kernel: waves, and MFMA column tiles (16 columns) per
// wave.  Up to 64 columns one tile per wave (2 or 4 waves); above, in the per-sequence pass, 4
// waves with two tiles each, which share every operand read and fp8 conversion (16 tokens on
// 64 query / 8 KV heads = 128 columns, against 8 waves with one tile: 8B-shaped lengths bf16
// 268 -> 247 us, fp8 258 -> 224 us, 70B-head-shaped fp8 batch 1614 -> 1216 us; with 64 columns
// two waves of two tiles are slower than four of one, 186 against 152 us).  The prefix pass
// keeps one tile per wave, up to 8 waves (two tiles measured 58.7 against 54.9 us per step).
struct WideShape {
    int nw, nct;
};

constexpr WideShape wide_shape(int cols, bool prefix)
{
    if (cols <= 32) return {2, 1};
    if (cols <= 64) return {4, 1};
    return prefix ? WideShape{8, 1} : WideShape{4, 2};
}

constexpr int wide_stages(int d, int kv, WideShape ws)
{
    if (d == 64) return kv == PA_KV_BF16 ? kWideStages64Bf16 : kWideStages64Fp8;
    const int cols = 16 * ws.nw * ws.nct;
    const int i = cols <= 32 ? 0 : (cols <= 64 ? 1 : 2);
    return kv == PA_KV_BF16 ? kWideStagesBf16[i] : kWideStagesFp8[i];
}

// workgroups of the multi-wave kernel resident per compute unit
int wide_groups_per_cu(int d, int kv, WideShape ws)
{
    const int fit = kLdsPerCu / pa::mfma_wide_lds_bytes(d, ws.nw, ws.nct, wide_stages(d, kv, ws), kv);
    const int want = wide_waves_per_cu(kv, ws.nw) / ws.nw;
    return fit < want ? fit : want;
}

// Compute units of the current device (cached per process; 256 when there is no device).
int compute_units()
{
    // initialised once, thread-safely; every GPU this library targets is the same part, so one
    // value per process is enough
    static const int cached = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            return n;
        (void)hipGetLastError();
        return kDefaultCus;
    }();
    return cached;
}

// tiles the per-sequence kernel can meet at most (those after a shared prefix, those a sliding
// window reaches), from what the host knows
int64_t tile_bound(const pa_shape* s)
{
    const int64_t max_ctx = s->max_context_len > 0 ? s->max_context_len : (int64_t)s->max_blocks_per_seq * s->block_size;
    int64_t tiles_per_seq = (max_ctx + pa::kTileTokens - 1) / pa::kTileTokens - shared_tiles(s);
    if (s->window > 0) {
        const int64_t reach_tiles = ((int64_t)s->window + query_len(s) - 1 + pa::kTileTokens - 1) / pa::kTileTokens + 1;
        if (tiles_per_seq > reach_tiles) tiles_per_seq = reach_tiles;
    }
    return (int64_t)s->batch * tiles_per_seq;
}

// resident waves of the one-wave kernel per compute unit
int one_wave_per_cu(const pa_shape* s, pa_kv_dtype kv)
{
    const int fit = kLdsPerCu / pa::mfma_lds_bytes(s->head_dim, mfma_stages(s->head_dim, (int)kv), mfma_col_pad(columns(s)), (int)kv);
    return fit < mfma_waves_per_cu(s->head_dim) ? fit : mfma_waves_per_cu(s->head_dim);
}

// Which kernel runs the per-sequence pass.  Up to 16 columns: one wave.  17 .. 32 columns, where
// both kernels apply: two column tiles in one wave once every partition has a long run of
// tiles, the two-wave workgroup for small calls, which are bound by the per-tile latency chain
// (one sequence, 64 query / 8 KV heads, 4 tokens: 16k context 33.4 against 27.5 us, 64k equal,
// 256k 188 against 208 us).
bool one_wave(const pa_shape* s, pa_kv_dtype kv)
{
    const int cols = columns(s);
    if (cols <= 16) return true;
    if (cols > max_cols_one_wave(s->head_dim, (int)kv)) return false;
    const int64_t P = s->num_partitions > 0 ? s->num_partitions
                                            : (int64_t)compute_units() * one_wave_per_cu(s, kv) / s->num_kv_heads;
    const int min_tiles = s->head_dim == 128 && s->precise_weights == 0 ? kMinTilesTwoColumnTilesStaged : kMinTilesTwoColumnTiles;
    return tile_bound(s) >= min_tiles * (P < 1 ? 1 : P);
}

// workgroups of up to 128 columns a call needs side by side (more than one: the cache is read once per group)
int column_groups(const pa_shape* s) { return (columns(s) + kMaxColsMfma - 1) / kMaxColsMfma; }

// The per-sequence pass of calls the one-wave kernel does not take runs on the stage-split kernel
// (score waves and value waves: two and two up to 64 columns, with two column tiles each above 32;
// four and four with two tiles each above 64), from 17 columns on -- unless the weights are to keep
// their low part, which its hand-over buffers have no room for.  Above 64 columns two cases stay on
// the multi-wave kernel: bf16 KV at head_dim 128, where only one stage-split workgroup would fit a
// compute unit's LDS (8B-shaped batch, 32 query tokens: 197 against 169 us per step), and fp8 KV
// at head_dim 64, whose tiles have two load instructions for four waves to share.
bool staged(const pa_shape* s, pa_kv_dtype kv)
{
    if (one_wave(s, kv) || s->precise_weights != 0 || columns(s) <= 16) return false;
    if (columns(s) <= 64) return true;
    // four and four waves with two column tiles each: where a tile's loads divide over them and two workgroups fit
    return s->head_dim == 128 ? kv == PA_KV_FP8_E4M3 : kv == PA_KV_BF16;
}

// score waves per workgroup and column tiles per wave of that kernel, and its resident workgroups
// per compute unit (sixteen waves, LDS permitting)
// (64 columns as two waves of two tiles, three workgroups per compute unit, against four waves of one
// tile, two workgroups: every K and V operand read and fp8 conversion serves two tiles.  fp8 KV:
// 70B-head-shaped batch, 8 tokens 521.5 -> 469.6 us per step, ragged batch, 16 tokens 330.5 -> 302.3;
// bf16 KV: long-context batch, 16 tokens 398.1 -> 388.2, 8B-shaped 133.7 -> 132.3)
int staged_ns(const pa_shape* s) { return columns(s) <= 64 ? 2 : 4; }
int staged_nct(const pa_shape* s) { return columns(s) > 32 ? 2 : 1; }
int staged_groups_per_cu(const pa_shape* s, pa_kv_dtype kv)
{
    const int fit = kLdsPerCu / pa::staged_lds_bytes(s->head_dim, staged_ns(s), staged_nct(s), (int)kv);
    const int want = 16 / (2 * staged_ns(s));
    return fit < want ? fit : want;
}

// waves (one-wave kernel) or workgroups (multi-wave kernel) resident per compute unit
int groups_per_cu(const pa_shape* s, pa_kv_dtype kv)
{
    const int cols = columns(s) < kMaxColsMfma ? columns(s) : kMaxColsMfma;
    if (staged(s, kv)) return staged_groups_per_cu(s, kv);
    return one_wave(s, kv) ? one_wave_per_cu(s, kv) : wide_groups_per_cu(s->head_dim, (int)kv, wide_shape(cols, false));
}

pa_status check_shape(const pa_shape* s, pa_kv_dtype kv)
{
    if (!s) return PA_ERR_INVALID_ARG;
    if (kv != PA_KV_BF16 && kv != PA_KV_FP8_E4M3) return PA_ERR_INVALID_ARG;
    if (s->batch < 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->head_dim <= 0 || s->block_size <= 0 ||
        s->max_blocks_per_seq <= 0 || s->num_blocks <= 0 || s->max_context_len < 0 || s->num_partitions < 0 ||
        s->q_len < 0 || s->shared_prefix_blocks < 0 || s->window < 0 || (s->precise_weights != 0 && s->precise_weights != 1) ||
        (s->out_dtype != PA_OUT_F32 && s->out_dtype != PA_OUT_BF16))
        return PA_ERR_INVALID_ARG;
    if (s->shared_prefix_blocks > s->max_blocks_per_seq) return PA_ERR_INVALID_ARG;
    if (s->num_q_heads % s->num_kv_heads != 0) return PA_ERR_INVALID_ARG;
    if ((int64_t)s->max_context_len > (int64_t)s->max_blocks_per_seq * s->block_size) return PA_ERR_INVALID_ARG;
    if (s->block_size != pa::kBlockSize) return PA_ERR_UNSUPPORTED;
    if (s->head_dim != 64 && s->head_dim != 128) return PA_ERR_UNSUPPORTED;
    if (s->q_len > kMaxQueryLen) return PA_ERR_UNSUPPORTED;
    if (columns(s) > kMaxCols) return PA_ERR_UNSUPPORTED;
    if (s->num_partitions > kMaxPartitions) return PA_ERR_UNSUPPORTED;
    if (s->batch > kMaxBatch) return PA_ERR_UNSUPPORTED;  // the merge kernels index sequences by blockIdx.y
    if (s->num_kv_heads > 65536) return PA_ERR_UNSUPPORTED;  // bytes between physical blocks fit 32 bits
    if (shared_tiles(s) > 0) {
        // the per-sequence pass takes one workgroup's columns, the prefix pass any number
        if (s->batch < 1 || columns(s) > kMaxColsMfma) return PA_ERR_UNSUPPORTED;
        // every query token lies after the prefix
        if (s->max_context_len > 0 && s->max_context_len < shared_tiles(s) * pa::kTileTokens + query_len(s) - 1) return PA_ERR_INVALID_ARG;
    }
    if ((int64_t)s->window + kMaxQueryLen > INT32_MAX / 2) return PA_ERR_UNSUPPORTED;
    if ((int64_t)s->max_blocks_per_seq * s->block_size > INT32_MAX) return PA_ERR_UNSUPPORTED;
    // the global tile index and the launch grid are 32-bit
    const int64_t max_ctx = s->max_context_len > 0 ? s->max_context_len : (int64_t)s->max_blocks_per_seq * s->block_size;
    const int64_t tile_bound = (int64_t)s->batch * ((max_ctx + pa::kTileTokens - 1) / pa::kTileTokens);
    if (tile_bound > INT32_MAX / 2) return PA_ERR_UNSUPPORTED;
    if ((int64_t)kMaxPartitions * s->num_kv_heads > INT32_MAX) return PA_ERR_UNSUPPORTED;
    return PA_OK;
}

pa_status make_plan(const pa_shape* s, pa_kv_dtype kv, Plan* plan)
{
    const pa_status st = check_shape(s, kv);
    if (st != PA_OK) return st;
    plan->max_ctx = s->max_context_len > 0 ? s->max_context_len : s->max_blocks_per_seq * s->block_size;
    plan->skip_tiles = shared_tiles(s);
    plan->one_wave = one_wave(s, kv);
    plan->staged = staged(s, kv);
    if (s->num_partitions > 0) {
        plan->P = s->num_partitions;
    } else {
        // one resident wave (or workgroup) per (partition, KV head): as many partitions as the device holds at once,
        // but never more than there can be tiles
        int64_t P = (int64_t)compute_units() * groups_per_cu(s, kv) / ((int64_t)s->num_kv_heads * column_groups(s));
        // small calls: a partition should have a few tiles to amortise its start-up, and every extra
        // partition is one more piece per row for the merge (measured on single-sequence calls)
        const int min_tiles = plan->one_wave ? kMinTilesOneWave : kMinTilesWide;
        int64_t most = tile_bound(s) / min_tiles;
        // ... and longer runs of tiles than that are better still, as long as every compute unit keeps a
        // wave (or workgroup): the stage-split workgroups, up to four per compute unit, most of all
        const int want_tiles = plan->staged ? kMinTilesStaged : (plan->one_wave ? kWantTilesOneWave : min_tiles);
        if (want_tiles > min_tiles) {
            const int64_t one_per_cu = (int64_t)compute_units() / ((int64_t)s->num_kv_heads * column_groups(s));
            const int64_t longer = tile_bound(s) / want_tiles;
            most = longer >= one_per_cu ? longer : (one_per_cu < most ? one_per_cu : most);
        }
        if (P > most) P = most;
        if (P > kMaxPartitions) P = kMaxPartitions;
        if (P < 1) P = 1;
        plan->P = (int32_t)P;
    }
    const size_t rows = (size_t)2 * plan->P * s->num_q_heads * query_len(s);
    const size_t o_bytes = plan->P == 1 ? 0 : rows * s->head_dim * sizeof(float);
    const auto pad = [](size_t n) { return (n + 255) / 256 * 256; };
    plan->lse_offset = pad(o_bytes);
    plan->desc_offset = plan->lse_offset + pad(rows * sizeof(float));
    plan->cut_offset = plan->desc_offset + pad((size_t)s->batch * 4 * sizeof(int32_t));
    plan->ws_bytes = plan->P == 1 ? 0 : plan->cut_offset + pad((size_t)plan->P * sizeof(int32_t));
    plan->Pp = 0;
    plan->prefix_waves = plan->prefix_groups = 0;
    plan->seq_o_offset = plan->seq_lse_offset = plan->prefix_o_offset = plan->prefix_lse_offset = 0;
    if (plan->skip_tiles > 0) {
        // the prefix pass: columns are the (sequence, head of the group) pairs, 16 per wave, at most
        // kMaxColsMfma per workgroup, further column groups beyond that
        const int64_t cols64 = (int64_t)s->batch * columns(s);  // (sequence, query token, head of the group)
        if (cols64 > INT32_MAX / 2) return PA_ERR_UNSUPPORTED;
        const int cols = (int)cols64;
        const int group_cols = cols < kMaxColsMfma ? cols : kMaxColsMfma;
        const WideShape ws = wide_shape(group_cols, true);
        plan->prefix_waves = ws.nw;
        plan->prefix_groups = (cols + 16 * ws.nw - 1) / (16 * ws.nw);
        const int per_cu = wide_groups_per_cu(s->head_dim, (int)kv, ws);
        int64_t Pp = (int64_t)compute_units() * per_cu / ((int64_t)s->num_kv_heads * plan->prefix_groups);
        if (s->num_partitions > 0) Pp = s->num_partitions;  // tests force both counts with one knob
        if (Pp > plan->skip_tiles) Pp = plan->skip_tiles;
        if (Pp < 1) Pp = 1;
        plan->Pp = (int32_t)Pp;
        const size_t out_rows = (size_t)s->batch * s->num_q_heads * query_len(s);
        plan->seq_o_offset = plan->ws_bytes;
        plan->seq_lse_offset = plan->seq_o_offset + pad(out_rows * s->head_dim * sizeof(float));
        plan->prefix_o_offset = plan->seq_lse_offset + pad(out_rows * sizeof(float));
        plan->prefix_lse_offset = plan->prefix_o_offset + pad((size_t)plan->Pp * out_rows * s->head_dim * sizeof(float));
        plan->ws_bytes = plan->prefix_lse_offset + pad((size_t)plan->Pp * out_rows * sizeof(float));
    }
    return PA_OK;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Does shape.precise_weights change the kernel?  Only where the default drops the low part.
constexpr bool precise_matters(int kv, int nct, bool multi_wave) { return !pa::p_has_low_part(kv, nct, multi_wave); }

template <int D, int CPAD, int KV>
void launch_mfma(const Params& p, bool trace, bool precise, dim3 grid, hipStream_t st)
{
    constexpr int NSTAGE = mfma_stages(D, KV);
    constexpr bool kMatters = precise_matters(KV, CPAD > 16 ? 2 : 1, false);
    if (kMatters && precise) {
        if (trace)
            hipLaunchKernelGGL((pa::partition_mfma_kernel<D, NSTAGE, CPAD, KV, true, kMatters>), grid, dim3(64), 0, st, p);
        else
            hipLaunchKernelGGL((pa::partition_mfma_kernel<D, NSTAGE, CPAD, KV, false, kMatters>), grid, dim3(64), 0, st, p);
    } else {
        if (trace)
            hipLaunchKernelGGL((pa::partition_mfma_kernel<D, NSTAGE, CPAD, KV, true, false>), grid, dim3(64), 0, st, p);
        else
            hipLaunchKernelGGL((pa::partition_mfma_kernel<D, NSTAGE, CPAD, KV, false, false>), grid, dim3(64), 0, st, p);
    }
}

template <int D, int NW, int NCT, int KV, bool PREFIX>
void launch_wide(const Params& p, bool trace, bool precise, dim3 grid, hipStream_t st)
{
    constexpr int NSTAGE = wide_stages(D, KV, WideShape{NW, NCT});
    if (precise) {
        if (trace)
            hipLaunchKernelGGL((pa::partition_mfma_wide_kernel<D, NW, NCT, NSTAGE, KV, true, PREFIX, true>), grid, dim3(NW * 64), 0, st, p);
        else
            hipLaunchKernelGGL((pa::partition_mfma_wide_kernel<D, NW, NCT, NSTAGE, KV, false, PREFIX, true>), grid, dim3(NW * 64), 0, st, p);
    } else {
        if (trace)
            hipLaunchKernelGGL((pa::partition_mfma_wide_kernel<D, NW, NCT, NSTAGE, KV, true, PREFIX, false>), grid, dim3(NW * 64), 0, st, p);
        else
            hipLaunchKernelGGL((pa::partition_mfma_wide_kernel<D, NW, NCT, NSTAGE, KV, false, PREFIX, false>), grid, dim3(NW * 64), 0, st, p);
    }
}

template <int D, int NS, int NCT, int KV>
void launch_staged(const Params& p, bool trace, dim3 grid, hipStream_t st)
{
    if (trace)
        hipLaunchKernelGGL((pa::partition_mfma_staged_kernel<D, NS, NCT, KV, true>), grid, dim3(2 * NS * 64), 0, st, p);
    else
        hipLaunchKernelGGL((pa::partition_mfma_staged_kernel<D, NS, NCT, KV, false>), grid, dim3(2 * NS * 64), 0, st, p);
}

// the per-sequence pass: one wave per (partition, KV head) up to 16 or 32 columns; above, the stage-split
// workgroup of 4 or 8 waves or the multi-wave workgroup of 2, 4 or 8
template <int D, int KV>
void launch_partition(const Params& p, bool one_wave, bool staged, bool trace, bool precise, dim3 grid, hipStream_t st)
{
    const int cols = p.Q * p.G;
    if (staged) {
        if (cols <= 32) {
            launch_staged<D, 2, 1, KV>(p, trace, grid, st);
        } else if (cols <= 64) {
            launch_staged<D, 2, 2, KV>(p, trace, grid, st);
        } else {
            if constexpr ((D == 128) == (KV == pa::KV_FP8)) launch_staged<D, 4, 2, KV>(p, trace, grid, st);
        }
        return;
    }
    if (cols <= 4)
        launch_mfma<D, 4, KV>(p, trace, precise, grid, st);
    else if (cols <= 8)
        launch_mfma<D, 8, KV>(p, trace, precise, grid, st);
    else if (cols <= 16)
        launch_mfma<D, 16, KV>(p, trace, precise, grid, st);
    else if (one_wave)
        launch_mfma<D, 32, KV>(p, trace, precise, grid, st);
    else if (cols <= 32)
        launch_wide<D, 2, 1, KV, false>(p, trace, precise, grid, st);
    else if (cols <= 64)
        launch_wide<D, 4, 1, KV, false>(p, trace, precise, grid, st);
    else
        launch_wide<D, 4, 2, KV, false>(p, trace, precise, grid, st);
    static_assert(wide_shape(32, false).nw == 2 && wide_shape(64, false).nw == 4 && wide_shape(128, false).nct == 2, "as launched");
}

// the pass over the prefix all sequences share
template <int D, int KV>
void launch_prefix(const Params& p, int nw, bool trace, bool precise, dim3 grid, hipStream_t st)
{
    if (nw == 2)
        launch_wide<D, 2, 1, KV, true>(p, trace, precise, grid, st);
    else if (nw == 4)
        launch_wide<D, 4, 1, KV, true>(p, trace, precise, grid, st);
    else
        launch_wide<D, 8, 1, KV, true>(p, trace, precise, grid, st);
}

// calls f with head_dim and the KV type as compile-time constants
template <typename F>
void with_head_dim_and_kv(int d, pa_kv_dtype kv, F&& f)
{
    using std::integral_constant;
    if (d == 128 && kv == PA_KV_BF16) f(integral_constant<int, 128>{}, integral_constant<int, pa::KV_BF16>{});
    else if (d == 128) f(integral_constant<int, 128>{}, integral_constant<int, pa::KV_FP8>{});
    else if (kv == PA_KV_BF16) f(integral_constant<int, 64>{}, integral_constant<int, pa::KV_BF16>{});
    else f(integral_constant<int, 64>{}, integral_constant<int, pa::KV_FP8>{});
}

struct Events {
    hipEvent_t before, between, after;
};

pa_status run(const void* q, const void* k_cache, const void* v_cache, const int32_t* block_tables,
              const int32_t* context_lens, float scale, pa_kv_dtype kv, void* out, const float* k_scale,
              const float* v_scale, const pa_shape* shape, void* workspace, size_t workspace_bytes, void* stream,
              int32_t* trace_blocks, bool trace, const Events* ev)
{
    Plan plan;
    const pa_status st = make_plan(shape, kv, &plan);
    if (st != PA_OK) return st;
    if (!q || !k_cache || !v_cache || !block_tables || !context_lens || !out) return PA_ERR_INVALID_ARG;
    if (kv == PA_KV_FP8_E4M3 && (!k_scale || !v_scale)) return PA_ERR_INVALID_ARG;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(block_tables, 4) || !aligned(context_lens, 4) || !aligned(k_scale, 4) || !aligned(v_scale, 4))
        return PA_ERR_INVALID_ARG;
    if (!(scale == scale) || scale * 0.f != 0.f) return PA_ERR_INVALID_ARG;  // NaN or infinite
    if (trace && !trace_blocks) return PA_ERR_INVALID_ARG;
    if (plan.ws_bytes > 0) {
        if (!workspace || !aligned(workspace, 256)) return PA_ERR_INVALID_ARG;
        if (workspace_bytes < plan.ws_bytes) return PA_ERR_WORKSPACE_TOO_SMALL;
    }
    if (shape->batch == 0) return PA_OK;

    Params p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k_cache = k_cache;
    p.v_cache = v_cache;
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.k_scale = k_scale;
    p.v_scale = v_scale;
    p.out = static_cast<float*>(out);
    p.out_bf16 = shape->out_dtype == PA_OUT_BF16 ? 1 : 0;
    p.part_o = plan.P > 1 ? static_cast<float*>(workspace) : nullptr;
    p.part_lse = plan.P > 1 ? reinterpret_cast<float*>(static_cast<char*>(workspace) + plan.lse_offset) : nullptr;
    p.merge_desc = plan.P > 1 ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + plan.desc_offset) : nullptr;
    // batches with at least as many sequences as boundaries: the merge looks its sequences up by boundary
    p.cut_list = (plan.P > 1 && shape->batch >= plan.P - 1)
                     ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + plan.cut_offset) : nullptr;
    p.trace_blocks = trace ? trace_blocks : nullptr;
    p.scale_log2 = scale * pa::kLog2e;
    p.B = shape->batch;
    p.Hq = shape->num_q_heads;
    p.Hkv = shape->num_kv_heads;
    p.G = shape->num_q_heads / shape->num_kv_heads;
    p.MB = shape->max_blocks_per_seq;
    p.num_blocks = shape->num_blocks;
    p.Q = query_len(shape);
    p.QH = p.Q * p.Hq;
    p.P = plan.P;
    p.window = shape->window;
    p.skip_tiles = plan.skip_tiles;
    p.Pp = plan.Pp;
    if (plan.skip_tiles > 0) {
        char* ws = static_cast<char*>(workspace);
        p.seq_o = reinterpret_cast<float*>(ws + plan.seq_o_offset);
        p.seq_lse = reinterpret_cast<float*>(ws + plan.seq_lse_offset);
        p.prefix_o = reinterpret_cast<float*>(ws + plan.prefix_o_offset);
        p.prefix_lse = reinterpret_cast<float*>(ws + plan.prefix_lse_offset);
    }

    const bool precise = shape->precise_weights != 0;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (ev && hipEventRecord(ev->before, hs) != hipSuccess) return PA_ERR_HIP;

    bool launched = true;
    with_head_dim_and_kv(shape->head_dim, kv, [&](auto d, auto kvt) {
        constexpr int D = decltype(d)::value, KV = decltype(kvt)::value;
        if (plan.skip_tiles > 0) {
            const dim3 pgrid((uint32_t)plan.Pp * (uint32_t)p.Hkv * (uint32_t)plan.prefix_groups);
            launch_prefix<D, KV>(p, plan.prefix_waves, trace, precise, pgrid, hs);
            if (hipGetLastError() != hipSuccess) { launched = false; return; }
        }
        const dim3 grid((uint32_t)plan.P * (uint32_t)p.Hkv * (uint32_t)column_groups(shape));
        launch_partition<D, KV>(p, plan.one_wave, plan.staged, trace, precise, grid, hs);
        if (hipGetLastError() != hipSuccess) { launched = false; return; }
        if (ev && hipEventRecord(ev->between, hs) != hipSuccess) { launched = false; return; }

        if (plan.skip_tiles > 0) {
            const dim3 mgrid(p.QH, p.B);
            hipLaunchKernelGGL((pa::merge_prefix_kernel<D>), mgrid, dim3(pa::kMergeWaves * pa::kWave), 0, hs, p);
        } else if (plan.P > 1) {
            const dim3 mgrid(p.QH, p.B < plan.P - 1 ? p.B : plan.P - 1);  // at most P - 1 sequences are cut
            // few sequences cut many times each: split a row's pieces over the waves of a workgroup
            if (plan.P >= kMergeManyPerSeq * (int64_t)p.B) {
                hipLaunchKernelGGL((pa::merge_many_kernel<D>), mgrid, dim3(pa::kMergeWaves * pa::kWave), 0, hs, p);
            } else if (p.QH >= kMergeRowsFrom) {
                // many rows per sequence: four rows per wave
                const dim3 rgrid((p.QH + pa::kMergeRowsPerWave - 1) / pa::kMergeRowsPerWave, mgrid.y);
                hipLaunchKernelGGL((pa::merge_rows_kernel<D>), rgrid, dim3(64), 0, hs, p);
            } else {
                hipLaunchKernelGGL((pa::merge_kernel<D>), mgrid, dim3(64), 0, hs, p);
            }
        }
        if (hipGetLastError() != hipSuccess) launched = false;
    });
    if (!launched) return PA_ERR_HIP;
    if (ev && hipEventRecord(ev->after, hs) != hipSuccess) return PA_ERR_HIP;
    return PA_OK;
}

// Device address of `scratch` on the current device: looked up once per device, with that device
// current (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];

pa_status static_scratch(void** ptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return PA_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return PA_OK;
}

}  // namespace

extern "C" {

int32_t pa_num_partitions(const pa_shape* shape, pa_kv_dtype kv_dtype)
{
    Plan plan;
    const pa_status st = make_plan(shape, kv_dtype, &plan);
    return st == PA_OK ? plan.P : -(int32_t)st;
}

int32_t pa_split_plan(const pa_shape* shape, pa_kv_dtype kv_dtype, const int32_t* context_lens,
                      int32_t* block_partition)
{
    Plan plan;
    const pa_status st = make_plan(shape, kv_dtype, &plan);
    if (st != PA_OK) return -(int32_t)st;
    if (shape->batch > 0 && (!context_lens || !block_partition)) return -(int32_t)PA_ERR_INVALID_ARG;
    const int skip = plan.skip_tiles;
    const int reach = shape->window > 0 ? shape->window + query_len(shape) - 1 : 0;
    const pa::Span sp{skip, reach};
    int64_t T = 0;
    for (int32_t b = 0; b < shape->batch; ++b) {
        if (context_lens[b] > plan.max_ctx) return -(int32_t)PA_ERR_INVALID_ARG;
        if (skip > 0 && context_lens[b] < skip * pa::kTileTokens + query_len(shape) - 1)
            return -(int32_t)PA_ERR_INVALID_ARG;  // a query token inside the shared prefix
        T += pa::tiles_of(context_lens[b], sp);
    }
    const int32_t MB = shape->max_blocks_per_seq;
    int32_t k = 0;
    int64_t t = 0;  // global index of the current tile
    for (int32_t b = 0; b < shape->batch; ++b) {
        const int32_t L = context_lens[b];
        const int32_t nblk = L > 0 ? (L + pa::kBlockSize - 1) / pa::kBlockSize : 0;
        for (int32_t j = 0; j < MB; ++j) block_partition[(int64_t)b * MB + j] = -1;
        for (int32_t pt = 0; pt < skip; ++pt) {  // shared prefix: range pt of the prefix pass, written as -2 - range
            const int32_t kp = pa::part_of(pt, skip, plan.Pp);
            block_partition[(int64_t)b * MB + 2 * pt] = -2 - kp;
            block_partition[(int64_t)b * MB + 2 * pt + 1] = -2 - kp;
        }
        const int32_t ft = pa::first_tile(L, sp);
        for (int32_t lt = ft; lt < ft + pa::tiles_of(L, sp); ++lt, ++t) {
            while (k + 1 < plan.P && pa::part_begin(k + 1, (int)T, plan.P) <= t) ++k;
            // a block that lies entirely before the window is not read
            if (!(reach > 0 && (2 * lt + 1) * pa::kBlockSize <= L - reach)) block_partition[(int64_t)b * MB + 2 * lt] = k;
            if (2 * lt + 1 < nblk) block_partition[(int64_t)b * MB + 2 * lt + 1] = k;
        }
    }
    return (int32_t)T;
}

size_t pa_decode_workspace_size(const pa_shape* shape, pa_kv_dtype kv_dtype)
{
    Plan plan;
    return make_plan(shape, kv_dtype, &plan) == PA_OK ? plan.ws_bytes : 0;
}

pa_status pa_decode(const void* q, const void* k_cache, const void* v_cache, const int32_t* block_tables,
                    const int32_t* context_lens, float scale, pa_kv_dtype kv_dtype, void* out, const float* k_scale,
                    const float* v_scale, const pa_shape* shape, void* workspace, size_t workspace_bytes, void* stream)
{
    return run(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape,
               workspace, workspace_bytes, stream, nullptr, false, nullptr);
}

pa_status pa_decode_static(const void* q, const void* k_cache, const void* v_cache, const int32_t* block_tables,
                           const int32_t* context_lens, float scale, pa_kv_dtype kv_dtype, void* out,
                           const float* k_scale, const float* v_scale, const pa_shape* shape, void* stream)
{
    Plan plan;
    const pa_status st = make_plan(shape, kv_dtype, &plan);
    if (st != PA_OK) return st;
    if (plan.ws_bytes > PA_STATIC_SCRATCH_BYTES) return PA_ERR_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    if (plan.ws_bytes > 0) {
        const pa_status ss = static_scratch(&ws);
        if (ss != PA_OK) return ss;
    }
    return run(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape, ws,
               plan.ws_bytes > 0 ? PA_STATIC_SCRATCH_BYTES : 0, stream, nullptr, false, nullptr);
}

pa_status pa_decode_trace(const void* q, const void* k_cache, const void* v_cache, const int32_t* block_tables,
                          const int32_t* context_lens, float scale, pa_kv_dtype kv_dtype, void* out,
                          const float* k_scale, const float* v_scale, const pa_shape* shape, void* workspace,
                          size_t workspace_bytes, void* stream, int32_t* visited_blocks)
{
    return run(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape,
               workspace, workspace_bytes, stream, visited_blocks, true, nullptr);
}

pa_status pa_decode_profile(const void* q, const void* k_cache, const void* v_cache, const int32_t* block_tables,
                            const int32_t* context_lens, float scale, pa_kv_dtype kv_dtype, void* out,
                            const float* k_scale, const float* v_scale, const pa_shape* shape, void* workspace,
                            size_t workspace_bytes, void* stream, int32_t steps, float* partition_ms, float* merge_ms)
{
    if (steps <= 0 || steps > 100000 || !partition_ms || !merge_ms) return PA_ERR_INVALID_ARG;
    std::vector<Events> evs((size_t)steps);
    pa_status st = PA_OK;
    size_t created = 0;
    for (; created < evs.size(); ++created) {
        Events& e = evs[created];
        if (hipEventCreate(&e.before) != hipSuccess) { st = PA_ERR_HIP; break; }
        if (hipEventCreate(&e.between) != hipSuccess) { (void)hipEventDestroy(e.before); st = PA_ERR_HIP; break; }
        if (hipEventCreate(&e.after) != hipSuccess) {
            (void)hipEventDestroy(e.before); (void)hipEventDestroy(e.between); st = PA_ERR_HIP; break;
        }
    }
    for (int32_t i = 0; st == PA_OK && i < steps; ++i)
        st = run(q, k_cache, v_cache, block_tables, context_lens, scale, kv_dtype, out, k_scale, v_scale, shape,
                 workspace, workspace_bytes, stream, nullptr, false, &evs[(size_t)i]);
    if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess && st == PA_OK) st = PA_ERR_HIP;
    if (st == PA_OK && shape->batch > 0) {
        double part = 0.0, merge = 0.0;
        for (const Events& e : evs) {
            float a = 0.f, b = 0.f;
            if (hipEventElapsedTime(&a, e.before, e.between) != hipSuccess ||
                hipEventElapsedTime(&b, e.between, e.after) != hipSuccess) { st = PA_ERR_HIP; break; }
            part += a;
            merge += b;
        }
        *partition_ms = (float)(part / steps);
        *merge_ms = (pa_num_partitions(shape, kv_dtype) > 1 || shared_tiles(shape) > 0) ? (float)(merge / steps) : 0.f;
    } else if (st == PA_OK) {
        *partition_ms = 0.f;
        *merge_ms = 0.f;
    }
    for (size_t i = 0; i < created; ++i) {
        (void)hipEventDestroy(evs[i].before);
        (void)hipEventDestroy(evs[i].between);
        (void)hipEventDestroy(evs[i].after);
    }
    return st;
}

pa_status pa_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache, const int32_t* block_tables,
                       const int32_t* context_lens, pa_kv_dtype kv_dtype, const float* k_scale, const float* v_scale,
                       const pa_shape* shape, void* stream)
{
    const pa_status st = check_shape(shape, kv_dtype);
    if (st != PA_OK) return st;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !context_lens) return PA_ERR_INVALID_ARG;
    if (kv_dtype == PA_KV_FP8_E4M3 && (!k_scale || !v_scale)) return PA_ERR_INVALID_ARG;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
        !aligned(block_tables, 4) || !aligned(context_lens, 4) || !aligned(k_scale, 4) || !aligned(v_scale, 4))
        return PA_ERR_INVALID_ARG;
    if (shape->batch == 0) return PA_OK;
    const int Q = query_len(shape);
    const int64_t threads = (int64_t)shape->batch * Q * shape->num_kv_heads * (shape->head_dim / 8);
    if ((threads + 255) / 256 > INT32_MAX) return PA_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)((threads + 255) / 256));
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const uint16_t* kn = static_cast<const uint16_t*>(k_new);
    const uint16_t* vn = static_cast<const uint16_t*>(v_new);
    const int B = shape->batch, Hkv = shape->num_kv_heads, MB = shape->max_blocks_per_seq;
    if (shape->head_dim == 128) {
        if (kv_dtype == PA_KV_BF16)
            hipLaunchKernelGGL((pa::kv_append_kernel<128, pa::KV_BF16>), grid, dim3(256), 0, hs, kn, vn, k_cache, v_cache,
                               block_tables, context_lens, k_scale, v_scale, B, Q, Hkv, MB);
        else
            hipLaunchKernelGGL((pa::kv_append_kernel<128, pa::KV_FP8>), grid, dim3(256), 0, hs, kn, vn, k_cache, v_cache,
                               block_tables, context_lens, k_scale, v_scale, B, Q, Hkv, MB);
    } else {
        if (kv_dtype == PA_KV_BF16)
            hipLaunchKernelGGL((pa::kv_append_kernel<64, pa::KV_BF16>), grid, dim3(256), 0, hs, kn, vn, k_cache, v_cache,
                               block_tables, context_lens, k_scale, v_scale, B, Q, Hkv, MB);
        else
            hipLaunchKernelGGL((pa::kv_append_kernel<64, pa::KV_FP8>), grid, dim3(256), 0, hs, kn, vn, k_cache, v_cache,
                               block_tables, context_lens, k_scale, v_scale, B, Q, Hkv, MB);
    }
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

pa_status pa_check_tables(const int32_t* block_tables, const int32_t* context_lens, const pa_shape* shape,
                          int32_t* report, void* stream)
{
    const pa_status st = check_shape(shape, PA_KV_BF16);  // nothing here depends on the KV type
    if (st != PA_OK) return st;
    if (!block_tables || !context_lens || !report) return PA_ERR_INVALID_ARG;
    if (!aligned(block_tables, 4) || !aligned(context_lens, 4) || !aligned(report, 16)) return PA_ERR_INVALID_ARG;
    pa::CheckParams c{};
    c.block_tables = block_tables;
    c.context_lens = context_lens;
    c.report = report;
    c.B = shape->batch;
    c.MB = shape->max_blocks_per_seq;
    c.num_blocks = shape->num_blocks;
    c.max_ctx = shape->max_context_len > 0 ? shape->max_context_len : shape->max_blocks_per_seq * shape->block_size;
    c.reach = shape->window > 0 ? shape->window + query_len(shape) - 1 : 0;
    c.shared_blocks = 2 * shared_tiles(shape);
    c.min_len = shared_tiles(shape) > 0 ? shared_tiles(shape) * pa::kTileTokens + query_len(shape) - 1 : 0;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(pa::check_tables_init, dim3(1), dim3(64), 0, hs, report);
    if (shape->batch > 0) {
        hipLaunchKernelGGL(pa::check_tables_scan, dim3((uint32_t)shape->batch), dim3(pa::kCheckThreads), 0, hs, c);
        hipLaunchKernelGGL(pa::check_tables_finish, dim3(1), dim3(64), 0, hs, c);
    }
    return hipGetLastError() == hipSuccess ? PA_OK : PA_ERR_HIP;
}

const char* pa_kernel_variant(const pa_shape* shape, pa_kv_dtype kv_dtype)
{
    if (check_shape(shape, kv_dtype) != PA_OK) return nullptr;
    return one_wave(shape, kv_dtype) ? "mfma" : (staged(shape, kv_dtype) ? "mfma-staged" : "mfma-wide");
}

const char* pa_source_digest(void)
{
#ifdef PA_SOURCE_DIGEST
    return PA_SOURCE_DIGEST;
#else
    return "";
#endif
}

const char* pa_status_string(pa_status status)
{
    switch (status) {
        case PA_OK: return "PA_OK";
        case PA_ERR_INVALID_ARG: return "PA_ERR_INVALID_ARG";
        case PA_ERR_UNSUPPORTED: return "PA_ERR_UNSUPPORTED";
        case PA_ERR_WORKSPACE_TOO_SMALL: return "PA_ERR_WORKSPACE_TOO_SMALL";
        case PA_ERR_HIP: return "PA_ERR_HIP";
    }
    return "PA_ERR_UNKNOWN";
}

}  // extern "C"
