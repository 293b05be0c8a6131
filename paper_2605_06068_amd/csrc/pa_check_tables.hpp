// Table check: does every block id that an attention call over these tables would follow lie
// inside the pool, is every length inside its bound, and (shared-prefix calls) does every row
// repeat row 0 over the prefix?  The kernels read block_tables and context_lens and nothing else:
// no id is ever turned into an address.  The release kernels trust what this checks.
//
// Three small launches on the caller's stream, no host synchronisation, no memset:
//   check_tables_init      report <- "nothing found"
//   check_tables_scan      one workgroup per sequence; every thread looks at some of the sequence's
//                          table entries, the workgroup keeps the smallest offending (b, j) as a
//                          64-bit key b * (MB + 1) + (j + 1) (j = -1: the length itself) with an
//                          integer atomic minimum, and counts the offending entries
//   check_tables_finish    one thread turns the key into {kind, b, j, value}
// "First" is batch order, then block order, so the answer does not depend on scheduling.
#pragma once
#include "pa_device.hpp"
#include "pa_plan.hpp"

namespace pa {

// report words (int32): 0 kind, 1 sequence, 2 logical block (-1: the length), 3 offending value,
// 4 number of offending entries, 5 unused, 6..7 the 64-bit key while the scan runs
constexpr int kReportKind = 0, kReportSeq = 1, kReportBlock = 2, kReportValue = 3, kReportCount = 4, kReportKey = 6;
constexpr int kTablesOk = 0, kTablesBadLength = 1, kTablesBadBlockId = 2, kTablesPrefixMismatch = 3;
constexpr unsigned long long kNoKey = ~0ull;
constexpr int kCheckThreads = 256;

struct CheckParams {
    const int32_t* block_tables;
    const int32_t* context_lens;
    int32_t* report;
    int32_t B, MB, num_blocks, max_ctx;
    int32_t reach;          // window + q_len - 1, or 0: how far back from the end of a context a query can see
    int32_t shared_blocks;  // leading table entries every row must share with row 0 (whole tiles)
    int32_t min_len;        // shortest length a shared prefix allows (prefix tokens + q_len - 1), else 0
};

__device__ __forceinline__ bool length_ok(const CheckParams& c, int L) { return L >= 0 && L <= c.max_ctx && L >= c.min_len; }

// 0, or what is wrong with entry j of row b (its value is id)
__device__ __forceinline__ int entry_kind(const CheckParams& c, int j, int id)
{
    if (id < 0 || id >= c.num_blocks) return kTablesBadBlockId;
    if (j < c.shared_blocks && id != c.block_tables[j]) return kTablesPrefixMismatch;
    return kTablesOk;
}

__global__ void check_tables_init(int32_t* report)
{
    if (threadIdx.x < 6) report[threadIdx.x] = threadIdx.x == kReportSeq || threadIdx.x == kReportBlock ? -1 : 0;
    if (threadIdx.x == 6) *reinterpret_cast<unsigned long long*>(report + kReportKey) = kNoKey;
}

__global__ __launch_bounds__(kCheckThreads) void check_tables_scan(const CheckParams c)
{
    const int b = blockIdx.x;
    const int L = c.context_lens[b];
    unsigned long long key = kNoKey;
    int bad = 0;
    if (!length_ok(c, L)) {
        if (threadIdx.x == 0) {
            key = (unsigned long long)b * ((unsigned long long)c.MB + 1ull);
            bad = 1;
        }
    } else if (L > 0) {
        const int t_first = (c.reach > 0 && L > c.reach) ? L - c.reach : 0;
        const int j_last = (L - 1) / kBlockSize;
        for (int j = t_first / kBlockSize + (int)threadIdx.x; j <= j_last; j += kCheckThreads) {
            if (entry_kind(c, j, c.block_tables[(int64_t)b * c.MB + j]) != kTablesOk) {
                const unsigned long long mine = (unsigned long long)b * ((unsigned long long)c.MB + 1ull) + (unsigned long long)(j + 1);
                key = mine < key ? mine : key;
                ++bad;
            }
        }
    }
    // the wave's smallest key and its count, then one pair of atomics per wave that found something
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const unsigned long long other = __shfl_xor(key, o, kWave);
        key = other < key ? other : key;
        bad += __shfl_xor(bad, o, kWave);
    }
    if ((threadIdx.x & (kWave - 1)) == 0 && bad > 0) {
        atomicMin(reinterpret_cast<unsigned long long*>(c.report + kReportKey), key);
        atomicAdd(c.report + kReportCount, bad);
    }
}

__global__ void check_tables_finish(const CheckParams c)
{
    if (threadIdx.x != 0) return;
    const unsigned long long key = *reinterpret_cast<const unsigned long long*>(c.report + kReportKey);
    if (key == kNoKey) return;  // the init kernel's "nothing found" stands
    const int b = (int)(key / ((unsigned long long)c.MB + 1ull));
    const int j = (int)(key % ((unsigned long long)c.MB + 1ull)) - 1;
    int kind, value;
    if (j < 0) {
        kind = kTablesBadLength;
        value = c.context_lens[b];
    } else {
        value = c.block_tables[(int64_t)b * c.MB + j];
        kind = entry_kind(c, j, value);
    }
    c.report[kReportKind] = kind;
    c.report[kReportSeq] = b;
    c.report[kReportBlock] = j;
    c.report[kReportValue] = value;
}

}  // namespace pa
