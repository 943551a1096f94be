// libnomad: how the deterministic edge pass is laid out for a problem -- tile size, LDS budgets of the three edge-pass
// kernels, which of them runs, whether a round's records are sorted, the number of record phases.  Plain C++ with no
// device code and no HIP types, so that the rules can be compiled and checked on a machine without a GPU; the kernels'
// header includes it for the constants and LDS sizes they share with the host.
#pragma once
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define NOMAD_HOST_DEVICE __host__ __device__
#else
#define NOMAD_HOST_DEVICE
#endif

namespace nomad {

constexpr int kMaxTileBits = 13;        // 8192 points: 128 KB of accumulators in the tile pass
constexpr int kMinTileBits = 8;
constexpr int kChunk = 128;             // records per chunk (1.5 KB): every (workgroup, tile) chain ends in a partly filled
                                        // chunk, so the pool carries workgroups x tiles x kChunk records of slack
constexpr int kBinBlock = 1024;         // threads of the tile pass and of the large edge-pass workgroup
constexpr int kMaxBinsPerThread = 8;    // tiles one thread owns in the per-round scan of the sorted form
constexpr size_t kMaxLdsBytes = 160 * 1024 - 256;   // per workgroup on gfx950, less the kernels' static LDS
constexpr int kDefaultFlushRounds = 2;  // unsorted binned edge pass: rounds between two flushes (5 % faster than one at
                                        // 60 M points; the records of four rounds do not fit the registers)

// ---- LDS of the edge-pass kernels
// binned: per tile (record count / first sorted slot, fill of the open chunk, open chunk, first chunk allocated this
// round) and, in the sorted form, the round's records sorted by tile
NOMAD_HOST_DEVICE inline size_t binned_records_per_round(int s, int block) { return (size_t)block * (s + 1) + 2 * (block / 64); }
NOMAD_HOST_DEVICE inline size_t binned_lds_bytes(uint32_t n_bins, int s, int block, bool sorted = true) {
    return ((size_t)4 * n_bins + 1 + (sorted ? 3 * binned_records_per_round(s, block) : 0)) * sizeof(uint32_t);
}
// pooled (16-bit picks): pool rows, points and 64-bit sums, the tile tables, the partial head sums of a block (two per
// wavefront and round)
NOMAD_HOST_DEVICE inline size_t pooled_side_records(int64_t block_edges) { return (size_t)(block_edges / 32); }
NOMAD_HOST_DEVICE inline size_t pooled_lds_bytes(uint32_t n_bins, int64_t block_edges, uint32_t pool_size) {
    return (size_t)pool_size * 28 + ((size_t)4 * n_bins + 3 * pooled_side_records(block_edges)) * sizeof(uint32_t);
}
// pooled with distinct picks: the same plus the starts of the next block's lines
NOMAD_HOST_DEVICE inline size_t distinct_lds_bytes(uint32_t n_bins, uint32_t pool_size, uint32_t lines, int rounds) {
    return (size_t)pool_size * 28 + ((size_t)lines + (size_t)4 * n_bins + 3 * (size_t)(32 * rounds)) * sizeof(uint32_t);
}

// ---- the plan
struct EdgePlanRequest {
    int64_t n = 0, E = 0;
    int s = 0;
    // pooled sampler (pool_size 0: none); distinct: picks in different lines (modes 1 and 2)
    int32_t pool_size = 0, pool_block = 0, pool_line = 1;
    bool pool_distinct = false;
    // nomad_tune (0 = the library's choice, except pool_kernel: 1 = use the pooled kernels)
    int tune_edge_block = 0, tune_wg_per_cu = 0, tune_pool_kernel = 1, tune_record_sort = 0, tune_flush_rounds = 0;
};

struct EdgePlan {
    int tile_bits = kMinTileBits;
    uint32_t n_bins = 0;
    int bin_block = 0;          // lanes per workgroup of the edge pass; 0: its tables do not fit LDS
    int wg_per_cu = 1;
    bool sorted = true;         // a round's records are counting-sorted by tile in LDS before they are written
    int flush_rounds = 1;       // unsorted form: rounds between two flushes
    int pool_rounds = 0;        // > 0: a pooled edge pass runs, pool_block = 1024 * pool_rounds
    bool distinct_kernel = false;
};

inline EdgePlan plan_edge_pass(const EdgePlanRequest& q) {
    EdgePlan p;
    // about a thousand tiles when n allows, never above 8192 points a tile
    while (p.tile_bits < kMaxTileBits && (q.n >> p.tile_bits) > 1024) ++p.tile_bits;
    p.n_bins = (uint32_t)((q.n + ((int64_t)1 << p.tile_bits) - 1) >> p.tile_bits);
    // One persistent workgroup of 1024 lanes per compute unit: the more records a round sorts, the longer the
    // contiguous run each tile receives.  (Two workgroups of 512 per compute unit measured 17 % slower at
    // 10 M points; nomad_tune(NOMAD_TUNE_EDGE_BLOCK, 512) selects them for experiments when their LDS fits.)
    // A round's records are counting-sorted by tile in LDS before they are written, unless there are more tiles than
    // a round has records (60 M points, s = 2): then no tile receives a run worth sorting for, and every lane
    // writes its own records (two barriers and the scan over the tiles less per round).
    p.sorted = q.tune_record_sort != 2 && (q.tune_record_sort == 1 || (size_t)p.n_bins <= binned_records_per_round(q.s, 1024));
    if ((!p.sorted || p.n_bins <= (uint32_t)kMaxBinsPerThread * 1024) && binned_lds_bytes(p.n_bins, q.s, 1024, p.sorted) <= kMaxLdsBytes)
        p.bin_block = 1024;
    if (q.tune_edge_block == 512 && (!p.sorted || p.n_bins <= (uint32_t)kMaxBinsPerThread * 512) &&
        2 * (binned_lds_bytes(p.n_bins, q.s, 512, p.sorted) + 256) <= 160 * 1024) { p.bin_block = 512; p.wg_per_cu = 2; }
    if (q.tune_wg_per_cu) p.wg_per_cu = q.tune_wg_per_cu;
    // Pooled samplers: their own edge pass (pool in LDS) when the block is 1, 2, 4 or 8 rounds of 1024 positions, one
    // workgroup per compute unit.  (Two workgroups of 512 lanes per compute unit, which lets one block's
    // bookkeeping overlap the other's rounds, measured 4 % slower: the rounds are bound by vector-ALU issue.)
    if (q.pool_size > 0 && q.pool_block % 1024 == 0 && q.tune_pool_kernel) {
        const int r = q.pool_block / 1024;
        if (r == 1 || r == 2 || r == 4 || r == 8) {
            if (q.pool_distinct) {
                // 32-bit byte offsets into col / head (4 E) and theta (8 n)
                if (distinct_lds_bytes(p.n_bins, (uint32_t)q.pool_size, (uint32_t)(q.pool_size / q.pool_line), r) <= kMaxLdsBytes &&
                    q.E < ((int64_t)1 << 30) && q.n < ((int64_t)1 << 29)) { p.pool_rounds = r; p.distinct_kernel = true; }
            } else if (pooled_lds_bytes(p.n_bins, q.pool_block, (uint32_t)q.pool_size) <= kMaxLdsBytes) {
                p.pool_rounds = r;
            }
        }
    }
    if (p.pool_rounds) { p.bin_block = 1024; p.wg_per_cu = 1; p.sorted = true; }
    p.flush_rounds = (!p.sorted && p.bin_block == 1024) ? (q.tune_flush_rounds ? q.tune_flush_rounds : kDefaultFlushRounds) : 1;
    return p;
}

// Record phases: the edge pass of a step runs over `phases` ranges of positions, each followed by the tile pass, so the
// pool holds the records of one range.  Default: as many (a power of two, at most 64) as keep one range's records under
// 8 GB, and under 4 GB for a step with more than 32 GB of records, where the pool would otherwise outweigh the graph
// (each further phase costs about half a per cent of an epoch: the tile pass walks shorter chains and carries its sums
// through memory).  Never more phases than the positions have blocks.
inline int plan_record_phases(int64_t E, int s, int bin_block, int tune_phases) {
    int phases = tune_phases;
    if (phases == 0) {
        const double step_bytes = (double)E * (s + 1) * 12.0;
        const double per_phase = step_bytes > 32e9 ? 4e9 : 8e9;
        phases = 1;
        while (phases < 64 && step_bytes / phases > per_phase) phases *= 2;
    }
    const int64_t blocks = (E + bin_block - 1) / bin_block;
    if (phases > blocks) phases = (int)blocks;
    return phases < 1 ? 1 : phases;
}

}  // namespace nomad
