// Internal layout of a scan plan (host side) and of the tables the kernels read.
#pragma once

#include <cstddef>
#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "ssm_prefill.h"

// One token tile: a run of consecutive tokens of one sequence that the scan
// kernel consumes in one step.  16 bytes, read by the kernels as an int4.
struct SsmTile {
    int32_t tok0;       // first token, index into the packed batch
    int32_t len;        // 1 .. tile_tokens
    int32_t ckpt_slot;  // state_out slot written after this tile, or -1
    int32_t seq;        // owning sequence
};

// Per sequence: its tiles are [tile_begin, tile_end) of the tile table.  The third field belongs to the table, not to
// the sequence: entry r names the sequence of rank r when the sequences are ordered by decreasing number of tiles.
struct SsmSeq {
    int32_t tile_begin;
    int32_t tile_end;
    int32_t by_length;
    int32_t reserved;
};

// Launch order of the matrix-core scan.  Its work items, one per (rank of a non-empty sequence, head, channel slice),
// form a line ordered by rank, then head, then slice: longest sequences first.  The hardware deals the workgroups of a
// launch round-robin to 8 dies (XCDs), each with its own L2 and 32 compute units that take one workgroup at a time.
// The line is cut into runs of 32 items (of an eighth of the items, if there are fewer than 256), one run per die and
// round; within a round the runs go to the dies in ascending order, in the next round in descending order, and so on,
// so that every die works through a similar mix of long and short items, starts its longest first, and neighbouring
// heads (which share operands) meet in one L2.
constexpr int kXcds = 8;
constexpr int kItemsPerRun = 32;

#ifdef __HIPCC__
#define SSM_HOST_DEVICE __host__ __device__
#else
#define SSM_HOST_DEVICE
#endif
// The item of workgroup `block` of the launch, or -1 if it has none.  The launch has ssm_launch_blocks(n_items) blocks.
SSM_HOST_DEVICE inline uint32_t ssm_launch_run_length(int64_t n_items)
{
    if (n_items >= kXcds * kItemsPerRun)
        return kItemsPerRun;
    return n_items > 0 ? (uint32_t)((n_items + kXcds - 1) / kXcds) : 1u;
}
SSM_HOST_DEVICE inline int32_t ssm_launch_item(uint32_t block, int32_t n_items)
{
    const uint32_t len = ssm_launch_run_length(n_items);
    const uint32_t xcd = block % kXcds, k = block / kXcds;  // k-th workgroup of this die
    const uint32_t round = k / len;
    const uint32_t run = round * kXcds + ((round & 1) ? kXcds - 1 - xcd : xcd);
    const uint32_t item = run * len + k % len;
    return item < (uint32_t)n_items ? (int32_t)item : -1;
}
inline int64_t ssm_launch_blocks(int64_t n_items)
{
    const int64_t per_round = (int64_t)kXcds * ssm_launch_run_length(n_items);
    return (n_items + per_round - 1) / per_round * per_round;
}

struct ssm_plan {
    ssm_shape_t shape;
    int32_t batch = 0;
    int32_t n_ckpt = 0;
    int64_t total_tokens = 0;
    int32_t tile_tokens = 0;
    int32_t path = SSM_PATH_VALU_F32;
    int32_t p_split = 1;          // workgroups per (sequence, head): headdim is cut in p_split parts
    int32_t n_workgroups = 0;
    int32_t n_items = 0;          // work items of the matrix-core scan: non-empty sequences x heads x p_split
    std::vector<SsmTile> tiles;
    std::vector<SsmSeq> seqs;
    // Device copies of the two tables and a buffer for the per-call state
    // pointers, one set per GPU the plan has been used on.  A cache behind a
    // logically constant plan: filled on first use under `mu`.
    struct DeviceTables {
        int device = -1;
        void *tiles = nullptr;  // SsmTile[n_tiles]
        void *seqs = nullptr;   // SsmSeq[batch]
        void *ptrs = nullptr;   // void*[batch], rewritten by every call that passes states
    };
    mutable std::mutex mu;
    mutable std::vector<DeviceTables> device_tables;
};

void ssm_set_error(const std::string &msg);

// (Re)builds seqs[].by_length and n_items from the tiles, the shape and p_split.
void ssm_plan_order_sequences(ssm_plan *plan);

// Tile lengths the two kernel families work with.
constexpr int kValuTileTokens = 16;
constexpr int kMfmaTileTokens = 64;

// Workspace of the matrix-core scan: per (tile, group) the operands the heads of a group share (C and B^T as fp16
// register images, 16 KiB each, and the raw score blocks, 6 KiB), then per (tile, head) the tile's dt, 64 bf16.
constexpr size_t kMfmaTileGroupBytes = 38912;
constexpr size_t kMfmaDtBytes = 128;

// The wide variant of the matrix-core scan (64 channels of a head per workgroup instead of 32) is chosen when it
// still has at least this many workgroups with work: one per compute unit of the GPU this library is written for.
constexpr int kMfmaWideChannels = 64;
constexpr int kMfmaWideMinWorkgroups = 256;

// The kernel in front of the scan works per (tile, group); below this many pairs each pair gets four workgroups.
constexpr int kMfmaPrepSplitBelow = 256;
