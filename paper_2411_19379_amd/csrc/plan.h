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

// Per sequence: its tiles are [tile_begin, tile_end) of the tile table.
struct SsmSeq {
    int32_t tile_begin;
    int32_t tile_end;
};

// What one workgroup of the matrix-core scan walks: a stretch of consecutive tiles of one sequence, either the whole
// sequence or, when a batch has too few sequences to fill the GPU, one of several stretches a long sequence is cut
// into.  A later stretch is scanned from a zero state at the same time as the ones before it; the state its
// predecessor ends with reaches a carry slot, and a second kernel adds what that state contributes to the stretch's
// outputs and checkpoints (the recurrence is linear in the state: the contribution to token t is the carried state
// decayed from the stretch's start to t, times C_t).  The last two fields belong to the table, not to the stretch.
struct SsmScanSeq {
    int32_t tile_begin;
    int32_t tile_end;
    int32_t init_seq;   // sequence of the batch whose initial state the stretch starts from; -1: it starts from zero
    int32_t carry_in;   // carry slot with the state the stretch truly starts from (a later stretch); -1: none
    int32_t carry_out;  // carry slot that receives the state after the stretch's last tile; -1: none
    int32_t by_length;  // entry r: the stretch of rank r when stretches are ordered by decreasing number of tiles
    int32_t of_slot;    // entry c: the stretch whose carry_in is c
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
    int32_t n_items = 0;          // work items of the matrix-core scan: non-empty stretches x heads x p_split
    int32_t n_carry = 0;          // carry slots: stretches that continue a sequence
    int32_t max_later_tiles = 0;  // most tiles in any such stretch
    bool carry_chains = false;    // some sequence is cut into three or more stretches
    std::vector<SsmTile> tiles;
    std::vector<SsmSeq> seqs;
    std::vector<SsmScanSeq> scan_seqs;  // matrix-core scan only
    // Device copies of the two tables and a buffer for the per-call state
    // pointers, one set per GPU the plan has been used on.  A cache behind a
    // logically constant plan: filled on first use under `mu`.
    struct DeviceTables {
        int device = -1;
        void *tiles = nullptr;  // SsmTile[n_tiles]
        void *seqs = nullptr;   // SsmSeq[batch]
        void *scan_seqs = nullptr;  // SsmScanSeq[stretches]
        void *ptrs = nullptr;   // void*[batch], rewritten by every call that passes states
    };
    mutable std::mutex mu;
    mutable std::vector<DeviceTables> device_tables;
};

void ssm_set_error(const std::string &msg);

// Matrix-core scan: (re)builds the stretches, p_split, the carry slots, the launch order and n_workgroups from the
// tiles and the shape.  `per_round` workgroups run at a time.  With s (sequence, head, 64-channel slice) streams, long
// sequences are cut into floor(per_round / s) stretches of at least `min_tiles` tiles each; the 64-channel variant is
// chosen if the 32-channel one would not fit one round.
void ssm_plan_build_stretches(ssm_plan *plan, int64_t per_round, int32_t min_tiles);

// Where the parts of the matrix-core scan's workspace start (bytes from its base), and its size.
struct SsmMfmaWorkspace {
    size_t images = 0;      // per (tile, group): kMfmaTileGroupBytes
    size_t dt_rows = 0;     // per (tile, head): kMfmaDtBytes
    size_t tile_decay = 0;  // per (head, tile): the tile's total log2 decay, fp32 (only with carry slots)
    size_t carry = 0;       // per carry slot: [H, P, N] fp32
    size_t total = 0;
};
SsmMfmaWorkspace ssm_mfma_workspace(const ssm_plan *plan);

// Tile lengths the two kernel families work with.
constexpr int kValuTileTokens = 16;
constexpr int kMfmaTileTokens = 64;

// Workspace of the matrix-core scan: per (tile, group) the operands the heads of a group share (C and B^T as fp16
// register images, 16 KiB each, and the raw score blocks, 6 KiB), then per (tile, head) the tile's dt, 64 bf16.
constexpr size_t kMfmaTileGroupBytes = 38912;
constexpr size_t kMfmaDtBytes = 128;

// The GPU this library is written for takes one workgroup of the matrix-core scan per compute unit, 256 at a time.
// The wide variant of the scan (64 channels of a head per workgroup instead of 32) is chosen when the narrow one would
// need more workgroups than that, i.e. a second round; long sequences are cut into as many stretches as still fit
// one round of the wide variant.
constexpr int kMfmaWideChannels = 64;
constexpr int kMfmaWorkgroupsPerRound = 256;

// A sequence is cut into stretches only if each gets at least this many tiles (the second kernel's work per stretch
// does not shrink with the stretch), and only if it has at least kMfmaMinCutTiles tiles: at 128 tiles two stretches
// of 64 were measured 2 to 8 % slower than no cut, at 192 tiles 5 % faster.
constexpr int kMfmaMinStretchTiles = 64;
constexpr int kMfmaMinCutTiles = 160;

// The kernel in front of the scan works per (tile, group); below this many pairs each pair gets four workgroups.
constexpr int kMfmaPrepSplitBelow = 256;
