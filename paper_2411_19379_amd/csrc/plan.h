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

struct ssm_plan {
    ssm_shape_t shape;
    int32_t batch = 0;
    int32_t n_ckpt = 0;
    int64_t total_tokens = 0;
    int32_t tile_tokens = 0;
    int32_t path = SSM_PATH_VALU_F32;
    int32_t p_split = 1;          // workgroups per (sequence, head): headdim is cut in p_split parts
    int32_t n_workgroups = 0;
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
