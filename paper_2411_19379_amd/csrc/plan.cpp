// Host side of the library: argument validation and the tile table.
// Nothing in this file touches the GPU.
#include "plan.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>

static thread_local std::string g_last_error;

void ssm_set_error(const std::string &msg) { g_last_error = msg; }

extern "C" const char *ssm_last_error(void) { return g_last_error.c_str(); }

static int fail(int code, const std::string &msg)
{
    ssm_set_error(msg);
    return code;
}

// LDS bytes of the fp32 VALU kernel for a given shape (must mirror the
// kernel's carve-up: state copy with padded rows, x/B/C tiles, score tile).
size_t ssm_valu_lds_bytes(int P, int N)
{
    const size_t q = kValuTileTokens;
    size_t floats = (size_t)P * (N + 1)   // state copy, rows padded by one float
                    + q * P               // x tile
                    + 2 * q * N           // B and C tiles
                    + q * q               // masked score tile
                    + 3 * q;              // dt, decay factors
    return floats * sizeof(float) + q * sizeof(double);
}

static int choose_path(const ssm_shape_t &s, ssm_plan *plan)
{
    const int P = s.headdim, N = s.d_state;
    if (s.io_dtype == SSM_DT_BF16 && N == 128 && P % 32 == 0 && P <= 256) {
        plan->path = SSM_PATH_MFMA_BF16;
        plan->p_split = P / 32;
        plan->tile_tokens = s.chunk < kMfmaTileTokens ? s.chunk : kMfmaTileTokens;
        return SSM_OK;
    }
    if ((size_t)P * N > 256u * 32u)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE,
                    "headdim*d_state above 8192 is only supported for bf16 I/O with d_state 128");
    if (ssm_valu_lds_bytes(P, N) > 64 * 1024)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "shape needs more than 64 KiB of LDS in the fp32 kernel");
    plan->path = SSM_PATH_VALU_F32;
    plan->p_split = 1;
    plan->tile_tokens = kValuTileTokens;
    return SSM_OK;
}

extern "C" int ssm_plan_create(const ssm_shape_t *shape, int32_t batch,
                               const int32_t *cu_seqlens_host,
                               const int32_t *cu_ckpt_host,
                               const int32_t *ckpt_pos_host,
                               ssm_plan_t **out)
{
    if (!out)
        return fail(SSM_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!shape)
        return fail(SSM_ERR_INVALID_ARG, "shape is NULL");
    if (batch < 0)
        return fail(SSM_ERR_INVALID_ARG, "batch is negative");
    if (!cu_seqlens_host)
        return fail(SSM_ERR_INVALID_ARG, "cu_seqlens is NULL");
    const ssm_shape_t &s = *shape;
    if (s.nheads <= 0 || s.headdim <= 0 || s.d_state <= 0 || s.ngroups <= 0)
        return fail(SSM_ERR_INVALID_ARG, "nheads, headdim, d_state and ngroups must be positive");
    if (s.nheads % s.ngroups != 0)
        return fail(SSM_ERR_INVALID_ARG, "ngroups must divide nheads");
    if (s.io_dtype != SSM_DT_F32 && s.io_dtype != SSM_DT_BF16)
        return fail(SSM_ERR_INVALID_ARG, "io_dtype must be SSM_DT_F32 or SSM_DT_BF16");
    if (s.state_dtype != SSM_ST_F32 && s.state_dtype != SSM_ST_F16 && s.state_dtype != SSM_ST_BF16)
        return fail(SSM_ERR_INVALID_ARG, "state_dtype must be SSM_ST_F32, SSM_ST_F16 or SSM_ST_BF16");
    if (s.chunk < 16 || s.chunk > 256 || s.chunk % 16 != 0)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "chunk must be a multiple of 16 in 16..256");
    if (s.nheads > 65535)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "nheads above 65535");
    // 16-byte alignment of every token row of x/y, B/C and of a head's state
    const int esz = s.io_dtype == SSM_DT_F32 ? 4 : 2;
    if ((s.headdim * esz) % 16 != 0 || (s.d_state * esz) % 16 != 0)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE,
                    "headdim and d_state rows must be multiples of 16 bytes");

    if (cu_seqlens_host[0] != 0)
        return fail(SSM_ERR_BAD_CU_SEQLENS, "cu_seqlens[0] must be 0");
    for (int32_t i = 0; i < batch; ++i)
        if (cu_seqlens_host[i + 1] < cu_seqlens_host[i])
            return fail(SSM_ERR_BAD_CU_SEQLENS, "cu_seqlens must be non-decreasing");

    int32_t n_ckpt = 0;
    if (cu_ckpt_host) {
        if (cu_ckpt_host[0] != 0)
            return fail(SSM_ERR_BAD_CHECKPOINT, "cu_ckpt[0] must be 0");
        for (int32_t i = 0; i < batch; ++i)
            if (cu_ckpt_host[i + 1] < cu_ckpt_host[i])
                return fail(SSM_ERR_BAD_CHECKPOINT, "cu_ckpt must be non-decreasing");
        n_ckpt = cu_ckpt_host[batch];
        if (n_ckpt > 0 && !ckpt_pos_host)
            return fail(SSM_ERR_INVALID_ARG, "ckpt_pos is NULL but checkpoints are requested");
        for (int32_t i = 0; i < batch; ++i) {
            const int64_t len = (int64_t)cu_seqlens_host[i + 1] - cu_seqlens_host[i];
            for (int32_t k = cu_ckpt_host[i]; k < cu_ckpt_host[i + 1]; ++k) {
                const int32_t p = ckpt_pos_host[k];
                if (p < 1 || p > len) {
                    char buf[160];
                    snprintf(buf, sizeof buf,
                             "checkpoint %d of sequence %d is at %d, outside 1..%lld", k, i, p,
                             (long long)len);
                    return fail(SSM_ERR_BAD_CHECKPOINT, buf);
                }
                if (k > cu_ckpt_host[i] && p <= ckpt_pos_host[k - 1])
                    return fail(SSM_ERR_BAD_CHECKPOINT,
                                "checkpoint positions must be strictly ascending per sequence");
            }
        }
    }

    ssm_plan *plan = new (std::nothrow) ssm_plan();
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "out of host memory");
    plan->shape = s;
    plan->batch = batch;
    plan->n_ckpt = n_ckpt;
    plan->total_tokens = cu_seqlens_host[batch];
    int rc = choose_path(s, plan);
    if (rc != SSM_OK) {
        delete plan;
        return rc;
    }

    // Cut each sequence into tiles.  Every stretch between two consecutive cut
    // points (sequence start, each checkpoint, sequence end) is tiled from its
    // own start, so a checkpoint is always the state at a tile end.
    const int32_t q = plan->tile_tokens;
    plan->seqs.resize(batch);
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t t0 = cu_seqlens_host[i];
        const int32_t len = cu_seqlens_host[i + 1] - t0;
        plan->seqs[i].tile_begin = (int32_t)plan->tiles.size();
        int32_t pos = 0;
        int32_t k = cu_ckpt_host ? cu_ckpt_host[i] : 0;
        const int32_t k_end = cu_ckpt_host ? cu_ckpt_host[i + 1] : 0;
        while (pos < len) {
            const int32_t stop = k < k_end ? ckpt_pos_host[k] : len;  // next cut point
            while (pos < stop) {
                SsmTile t;
                t.tok0 = t0 + pos;
                t.len = stop - pos < q ? stop - pos : q;
                t.seq = i;
                pos += t.len;
                t.ckpt_slot = (pos == stop && k < k_end) ? k : -1;
                plan->tiles.push_back(t);
            }
            if (k < k_end)
                ++k;
        }
        plan->seqs[i].tile_end = (int32_t)plan->tiles.size();
    }
    const int64_t wgs = (int64_t)batch * s.nheads * plan->p_split;
    if (wgs > 0x7fffffffLL / 4) {
        delete plan;
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "batch*nheads too large for one launch");
    }
    plan->n_workgroups = (int32_t)wgs;
    if (plan->path == SSM_PATH_MFMA_BF16)
        ssm_plan_build_stretches(plan, kMfmaWorkgroupsPerRound, kMfmaMinStretchTiles);
    *out = plan;
    return SSM_OK;
}

static void ssm_plan_order_sequences(ssm_plan *plan);

void ssm_plan_build_stretches(ssm_plan *plan, int64_t per_round, int32_t min_tiles)
{
    const ssm_shape_t &s = plan->shape;
    const int32_t batch = plan->batch;
    auto seq_tiles = [&](int32_t i) { return plan->seqs[i].tile_end - plan->seqs[i].tile_begin; };
    // A batch with too few (sequence, head, 64-channel slice) streams to occupy the GPU has its long sequences cut
    // into stretches, as many as still run in one round.  The scan has a variant whose workgroups own 64 channels of
    // a head instead of 32: one set of operand loads serves twice the rows, at half the number of workgroups; it
    // runs where the 32-channel variant would need a second round.
    std::vector<int32_t> parts(batch, 1);
    plan->p_split = s.headdim / 32;
    if (s.headdim % kMfmaWideChannels == 0) {
        const int64_t per_seq = (int64_t)s.nheads * (s.headdim / kMfmaWideChannels);
        int64_t active = 0;
        for (int32_t i = 0; i < batch; ++i)
            active += seq_tiles(i) > 0;
        int64_t stretches = active;
        const int64_t k_want = active > 0 ? per_round / (active * per_seq) : 0;
        if (k_want >= 2 && min_tiles > 0) {
            stretches = 0;
            for (int32_t i = 0; i < batch; ++i)
                if (seq_tiles(i) > 0) {
                    // kMfmaMinCutTiles belongs to the default min_tiles; a caller that passes a smaller one means it
                    const int64_t min_cut = min_tiles >= kMfmaMinStretchTiles ? kMfmaMinCutTiles : 2 * (int64_t)min_tiles;
                    if (seq_tiles(i) >= min_cut)
                        parts[i] = (int32_t)std::max<int64_t>(1, std::min<int64_t>(k_want, seq_tiles(i) / min_tiles));
                    stretches += parts[i];
                }
        }
        if (2 * stretches * per_seq > per_round)
            plan->p_split = s.headdim / kMfmaWideChannels;
    }
    plan->scan_seqs.clear();
    plan->n_carry = 0;
    plan->max_later_tiles = 0;
    plan->carry_chains = false;
    for (int32_t i = 0; i < batch; ++i) {
        const int64_t begin = plan->seqs[i].tile_begin, n = seq_tiles(i);
        for (int32_t k = 0; k < parts[i]; ++k) {
            SsmScanSeq q = {};
            q.tile_begin = (int32_t)(begin + n * k / parts[i]);
            q.tile_end = (int32_t)(begin + n * (k + 1) / parts[i]);
            q.init_seq = k == 0 ? i : -1;
            q.carry_in = q.carry_out = -1;
            if (k > 0) {
                q.carry_in = plan->n_carry++;
                plan->scan_seqs.back().carry_out = q.carry_in;
                plan->max_later_tiles = std::max(plan->max_later_tiles, q.tile_end - q.tile_begin);
                plan->carry_chains = plan->carry_chains || k > 1;
            }
            plan->scan_seqs.push_back(q);
        }
    }
    for (size_t j = 0; j < plan->scan_seqs.size(); ++j)
        if (plan->scan_seqs[j].carry_in >= 0)
            plan->scan_seqs[plan->scan_seqs[j].carry_in].of_slot = (int32_t)j;
    plan->n_workgroups = (int32_t)((int64_t)plan->scan_seqs.size() * s.nheads * plan->p_split);
    ssm_plan_order_sequences(plan);
}

// Launch order of the stretches: longest first (ties: lower index first); stretches without tiles get no work item.
static void ssm_plan_order_sequences(ssm_plan *plan)
{
    const int32_t n = (int32_t)plan->scan_seqs.size();
    std::vector<int32_t> order(n);
    std::iota(order.begin(), order.end(), 0);
    auto n_tiles = [&](int32_t i) { return plan->scan_seqs[i].tile_end - plan->scan_seqs[i].tile_begin; };
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return n_tiles(a) > n_tiles(b); });
    int64_t n_active = 0;
    for (int32_t r = 0; r < n; ++r) {
        plan->scan_seqs[r].by_length = order[r];
        n_active += n_tiles(order[r]) > 0;
    }
    plan->n_items = (int32_t)(n_active * plan->shape.nheads * plan->p_split);
}

SsmMfmaWorkspace ssm_mfma_workspace(const ssm_plan *plan)
{
    auto round256 = [](size_t n) { return (n + 255) / 256 * 256; };
    SsmMfmaWorkspace w;
    if (plan->path != SSM_PATH_MFMA_BF16)
        return w;
    const size_t n_tiles = plan->tiles.size(), H = (size_t)plan->shape.nheads;
    w.images = 0;
    w.dt_rows = w.images + n_tiles * (size_t)plan->shape.ngroups * kMfmaTileGroupBytes;
    w.tile_decay = round256(w.dt_rows + n_tiles * H * kMfmaDtBytes);
    w.carry = w.tile_decay;
    w.total = w.tile_decay;
    if (plan->n_carry > 0) {
        w.carry = round256(w.tile_decay + n_tiles * H * sizeof(float));
        w.total = round256(w.carry + (size_t)plan->n_carry * H * plan->shape.headdim * plan->shape.d_state * sizeof(float));
    }
    return w;
}

extern "C" int ssm_plan_info(const ssm_plan_t *plan, ssm_plan_info_t *info)
{
    if (!plan || !info)
        return fail(SSM_ERR_INVALID_ARG, "plan or info is NULL");
    info->batch = plan->batch;
    info->n_ckpt = plan->n_ckpt;
    info->total_tokens = plan->total_tokens;
    info->n_tiles = (int32_t)plan->tiles.size();
    info->tile_tokens = plan->tile_tokens;
    info->path = plan->path;
    info->n_workgroups = plan->n_workgroups;
    info->n_stretches = plan->path == SSM_PATH_MFMA_BF16 ? (int32_t)plan->scan_seqs.size() : plan->batch;
    return SSM_OK;
}

extern "C" int ssm_plan_tile(const ssm_plan_t *plan, int32_t i, int32_t *tok0, int32_t *len,
                             int32_t *seq, int32_t *ckpt_slot)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (i < 0 || (size_t)i >= plan->tiles.size())
        return fail(SSM_ERR_INVALID_ARG, "tile index out of range");
    const SsmTile &t = plan->tiles[i];
    if (tok0) *tok0 = t.tok0;
    if (len) *len = t.len;
    if (seq) *seq = t.seq;
    if (ckpt_slot) *ckpt_slot = t.ckpt_slot;
    return SSM_OK;
}

extern "C" int ssm_plan_launch_order(const ssm_plan_t *plan, int32_t *by_length, int32_t *slices, int32_t *n_items,
                                     int64_t *n_blocks)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (by_length)
        for (size_t r = 0; r < plan->scan_seqs.size(); ++r)
            by_length[r] = plan->scan_seqs[r].by_length;
    if (slices)
        *slices = plan->p_split;
    if (n_items)
        *n_items = plan->n_items;
    if (n_blocks)
        *n_blocks = ssm_launch_blocks(plan->n_items);
    return SSM_OK;
}

extern "C" int ssm_plan_launch_item(const ssm_plan_t *plan, int64_t block, int32_t *item)
{
    if (!plan || !item)
        return fail(SSM_ERR_INVALID_ARG, "plan or item is NULL");
    if (block < 0 || block >= ssm_launch_blocks(plan->n_items))
        return fail(SSM_ERR_INVALID_ARG, "block outside the launch");
    *item = ssm_launch_item((uint32_t)block, plan->n_items);
    return SSM_OK;
}

extern "C" int ssm_plan_stretch(const ssm_plan_t *plan, int32_t i, int32_t *tile_begin, int32_t *tile_end,
                                int32_t *starts_from_zero)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->path != SSM_PATH_MFMA_BF16) {
        if (i < 0 || i >= plan->batch)
            return fail(SSM_ERR_INVALID_ARG, "stretch index out of range");
        if (tile_begin) *tile_begin = plan->seqs[i].tile_begin;
        if (tile_end) *tile_end = plan->seqs[i].tile_end;
        if (starts_from_zero) *starts_from_zero = 0;
        return SSM_OK;
    }
    if (i < 0 || (size_t)i >= plan->scan_seqs.size())
        return fail(SSM_ERR_INVALID_ARG, "stretch index out of range");
    const SsmScanSeq &q = plan->scan_seqs[i];
    if (tile_begin) *tile_begin = q.tile_begin;
    if (tile_end) *tile_end = q.tile_end;
    if (starts_from_zero) *starts_from_zero = q.carry_in >= 0;
    return SSM_OK;
}

extern "C" int ssm_plan_workspace_bytes(const ssm_plan_t *plan, size_t *bytes)
{
    if (!plan || !bytes)
        return fail(SSM_ERR_INVALID_ARG, "plan or bytes is NULL");
    // The running state never leaves the chip between tiles; the matrix-core scan needs room for the operands
    // that the heads of a group share (written by its first kernel, read by its second) and, when it cuts long
    // sequences into stretches, for the states carried from one stretch to the next and each tile's total decay.
    *bytes = ssm_mfma_workspace(plan).total;
    return SSM_OK;
}
