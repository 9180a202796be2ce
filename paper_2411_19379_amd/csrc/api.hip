// ssm_prefill: argument checks, upload of the plan's tables, kernel launch.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <string>

#include "device_utils.h"
#include "plan.h"

static int fail(int code, const std::string &msg)
{
    ssm_set_error(msg);
    return code;
}

static int hip_fail(const char *what, hipError_t e)
{
    return fail(SSM_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// First use of a plan on the GPU: copy its tables to device memory.
static int upload_plan(ssm_plan *plan)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail("hipGetDevice", e);
    if (plan->d_tiles && plan->device == dev)
        return SSM_OK;
    if (plan->d_tiles)
        return fail(SSM_ERR_INVALID_ARG, "plan was first used on another device");
    const size_t tile_bytes = plan->tiles.size() * sizeof(SsmTile);
    const size_t seq_bytes = plan->seqs.size() * sizeof(SsmSeq);
    const size_t ptr_bytes = (size_t)plan->batch * sizeof(const float *);
    void *dt = nullptr, *ds = nullptr, *dp = nullptr;
    if ((e = hipMalloc(&dt, tile_bytes ? tile_bytes : 16)) != hipSuccess)
        return hip_fail("hipMalloc(tiles)", e);
    if ((e = hipMalloc(&ds, seq_bytes ? seq_bytes : 16)) != hipSuccess) {
        (void)hipFree(dt);
        return hip_fail("hipMalloc(seqs)", e);
    }
    if ((e = hipMalloc(&dp, ptr_bytes ? ptr_bytes : 16)) != hipSuccess) {
        (void)hipFree(dt);
        (void)hipFree(ds);
        return hip_fail("hipMalloc(init ptrs)", e);
    }
    if (tile_bytes)
        e = hipMemcpy(dt, plan->tiles.data(), tile_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess && seq_bytes)
        e = hipMemcpy(ds, plan->seqs.data(), seq_bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(dt);
        (void)hipFree(ds);
        (void)hipFree(dp);
        return hip_fail("hipMemcpy(plan tables)", e);
    }
    plan->d_tiles = dt;
    plan->d_seqs = ds;
    plan->d_init_ptrs = dp;
    plan->device = dev;
    return SSM_OK;
}

extern "C" int ssm_prefill(ssm_plan_t *plan,
                           const void *x, const void *dt, const float *A,
                           const void *B, const void *C, const float *D,
                           const float *const *init_state_ptrs,
                           void *y_out, float *state_out,
                           void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 || plan->batch == 0)
        return SSM_OK;
    if (!x || !dt || !A || !B || !C || !D || !y_out)
        return fail(SSM_ERR_INVALID_ARG, "a required tensor pointer is NULL");
    if (plan->n_ckpt > 0 && !state_out)
        return fail(SSM_ERR_INVALID_ARG, "state_out is NULL but the plan has checkpoints");
    const void *ptrs[] = {x, dt, A, B, C, D, y_out, state_out};
    for (const void *p : ptrs)
        if (!aligned16(p))
            return fail(SSM_ERR_MISALIGNED, "device pointers must be 16-byte aligned");
    bool any_init = false;
    if (init_state_ptrs)
        for (int32_t i = 0; i < plan->batch; ++i) {
            if (!aligned16(init_state_ptrs[i]))
                return fail(SSM_ERR_MISALIGNED, "initial states must be 16-byte aligned");
            any_init = any_init || init_state_ptrs[i] != nullptr;
        }

    int rc = upload_plan(plan);
    if (rc != SSM_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (any_init) {
        // pageable source: the runtime has taken its copy when this returns
        hipError_t e = hipMemcpyAsync(plan->d_init_ptrs, init_state_ptrs,
                                      (size_t)plan->batch * sizeof(const float *),
                                      hipMemcpyHostToDevice, stream);
        if (e != hipSuccess)
            return hip_fail("hipMemcpyAsync(init ptrs)", e);
    }

    ScanArgs args;
    args.x = x;
    args.dt = dt;
    args.A = A;
    args.B = B;
    args.C = C;
    args.D = D;
    args.y = y_out;
    args.state_out = state_out;
    args.init_ptrs = any_init ? static_cast<const float *const *>(plan->d_init_ptrs) : nullptr;
    args.tiles = static_cast<const SsmTile *>(plan->d_tiles);
    args.seqs = static_cast<const SsmSeq *>(plan->d_seqs);
    args.H = plan->shape.nheads;
    args.P = plan->shape.headdim;
    args.N = plan->shape.d_state;
    args.G = plan->shape.ngroups;
    args.p_split = plan->p_split;

    hipError_t e = plan->path == SSM_PATH_MFMA_BF16 ? launch_scan_mfma(plan, args, stream)
                                                     : launch_scan_valu(plan, args, stream);
    if (e != hipSuccess)
        return hip_fail("kernel launch", e);
    return SSM_OK;
}

extern "C" void ssm_plan_destroy(ssm_plan_t *plan)
{
    if (!plan)
        return;
    if (plan->d_tiles)
        (void)hipFree(plan->d_tiles);
    if (plan->d_seqs)
        (void)hipFree(plan->d_seqs);
    if (plan->d_init_ptrs)
        (void)hipFree(plan->d_init_ptrs);
    delete plan;
}
