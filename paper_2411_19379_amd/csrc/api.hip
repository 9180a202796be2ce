// Entry points that touch the GPU: argument checks, the plan's device tables, kernel launches.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
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

// ---------------------------------------------------------------- small host tables -> device memory
// Tables (tile descriptors, sequence descriptors, per-call state pointers) reach the GPU as kernel arguments of a
// one-workgroup copy kernel, 3 KiB per launch: the runtime takes its copy of the arguments when the launch is
// enqueued, so the host buffer may be pageable and may change right after the call, nothing blocks, nothing is
// allocated, and the launch can be captured into a graph like any other.
constexpr int kPayloadWords = 192;  // uint4 words per launch
struct TablePayload {
    uint4 w[kPayloadWords];
};

__global__ __launch_bounds__(kPayloadWords) void ssm_table_write_kernel(TablePayload p, uint4 *__restrict__ dst, int n_words)
{
    const int i = threadIdx.x;
    if (i < n_words)
        dst[i] = p.w[i];
}

// `dst` is 16-byte aligned device memory with room for `bytes` rounded up to 16.
static hipError_t upload_table(void *dst, const void *src_host, size_t bytes, hipStream_t stream)
{
    const unsigned char *src = static_cast<const unsigned char *>(src_host);
    unsigned char *d = static_cast<unsigned char *>(dst);
    while (bytes > 0) {
        const size_t chunk = bytes < sizeof(TablePayload) ? bytes : sizeof(TablePayload);
        TablePayload p;
        memset(&p, 0, sizeof p);
        memcpy(&p, src, chunk);
        hipLaunchKernelGGL(ssm_table_write_kernel, dim3(1), dim3(kPayloadWords), 0, stream, p,
                           reinterpret_cast<uint4 *>(d), (int)((chunk + 15) / 16));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
        src += chunk;
        d += chunk;
        bytes -= chunk;
    }
    return hipSuccess;
}

static size_t round16(size_t n) { return (n + 15) / 16 * 16; }

// Device copies of a plan's tables on the current GPU; made on first use (four device allocations, the uploads
// enqueued on `stream` and waited for once, so that later calls on any stream find them complete).
static int device_tables(const ssm_plan *plan, hipStream_t stream, ssm_plan::DeviceTables *out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail("hipGetDevice", e);
    std::lock_guard<std::mutex> lock(plan->mu);
    for (const ssm_plan::DeviceTables &t : plan->device_tables)
        if (t.device == dev) {
            *out = t;
            return SSM_OK;
        }
    const size_t tile_bytes = round16(plan->tiles.size() * sizeof(SsmTile));
    const size_t seq_bytes = round16(plan->seqs.size() * sizeof(SsmSeq));
    const size_t ptr_bytes = round16((size_t)plan->batch * sizeof(void *));
    const size_t scan_seq_bytes = round16(plan->scan_seqs.size() * sizeof(SsmScanSeq));
    ssm_plan::DeviceTables t;
    t.device = dev;
    auto release = [&]() {
        (void)hipFree(t.tiles);
        (void)hipFree(t.seqs);
        (void)hipFree(t.scan_seqs);
        (void)hipFree(t.ptrs);
    };
    if ((e = hipMalloc(&t.tiles, tile_bytes ? tile_bytes : 16)) != hipSuccess)
        return hip_fail("hipMalloc(tile table)", e);
    if ((e = hipMalloc(&t.seqs, seq_bytes ? seq_bytes : 16)) != hipSuccess) {
        release();
        return hip_fail("hipMalloc(sequence table)", e);
    }
    if ((e = hipMalloc(&t.ptrs, ptr_bytes ? ptr_bytes : 16)) != hipSuccess) {
        release();
        return hip_fail("hipMalloc(state pointers)", e);
    }
    if ((e = hipMalloc(&t.scan_seqs, scan_seq_bytes ? scan_seq_bytes : 16)) != hipSuccess) {
        release();
        return hip_fail("hipMalloc(stretch table)", e);
    }
    e = upload_table(t.tiles, plan->tiles.data(), plan->tiles.size() * sizeof(SsmTile), stream);
    if (e == hipSuccess)
        e = upload_table(t.seqs, plan->seqs.data(), plan->seqs.size() * sizeof(SsmSeq), stream);
    if (e == hipSuccess)
        e = upload_table(t.scan_seqs, plan->scan_seqs.data(), plan->scan_seqs.size() * sizeof(SsmScanSeq), stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        release();
        return hip_fail("upload of the plan's tables", e);
    }
    plan->device_tables.push_back(t);
    *out = t;
    return SSM_OK;
}

// ---------------------------------------------------------------- the scan
static int check_state_ptrs(const ssm_plan *plan, const void *const *ptrs, bool *any)
{
    *any = false;
    if (ptrs)
        for (int32_t i = 0; i < plan->batch; ++i) {
            if (!aligned16(ptrs[i]))
                return fail(SSM_ERR_MISALIGNED, "states must be 16-byte aligned");
            *any = *any || ptrs[i] != nullptr;
        }
    return SSM_OK;
}

// Checks shared by ssm_prefill and ssm_prefill_noalloc.  *any_init: a non-null initial state was passed.
static int check_prefill(const ssm_plan *plan, const void *x, const void *dt, const float *A, const void *B,
                         const void *C, const float *D, const void *const *init_state_ptrs, void *y_out,
                         void *state_out, void *workspace, size_t workspace_bytes, bool *any_init)
{
    if (!x || !dt || !A || !B || !C || !D || !y_out)
        return fail(SSM_ERR_INVALID_ARG, "a required tensor pointer is NULL");
    if (plan->n_ckpt > 0 && !state_out)
        return fail(SSM_ERR_INVALID_ARG, "state_out is NULL but the plan has checkpoints");
    const void *ptrs[] = {x, dt, A, B, C, D, y_out, state_out};
    for (const void *p : ptrs)
        if (!aligned16(p))
            return fail(SSM_ERR_MISALIGNED, "device pointers must be 16-byte aligned");
    int rc = check_state_ptrs(plan, init_state_ptrs, any_init);
    if (rc != SSM_OK)
        return rc;
    size_t need = 0;
    (void)ssm_plan_workspace_bytes(plan, &need);
    if (need) {
        if (!workspace || workspace_bytes < need)
            return fail(SSM_ERR_WORKSPACE_TOO_SMALL, "workspace is NULL or smaller than ssm_plan_workspace_bytes");
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
            return fail(SSM_ERR_MISALIGNED, "workspace is not 256-byte aligned");
    }
    return SSM_OK;
}

static void fill_args(const ssm_plan *plan, ScanArgs &args, const void *tiles, const void *seqs,
                      const void *scan_seqs = nullptr)
{
    args.tiles = static_cast<const SsmTile *>(tiles);
    args.seqs = static_cast<const SsmSeq *>(seqs);
    args.scan_seqs = static_cast<const SsmScanSeq *>(scan_seqs);
    args.H = plan->shape.nheads;
    args.P = plan->shape.headdim;
    args.N = plan->shape.d_state;
    args.G = plan->shape.ngroups;
    args.p_split = plan->p_split;
    args.state_dtype = plan->shape.state_dtype;
}

// Launch the scan with the plan's tables at the given device addresses; `d_init_ptrs` is null when no sequence
// starts from a cached state.
static int launch_scan(const ssm_plan *plan, const void *x, const void *dt, const float *A, const void *B,
                       const void *C, const float *D, void *y_out, void *state_out, void *workspace,
                       const void *d_tiles, const void *d_seqs, const void *d_scan_seqs, const void *d_init_ptrs,
                       hipStream_t stream)
{
    ScanArgs args;
    args.x = x;
    args.dt = dt;
    args.A = A;
    args.B = B;
    args.C = C;
    args.D = D;
    args.y = y_out;
    args.state_out = state_out;
    args.init_ptrs = static_cast<const void *const *>(d_init_ptrs);
    fill_args(plan, args, d_tiles, d_seqs, d_scan_seqs);
    const hipError_t e = plan->path == SSM_PATH_MFMA_BF16 ? launch_scan_mfma(plan, args, workspace, stream)
                                                          : launch_scan_valu(plan, args, stream);
    if (e != hipSuccess)
        return hip_fail("kernel launch", e);
    return SSM_OK;
}

extern "C" int ssm_prefill(const ssm_plan_t *plan,
                           const void *x, const void *dt, const float *A,
                           const void *B, const void *C, const float *D,
                           const void *const *init_state_ptrs,
                           void *y_out, void *state_out,
                           void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 || plan->batch == 0)
        return SSM_OK;
    bool any_init = false;
    int rc = check_prefill(plan, x, dt, A, B, C, D, init_state_ptrs, y_out, state_out, workspace, workspace_bytes,
                           &any_init);
    if (rc != SSM_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ssm_plan::DeviceTables t;
    rc = device_tables(plan, stream, &t);
    if (rc != SSM_OK)
        return rc;
    if (any_init) {
        const hipError_t e = upload_table(t.ptrs, init_state_ptrs, (size_t)plan->batch * sizeof(void *), stream);
        if (e != hipSuccess)
            return hip_fail("upload of the initial-state pointers", e);
    }
    return launch_scan(plan, x, dt, A, B, C, D, y_out, state_out, workspace, t.tiles, t.seqs, t.scan_seqs,
                       any_init ? t.ptrs : nullptr, stream);
}

// ---------------------------------------------------------------- the scan for callers that cannot allocate
// The plan's tile table, its sequence and stretch tables and the per-call state pointers go into a fixed device array
// that is part of the library image, in place of the buffers ssm_prefill allocates on a plan's first use.  Every call
// on a GPU shares that GPU's array: calls that overlap on one GPU race.  All tables are rewritten by every call, so
// nothing of an earlier call is read.
constexpr size_t kNoAllocMaxTiles = 16384;
constexpr size_t kNoAllocMaxBatch = 1024;
constexpr size_t kNoAllocMaxStretches = kNoAllocMaxBatch + 256;  // cutting adds fewer than 256 stretches to a batch
constexpr size_t kScratchSeqsOff = kNoAllocMaxTiles * sizeof(SsmTile);
constexpr size_t kScratchPtrsOff = kScratchSeqsOff + kNoAllocMaxBatch * sizeof(SsmSeq);
constexpr size_t kScratchScanSeqsOff = kScratchPtrsOff + kNoAllocMaxBatch * sizeof(void *);
constexpr size_t kScratchBytes = kScratchScanSeqsOff + kNoAllocMaxStretches * sizeof(SsmScanSeq);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, set on first use there
static std::mutex g_scratch_mutex;

static int scratch_on_current_device(unsigned char **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail("hipGetDevice", e);
    if (dev < 0 || dev >= kMaxDevices)
        return fail(SSM_ERR_INVALID_ARG, "device ordinal above 63");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return hip_fail("hipGetSymbolAddress(scratch)", e);
        if (!ptr)
            return fail(SSM_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return SSM_OK;
}

extern "C" int ssm_prefill_noalloc(const ssm_plan_t *plan,
                                   const void *x, const void *dt, const float *A,
                                   const void *B, const void *C, const float *D,
                                   const void *const *init_state_ptrs,
                                   void *y_out, void *state_out,
                                   void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 || plan->batch == 0)
        return SSM_OK;
    if (plan->tiles.size() > kNoAllocMaxTiles || (size_t)plan->batch > kNoAllocMaxBatch ||
        plan->scan_seqs.size() > kNoAllocMaxStretches)
        return fail(SSM_ERR_UNSUPPORTED_SHAPE,
                    "ssm_prefill_noalloc handles at most 16384 tiles and 1024 sequences per call");
    bool any_init = false;
    int rc = check_prefill(plan, x, dt, A, B, C, D, init_state_ptrs, y_out, state_out, workspace, workspace_bytes,
                           &any_init);
    if (rc != SSM_OK)
        return rc;
    unsigned char *base = nullptr;
    rc = scratch_on_current_device(&base);
    if (rc != SSM_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = upload_table(base, plan->tiles.data(), plan->tiles.size() * sizeof(SsmTile), stream);
    if (e == hipSuccess)
        e = upload_table(base + kScratchSeqsOff, plan->seqs.data(), plan->seqs.size() * sizeof(SsmSeq), stream);
    if (e == hipSuccess)
        e = upload_table(base + kScratchScanSeqsOff, plan->scan_seqs.data(), plan->scan_seqs.size() * sizeof(SsmScanSeq),
                         stream);
    if (e == hipSuccess && any_init)
        e = upload_table(base + kScratchPtrsOff, init_state_ptrs, (size_t)plan->batch * sizeof(void *), stream);
    if (e != hipSuccess)
        return hip_fail("upload of the plan's tables into the fixed device array", e);
    return launch_scan(plan, x, dt, A, B, C, D, y_out, state_out, workspace, base, base + kScratchSeqsOff,
                       base + kScratchScanSeqsOff, any_init ? base + kScratchPtrsOff : nullptr, stream);
}

// ---------------------------------------------------------------- roll-forward / decode step
extern "C" int ssm_state_advance(const ssm_plan_t *plan,
                                 const void *x, const void *dt, const float *A,
                                 const void *B, const void *C, const float *D,
                                 void *const *state_ptrs, void *y_out, void *hip_stream)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 || plan->batch == 0)
        return SSM_OK;
    if (!state_advance_supports(plan->shape))
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "ssm_state_advance needs d_state a power of two in 4..256");
    if (!x || !dt || !A || !B || !C || !D || !state_ptrs)
        return fail(SSM_ERR_INVALID_ARG, "a required pointer is NULL");
    const void *ptrs[] = {x, dt, A, B, C, D, y_out};
    for (const void *p : ptrs)
        if (!aligned16(p))
            return fail(SSM_ERR_MISALIGNED, "device pointers must be 16-byte aligned");
    bool any = false;
    int rc = check_state_ptrs(plan, state_ptrs, &any);
    if (rc != SSM_OK)
        return rc;
    if (!any)
        return SSM_OK;  // every sequence is left alone
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ssm_plan::DeviceTables t;
    rc = device_tables(plan, stream, &t);
    if (rc != SSM_OK)
        return rc;
    hipError_t e = upload_table(t.ptrs, state_ptrs, (size_t)plan->batch * sizeof(void *), stream);
    if (e != hipSuccess)
        return hip_fail("upload of the state pointers", e);
    ScanArgs args;
    args.x = x;
    args.dt = dt;
    args.A = A;
    args.B = B;
    args.C = C;
    args.D = D;
    args.y = y_out;
    args.state_out = nullptr;
    args.init_ptrs = nullptr;
    fill_args(plan, args, t.tiles, t.seqs);
    e = launch_state_advance(plan, args, static_cast<void *const *>(t.ptrs), stream);
    if (e != hipSuccess)
        return hip_fail("kernel launch", e);
    return SSM_OK;
}

// ---------------------------------------------------------------- causal convolution in front of the scan
extern "C" int ssm_conv1d_prefill(const ssm_plan_t *plan, int32_t channels, int32_t kernel_width,
                                  const void *in, const float *weight, const float *bias,
                                  const void *const *init_state_ptrs, void *out, void *state_out,
                                  int32_t activation, void *hip_stream)
{
    if (!plan)
        return fail(SSM_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 || plan->batch == 0)
        return SSM_OK;
    if (!conv1d_supports(channels, kernel_width, plan->shape.io_dtype))
        return fail(SSM_ERR_UNSUPPORTED_SHAPE, "kernel width must be 1..4 and a channel row a multiple of 16 bytes");
    if (activation != 0 && activation != 1)
        return fail(SSM_ERR_INVALID_ARG, "activation is 0 (identity) or 1 (SiLU)");
    if (!in || !weight || !out)
        return fail(SSM_ERR_INVALID_ARG, "a required pointer is NULL");
    if (plan->n_ckpt > 0 && !state_out)
        return fail(SSM_ERR_INVALID_ARG, "state_out is NULL but the plan has checkpoints");
    const void *ptrs[] = {in, weight, bias, out, state_out};
    for (const void *p : ptrs)
        if (!aligned16(p))
            return fail(SSM_ERR_MISALIGNED, "device pointers must be 16-byte aligned");
    bool any_init = false;
    int rc = check_state_ptrs(plan, init_state_ptrs, &any_init);
    if (rc != SSM_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ssm_plan::DeviceTables t;
    rc = device_tables(plan, stream, &t);
    if (rc != SSM_OK)
        return rc;
    if (any_init) {
        const hipError_t e = upload_table(t.ptrs, init_state_ptrs, (size_t)plan->batch * sizeof(void *), stream);
        if (e != hipSuccess)
            return hip_fail("upload of the initial-state pointers", e);
    }
    const hipError_t e = launch_conv1d_prefill(
        plan, static_cast<const SsmTile *>(t.tiles), static_cast<const SsmSeq *>(t.seqs), channels, kernel_width, in,
        weight, bias, any_init ? static_cast<const void *const *>(t.ptrs) : nullptr, out, state_out, activation,
        stream);
    if (e != hipSuccess)
        return hip_fail("kernel launch", e);
    return SSM_OK;
}

static thread_local hipEvent_t g_profile_event[2] = {nullptr, nullptr};

hipEvent_t ssm_profile_event(int which) { return g_profile_event[which & 1]; }

extern "C" void ssm_profile_mark(void *after_first_kernel, void *after_second_kernel)
{
    g_profile_event[0] = static_cast<hipEvent_t>(after_first_kernel);
    g_profile_event[1] = static_cast<hipEvent_t>(after_second_kernel);
}

extern "C" void ssm_plan_destroy(ssm_plan_t *plan)
{
    if (!plan)
        return;
    for (const ssm_plan::DeviceTables &t : plan->device_tables) {
        (void)hipFree(t.tiles);
        (void)hipFree(t.seqs);
        (void)hipFree(t.scan_seqs);
        (void)hipFree(t.ptrs);
    }
    delete plan;
}
