// Roll-forward of cached states (Section 4.1: a kernel that rolls a checkpointed state forward by a few tokens to
// reach an exact position; with one token per sequence it is the decode step).  Every sequence of the batch brings
// its own [H,P,N] state (fp32, or fp16 / bf16 as a cache stores it), which is advanced IN PLACE by the sequence's
// tokens with the token recurrence itself,
//
//     a = exp(dt A),   S[p,n] = a S[p,n] + (dt x[p]) B[n],   y[p] = sum_n C[n] S[p,n] + D x[p],
//
// in fp32 on the vector ALUs: for a handful of tokens the work is reading and writing the state once (2 x 4 MiB per
// sequence at H=128, P=64, N=128), i.e. HBM-bound streaming, and the chunked machinery of the scan buys nothing.
//
// One workgroup of 256 threads owns (sequence, head, slice of state rows).  A state row of N floats is spread over
// N/4 neighbouring lanes (16 bytes each, so every state access is a contiguous run of 16-byte pieces); a thread keeps
// up to 8 rows in registers across the sequence's tokens.  y needs the sum over a row: a DPP prefix sum inside the
// lane group, taken from the group's last lane.
#include "device_utils.h"

namespace {

constexpr int kAdvThreads = 256;
constexpr int kAdvMaxRows = 8;  // state rows per thread
constexpr float kAdvLog2e = 1.4426950408889634f;

#define ADV_DPP(v, ctrl, row_mask)                                                                            \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (float)(v)), (ctrl),     \
                                                          (row_mask), 0xF, true))

// Sum over each group of LPR neighbouring lanes (LPR a power of two, groups aligned); valid in the last lane of a group.
template <int LPR>
__device__ __forceinline__ float group_sum_in_last_lane(float v)
{
    if (LPR >= 2)
        v += ADV_DPP(v, 0x111, 0xF);  // row_shr:1
    if (LPR >= 4)
        v += ADV_DPP(v, 0x112, 0xF);  // row_shr:2
    if (LPR >= 8)
        v += ADV_DPP(v, 0x114, 0xF);  // row_shr:4
    if (LPR >= 16)
        v += ADV_DPP(v, 0x118, 0xF);  // row_shr:8
    if (LPR >= 32)
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF,
                                                                   false));  // row_bcast:15 into rows 1 and 3
    if (LPR >= 64)
        v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF,
                                                                   false));  // row_bcast:31 into rows 2 and 3
    return v;
}

template <typename IO> struct Vec4;
template <> struct Vec4<float> {
    static __device__ __forceinline__ float4 load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
};
template <> struct Vec4<bf16_t> {
    static __device__ __forceinline__ float4 load(const bf16_t *p)
    {
        const uint2 u = *reinterpret_cast<const uint2 *>(p);
        return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                           __uint_as_float(u.y & 0xffff0000u));
    }
};

// Storage type of the cached states: fp32, or fp16 / bf16 as a cache keeps them (Section 5.1: FP16 everywhere;
// Appendix A.1: 2 bytes per state element), which halves the bytes this kernel moves.  Arithmetic stays fp32; a
// reduced-precision state is rounded once, to nearest even, when it is written back.
enum { ADV_STATE_F32 = SSM_ST_F32, ADV_STATE_F16 = SSM_ST_F16, ADV_STATE_BF16 = SSM_ST_BF16 };
template <int ST> struct StateVec;
template <> struct StateVec<ADV_STATE_F32> {
    typedef float elem;
    static __device__ __forceinline__ float4 load(const elem *p) { return *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ void store(elem *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
};
template <> struct StateVec<ADV_STATE_F16> {
    typedef _Float16 elem;
    typedef __attribute__((ext_vector_type(4))) _Float16 h4;
    static __device__ __forceinline__ float4 load(const elem *p)
    {
        const h4 h = *reinterpret_cast<const h4 *>(p);
        return make_float4((float)h[0], (float)h[1], (float)h[2], (float)h[3]);
    }
    static __device__ __forceinline__ void store(elem *p, float4 v)
    {
        const h4 h = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
        *reinterpret_cast<h4 *>(p) = h;
    }
};
template <> struct StateVec<ADV_STATE_BF16> {
    typedef bf16_t elem;
    static __device__ __forceinline__ float4 load(const elem *p) { return Vec4<bf16_t>::load(p); }
    static __device__ __forceinline__ void store(elem *p, float4 v)
    {
        *reinterpret_cast<uint2 *>(p) = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                                                   (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
    }
};

struct AdvanceArgs {
    const void *x, *dt, *B, *C;
    const float *A, *D;
    void *y;                   // may be null
    void *const *state_ptrs;   // [batch] device pointers, each [H,P,N] in the state type; null = leave the sequence alone
    const SsmTile *tiles;
    const SsmSeq *seqs;
    int H, P, N, G;
    int rows_per_thread;       // 1..kAdvMaxRows
    int slices;                // workgroups per (sequence, head)
};

template <typename IO, int LPR, int ST>
__global__ __launch_bounds__(kAdvThreads) void ssm_advance_kernel(AdvanceArgs a)
{
    typedef typename StateVec<ST>::elem state_t;
    constexpr int kRowsPerPass = kAdvThreads / LPR;
    const int H = a.H, P = a.P, N = a.N, G = a.G;
    const int slice = blockIdx.x % a.slices;
    const int h = (blockIdx.x / a.slices) % H;
    const int seq = blockIdx.x / (a.slices * H);
    const int g = h / (H / G);
    const int c = threadIdx.x % LPR;   // this thread holds state columns 4c .. 4c+3
    const int rs = threadIdx.x / LPR;  // row slot inside a pass
    const int R = a.rows_per_thread;
    const int p_first = slice * kRowsPerPass * R + rs;  // rows p_first + kRowsPerPass * r

    const SsmSeq sq = a.seqs[seq];
    state_t *state = static_cast<state_t *>(a.state_ptrs[seq]);
    if (sq.tile_end <= sq.tile_begin || state == nullptr)
        return;  // nothing to advance; the whole workgroup leaves

    const IO *x = static_cast<const IO *>(a.x);
    const IO *dt = static_cast<const IO *>(a.dt);
    const IO *Bg = static_cast<const IO *>(a.B);
    const IO *Cg = static_cast<const IO *>(a.C);
    IO *y = static_cast<IO *>(a.y);
    const float Ah = a.A[h] * kAdvLog2e;
    const float Dh = a.D[h];

    float4 S[kAdvMaxRows];
#pragma unroll
    for (int r = 0; r < kAdvMaxRows; ++r) {
        const int p = p_first + kRowsPerPass * r;
        S[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < R && p < P)
            S[r] = StateVec<ST>::load(state + ((size_t)h * P + p) * N + 4 * c);
    }

    for (int ti = sq.tile_begin; ti < sq.tile_end; ++ti) {
        const SsmTile t = a.tiles[ti];
        for (int i = 0; i < t.len; ++i) {
            const size_t tok = (size_t)t.tok0 + i;
            const float dtv = IoTraits<IO>::load(dt + tok * H + h);
            const float decay = __builtin_amdgcn_exp2f(dtv * Ah);
            const float4 b4 = Vec4<IO>::load(Bg + (tok * G + g) * N + 4 * c);
            const float4 c4 = Vec4<IO>::load(Cg + (tok * G + g) * N + 4 * c);
#pragma unroll
            for (int r = 0; r < kAdvMaxRows; ++r) {
                const int p = p_first + kRowsPerPass * r;
                // the row guard is uniform over a lane group, and groups never straddle DPP rows they do not own
                const bool live = r < R && p < P;
                const float xv = live ? IoTraits<IO>::load(x + (tok * H + h) * P + p) : 0.f;
                const float dx = dtv * xv;
                S[r].x = decay * S[r].x + dx * b4.x;
                S[r].y = decay * S[r].y + dx * b4.y;
                S[r].z = decay * S[r].z + dx * b4.z;
                S[r].w = decay * S[r].w + dx * b4.w;
                if (y != nullptr && r < R) {  // uniform over the wave: every lane takes part in the DPP steps
                    const float part = c4.x * S[r].x + c4.y * S[r].y + c4.z * S[r].z + c4.w * S[r].w;
                    const float row = group_sum_in_last_lane<LPR>(part);
                    if (live && c == LPR - 1)
                        IoTraits<IO>::store(y + (tok * H + h) * P + p, row + Dh * xv);
                }
            }
        }
    }

#pragma unroll
    for (int r = 0; r < kAdvMaxRows; ++r) {
        const int p = p_first + kRowsPerPass * r;
        if (r < R && p < P)
            StateVec<ST>::store(state + ((size_t)h * P + p) * N + 4 * c, S[r]);
    }
}

template <typename IO, int LPR>
void launch_lpr(const AdvanceArgs &a, int batch, int state_type, hipStream_t stream)
{
    const dim3 grid((unsigned)(batch * a.H * a.slices)), block(kAdvThreads);
    switch (state_type) {
    case ADV_STATE_F16: hipLaunchKernelGGL((ssm_advance_kernel<IO, LPR, ADV_STATE_F16>), grid, block, 0, stream, a); break;
    case ADV_STATE_BF16: hipLaunchKernelGGL((ssm_advance_kernel<IO, LPR, ADV_STATE_BF16>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((ssm_advance_kernel<IO, LPR, ADV_STATE_F32>), grid, block, 0, stream, a); break;
    }
}

template <typename IO>
hipError_t launch_io(AdvanceArgs &a, int batch, int state_type, hipStream_t stream)
{
    const int lpr = a.N / 4;
    const int rows_per_pass = kAdvThreads / lpr;
    int R = (a.P + rows_per_pass - 1) / rows_per_pass;
    if (R > kAdvMaxRows)
        R = kAdvMaxRows;
    a.rows_per_thread = R;
    a.slices = (a.P + rows_per_pass * R - 1) / (rows_per_pass * R);
    switch (lpr) {
    case 1: launch_lpr<IO, 1>(a, batch, state_type, stream); break;
    case 2: launch_lpr<IO, 2>(a, batch, state_type, stream); break;
    case 4: launch_lpr<IO, 4>(a, batch, state_type, stream); break;
    case 8: launch_lpr<IO, 8>(a, batch, state_type, stream); break;
    case 16: launch_lpr<IO, 16>(a, batch, state_type, stream); break;
    case 32: launch_lpr<IO, 32>(a, batch, state_type, stream); break;
    case 64: launch_lpr<IO, 64>(a, batch, state_type, stream); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

// True if the roll-forward kernel handles this shape: d_state a power of two between 4 and 256.
bool state_advance_supports(const ssm_shape_t &s)
{
    const int n = s.d_state;
    return n >= 4 && n <= 256 && (n & (n - 1)) == 0;
}

// Advance the state of every sequence of the plan in place by the sequence's tokens; `d_state_ptrs` is a device array
// of plan->batch device pointers to states in the plan's state type.  y may be null.
// Checkpoints of the plan are ignored (the result is the in-place state after the last token).
hipError_t launch_state_advance(const ssm_plan *plan, const ScanArgs &args, void *const *d_state_ptrs,
                                hipStream_t stream)
{
    const int state_type = args.state_dtype;
    if (!state_advance_supports(plan->shape) || state_type < ADV_STATE_F32 || state_type > ADV_STATE_BF16)
        return hipErrorInvalidValue;
    if (plan->batch == 0 || plan->tiles.empty())
        return hipSuccess;
    AdvanceArgs a;
    a.x = args.x;
    a.dt = args.dt;
    a.B = args.B;
    a.C = args.C;
    a.A = args.A;
    a.D = args.D;
    a.y = args.y;
    a.state_ptrs = d_state_ptrs;
    a.tiles = args.tiles;
    a.seqs = args.seqs;
    a.H = args.H;
    a.P = args.P;
    a.N = args.N;
    a.G = args.G;
    return plan->shape.io_dtype == SSM_DT_F32 ? launch_io<float>(a, plan->batch, state_type, stream)
                                              : launch_io<bf16_t>(a, plan->batch, state_type, stream);
}
