// Causal depthwise convolution in front of the SSM scan, with cached-state resume and state checkpoints (the
// conv_1d state of Appendix A.1, "Memory footprint").  For channel c, kernel width K <= 4 and the sequence-local
// token t:
//
//     out[t,c] = act( bias[c] + sum_{j<K} w[c,j] z[t-K+1+j, c] ),   act = identity or SiLU
//
// where z is the sequence's input, continued to the left by the cached prefix's last inputs (or zeros).  The state
// after p tokens is the last K inputs of every channel, oldest first, in the storage type of the input (a copy of
// inputs, so nothing is lost); a resumed sequence passes such a state back.
//
// The work is streaming: 2 bytes in and 2 bytes out per (token, channel) in bf16.  It uses the tile table of the
// scan's plan, whose tiles never cross a sequence boundary and end at every checkpoint: one workgroup takes one tile
// and a block of channels, a thread walks the tile's tokens for 16 bytes' worth of neighbouring channels with the
// last K inputs in registers, so every access is a contiguous run of 16-byte pieces.  The K-1 tokens in front of a
// tile are read again (from the previous tile's tokens, or from the cached state at the start of a sequence).
#include "device_utils.h"

namespace {

constexpr int kConvThreads = 256;
constexpr int kConvMaxK = 4;

template <typename IO> struct ConvVec;
template <> struct ConvVec<float> {
    static constexpr int kLanes = 4;  // channels per thread: 16 bytes
    static __device__ __forceinline__ void load(const float *p, float *v)
    {
        const float4 f = *reinterpret_cast<const float4 *>(p);
        v[0] = f.x, v[1] = f.y, v[2] = f.z, v[3] = f.w;
    }
    static __device__ __forceinline__ void store(float *p, const float *v)
    {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct ConvVec<bf16_t> {
    static constexpr int kLanes = 8;
    static __device__ __forceinline__ void load(const bf16_t *p, float *v)
    {
        const uint4 u = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __uint_as_float(w[e] << 16);
            v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float *v)
    {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            w[e] = (uint32_t)f32_to_bf16(v[2 * e]) | ((uint32_t)f32_to_bf16(v[2 * e + 1]) << 16);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

struct ConvArgs {
    const void *in;                 // [T,Cch] storage type
    const float *w;                 // [Cch,K]
    const float *bias;              // [Cch] or null
    void *out;                      // [T,Cch] storage type
    const void *const *init_ptrs;   // null, or [batch] device pointers (null entry = zeros) to [Cch,K] storage type
    void *state_out;                // [n_ckpt,Cch,K] storage type
    const SsmTile *tiles;
    const SsmSeq *seqs;
    int Cch, act, n_tiles, blocks_per_tile;
};

template <typename IO, int K>
__global__ __launch_bounds__(kConvThreads) void ssm_conv1d_kernel(ConvArgs a)
{
    constexpr int V = ConvVec<IO>::kLanes;
    const int tile = blockIdx.x / a.blocks_per_tile;
    const int cb = blockIdx.x % a.blocks_per_tile;
    const int c0 = (cb * kConvThreads + threadIdx.x) * V;  // first channel of this thread
    const int Cch = a.Cch;
    if (tile >= a.n_tiles || c0 >= Cch)
        return;  // no barriers in this kernel: threads may leave on their own
    const SsmTile t = a.tiles[tile];
    const int seq_tok0 = a.tiles[a.seqs[t.seq].tile_begin].tok0;
    const int lp = t.tok0 - seq_tok0;  // tokens of this sequence in front of the tile

    const IO *__restrict__ in = static_cast<const IO *>(a.in);  // the caller keeps in and out apart
    IO *__restrict__ out = static_cast<IO *>(a.out);
    const IO *init = a.init_ptrs ? static_cast<const IO *>(a.init_ptrs[t.seq]) : nullptr;

    float wk[K][V], bias[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        bias[e] = a.bias ? a.bias[c0 + e] : 0.f;
#pragma unroll
        for (int j = 0; j < K; ++j)
            wk[j][e] = a.w[(size_t)(c0 + e) * K + j];
    }

    // hist[j] = the input j+1 tokens in front of the current one (j = 0 newest); K entries so that the state,
    // which also holds the input K-1 places back from its last token, can be written from registers
    float hist[K][V];
#pragma unroll
    for (int j = 0; j < K; ++j) {
#pragma unroll
        for (int e = 0; e < V; ++e)
            hist[j][e] = 0.f;
        const int back = j + 1;  // tokens back from the tile's first token
        if (lp - back >= 0) {
            ConvVec<IO>::load(in + (size_t)(t.tok0 - back) * Cch + c0, hist[j]);
        } else if (init) {
            // sequence-local index lp + 1 - back <= 0 is entry K - 1 + (lp + 1 - back) of the cached state
            const int m = K - 1 + (lp + 1 - back);
            if (m >= 0) {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    hist[j][e] = IoTraits<IO>::load(init + (size_t)(c0 + e) * K + m);
            }
        }
    }

    // Groups of kAhead tokens: the group's rows are requested together, then consumed in order, so that a thread has
    // several loads in flight instead of one per trip.
    constexpr int kAhead = 8;
    for (int i0 = 0; i0 < t.len; i0 += kAhead) {
      float row[kAhead][V];
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
          const int i = i0 + u < t.len ? i0 + u : t.len - 1;  // past the end: the last row again, unused
          ConvVec<IO>::load(in + ((size_t)t.tok0 + i) * Cch + c0, row[u]);
      }
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        if (i0 + u >= t.len)
            break;
        const size_t tok = (size_t)t.tok0 + i0 + u;
        float cur[V], v[V];
#pragma unroll
        for (int e = 0; e < V; ++e)
            cur[e] = row[u][e];
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float acc = bias[e];
            // oldest first, as the definition is written: w[c,j] meets the input K-1-j places back
#pragma unroll
            for (int j = 0; j < K - 1; ++j)
                acc += wk[j][e] * hist[K - 2 - j][e];
            acc += wk[K - 1][e] * cur[e];
            if (a.act == 1)
                acc = acc * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * acc));
            v[e] = acc;
        }
        ConvVec<IO>::store(out + tok * Cch + c0, v);
#pragma unroll
        for (int j = K - 1; j > 0; --j)
#pragma unroll
            for (int e = 0; e < V; ++e)
                hist[j][e] = hist[j - 1][e];
#pragma unroll
        for (int e = 0; e < V; ++e)
            hist[0][e] = cur[e];
      }
    }

    if (t.ckpt_slot >= 0) {
        // the last K inputs, oldest first: hist[K-1] .. hist[0]
        IO *st = static_cast<IO *>(a.state_out) + ((size_t)t.ckpt_slot * Cch + c0) * K;
#pragma unroll
        for (int e = 0; e < V; ++e)
#pragma unroll
            for (int m = 0; m < K; ++m)
                IoTraits<IO>::store(st + (size_t)e * K + m, hist[K - 1 - m][e]);
    }
}

}  // namespace

// True if the convolution kernel handles the request: width 1..4 and channel rows that are whole 16-byte pieces.
bool conv1d_supports(int channels, int K, int io_dtype)
{
    const int v = io_dtype == SSM_DT_F32 ? 4 : 8;
    return K >= 1 && K <= kConvMaxK && channels > 0 && channels % v == 0;
}

// Launch over the tiles of `plan` (any shape: only its tile table, sequence table and storage type are used).
// `d_init_ptrs` is null or a device array of plan->batch device pointers; `state_out` may be null if the plan has no
// checkpoints.
hipError_t launch_conv1d_prefill(const ssm_plan *plan, const SsmTile *d_tiles, const SsmSeq *d_seqs, int channels,
                                 int K, const void *in, const float *w, const float *bias,
                                 const void *const *d_init_ptrs, void *out, void *state_out, int act,
                                 hipStream_t stream)
{
    if (!conv1d_supports(channels, K, plan->shape.io_dtype))
        return hipErrorInvalidValue;
    const int n_tiles = (int)plan->tiles.size();
    if (n_tiles == 0)
        return hipSuccess;
    const int v = plan->shape.io_dtype == SSM_DT_F32 ? 4 : 8;
    ConvArgs a;
    a.in = in;
    a.w = w;
    a.bias = bias;
    a.out = out;
    a.init_ptrs = d_init_ptrs;
    a.state_out = state_out;
    a.tiles = d_tiles;
    a.seqs = d_seqs;
    a.Cch = channels;
    a.act = act;
    a.n_tiles = n_tiles;
    a.blocks_per_tile = (channels + kConvThreads * v - 1) / (kConvThreads * v);
    const dim3 grid((unsigned)n_tiles * (unsigned)a.blocks_per_tile);
    const bool f32 = plan->shape.io_dtype == SSM_DT_F32;
#define SSM_CONV_LAUNCH(KW)                                                                                  \
    case KW:                                                                                                 \
        if (f32)                                                                                             \
            hipLaunchKernelGGL((ssm_conv1d_kernel<float, KW>), grid, dim3(kConvThreads), 0, stream, a);      \
        else                                                                                                 \
            hipLaunchKernelGGL((ssm_conv1d_kernel<bf16_t, KW>), grid, dim3(kConvThreads), 0, stream, a);     \
        break;
    switch (K) {
        SSM_CONV_LAUNCH(1)
        SSM_CONV_LAUNCH(2)
        SSM_CONV_LAUNCH(3)
        SSM_CONV_LAUNCH(4)
    default: return hipErrorInvalidValue;
    }
#undef SSM_CONV_LAUNCH
    return hipGetLastError();
}
