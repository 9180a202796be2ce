// Matrix-core scan for gfx950: d_state 128, headdim a multiple of 32, bf16 x/dt/B/C/y, fp32 A/D, cached states in
// fp32, fp16 or bf16.
//
// Per tile of q <= 64 tokens starting after token s, with l_i = A * sum_{k<=i} dt_k inside the tile:
//
//   Gm[i,j] = (C_i.B_j) e^{l_i-l_j} dt_j   for j <= i, else 0   (masked score)
//   y_i     = e^{l_i} (S_s C_i) + sum_j Gm[i,j] x_j + D x_i
//   S_e     = e^{l_q} S_s + sum_j (e^{l_q-l_j} dt_j x_j) B_j^T
//
// Only the last line chains one tile to the next, and only through an element-wise update of S; everything else
// of a tile (scores, Gm.x, the tile-local state sum_j (...) B_j^T) is independent of the tiles before it.
//
// Two kernels.
//
// ssm_prep_kernel, one workgroup per (tile, group): what the heads of a group share.  B and C of the tile are read
// once with coalesced rows, converted bf16 -> fp16 (exact for normal values) and written back in the register image
// of the matrix-core operands the scan needs (B^T for the state update, C for S.C), together with the raw score
// blocks C_i.B_j and the tile's dt transposed to head-major.  The scan then loads every operand with fully
// contiguous 1 KiB wave loads straight into registers: B and C never pass through its LDS.
//
// ssm_scan_mfma_kernel, one workgroup per (sequence, head, slice of 32 or 64 channels).  The waves of a workgroup
// take the sequence's tiles round-robin and each wave computes ALL of its tile: tables of decay factors, the
// tile-local state, S.C, the masked scores, Gm.x, y.  The running state S lives in LDS as the register image of the
// accumulators of the tile-local state; the wave whose turn it is reads it, adds its tile-local state
// (S <- e^{l_q} S + local), writes it back and uses the value it read for S.C.  The hand-off goes block by block of
// 32 state indices; a counter per block in LDS says how many tiles have left their state there, and the wave of tile
// k waits for the counter to reach k before it touches the block.  Nothing else orders the waves: there is no
// workgroup barrier in the loop, each wave runs at its own pace, and 8 or 12 tiles are in flight per workgroup to
// hide latencies.  A wave waits only for the wave of the tile before its own, which never waits for it, so the
// waits cannot form a cycle; they are bounded all the same.
//
// The blocks of 32 state indices are streamed through the registers: the B^T operand of a block, its part of the
// tile-local state, its hand-off and its part of S.C, then the next block; the intra-tile term comes last and is
// added onto e^{l_i} (S C_i) in the same accumulators.  x and y of a tile share one LDS tile per wave.
//
// With 64 channels per workgroup (two halves of 32) one set of operand loads (B^T, C, raw scores: 38 KiB per tile)
// serves twice the rows: 54 KiB per 64 channels and tile instead of 2 x 47 KiB.  What limits the scan is the rate at
// which a compute unit can pull operands through its L1, so this is the better variant whenever it still has enough
// workgroups to fill the GPU (the plan decides); otherwise 32 channels per workgroup.
//
// Rounding: operands of the two long contractions (state update, S.C) are fp16 (11 bits: the decay-weighted x, the
// copy of S, B and C), those of Gm.x are bf16 (x as stored, Gm rounded once); decay exponents, accumulators, the
// carried state and checkpoints are fp32.
#include <mutex>

#include "device_utils.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kQ = kMfmaTileTokens;  // 64 tokens per tile
constexpr int kN = 128;              // d_state
#ifndef SSM_SCAN_WAVES
#define SSM_SCAN_WAVES 8
#endif
#ifndef SSM_SCAN_WAVES_NARROW
#define SSM_SCAN_WAVES_NARROW 12
#endif
constexpr int kWavesWide = SSM_SCAN_WAVES;           // waves per workgroup of the scan, 64 channels per workgroup
constexpr int kWavesNarrow = SSM_SCAN_WAVES_NARROW;  // 32 channels per workgroup
constexpr int kSpinLimit = 1 << 16;      // polls of a hand-off counter before a wave gives up waiting (milliseconds)
constexpr float kLog2e = 1.4426950408889634f;

// Operand images of one (tile, group) in the workspace, in uint4 units of 64 lanes each.
constexpr int kCfWords = 2 * 8 * 64;  // C:   [token half][k-step of 16 state indices][lane]
constexpr int kBfWords = 4 * 4 * 64;  // B^T: [block of 32 state indices][k-step of 16 tokens][lane]
constexpr int kCbWords = 3 * 2 * 64;  // raw score blocks: [block][half of the 16 accumulator elements][lane]
static_assert((kCfWords + kBfWords + kCbWords) * 16 == kMfmaTileGroupBytes, "workspace layout");

__device__ __forceinline__ s16x4 lds_tr4(const void *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
}

// 8 k-values of a transposed operand: two groups of 4 consecutive rows of a row-major tile of 16-bit elements.
// The 16 lanes of a group pass the addresses of 4 rows x (4 lanes x 4 elements); lane i of the group receives
// column i of that 4x16 block.
__device__ __forceinline__ uint4 lds_frag_tr(const void *p_lo, const void *p_hi)
{
    const s16x4 lo = lds_tr4(p_lo), hi = lds_tr4(p_hi);
    return __builtin_bit_cast(uint4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ uint32_t pack2_f16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

__device__ __forceinline__ float f16_lo(uint32_t u) { return (float)__builtin_bit_cast(f16x2, u)[0]; }
__device__ __forceinline__ float f16_hi(uint32_t u) { return (float)__builtin_bit_cast(f16x2, u)[1]; }
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Loads and stores of the tile loop go through buffer descriptors: a wave-uniform base and size in scalar registers,
// one 32-bit byte offset per lane and a uniform offset, so that no address arithmetic runs on the vector ALUs.  The
// loads are issued phases ahead of their use; the scheduling fences at the phase ends keep them where they are
// written.  Every access stays inside its descriptor's range.  The one use of the hardware's range check is a
// descriptor of size zero, through which a wave that has no next tile issues its look-ahead loads: they return
// zeros without touching memory (and their base address is valid memory in any case).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    // raw buffer (stride 0) of `bytes` bytes; the flags word selects 32-bit data, as for any untyped access on gfx9
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    const auto v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)uniform_off, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void buf_store16(rsrc_t r, uint32_t lane_off, uint32_t uniform_off, const uint4 &d)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = {d.x, d.y, d.z, d.w};
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_off, (int)uniform_off, 0);
}

// Wait for this wave's own LDS traffic (LDS executes a wave's accesses in order).
__device__ __forceinline__ void lds_wait()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// Workgroup barrier that orders LDS traffic only: global loads issued for later phases stay in flight.  Global
// memory written by these kernels is never read back by the same launch.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Boundary between two stretches of the scan's tile routine: the instruction scheduler moves nothing across it, so
// loads are issued where they are written, stretches ahead of their use.
__device__ __forceinline__ void phase_end()
{
    __builtin_amdgcn_sched_barrier(0);
}

// The hand-off counters are read and written as LDS words, with DS instructions.  Through a generic pointer a volatile
// access becomes a FLAT instruction, and the wait for a FLAT load also waits for every load from device memory that the
// wave has in flight: the prefetched operands would sit on the chain from one tile's hand-off to the next.
typedef __attribute__((address_space(3))) int lds_int_t;

// Wait until `*counter` (in LDS) has reached `want`.  Bounded: a wave that gives up goes on with what is there, so
// that every wave of the grid ends whatever happens.
__device__ __forceinline__ void wait_counter(const int *counter, int want)
{
    const volatile lds_int_t *c = (const volatile lds_int_t *)counter;
    int polls = 0;
    while (__builtin_amdgcn_readfirstlane(*c) < want) {
        if (++polls > kSpinLimit)
            break;
        __builtin_amdgcn_s_sleep(1);
    }
    asm volatile("" ::: "memory");  // what follows in the source reads LDS after the counter
}

// Publish `value` in `*counter` after this wave's earlier LDS writes (LDS executes a wave's accesses in order).
__device__ __forceinline__ void publish_counter(int *counter, int value, int lane)
{
    asm volatile("" ::: "memory");
    if (lane == 0)
        *(volatile lds_int_t *)counter = value;
}

#define SSM_DPP(old, v, ctrl, row_mask, bound)                                                        \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, (float)(old)),       \
                                                          __builtin_bit_cast(int, (float)(v)), (ctrl), \
                                                          (row_mask), 0xF, (bound)))
// Inclusive prefix sum over the 64 lanes of a wave with DPP row shifts and the two row broadcasts.
__device__ __forceinline__ float wave_inclusive_sum(float v)
{
    v += SSM_DPP(0.f, v, 0x111, 0xF, true);   // row_shr:1
    v += SSM_DPP(0.f, v, 0x112, 0xF, true);   // row_shr:2
    v += SSM_DPP(0.f, v, 0x114, 0xF, true);   // row_shr:4
    v += SSM_DPP(0.f, v, 0x118, 0xF, true);   // row_shr:8
    v += SSM_DPP(0.f, v, 0x142, 0xA, false);  // row_bcast:15 into rows 1 and 3
    v += SSM_DPP(0.f, v, 0x143, 0xC, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ float read_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

__device__ __forceinline__ f32x16 zero16()
{
    const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    return z;
}

__device__ __forceinline__ f32x16 mfma_bf16(uint4 a, uint4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                   0);
}

__device__ __forceinline__ f32x16 mfma_f16(uint4 a, uint4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
}

// Four neighbouring elements of a cached state (element index idx) in its storage type.
__device__ __forceinline__ float4 load_state4(const void *base, size_t idx, int state_dtype)
{
    if (state_dtype == SSM_ST_F16) {
        const f16x4 h = *reinterpret_cast<const f16x4 *>(static_cast<const _Float16 *>(base) + idx);
        return make_float4((float)h[0], (float)h[1], (float)h[2], (float)h[3]);
    }
    if (state_dtype == SSM_ST_BF16) {
        const uint2 u = *reinterpret_cast<const uint2 *>(static_cast<const bf16_t *>(base) + idx);
        return make_float4(bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y));
    }
    return *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + idx);
}

__device__ __forceinline__ void store_state4(void *base, size_t idx, float4 v, int state_dtype)
{
    if (state_dtype == SSM_ST_F16) {
        const f16x4 h = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
        *reinterpret_cast<f16x4 *>(static_cast<_Float16 *>(base) + idx) = h;
    } else if (state_dtype == SSM_ST_BF16) {
        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(base) + idx) =
            make_uint2(pack2_bf16(v.x, v.y), pack2_bf16(v.z, v.w));
    } else {
        *reinterpret_cast<float4 *>(static_cast<float *>(base) + idx) = v;
    }
}

// ================================================================ per-(tile, group) operands
constexpr int kPrepThreads = 256;
constexpr int LDPB = kN + 32;  // row stride (halves) of the B tile: transpose reads and 16-byte row reads
constexpr int LDPC = kN + 8;   // row stride of the C tile: row reads only
constexpr int kDtHeads = 64;   // heads per pass of the dt transposition

struct PrepLds {
    _Float16 Bs[kQ][LDPB];
    _Float16 Cs[kQ][LDPC];
    bf16_t dts[kDtHeads][kQ + 2];
};

// 8 bf16 -> 8 fp16 (exact for values whose exponent fp16 can hold)
__device__ __forceinline__ uint4 bf16x8_to_f16x8(uint4 v)
{
    return make_uint4(pack2_f16(bf16_lo(v.x), bf16_hi(v.x)), pack2_f16(bf16_lo(v.y), bf16_hi(v.y)),
                      pack2_f16(bf16_lo(v.z), bf16_hi(v.z)), pack2_f16(bf16_lo(v.w), bf16_hi(v.w)));
}

__global__ __launch_bounds__(kPrepThreads) void ssm_prep_kernel(
    const bf16_t *__restrict__ Bg, const bf16_t *__restrict__ Cg, const bf16_t *__restrict__ dt,
    const SsmTile *__restrict__ tiles, uint4 *__restrict__ frags, bf16_t *__restrict__ dt_t, int H, int G, int n_tiles,
    int parts)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    PrepLds &L = *reinterpret_cast<PrepLds *>(lds_raw);
    // parts = 1: one workgroup per (tile, group), its wave w writes quarter w of the operand images.  parts = 4 (small
    // grids, which would leave most of the GPU idle): four workgroups per (tile, group), workgroup `part` writes
    // quarter `part`, a sixteenth per wave, and transposes a quarter of the heads' dt.
    const int tg = blockIdx.x / parts, part = blockIdx.x % parts;
    const int tile = tg / G, g = tg % G;
    if (tile >= n_tiles)
        return;
    const SsmTile t = tiles[tile];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hg = H / G;  // heads of this group: g * hg .. g * hg + hg - 1
    const int quarter = parts == 1 ? w : part;                 // which quarter of the images this wave works on
    const int sub0 = parts == 1 ? 0 : w, sub1 = parts == 1 ? 4 : w + 1;  // and which sixteenths of it
    const int h_lo = hg * part / parts, h_hi = hg * (part + 1) / parts;   // heads whose dt this workgroup transposes

    // B and C rows, 16 lanes per 256-byte row; rows past the end of a partial tile are zero
    {
        const int row_l = tid >> 4, col = 8 * (tid & 15);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int row = row_l + 16 * kk;
            uint4 vb = make_uint4(0, 0, 0, 0), vc = vb;
            if (row < t.len) {
                const size_t off = (((size_t)t.tok0 + row) * G + g) * kN + col;
                vb = *reinterpret_cast<const uint4 *>(Bg + off);
                vc = *reinterpret_cast<const uint4 *>(Cg + off);
            }
            *reinterpret_cast<uint4 *>(&L.Bs[row][col]) = bf16x8_to_f16x8(vb);
            *reinterpret_cast<uint4 *>(&L.Cs[row][col]) = bf16x8_to_f16x8(vc);
        }
    }
    // dt of the tile, transposed to head-major rows of 64 tokens, kDtHeads heads at a time.  The barrier after the
    // first pass's loads also publishes the B and C tiles.
    for (int h0 = h_lo; h0 < h_hi || h0 == h_lo; h0 += kDtHeads) {  // at least one pass: its barrier is needed
        const int nh = h_hi - h0 < kDtHeads ? (h_hi - h0 > 0 ? h_hi - h0 : 0) : kDtHeads;
        if (h0 > h_lo)
            __syncthreads();  // the previous pass has been written out
        for (int idx = tid; idx < kQ * nh; idx += kPrepThreads) {
            const int tok = idx / nh, hh = idx % nh;
            bf16_t v = 0;
            if (tok < t.len)
                v = dt[((size_t)t.tok0 + tok) * H + g * hg + h0 + hh];
            L.dts[hh][tok] = v;
        }
        __syncthreads();
        for (int idx = tid; idx < kQ * nh; idx += kPrepThreads) {
            const int hh = idx / kQ, tok = idx % kQ;
            dt_t[((size_t)tile * H + g * hg + h0 + hh) * kQ + tok] = L.dts[hh][tok];
        }
    }

    uint4 *out = frags + (size_t)tg * (kCfWords + kBfWords + kCbWords);
    const int i = lane & 31, q = lane >> 5;
    // C operand of S.C: lane (token i of a half, q), k-step ks: state indices 16 ks + 8 (e/4) + 4 q + e%4, the order
    // in which a lane holds a block of the state in its accumulators
    for (int f = sub0; f < sub1; ++f) {
        const int idx = 4 * quarter + f, ih = idx >> 3, ks = idx & 7;
        const _Float16 *row = &L.Cs[32 * ih + i][16 * ks + 4 * q];
        const uint2 lo = *reinterpret_cast<const uint2 *>(row), hi = *reinterpret_cast<const uint2 *>(row + 8);
        out[(ih * 8 + ks) * 64 + lane] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
    // B^T operand of the state update: lane (state index n%32, q), k-step ks: tokens 16 ks + 8 q + e
    {
        const int g4 = lane >> 4;
        const int tr_row = 8 * (g4 >> 1) + ((lane & 15) >> 2);
        const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
        const _Float16 *pb = &L.Bs[tr_row][32 * quarter + tr_col];
        for (int ks = sub0; ks < sub1; ++ks)
            out[kCfWords + (quarter * 4 + ks) * 64 + lane] = lds_frag_tr(pb + 16 * ks * LDPB, pb + (16 * ks + 4) * LDPB);
    }
    // raw score blocks Gm^T[j, i] = B_j . C_i: block 0 keys and queries 0..31, block 1 keys and queries 32..63,
    // block 2 keys 0..31 and queries 32..63; kept as the 16 accumulator elements of every lane, in fp16
    if (quarter < 3 && (parts == 1 || w == 0)) {
        const _Float16 *pb = &L.Bs[(quarter == 1 ? 32 : 0) + i][8 * q];
        const _Float16 *pc = &L.Cs[(quarter == 0 ? 0 : 32) + i][8 * q];
        f32x16 acc = zero16();
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            acc = mfma_f16(*reinterpret_cast<const uint4 *>(pb + 16 * ks), *reinterpret_cast<const uint4 *>(pc + 16 * ks),
                           acc);
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
            out[kCfWords + kBfWords + (quarter * 2 + hf) * 64 + lane] =
                make_uint4(pack2_f16(acc[8 * hf + 0], acc[8 * hf + 1]), pack2_f16(acc[8 * hf + 2], acc[8 * hf + 3]),
                           pack2_f16(acc[8 * hf + 4], acc[8 * hf + 5]), pack2_f16(acc[8 * hf + 6], acc[8 * hf + 7]));
    }
}

// ================================================================ the scan
// The 16 raw scores of a lane (accumulator image of a 32x32 block of Gm^T, fp16) as floats.
__device__ __forceinline__ void unpack_scores(const uint4 &raw0, const uint4 &raw1, float (&v)[16])
{
    const uint32_t rw[8] = {raw0.x, raw0.y, raw0.z, raw0.w, raw1.x, raw1.y, raw1.z, raw1.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        v[2 * e] = f16_lo(rw[e]);
        v[2 * e + 1] = f16_hi(rw[e]);
    }
}

__device__ __forceinline__ void pack_scores(const float (&v)[16], uint4 &g0, uint4 &g1)
{
    g0 = make_uint4(pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]), pack2_bf16(v[4], v[5]), pack2_bf16(v[6], v[7]));
    g1 = make_uint4(pack2_bf16(v[8], v[9]), pack2_bf16(v[10], v[11]), pack2_bf16(v[12], v[13]), pack2_bf16(v[14], v[15]));
}

// Mask and decay a diagonal 32x32 block of raw scores held as the accumulator image of Gm^T (element r of lane
// (i = lane%32, q = lane/32) is key j = 8(r/4) + 4q + r%4), add D on the diagonal, and pack it as the two bf16
// operands of the Gm.x MFMAs.
//   FAST: e^{l_i-l_j} dt_j = e^{l_i-l_31} * e^{l_31-l_j} dt_j from the two factor tables; the caller has checked that
//         the decay over the whole tile stays inside the fp32 exponent range, so neither factor over- or underflows.
//   else: one exponential of l_i - l_j per entry; no factor can overflow whatever the decay.
template <bool FAST, typename Tables>
__device__ __forceinline__ void mask_diag(const uint4 &raw0, const uint4 &raw1, const Tables &tb, int off, int i, int q,
                                          float Dh, uint4 &g0, uint4 &g1)
{
    float v[16];
    unpack_scores(raw0, raw1, v);
    const float fi = FAST ? tb.ri[off + i] : tb.ell2[off + i];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const float4 c4 = *reinterpret_cast<const float4 *>(FAST ? &tb.cf[off + 8 * a + 4 * q] : &tb.cj[off + 8 * a + 4 * q]);
        const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int jl = 8 * a + 4 * q + r;
            const float f = FAST ? fi * cc[r] : exp2_fast(fi - cc[r]);
            float gv = __builtin_fmaf(v[4 * a + r], f, jl == i ? Dh : 0.f);
            v[4 * a + r] = jl <= i ? gv : 0.f;
        }
    }
    pack_scores(v, g0, g1);
}

template <int NC>
struct WaveLdsT {                  // private to one wave
    bf16_t XY[kQ][32 * NC + 8];    // x of the tile as loaded, token major; later y on its way to coalesced stores
    float ell2[kQ];                // l_i * log2(e)
    float cj[kQ];                  // l_j * log2(e) - log2(dt_j)
    float ei[kQ];                  // e^{l_i}
    float wt[kQ];                  // e^{l_q - l_j} dt_j: weight of token j in the state update
    float ri[kQ];                  // e^{l_i - l_31}
    float cf[kQ];                  // e^{l_31 - l_j} dt_j
};

template <int NC, int NW>
struct LdsT {
    float4 S[NC][4][4][64];        // the running state: [channel half][block of 32 n][element group a][lane]
    int done[4];                   // per block of 32 n: how many tiles of the sequence have left their state in it
    int pad[12];
    WaveLdsT<NC> wv[NW];
};

// ST: storage type of cached states (ssm_state_dtype_t); NC: channel halves of 32 per workgroup; NW: waves.
template <int ST, int NC, int NW>
__global__ __launch_bounds__(64 * NW) void ssm_scan_mfma_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ A_, const float *__restrict__ D_, bf16_t *__restrict__ y,
    void *__restrict__ state_out, const void *const *__restrict__ init_ptrs, const uint4 *__restrict__ frags,
    const bf16_t *__restrict__ dt_t, const SsmTile *__restrict__ tiles, const SsmScanSeq *__restrict__ scan_seqs,
    float *__restrict__ tile_decay, float *__restrict__ carry, int H, int P, int G, int p_split, int n_items,
    int n_tiles_all)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int kCh = 32 * NC, LDXY = kCh + 8, kWaves = NW;
    // rows of x / y: 4 NC lanes x 16 bytes per row, 64 / (4 NC) rows per wave instruction
    constexpr int kLanesPerRow = 4 * NC, kRowsPerInstr = 64 / kLanesPerRow, kRowInstrs = kQ / kRowsPerInstr;
    LdsT<NC, NW> &L = *reinterpret_cast<LdsT<NC, NW> *>(lds_raw);

    // The item of this workgroup in the launch order (longest sequences first; same head, then same group, next to
    // each other on one XCD, so that they share its L2).
    const int wg = ssm_launch_item(blockIdx.x, n_items);
    if (wg < 0)
        return;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const int ps = wg % p_split;
    const int h = (wg / p_split) % H;
    const int stretch = scan_seqs[wg / (p_split * H)].by_length;
    const int g = h / (H / G);
    const int pbase = ps * kCh;
    const float Ah = A_[h], Dh = D_[h];
    const SsmScanSeq sq = scan_seqs[stretch];
    const void *init = init_ptrs && sq.init_seq >= 0 ? init_ptrs[sq.init_seq] : nullptr;
    const int tile_begin = sq.tile_begin;
    const int n_tiles = sq.tile_end - sq.tile_begin;
    if (n_tiles <= 0)
        return;  // empty sequence: the whole workgroup leaves before any barrier
    // a stretch that another one continues leaves its last state in a carry slot: fp32, as the register image of the
    // accumulators ([head][block of 32 channels][block of 32 state indices][a][lane] float4), which the kernel that
    // uses it reads back with contiguous wave loads
    const bool carries = carry && sq.carry_out >= 0;
    const rsrc_t carry_to = make_rsrc(
        carry + (carries ? (size_t)sq.carry_out * H * P * kN + ((size_t)h * (P / 32) + pbase / 32) * (16 * 64 * 4) : 0),
        carries ? NC * 16 * 1024 : 0);

    WaveLdsT<NC> &W = L.wv[w];
    const int i = lane & 31, q = lane >> 5;
    const int g4 = lane >> 4;
    const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
    const int tr_row_nat = 8 * (g4 >> 1) + ((lane & 15) >> 2);  // tokens 16 ks + 8 q + e (state update)
    const int tr_row_sc = 4 * (g4 >> 1) + ((lane & 15) >> 2);   // tokens 8 (e/4) + 4 q + e%4 (score order)
    const int tok_l = lane / kLanesPerRow, xcol = 8 * (lane % kLanesPerRow);
    // + 32 c kN (channel half) + 32 nb + 8 a: this lane's 4 state values
    const size_t state_row = ((size_t)h * P + pbase + i) * kN + 4 * q;
    const uint32_t xrow_b = (uint32_t)H * P * 2;                         // bytes per token row of x and y
    const unsigned char *xh = reinterpret_cast<const unsigned char *>(x) + ((size_t)h * P + pbase) * 2;  // uniform
    unsigned char *yh = reinterpret_cast<unsigned char *>(y) + ((size_t)h * P + pbase) * 2;
    const uint32_t xoff_lane = tok_l * xrow_b + xcol * 2;               // row tok_l, this lane's 16 bytes
    const uint32_t lane16 = lane * 16;

    // The state the sequence starts from (its cached state or zero) goes into LDS the way a tile would have left it.
    for (int blk = w; blk < 16 * NC; blk += kWaves) {
        const int c = blk >> 4, nb = (blk >> 2) & 3, a = blk & 3;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (init)
            v = load_state4(init, state_row + (size_t)32 * c * kN + 32 * nb + 8 * a, ST);
        L.S[c][nb][a][lane] = v;
    }
    if (threadIdx.x < 4)
        L.done[threadIdx.x] = 0;
    lds_barrier();  // the only workgroup barrier: the starting state and the counters are in place
    constexpr uint32_t kBfOff = kCfWords * 16, kCbOff = (kCfWords + kBfWords) * 16;
    const unsigned char *img_g = reinterpret_cast<const unsigned char *>(frags) + (size_t)g * kMfmaTileGroupBytes;

    // dt and x of a tile are loaded one tile of this wave ahead (before the epilogue of the current one).  Rows past
    // the end of a partial tile re-read the tile's last row: their weights are zero, so any finite value will do.
    // After its last tile the wave issues these loads once more through descriptors of size zero (on the current
    // tile's addresses): they return zeros without touching memory, and the loop needs no second copy of its tail.
    uint32_t dt_raw = 0;
    uint4 xr[kRowInstrs];
    auto issue_first_loads = [&](int tile_idx, const SsmTile &tl, bool live) {
        const rsrc_t dtr = make_rsrc(dt_t + ((size_t)tile_idx * H + h) * kQ, live ? kQ * 2 : 0);
        dt_raw = __builtin_amdgcn_raw_buffer_load_b16(dtr, lane * 2, 0, 0);
        const rsrc_t xrs =
            make_rsrc(xh + (size_t)tl.tok0 * xrow_b, live ? (uint32_t)(tl.len - 1) * xrow_b + kCh * 2 : 0);
        if (tl.len == kQ) {
#pragma unroll
            for (int kk = 0; kk < kRowInstrs; ++kk)
                xr[kk] = buf_load16(xrs, xoff_lane, (uint32_t)(kRowsPerInstr * kk) * xrow_b);
        } else {
#pragma unroll
            for (int kk = 0; kk < kRowInstrs; ++kk) {
                const int tok = tok_l + kRowsPerInstr * kk < tl.len ? tok_l + kRowsPerInstr * kk : tl.len - 1;
                xr[kk] = buf_load16(xrs, (uint32_t)tok * xrow_b + xcol * 2, 0);
            }
        }
    };
    if (w >= n_tiles)
        return;  // a wave without tiles; no barrier follows
    int tile_idx = __builtin_amdgcn_readfirstlane(tile_begin + w);
    SsmTile t = tiles[tile_idx], t_next = t;
    issue_first_loads(tile_idx, t, true);
    for (int k = w; k < n_tiles; k += kWaves) {  // this wave's tiles
        __builtin_amdgcn_sched_barrier(0);
        const rsrc_t img = make_rsrc(img_g + (size_t)tile_idx * G * kMfmaTileGroupBytes, kMfmaTileGroupBytes);
        // B^T and C for one block of 32 state indices
        uint4 bfb[4], cfr[2][2];
        auto load_b = [&](int nb) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                bfb[ks] = buf_load16(img, lane16, kBfOff + (nb * 4 + ks) * 1024);
        };
        auto load_c = [&](int nb) {
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
                    cfr[ih][hf] = buf_load16(img, lane16, (ih * 8 + 2 * nb + hf) * 1024);
        };
        load_b(0);
        load_c(0);
        phase_end();

        // ---------------- factor tables, x into LDS, decay-weighted x of both channel halves as fp16 operands
        float dl;
        bool fast;
        {
            const float dtj = __uint_as_float(dt_raw << 16);
            const float ell2 = wave_inclusive_sum(dtj * Ah) * kLog2e;
            const float last = read_lane(ell2, 63), e31 = read_lane(ell2, 31);
            dl = exp2_fast(last);   // padded tokens have dt = 0, so this is e^{l_len}
            if (tile_decay && lane == 0)
                tile_decay[(size_t)h * n_tiles_all + tile_idx] = last;  // head-major: a head's tiles side by side
            fast = last > -100.f;   // 2^+-100 is far inside the fp32 range: the two-factor form of the decay is safe
            W.ell2[lane] = ell2;
            W.cj[lane] = ell2 - __builtin_amdgcn_logf(dtj);
            W.ei[lane] = exp2_fast(ell2);
            W.wt[lane] = exp2_fast(last - ell2) * dtj;
            W.ri[lane] = exp2_fast(ell2 - e31);
            W.cf[lane] = exp2_fast(e31 - ell2) * dtj;
#pragma unroll
            for (int kk = 0; kk < kRowInstrs; ++kk)
                *reinterpret_cast<uint4 *>(&W.XY[tok_l + kRowsPerInstr * kk][xcol]) = xr[kk];
        }
        lds_wait();
        uint4 xw[NC][4];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const bf16_t *px = &W.XY[tr_row_nat][32 * c + tr_col];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const uint4 xv = lds_frag_tr(px + 16 * ks * LDXY, px + (16 * ks + 4) * LDXY);
                const float4 w0 = *reinterpret_cast<const float4 *>(&W.wt[16 * ks + 8 * q]);
                const float4 w1 = *reinterpret_cast<const float4 *>(&W.wt[16 * ks + 8 * q + 4]);
                xw[c][ks] = make_uint4(pack2_f16(w0.x * bf16_lo(xv.x), w0.y * bf16_hi(xv.x)),
                                       pack2_f16(w0.z * bf16_lo(xv.y), w0.w * bf16_hi(xv.y)),
                                       pack2_f16(w1.x * bf16_lo(xv.z), w1.y * bf16_hi(xv.z)),
                                       pack2_f16(w1.z * bf16_lo(xv.w), w1.w * bf16_hi(xv.w)));
            }
        }
        const bool more = k + kWaves < n_tiles;
        if (more)  // the descriptor of this wave's next tile
            t_next = tiles[tile_idx + kWaves];
        phase_end();

        // ---------------- per block of 32 state indices: tile-local state, hand-off, S.C
        f32x16 Yo[NC][2];  // [channel half][token half]
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
                Yo[c][ih] = zero16();
        auto block = [&](int nb) {
            f32x16 Sl[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c)
                Sl[c] = zero16();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    Sl[c] = mfma_f16(bfb[ks], xw[c][ks], Sl[c]);
            __builtin_amdgcn_sched_barrier(0);
            if (nb < 3)
                load_b(nb + 1);  // into the registers the MFMAs above have just read
            // S as it was before this tile comes from LDS, where the wave of the previous tile left the block; this
            // tile's S goes back in its place.  The value read also feeds S.C.  The tile-local state is pinned in front
            // of the wait: everything that does not depend on the previous tile is issued before the wave starts to
            // poll, so that only the read, the multiply-add and the write of the block lie between one tile's hand-off
            // and the next.
#pragma unroll
            for (int c = 0; c < NC; ++c)
                asm volatile("" : "+v"(Sl[c]));
            wait_counter(&L.done[nb], k);
            // between one tile's hand-off and the next: read the block, multiply-add, write it back, publish.  What
            // else needs the old or the new value (checkpoint, carry slot, the operand of S.C) comes after.
            float4 sp[NC][4], sn[NC][4];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    sp[c][a] = L.S[c][nb][a][lane];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    sn[c][a] = make_float4(
                        __builtin_fmaf(dl, sp[c][a].x, Sl[c][4 * a + 0]), __builtin_fmaf(dl, sp[c][a].y, Sl[c][4 * a + 1]),
                        __builtin_fmaf(dl, sp[c][a].z, Sl[c][4 * a + 2]), __builtin_fmaf(dl, sp[c][a].w, Sl[c][4 * a + 3]));
                    L.S[c][nb][a][lane] = sn[c][a];
                }
            publish_counter(&L.done[nb], k + 1, lane);
            if (t.ckpt_slot >= 0) {
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const size_t slot_row = (size_t)t.ckpt_slot * H * P * kN + state_row + (size_t)32 * c * kN + 32 * nb;
#pragma unroll
                    for (int a = 0; a < 4; ++a)
                        store_state4(state_out, slot_row + 8 * a, sn[c][a], ST);
                }
            }
            if (carries && k == n_tiles - 1) {
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int a = 0; a < 4; ++a)
                        buf_store16(carry_to, lane16, ((c * 4 + nb) * 4 + a) * 1024, __builtin_bit_cast(uint4, sn[c][a]));
            }
            uint4 s16[NC][2];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
                    s16[c][hf] = make_uint4(pack2_f16(sp[c][2 * hf].x, sp[c][2 * hf].y),
                                            pack2_f16(sp[c][2 * hf].z, sp[c][2 * hf].w),
                                            pack2_f16(sp[c][2 * hf + 1].x, sp[c][2 * hf + 1].y),
                                            pack2_f16(sp[c][2 * hf + 1].z, sp[c][2 * hf + 1].w));
            // S_s C_i over the 32 state indices of this block: two k-steps of 16
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    Yo[c][0] = mfma_f16(s16[c][hf], cfr[0][hf], Yo[c][0]);
                    Yo[c][1] = mfma_f16(s16[c][hf], cfr[1][hf], Yo[c][1]);
                }
            __builtin_amdgcn_sched_barrier(0);
            if (nb < 3)
                load_c(nb + 1);
        };
        block(0);
        block(1);
        phase_end();
        block(2);
        block(3);
        phase_end();

        // ---------------- the intra-tile term, added onto e^{l_i} (S C_i) in the same accumulators: raw scores,
        // decay mask (+ D on the diagonal), x in score order, Gm.x
        uint4 cb[3][2];
#pragma unroll
        for (int blk = 0; blk < 3; ++blk)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                cb[blk][hf] = buf_load16(img, lane16, kCbOff + (blk * 2 + hf) * 1024);
        phase_end();
#pragma unroll
        for (int ih = 0; ih < 2; ++ih) {
            const float ei = W.ei[32 * ih + i];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Yo[c][ih][r] *= ei;
        }
        {
            uint4 gd[2][2], go[2];
            if (fast) {
                mask_diag<true>(cb[0][0], cb[0][1], W, 0, i, q, Dh, gd[0][0], gd[0][1]);
                mask_diag<true>(cb[1][0], cb[1][1], W, 32, i, q, Dh, gd[1][0], gd[1][1]);
            } else {
                mask_diag<false>(cb[0][0], cb[0][1], W, 0, i, q, Dh, gd[0][0], gd[0][1]);
                mask_diag<false>(cb[1][0], cb[1][1], W, 32, i, q, Dh, gd[1][0], gd[1][1]);
            }
            {
                // off-diagonal block (keys 0..31, queries 32..63): unmasked, and both factors of
                // e^{l_i-l_31} * e^{l_31-l_j} dt_j are <= 1 whatever the decay
                float v[16];
                unpack_scores(cb[2][0], cb[2][1], v);
                const float ri = W.ri[32 + i];
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 f4 = *reinterpret_cast<const float4 *>(&W.cf[8 * a + 4 * q]);
                    v[4 * a + 0] *= ri * f4.x;
                    v[4 * a + 1] *= ri * f4.y;
                    v[4 * a + 2] *= ri * f4.z;
                    v[4 * a + 3] *= ri * f4.w;
                }
                pack_scores(v, go[0], go[1]);
            }
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                uint4 xs[2][2];  // x^T of each token half, tokens in the order of the score blocks' rows
#pragma unroll
                for (int ih = 0; ih < 2; ++ih) {
                    const bf16_t *px = &W.XY[32 * ih + tr_row_sc][32 * c + tr_col];
                    xs[ih][0] = lds_frag_tr(px, px + 8 * LDXY);
                    xs[ih][1] = lds_frag_tr(px + 16 * LDXY, px + 24 * LDXY);
                }
                Yo[c][0] = mfma_bf16(xs[0][0], gd[0][0], Yo[c][0]);
                Yo[c][1] = mfma_bf16(xs[1][0], gd[1][0], Yo[c][1]);
                Yo[c][0] = mfma_bf16(xs[0][1], gd[0][1], Yo[c][0]);
                Yo[c][1] = mfma_bf16(xs[1][1], gd[1][1], Yo[c][1]);
                Yo[c][1] = mfma_bf16(xs[0][0], go[0], Yo[c][1]);
                Yo[c][1] = mfma_bf16(xs[0][1], go[1], Yo[c][1]);
            }
        }
        phase_end();
        // the first loads of this wave's next tile, in flight under the epilogue
        issue_first_loads(more ? tile_idx + kWaves : tile_idx, t_next, more);
        phase_end();
        // y on its way to LDS, over the x tile (every read of it has been issued, and LDS runs a wave's accesses in
        // order).  Y^T[p, i]: element r of this lane is channel 32 c + 8(r/4) + 4q + r%4 of token 32 ih + i
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    *reinterpret_cast<uint2 *>(&W.XY[32 * ih + i][32 * c + 8 * a + 4 * q]) =
                        make_uint2(pack2_bf16(Yo[c][ih][4 * a + 0], Yo[c][ih][4 * a + 1]),
                                   pack2_bf16(Yo[c][ih][4 * a + 2], Yo[c][ih][4 * a + 3]));
        lds_wait();

        // ---------------- y from LDS to device memory in whole 128-byte rows
        {
            const rsrc_t yrs = make_rsrc(yh + (size_t)t.tok0 * xrow_b, (uint32_t)(t.len - 1) * xrow_b + kCh * 2);
            if (t.len == kQ) {  // full tile: no predication
#pragma unroll
                for (int m = 0; m < kRowInstrs; ++m)
                    buf_store16(yrs, xoff_lane, (uint32_t)(kRowsPerInstr * m) * xrow_b,
                                *reinterpret_cast<const uint4 *>(&W.XY[tok_l + kRowsPerInstr * m][xcol]));
            } else {
#pragma unroll
                for (int m = 0; m < kRowInstrs; ++m) {
                    const int tok = tok_l + kRowsPerInstr * m;
                    if (tok < t.len)
                        buf_store16(yrs, xoff_lane, (uint32_t)(kRowsPerInstr * m) * xrow_b,
                                    *reinterpret_cast<const uint4 *>(&W.XY[tok][xcol]));
                }
            }
        }
        phase_end();
        t = t_next;
        tile_idx += kWaves;
    }
}


// ================================================================ sequences cut into stretches: the carried states
// A later stretch of a cut sequence was scanned from a zero state.  The recurrence is linear in the state, so what is
// missing is, for token t of the stretch, C_t applied to the state S the stretch truly starts from, decayed from the
// stretch's start to t; for a checkpoint after t the decayed S itself.  S is the state its predecessor ended with (in
// its carry slot, where the scan left it, completed by ssm_carry_kernel when the predecessor is itself a later
// stretch).  The decay only shrinks along the stretch: once it is below 2^-150 nothing is added in fp32 and the rest
// of the stretch is left alone, which for decay rates as trained models have them is all but its first few tiles.
constexpr int kFixThreads = 256;
// A stretch's first kFixFineTiles tiles, where the carried state usually still counts, go to workgroups of 8 tiles
// (two per wave); the rest, which it reaches only when decay is unusually slow, to workgroups of 32 (eight per wave).
#ifndef SSM_FIX_FINE_TILES
#define SSM_FIX_FINE_TILES 96
#endif
constexpr int kFixFineTiles = SSM_FIX_FINE_TILES;
constexpr int kFixFineGroup = 8, kFixCoarseGroup = 32;
static_assert(kFixFineTiles % kFixFineGroup == 0, "whole groups");
// workgroups per (carry slot, head, 64 channels) for stretches of up to `tiles` tiles
__host__ __device__ inline int fix_groups(int tiles)
{
    if (tiles <= kFixFineTiles)
        return (tiles + kFixFineGroup - 1) / kFixFineGroup;
    return kFixFineTiles / kFixFineGroup + (tiles - kFixFineTiles + kFixCoarseGroup - 1) / kFixCoarseGroup;
}
constexpr float kFixCutoffLog2 = -150.f;

constexpr int LDYT = 64 + 4;  // row stride (floats) of a wave's tile of contributions: 32 tokens x 64 channels
struct FixLds {
    float ell2[kFixThreads / 64][kQ];
    uint4 s16[2][4][2][64];  // the carried state of 64 channels as fp16 operands: [channel half][block][k-step][lane]
    float yt[kFixThreads / 64][32][LDYT];
};
struct CarryLds {
    float red[kFixThreads / 64];
};
// The tiles of the first later stretches, by carry slot, as a kernel argument: with few slots (the usual case: one
// long sequence in two to four stretches) a wave of ssm_fix_kernel knows its stretch without a dependent chain of
// loads from the stretch table in front of the one load it needs to decide whether it has work.
constexpr int kFixSlotsInArgs = 8;
struct FixSlots {
    int32_t tile_begin[kFixSlotsInArgs];
    int32_t tile_end[kFixSlotsInArgs];
};

// Turns the carry slots of a sequence cut into three or more stretches into true states: the slot a later stretch
// filled holds what that stretch adds from zero; the state it starts from, decayed over the stretch, is added, one
// stretch after the other.  One workgroup per (carry slot, head); only the one of a sequence's first slot works.
__global__ __launch_bounds__(kFixThreads) void ssm_carry_kernel(float *__restrict__ carry,
                                                                const float *__restrict__ tile_decay,
                                                                const SsmScanSeq *__restrict__ scan_seqs, int H, int P,
                                                                int n_tiles_all)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    CarryLds &L = *reinterpret_cast<CarryLds *>(lds_raw);
    const int c = blockIdx.x / H, h = blockIdx.x % H;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int st = scan_seqs[c].of_slot;           // the stretch that starts from slot c
    if (scan_seqs[st - 1].carry_in >= 0)
        return;                              // not the first later stretch of its sequence
    const size_t hpn = (size_t)H * P * kN, head = (size_t)h * P * kN;
    for (; scan_seqs[st].carry_out >= 0; ++st) {
        const SsmScanSeq sq = scan_seqs[st];
        float part = 0.f;
        for (int t = sq.tile_begin + tid; t < sq.tile_end; t += kFixThreads)
            part += tile_decay[(size_t)h * n_tiles_all + t];
        part = read_lane(wave_inclusive_sum(part), 63);
        lds_barrier();  // the previous round has read the partial sums
        if (lane == 0)
            L.red[w] = part;
        lds_barrier();
        const float f = exp2_fast(L.red[0] + L.red[1] + L.red[2] + L.red[3]);
        const float *in = carry + (size_t)sq.carry_in * hpn + head;
        float *out = carry + (size_t)sq.carry_out * hpn + head;
        for (int idx = 4 * tid; idx < P * kN; idx += 4 * kFixThreads) {
            const float4 a = *reinterpret_cast<const float4 *>(in + idx);
            float4 b = *reinterpret_cast<float4 *>(out + idx);
            b.x = __builtin_fmaf(f, a.x, b.x);
            b.y = __builtin_fmaf(f, a.y, b.y);
            b.z = __builtin_fmaf(f, a.z, b.z);
            b.w = __builtin_fmaf(f, a.w, b.w);
            *reinterpret_cast<float4 *>(out + idx) = b;
        }
    }
}

// One workgroup per (carry slot, head, 64 channels, group of tiles of the stretch that starts from the slot).  The
// workgroup leaves at once if the decay in front of its first tile is below the cutoff; else its four waves convert
// the carried state to fp16 operands in LDS, a quarter each, and then take every fourth tile of the group each.
template <int ST>
__global__ __launch_bounds__(kFixThreads) void ssm_fix_kernel(
    bf16_t *__restrict__ y, void *__restrict__ state_out, const float *__restrict__ carry,
    const float *__restrict__ tile_decay, const uint4 *__restrict__ frags, const bf16_t *__restrict__ dt_t,
    const float *__restrict__ A_, const SsmTile *__restrict__ tiles, const SsmScanSeq *__restrict__ scan_seqs, int H,
    int P, int G, int max_tiles, int n_tiles_all, FixSlots slots, int n_slots)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    FixLds &L = *reinterpret_cast<FixLds *>(lds_raw);
    const int slices = P / 64, groups = fix_groups(max_tiles);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int b = blockIdx.x;
    const int grp = b % groups;
    const bool fine = grp < kFixFineTiles / kFixFineGroup;
    const int j0 = fine ? kFixFineGroup * grp : kFixFineTiles + kFixCoarseGroup * (grp - kFixFineTiles / kFixFineGroup);
    const int group_tiles = fine ? kFixFineGroup : kFixCoarseGroup;
    b /= groups;
    const int slice = b % slices;
    b /= slices;
    const int h = b % H, c = b / H;
    int tile_begin, tile_end;
    if (n_slots <= kFixSlotsInArgs) {
        tile_begin = slots.tile_begin[c];
        tile_end = slots.tile_end[c];
    } else {
        const SsmScanSeq later = scan_seqs[scan_seqs[c].of_slot];
        tile_begin = later.tile_begin;
        tile_end = later.tile_end;
    }
    const int n_tiles = tile_end - tile_begin;
    if (j0 >= n_tiles)
        return;
    const int i = lane & 31, q = lane >> 5;
    const int g = h / (H / G);
    const float Ah = A_[h];

    // Decay from the stretch's start to the start of each of the group's tiles: the sum of the tile decays in front
    // of the group (contiguous wave loads) plus the inclusive sums inside it (at most 32), every wave for itself.
    float before_group, incl;
    {
        const float *d = tile_decay + (size_t)h * n_tiles_all + tile_begin;
        float part = 0.f;
        for (int k = lane; k < j0; k += 64)
            part += d[k];
        before_group = read_lane(wave_inclusive_sum(part), 63);
        incl = wave_inclusive_sum(lane < group_tiles && j0 + lane < n_tiles ? d[j0 + lane] : 0.f);
    }
    auto decay_before = [&](int j) {  // j is uniform in the wave, j0 <= j < j0 + group_tiles
        return j == j0 ? before_group : before_group + read_lane(incl, j - j0 - 1);
    };
    if (before_group < kFixCutoffLog2)
        return;  // the whole workgroup: every wave computes the same value

    // the carried state of the 64 channels as fp16 operands, in the order the scan uses for S.C; the slot holds the
    // register image the scan left: [head][block of 32 channels][block of 32 state indices][a][lane] float4
    const size_t state_row = ((size_t)h * P + 64 * slice + i) * kN + 4 * q;  // + 32 cc kN: channel half cc
    const float4 *S = reinterpret_cast<const float4 *>(carry + (size_t)c * H * P * kN) +
                      ((size_t)h * (P / 32) + 2 * slice) * (16 * 64) + lane;
    {
        const int cc = w >> 1;
#pragma unroll
        for (int n2 = 0; n2 < 2; ++n2)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int nb = 2 * (w & 1) + n2;
                const float4 lo = S[((cc * 4 + nb) * 4 + 2 * hf) * 64], hi = S[((cc * 4 + nb) * 4 + 2 * hf + 1) * 64];
                L.s16[cc][nb][hf][lane] = make_uint4(pack2_f16(lo.x, lo.y), pack2_f16(lo.z, lo.w),
                                                     pack2_f16(hi.x, hi.y), pack2_f16(hi.z, hi.w));
            }
    }
    lds_barrier();  // the only one; after it the waves go their own ways
    const int yrow = lane >> 3, ycol = 8 * (lane & 7);  // rows of y: 8 lanes x 16 bytes, 8 rows per wave instruction
    const uint32_t lane16 = lane * 16;
    for (int r = 0; r < group_tiles / 4; ++r) {
      const int j = j0 + 4 * r + w;
      if (j >= n_tiles)
          break;
      float cum = decay_before(j);
      if (cum < kFixCutoffLog2)
          break;
      {
        const int tile_idx = tile_begin + j;
        const SsmTile t = tiles[tile_idx];
        const rsrc_t img = make_rsrc(reinterpret_cast<const unsigned char *>(frags) +
                                         ((size_t)tile_idx * G + g) * kMfmaTileGroupBytes,
                                     kMfmaTileGroupBytes);
        // per token half: C operands and y as it stands (whole 128-byte rows; rows past the end of a partial tile
        // re-read its last row); the loads of the second half are issued before the first half's y is updated
        uint4 cfr[8], yo[2][4];
        auto issue_loads = [&](int ih) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                cfr[ks] = buf_load16(img, lane16, (ih * 8 + ks) * 1024);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int tok = 32 * ih + 8 * m + yrow < t.len ? 32 * ih + 8 * m + yrow : t.len - 1;
                yo[ih][m] = *reinterpret_cast<const uint4 *>(y + ((size_t)(t.tok0 + tok) * H + h) * P + 64 * slice + ycol);
            }
        };
        // element r of an accumulator: channel 32 cc + 8 (r / 4) + 4 q + r % 4 of token 32 ih + i
        auto contribution_to_lds = [&](float f) {
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                f32x16 acc = zero16();
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    acc = mfma_f16(L.s16[cc][ks >> 1][ks & 1][lane], cfr[ks], acc);
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    *reinterpret_cast<float4 *>(&L.yt[w][i][32 * cc + 8 * a + 4 * q]) =
                        make_float4(f * acc[4 * a + 0], f * acc[4 * a + 1], f * acc[4 * a + 2], f * acc[4 * a + 3]);
            }
            lds_wait();
        };
        auto update_y = [&](int ih) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float4 d0 = *reinterpret_cast<const float4 *>(&L.yt[w][8 * m + yrow][ycol]);
                const float4 d1 = *reinterpret_cast<const float4 *>(&L.yt[w][8 * m + yrow][ycol + 4]);
                const uint4 o = yo[ih][m];
                if (32 * ih + 8 * m + yrow < t.len)
                    *reinterpret_cast<uint4 *>(y + ((size_t)(t.tok0 + 32 * ih + 8 * m + yrow) * H + h) * P + 64 * slice + ycol) =
                        make_uint4(pack2_bf16(bf16_lo(o.x) + d0.x, bf16_hi(o.x) + d0.y),
                                   pack2_bf16(bf16_lo(o.y) + d0.z, bf16_hi(o.y) + d0.w),
                                   pack2_bf16(bf16_lo(o.z) + d1.x, bf16_hi(o.z) + d1.y),
                                   pack2_bf16(bf16_lo(o.w) + d1.z, bf16_hi(o.w) + d1.w));
            }
            lds_wait();  // the tile of contributions is rewritten next
        };
        issue_loads(0);
        const float dtj = __uint_as_float((uint32_t)dt_t[((size_t)tile_idx * H + h) * kQ + lane] << 16);
        phase_end();
        const float ell2 = wave_inclusive_sum(dtj * Ah) * kLog2e;
        const float last = read_lane(ell2, 63);
        L.ell2[w][lane] = ell2;
        lds_wait();
        const float f0 = exp2_fast(cum + L.ell2[w][i]), f1 = exp2_fast(cum + L.ell2[w][32 + i]);
        lds_wait();  // the row is rewritten in the next round
        contribution_to_lds(f0);
        phase_end();
        issue_loads(1);
        phase_end();
        update_y(0);
        contribution_to_lds(f1);
        update_y(1);
        cum += last;
        if (t.ckpt_slot >= 0 && cum >= kFixCutoffLog2) {  // the state after the tile: + the decayed carried state
            const float fs = exp2_fast(cum);
            const size_t slot = (size_t)t.ckpt_slot * H * P * kN;
#pragma unroll 1
            for (int cn = 0; cn < 8; ++cn)  // rare, and kept small: not unrolled
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const int cc = cn >> 2, nb = cn & 3;
                        const size_t idx = state_row + (size_t)32 * cc * kN + 32 * nb + 8 * a;
                        const float4 sv = S[((cc * 4 + nb) * 4 + a) * 64];
                        float4 v = load_state4(state_out, slot + idx, ST);
                        v.x = __builtin_fmaf(fs, sv.x, v.x);
                        v.y = __builtin_fmaf(fs, sv.y, v.y);
                        v.z = __builtin_fmaf(fs, sv.z, v.z);
                        v.w = __builtin_fmaf(fs, sv.w, v.w);
                        store_state4(state_out, slot + idx, v, ST);
                    }
        }
      }
    }
}

// NC channel halves of 32 per workgroup, NW waves.
template <int ST, int NC, int NW>
hipError_t launch_scan_st(const ssm_plan *plan, const ScanArgs &args, const uint4 *frags, const bf16_t *dt_t,
                          float *tile_decay, float *carry, hipStream_t stream)
{
    static std::once_flag attr_once[64];
    static hipError_t attr_err[64];
    constexpr size_t lds = sizeof(LdsT<NC, NW>);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    std::call_once(attr_once[dev], [&]() {
        attr_err[dev] = hipFuncSetAttribute(reinterpret_cast<const void *>(ssm_scan_mfma_kernel<ST, NC, NW>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err[dev] != hipSuccess)
        return attr_err[dev];
    if (plan->n_items == 0)
        return hipSuccess;  // every sequence is empty
    hipLaunchKernelGGL((ssm_scan_mfma_kernel<ST, NC, NW>), dim3((unsigned)ssm_launch_blocks(plan->n_items)), dim3(64 * NW), lds,
                       stream, static_cast<const bf16_t *>(args.x), args.A, args.D, static_cast<bf16_t *>(args.y),
                       args.state_out, args.init_ptrs, frags, dt_t, args.tiles, args.scan_seqs, tile_decay, carry, args.H,
                       args.P, args.G, args.p_split, plan->n_items, (int)plan->tiles.size());
    return hipGetLastError();
}

template <int NC, int NW>
hipError_t launch_scan_width(const ssm_plan *plan, const ScanArgs &args, const uint4 *frags, const bf16_t *dt_t,
                             float *tile_decay, float *carry, hipStream_t stream)
{
    switch (args.state_dtype) {
    case SSM_ST_F16: return launch_scan_st<SSM_ST_F16, NC, NW>(plan, args, frags, dt_t, tile_decay, carry, stream);
    case SSM_ST_BF16: return launch_scan_st<SSM_ST_BF16, NC, NW>(plan, args, frags, dt_t, tile_decay, carry, stream);
    default: return launch_scan_st<SSM_ST_F32, NC, NW>(plan, args, frags, dt_t, tile_decay, carry, stream);
    }
}

template <int ST>
void launch_fix_st(const ScanArgs &args, const float *carry, const float *tile_decay, const uint4 *frags,
                   const bf16_t *dt_t, unsigned blocks, int max_tiles, int n_tiles_all, const FixSlots &slots,
                   int n_slots, hipStream_t stream)
{
    hipLaunchKernelGGL(ssm_fix_kernel<ST>, dim3(blocks), dim3(kFixThreads), sizeof(FixLds), stream,
                       static_cast<bf16_t *>(args.y), args.state_out, carry, tile_decay, frags, dt_t, args.A, args.tiles,
                       args.scan_seqs, args.H, args.P, args.G, max_tiles, n_tiles_all, slots, n_slots);
}

}  // namespace

hipError_t launch_scan_mfma(const ssm_plan *plan, const ScanArgs &args, void *workspace, hipStream_t stream)
{
    const int n_tiles = (int)plan->tiles.size();
    if (n_tiles == 0 || plan->n_items == 0)
        return hipSuccess;
    const SsmMfmaWorkspace ws = ssm_mfma_workspace(plan);
    unsigned char *base = static_cast<unsigned char *>(workspace);
    uint4 *frags = reinterpret_cast<uint4 *>(base + ws.images);
    bf16_t *dt_t = reinterpret_cast<bf16_t *>(base + ws.dt_rows);
    float *tile_decay = plan->n_carry > 0 ? reinterpret_cast<float *>(base + ws.tile_decay) : nullptr;
    float *carry = plan->n_carry > 0 ? reinterpret_cast<float *>(base + ws.carry) : nullptr;
    // few (tile, group) pairs: four workgroups each, so that the preparation does not run on a corner of the GPU
    const int parts = (long long)n_tiles * args.G < kMfmaPrepSplitBelow ? 4 : 1;
    hipLaunchKernelGGL(ssm_prep_kernel, dim3((unsigned)n_tiles * (unsigned)args.G * (unsigned)parts), dim3(kPrepThreads),
                       sizeof(PrepLds), stream, static_cast<const bf16_t *>(args.B), static_cast<const bf16_t *>(args.C),
                       static_cast<const bf16_t *>(args.dt), args.tiles, frags, dt_t, args.H, args.G, n_tiles, parts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    if (hipEvent_t mark = ssm_profile_event(0)) {
        e = hipEventRecord(mark, stream);
        if (e != hipSuccess)
            return e;
    }
    if (args.P / args.p_split == 64)
        e = launch_scan_width<2, kWavesWide>(plan, args, frags, dt_t, tile_decay, carry, stream);
    else
        e = launch_scan_width<1, kWavesNarrow>(plan, args, frags, dt_t, tile_decay, carry, stream);
    if (e != hipSuccess)
        return e;
    if (hipEvent_t mark = ssm_profile_event(1)) {
        e = hipEventRecord(mark, stream);
        if (e != hipSuccess)
            return e;
    }
    if (plan->n_carry == 0)
        return hipSuccess;
    // sequences cut into stretches: complete the carried states (three or more stretches), then add what they
    // contribute to the later stretches
    if (plan->carry_chains) {
        hipLaunchKernelGGL(ssm_carry_kernel, dim3((unsigned)plan->n_carry * (unsigned)args.H), dim3(kFixThreads),
                           sizeof(CarryLds), stream, carry, tile_decay, args.scan_seqs, args.H, args.P, n_tiles);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    const int per_stretch = plan->max_later_tiles;
    const unsigned blocks =
        (unsigned)plan->n_carry * (unsigned)args.H * (unsigned)(args.P / 64) * (unsigned)fix_groups(per_stretch);
    FixSlots slots = {};
    for (int c = 0; c < plan->n_carry && c < kFixSlotsInArgs; ++c) {
        const SsmScanSeq &later = plan->scan_seqs[plan->scan_seqs[c].of_slot];
        slots.tile_begin[c] = later.tile_begin;
        slots.tile_end[c] = later.tile_end;
    }
    switch (args.state_dtype) {
    case SSM_ST_F16: launch_fix_st<SSM_ST_F16>(args, carry, tile_decay, frags, dt_t, blocks, per_stretch, n_tiles, slots, plan->n_carry, stream); break;
    case SSM_ST_BF16: launch_fix_st<SSM_ST_BF16>(args, carry, tile_decay, frags, dt_t, blocks, per_stretch, n_tiles, slots, plan->n_carry, stream); break;
    default: launch_fix_st<SSM_ST_F32>(args, carry, tile_decay, frags, dt_t, blocks, per_stretch, n_tiles, slots, plan->n_carry, stream); break;
    }
    return hipGetLastError();
}
