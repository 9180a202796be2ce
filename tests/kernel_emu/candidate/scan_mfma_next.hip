// bf16 MFMA scan kernel for gfx950: d_state 128, headdim a multiple of 32,
// bf16 x/dt/B/C/y, fp32 A/D/state.
//
// One workgroup owns one (sequence, head, 32-channel slice) and walks the
// sequence's tiles in order; the slice's [32,128] state stays in MFMA
// accumulators from the first token to the last, so states reach device
// memory only as requested checkpoints.  Per tile of q <= 64 tokens starting
// after token s, with l_i = A * sum_{k<=i} dt_k inside the tile:
//
//   Gm[i,j] = (C_i.B_j) e^{l_i-l_j} dt_j   for j <= i, else 0   (masked score)
//   y_i     = e^{l_i} (S_s C_i) + sum_j Gm[i,j] x_j + D x_i
//   S_e     = e^{l_q} S_s + sum_j (e^{l_q-l_j} dt_j x_j) B_j^T
//
// All contractions run on the matrix cores with bf16 operands and fp32
// accumulation; bf16 rounding touches only MFMA operands (Gm with D added on
// its diagonal, the decay-weighted x, the copy of S used for S.C).  Decay
// exponents, accumulators and checkpoints are fp32.
//
// STATUS: candidate revision of scan_mfma.hip.  It is not built into the library and has never run on a GPU; it
// lives next to the CPU emulator so that the emulation tests can check it (oracle parity, wave-order independence,
// bounds) before it replaces the shipped kernel.  Same interface as the shipped kernel plus a workspace.
//
// A wave issues roughly one vector instruction every 5-8 cycles, whatever else
// runs beside it, so the work of a tile is cut into short instruction streams:
// the 12 waves of a workgroup (three per SIMD) are specialised and form a
// software pipeline over tiles with ONE workgroup barrier per tile.  In step k:
//
//   waves  6..9     B and C of tile k+1 -> LDS.  Two waves per stream take
//                   alternate tiles, so each load has two steps to arrive.
//   waves  10,11    (alternate tiles) x of tile k+1, raw and decay-weighted;
//                   dt of tile k+2: prefix sums and the per-token factor tables
//   waves  4,5      masked score blocks of tile k+1 (alternate tiles): the raw
//                   products C_i.B_j come from the workspace, where a small
//                   kernel in front of the scan left them once per group; here
//                   they get this head's decay, the mask and D on the diagonal
//   waves  0,1      tile k, token half 0 / 1: S.C, Gm.x, y staged through LDS
//                   and stored with coalesced writes
//   waves  2,3      tile k: state update for 64 state indices each, bf16 copy
//                   of the new state for tile k+1, checkpoint stores
//
// Score blocks travel from the score waves to the output waves through
// per-lane LDS mailboxes that already hold the consumer's MFMA operand.
// Every global access of the scan keeps four neighbouring lanes inside one
// 64-byte segment; its MFMA operand layouts are produced from LDS, never from
// global memory directly.
#include <type_traits>

#include "device_utils.h"

// Optional cycle-trace hooks for profiling builds; they expand to nothing here.
#ifndef SSM_TRACE
#define SSM_TRACE(slot)
#define SSM_TRACE_DECL
#endif

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 768;         // 12 waves, three per SIMD (waves of a workgroup go to the SIMDs round-robin)
constexpr int kQ = kMfmaTileTokens;  // 64 tokens per tile
// Raw score blocks of one (tile, group) in the workspace: keys 0..31 x queries 0..31, keys 32..63 x queries 32..63,
// keys 0..31 x queries 32..63; fp32 or bf16.
#ifndef SSM_CB_BF16
#define SSM_CB_BF16 1
#endif
constexpr int kScoreBlocksPerTile = 3;
constexpr size_t kScoreBlockBytes = 32 * 32 * (SSM_CB_BF16 ? 2 : 4);
constexpr int kN = 128;              // d_state
constexpr int kPW = 32;              // channels per workgroup
#ifndef SSM_LDB_PAD
#define SSM_LDB_PAD 8
#endif
#ifndef SSM_XS_SPLIT
#define SSM_XS_SPLIT 1  // 1: the decay-weighted x enters the state update as a bf16 pair (value, rounding remainder)
#endif
#ifndef SSM_DEFER_Y
#define SSM_DEFER_Y 0  // 1: an output wave stores the y of a tile at the start of its next step, under the LDS reads
#endif
#ifndef SSM_WAVE_PRIO
#define SSM_WAVE_PRIO 0  // 1: the output and state waves (the long dependent chains) run at a raised wave priority
#endif
#ifndef SSM_SS_SPLIT
#define SSM_SS_SPLIT 0  // 1: the copy of S used for S.C is a bf16 pair too (y after a resume from a large cached state)
#endif
#ifndef SSM_LDBS_PAD
#define SSM_LDBS_PAD 8
#endif
constexpr int LDB = kN + SSM_LDB_PAD;    // row stride (elements) of the C and state tiles (16-byte operand reads)
constexpr int LDBS = kN + SSM_LDBS_PAD;  // row stride of the B tiles (transpose reads only)
constexpr int LDX = kPW;             // row stride of the x tiles (unpadded on purpose)
constexpr int LDY = kPW + 8;         // row stride of the y staging tiles
constexpr float kLog2e = 1.4426950408889634f;

// per-token factors of one tile
struct Tables {
    float ell2[kQ];    // l_i * log2(e)
    float cj[kQ];      // l_j * log2(e) - log2(dt_j)
    float ei[kQ];      // e^{l_i}
    float ri[kQ / 2];  // i >= 32: e^{l_i - l_31}
    float cf[kQ / 2];  // j <  32: e^{l_31 - l_j} dt_j
    float w[kQ];       // e^{l_q - l_j} dt_j: weight of token j in the state update
};

struct Lds {
    bf16_t Bs[2][kQ][LDBS];       // B tile, token major
    bf16_t Cs[2][kQ][LDB];        // C tile, token major
    bf16_t Xr[2][kQ][LDX];        // x as loaded, token major
    bf16_t Xs[2][kQ][LDX];        // e^{l_q-l_j} dt_j x_j, token major
#if SSM_XS_SPLIT
    bf16_t Xl[2][kQ][LDX];        // what bf16 rounding took away from Xs
#endif
    bf16_t Ss[2][kPW][LDB];       // bf16 copy of the running state, channel major
#if SSM_SS_SPLIT
    bf16_t Sl[2][kPW][LDB];       // what bf16 rounding took away from Ss
#endif
    uint4 Md[2][2][64][2];        // [half][parity] masked diagonal score block as the output lane's two MFMA operands
    uint4 M10[2][64][2];          // off-diagonal score block, same form
    bf16_t Ys[2][kQ / 2][LDY];    // y of one token half on its way to coalesced stores
    Tables tab[3];
};

__device__ __forceinline__ bf16x8 lds_frag(const bf16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

// LDS transpose read: the 16 lanes of a group pass the addresses of 4 rows x
// (4 lanes x 4 elements); lane i of the group receives column i of that 4x16
// block, i.e. 4 elements that sit in 4 consecutive rows.
__device__ __forceinline__ s16x4 lds_tr4(const bf16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
}

// 8 k-values of a transposed operand: two groups of 4 consecutive rows of a token-major tile
__device__ __forceinline__ bf16x8 lds_frag_tr(const bf16_t *p_lo, const bf16_t *p_hi)
{
    const s16x4 lo = lds_tr4(p_lo), hi = lds_tr4(p_hi);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also
// wait for every outstanding global load, i.e. for the prefetches of later
// tiles.  Global memory written by this kernel is never read back by it, so
// LDS ordering is all the pipeline stages need.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#define SSM_DPP(old, v, ctrl, row_mask, bound)                                                        \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, (float)(old)),       \
                                                          __builtin_bit_cast(int, (float)(v)), (ctrl), \
                                                          (row_mask), 0xF, (bound)))
// Inclusive prefix sum over the 64 lanes of a wave with DPP row shifts and the
// two row broadcasts (no LDS round trips).
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

__device__ __forceinline__ bf16x8 pack8(float v0, float v1, float v2, float v3, float v4, float v5, float v6,
                                        float v7)
{
    const uint4 u = make_uint4(pack2(v0, v1), pack2(v2, v3), pack2(v4, v5), pack2(v6, v7));
    return __builtin_bit_cast(bf16x8, u);
}

// What every role needs to know; all members are wave-uniform.
struct Ctx {
    const bf16_t *__restrict__ x;
    const bf16_t *__restrict__ dt;
    const bf16_t *__restrict__ Bg;
    const bf16_t *__restrict__ Cg;
    bf16_t *__restrict__ y;
    void *__restrict__ state_out;  // checkpoints, [slot][H][P][N] in the state type
    const float *__restrict__ cb;  // raw score blocks, [tile][group][3][16 x 64 lanes] fp32
    const SsmTile *__restrict__ tiles;
    const void *init;   // this sequence's initial state (state type) or nullptr
    int state_type;     // 0 fp32, 1 fp16, 2 bf16: how cached states are stored; the running state is fp32
    int H, P, G, h, g, pbase;
    int tile_begin, n_tiles;
    float Ah, Dh;
};

// Descriptor of tile k of this sequence; indices past the end are clamped
// (those descriptors are never used).  Uniform index, so a scalar load.
__device__ __forceinline__ SsmTile tile_at(const Ctx &c, int k)
{
    const int kk = k < c.n_tiles ? k : c.n_tiles - 1;
    return c.tiles[__builtin_amdgcn_readfirstlane(c.tile_begin + kk)];
}

// The pipeline loop shared by all roles: steps s = -2 .. n_tiles-1, one
// workgroup barrier after each.  Steps come in groups of three so that
// everything indexed by a tile number modulo 3 (LDS buffers, register rings
// of prefetched data) is addressed statically: in step s = 3m - 2 + u,
// (s + 2) % 3 == u.
template <typename F>
__device__ __forceinline__ void pipe_loop(int n_tiles, F &&body)
{
    for (int s0 = -2; s0 < n_tiles; s0 += 3) {
        if (s0 + 0 < n_tiles) {
            body(s0 + 0, std::integral_constant<int, 0>{});
            lds_barrier();
        }
        if (s0 + 1 < n_tiles) {
            body(s0 + 1, std::integral_constant<int, 1>{});
            lds_barrier();
        }
        if (s0 + 2 < n_tiles) {
            body(s0 + 2, std::integral_constant<int, 2>{});
            lds_barrier();
        }
    }
}

// ---------------------------------------------------------------- loaders
// Global loads take a couple of thousand cycles when they miss in L2, more
// than a pipeline step is meant to last, and a wave can only wait for all of
// its outstanding loads at once.  Each stream (B, C, x with dt) is therefore
// served by two waves that take alternate tiles: in its active step a wave
// writes the tile it loaded two steps ago into LDS and then issues the loads
// of the tile after the next one, so every load has two full steps to arrive
// and a wave never waits with younger loads in flight.
//
// One 64 x 128 bf16 tile (B or C): 16 coalesced 16-byte loads per lane (16
// lanes per token row), in LDS one tile ahead of its readers.
template <bool IS_C, int PAR>
__device__ __forceinline__ void role_load_bc(const Ctx &c, Lds &L, int lane)
{
    uint4 r[16];
    const char *src = reinterpret_cast<const char *>(IS_C ? c.Cg : c.Bg);
    const int row_l = lane >> 4, col = 8 * (lane & 15);
    const uint32_t voff = (uint32_t)((row_l * c.G * kN + col) * 2);  // lane part of the address
    const uint32_t step = (uint32_t)(4 * c.G * kN * 2);              // 4 token rows
    auto issue = [&](const SsmTile &t) {
        const char *base = src + ((size_t)t.tok0 * c.G + c.g) * (kN * 2);  // uniform part
        if (t.len == kQ) {  // full tile: no predication
#pragma unroll
            for (int kk = 0; kk < 16; ++kk)
                r[kk] = *reinterpret_cast<const uint4 *>(base + kk * step + voff);
        } else {
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                r[kk] = make_uint4(0, 0, 0, 0);
                if (row_l + 4 * kk < t.len)
                    r[kk] = *reinterpret_cast<const uint4 *>(base + kk * step + voff);
            }
        }
    };
    if (PAR < c.n_tiles)
        issue(tile_at(c, PAR));
    SsmTile dpf = tile_at(c, PAR + 2);
    SSM_TRACE_DECL
    pipe_loop(c.n_tiles, [&](int s, auto) {
        SSM_TRACE(2);
        const int k = s + 1;
        if (k >= 0 && k < c.n_tiles && (k & 1) == PAR) {
#pragma unroll
            for (int kk = 0; kk < 16; ++kk)
                *reinterpret_cast<uint4 *>(IS_C ? &L.Cs[PAR][row_l + 4 * kk][col] : &L.Bs[PAR][row_l + 4 * kk][col]) = r[kk];
            if (k + 2 < c.n_tiles)
                issue(dpf);
            dpf = tile_at(c, k + 4);
        }
        SSM_TRACE(1);
    });
}

// x and dt.  The wave of parity PAR is active in the steps before tiles
// k = PAR, PAR+2, ...: it puts x of tile k into LDS, raw and weighted by
// e^{l_q - l_j} dt_j (weights from the tile's factor table, written one step
// earlier by the other wave), and turns dt of tile k+1 into that tile's prefix
// sums and factor tables, which the score waves and the other x wave need one
// step later.
template <int PAR>
__device__ __forceinline__ void role_load_x(const Ctx &c, Lds &L, int lane)
{
    uint4 xr[4];
    uint32_t dt_raw = 0;
    const int tok_l = lane >> 2, col = 8 * (lane & 3);
    auto issue_x = [&](const SsmTile &t) {
        const bf16_t *px = c.x + (((size_t)t.tok0 + tok_l) * c.H + c.h) * c.P + c.pbase + col;
        const size_t xstep = (size_t)16 * c.H * c.P;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            xr[kk] = make_uint4(0, 0, 0, 0);
            if (tok_l + 16 * kk < t.len)
                xr[kk] = *reinterpret_cast<const uint4 *>(px + kk * xstep);
        }
    };
    auto issue_dt = [&](const SsmTile &t) {
        dt_raw = 0;
        if (lane < t.len)
            dt_raw = c.dt[((size_t)t.tok0 + lane) * c.H + c.h];
    };
    // first active step: s = PAR - 1 for PAR 0 (tile 0), s = -2 for PAR 1 (no x tile yet, tables of tile 0)
    constexpr int k_first = PAR == 0 ? 0 : -1;
    if (k_first >= 0 && k_first < c.n_tiles)
        issue_x(tile_at(c, k_first));
    if (k_first + 1 < c.n_tiles)
        issue_dt(tile_at(c, k_first + 1));
    SsmTile xpf = tile_at(c, k_first + 2), dpf = tile_at(c, k_first + 3);
    SSM_TRACE_DECL
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        SSM_TRACE(2);
        constexpr int u = decltype(U)::value;   // == (s + 2) % 3: factor table of tile k + 1
        constexpr int b = (u + 2) % 3;          // == (s + 1) % 3: factor table of tile k
        const int k = s + 1;
        if (((k + 2) & 1) == PAR) {             // k may be -1: parity of k taken on k + 2
            if (k >= 0 && k < c.n_tiles) {
                float wt[4];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    wt[kk] = L.tab[b].w[tok_l + 16 * kk];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const int tok = tok_l + 16 * kk;
                    const uint4 xq = xr[kk];
                    *reinterpret_cast<uint4 *>(&L.Xr[PAR][tok][col]) = xq;
                    const uint32_t xv[4] = {xq.x, xq.y, xq.z, xq.w};
                    uint32_t o[4];
#if SSM_XS_SPLIT
                    uint32_t ol[4];
#endif
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p0 = wt[kk] * __uint_as_float(xv[e] << 16);
                        const float p1 = wt[kk] * __uint_as_float(xv[e] & 0xffff0000u);
                        o[e] = pack2(p0, p1);
#if SSM_XS_SPLIT
                        ol[e] = pack2(p0 - __uint_as_float(o[e] << 16), p1 - __uint_as_float(o[e] & 0xffff0000u));
#endif
                    }
                    *reinterpret_cast<uint4 *>(&L.Xs[PAR][tok][col]) = make_uint4(o[0], o[1], o[2], o[3]);
#if SSM_XS_SPLIT
                    *reinterpret_cast<uint4 *>(&L.Xl[PAR][tok][col]) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
#endif
                }
            }
            if (k + 1 < c.n_tiles) {
                Tables &tb = L.tab[u];
                const float dtj = __uint_as_float(dt_raw << 16);
                const float ell2 = wave_inclusive_sum(dtj * c.Ah) * kLog2e;
                const float last = read_lane(ell2, 63), e31 = read_lane(ell2, 31);
                tb.ell2[lane] = ell2;
                tb.cj[lane] = ell2 - __builtin_amdgcn_logf(dtj);
                tb.ei[lane] = exp2_fast(ell2);
                tb.w[lane] = exp2_fast(last - ell2) * dtj;
                if (lane >= 32)
                    tb.ri[lane - 32] = exp2_fast(ell2 - e31);
                else
                    tb.cf[lane] = exp2_fast(e31 - ell2) * dtj;
            }
            if (k + 2 < c.n_tiles)
                issue_x(xpf);
            if (k + 3 < c.n_tiles)
                issue_dt(dpf);
            xpf = tile_at(c, k + 4);
            dpf = tile_at(c, k + 5);
        }
        SSM_TRACE(1);
    });
}

// ---------------------------------------------------------------- score blocks of tile k+1
// All score blocks are kept transposed, Gm^T[j, i] = B_j . C_i.  Element r of
// the accumulator of lane (i = lane%32, q = lane/32) is key
// j = 8(r/4) + 4q + r%4; the output wave's Gm.x MFMA takes exactly these values
// as its operand when its other operand lists tokens in the same order, so the
// packed block is mailed lane to lane.
//
// The raw products do not depend on the head: ssm_cb_kernel computes them once
// per (tile, group) and stores each block as the 16 accumulator elements of
// the 64 lanes, four at a time, so that a lane reads back its own elements
// with four coalesced 16-byte loads per block.  The two score waves take
// alternate tiles; a wave issues the loads of its next tile right after it
// has finished the current one, two steps before it needs them.
//
// Diagonal blocks: masked (j <= i), one exponential of l_i - l_j per entry (no
// factor can overflow), D added on the diagonal so that D x_i rides through
// the Gm.x product.  Off-diagonal block (keys 0..31, queries 32..63): unmasked,
// and the decay factorises as e^{l_i-l_31} * e^{l_31-l_j} dt_j, both <= 1.
template <int PAR>
__device__ __forceinline__ void role_scores(const Ctx &c, Lds &L, int lane)
{
    const int i = lane & 31, q = lane >> 5;
#if SSM_CB_BF16
    uint4 rawp[kScoreBlocksPerTile][2];  // 16 bf16 per block and lane
    auto issue = [&](int k) {
        const uint4 *src = reinterpret_cast<const uint4 *>(c.cb) +
                           ((size_t)(c.tile_begin + k) * c.G + c.g) * (kScoreBlocksPerTile * 128) + lane;
#pragma unroll
        for (int blk = 0; blk < kScoreBlocksPerTile; ++blk)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                rawp[blk][hf] = src[blk * 128 + hf * 64];
    };
    // element 4a+r of block blk
    auto raw_at = [&](int blk, int a, int r) {
        const uint4 u4 = rawp[blk][a >> 1];
        const uint32_t w2[4] = {u4.x, u4.y, u4.z, u4.w};
        const uint32_t w = w2[2 * (a & 1) + (r >> 1)];
        return __uint_as_float((r & 1) ? (w & 0xffff0000u) : (w << 16));
    };
#else
    float4 raw[kScoreBlocksPerTile][4];
    auto issue = [&](int k) {
        const float *src = c.cb + ((size_t)(c.tile_begin + k) * c.G + c.g) * (kScoreBlocksPerTile * 1024) + 4 * lane;
#pragma unroll
        for (int blk = 0; blk < kScoreBlocksPerTile; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                raw[blk][a] = *reinterpret_cast<const float4 *>(src + blk * 1024 + a * 256);
    };
    auto raw_at = [&](int blk, int a, int r) {
        const float4 f = raw[blk][a];
        const float v4[4] = {f.x, f.y, f.z, f.w};
        return v4[r];
    };
#endif
    if (PAR < c.n_tiles)
        issue(PAR);
    SSM_TRACE_DECL
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        SSM_TRACE(2);
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 2) % 3;  // == (s + 1) % 3
        const int k = s + 1;
        if (k >= 0 && k < c.n_tiles && (k & 1) == PAR) {
            const Tables &tb = L.tab[b];
            // diagonal blocks of the two token halves
#pragma unroll
            for (int ih = 0; ih < 2; ++ih) {
                const float ell2_i = tb.ell2[32 * ih + i];
                float v[16];
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 c4 = *reinterpret_cast<const float4 *>(&tb.cj[32 * ih + 8 * a + 4 * q]);
                    const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
                    const float rr[4] = {raw_at(ih, a, 0), raw_at(ih, a, 1), raw_at(ih, a, 2), raw_at(ih, a, 3)};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int jl = 8 * a + 4 * q + r;
                        const float g = __builtin_fmaf(rr[r], exp2_fast(ell2_i - cc[r]), jl == i ? c.Dh : 0.f);
                        v[4 * a + r] = jl <= i ? g : 0.f;
                    }
                }
                L.Md[ih][k & 1][lane][0] =
                    make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
                L.Md[ih][k & 1][lane][1] =
                    make_uint4(pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
            }
            // off-diagonal block
            {
                const float ri = tb.ri[i];
                float v[16];
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 f4 = *reinterpret_cast<const float4 *>(&tb.cf[8 * a + 4 * q]);
                    v[4 * a + 0] = raw_at(2, a, 0) * (ri * f4.x);
                    v[4 * a + 1] = raw_at(2, a, 1) * (ri * f4.y);
                    v[4 * a + 2] = raw_at(2, a, 2) * (ri * f4.z);
                    v[4 * a + 3] = raw_at(2, a, 3) * (ri * f4.w);
                }
                L.M10[k & 1][lane][0] =
                    make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
                L.M10[k & 1][lane][1] =
                    make_uint4(pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
            }
            if (k + 2 < c.n_tiles)
                issue(k + 2);
        }
        SSM_TRACE(1);
    });
}

// Four neighbouring elements of a cached state (element index idx), in the storage type of the cache: fp32, or
// fp16 / bf16 as caches keep them (Section 5.1: FP16).  A reduced-precision checkpoint is the fp32 running state
// rounded once to nearest even; the running state itself is never rounded.
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
__device__ __forceinline__ float4 load_state4(const void *base, size_t idx, int state_type)
{
    if (state_type == 1) {
        const f16x4 h = *reinterpret_cast<const f16x4 *>(static_cast<const _Float16 *>(base) + idx);
        return make_float4((float)h[0], (float)h[1], (float)h[2], (float)h[3]);
    }
    if (state_type == 2) {
        const uint2 u = *reinterpret_cast<const uint2 *>(static_cast<const bf16_t *>(base) + idx);
        return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                           __uint_as_float(u.y & 0xffff0000u));
    }
    return *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + idx);
}
__device__ __forceinline__ void store_state4(void *base, size_t idx, float v0, float v1, float v2, float v3, int state_type)
{
    if (state_type == 1) {
        const f16x4 h = {(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};
        *reinterpret_cast<f16x4 *>(static_cast<_Float16 *>(base) + idx) = h;
    } else if (state_type == 2) {
        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(base) + idx) = make_uint2(pack2(v0, v1), pack2(v2, v3));
    } else {
        *reinterpret_cast<float4 *>(static_cast<float *>(base) + idx) = make_float4(v0, v1, v2, v3);
    }
}

// bf16 copy of four neighbouring state values (and, if asked for, of what the rounding took away)
__device__ __forceinline__ void store_state_copy(Lds &L, int buf, int p, int n0, float v0, float v1, float v2, float v3)
{
    const uint32_t h0 = pack2(v0, v1), h1 = pack2(v2, v3);
    *reinterpret_cast<uint2 *>(&L.Ss[buf][p][n0]) = make_uint2(h0, h1);
#if SSM_SS_SPLIT
    *reinterpret_cast<uint2 *>(&L.Sl[buf][p][n0]) =
        make_uint2(pack2(v0 - __uint_as_float(h0 << 16), v1 - __uint_as_float(h0 & 0xffff0000u)),
                   pack2(v2 - __uint_as_float(h1 << 16), v3 - __uint_as_float(h1 & 0xffff0000u)));
#endif
}

// ---------------------------------------------------------------- outputs of tile k, token half IH
template <int IH>
__device__ __forceinline__ void role_output(const Ctx &c, Lds &L, int lane)
{
    const int i = lane & 31, q = lane >> 5;
    // transpose-read addressing: lane group g4 = lane/16 covers channel block
    // g4&1; tokens come in the order 8(e/4) + 4q + e%4, as in the scores
    const int g4 = lane >> 4;
    const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
    const int tr_row = 4 * (g4 >> 1) + ((lane & 15) >> 2);
#if SSM_WAVE_PRIO
    __builtin_amdgcn_s_setprio(2);
#endif
    bf16_t(*ys)[LDY] = L.Ys[IH];
    // rows of this wave's staging tile to device memory: 16 bytes per lane, four lanes per 64-byte row of y
    auto flush_y = [&](const SsmTile &t) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int tok = (lane >> 2) + 16 * m;
            const uint4 o = *reinterpret_cast<const uint4 *>(&ys[tok][8 * (lane & 3)]);
            if (32 * IH + tok < t.len)
                *reinterpret_cast<uint4 *>(c.y + (((size_t)t.tok0 + 32 * IH + tok) * c.H + c.h) * c.P + c.pbase +
                                           8 * (lane & 3)) = o;
        }
    };
#if SSM_DEFER_Y
    SsmTile t_prev = tile_at(c, 0);
#endif
    SSM_TRACE_DECL
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        SSM_TRACE(2);
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 1) % 3;  // == s % 3 for s >= 0
        if (s >= 0) {
            const SsmTile t = tile_at(c, s);
            // all LDS reads of the step are issued up front
            const bf16_t *ps = &L.Ss[(s + 1) & 1][i][8 * q];
            const bf16_t *pc = &L.Cs[s & 1][32 * IH + i][8 * q];
            bf16x8 fs[8], fc[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                fs[ks] = lds_frag(ps + 16 * ks);
                fc[ks] = lds_frag(pc + 16 * ks);
            }
#if SSM_SS_SPLIT
            const bf16_t *pl = &L.Sl[(s + 1) & 1][i][8 * q];
            bf16x8 fsl[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                fsl[ks] = lds_frag(pl + 16 * ks);
#endif
            const uint4 g0 = L.Md[IH][s & 1][lane][0], g1 = L.Md[IH][s & 1][lane][1];
            const bf16_t *px = &L.Xr[s & 1][32 * IH + tr_row][tr_col];
            const bf16x8 x0 = lds_frag_tr(px, px + 8 * LDX), x1 = lds_frag_tr(px + 16 * LDX, px + 24 * LDX);
            bf16x8 x2, x3;
            uint4 m0, m1;
            if (IH == 1) {
                const bf16_t *px0 = &L.Xr[s & 1][tr_row][tr_col];
                x2 = lds_frag_tr(px0, px0 + 8 * LDX);
                x3 = lds_frag_tr(px0 + 16 * LDX, px0 + 24 * LDX);
                m0 = L.M10[s & 1][lane][0];
                m1 = L.M10[s & 1][lane][1];
            }
            const float ei = L.tab[b].ei[32 * IH + i];
#if SSM_DEFER_Y
            // y of the previous tile: staged before the last barrier, stored now, under the reads just issued
            if (s > 0)
                flush_y(t_prev);
            t_prev = t;
#endif
            // S_s C_i with the state as it was before this tile
            f32x16 Y = zero16();
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fs[ks], fc[ks], Y, 0, 0, 0);
#if SSM_SS_SPLIT
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fsl[ks], fc[ks], Y, 0, 0, 0);
#endif
#pragma unroll
            for (int r = 0; r < 16; ++r)
                Y[r] *= ei;
            // intra-tile term: x^T through transpose reads, masked scores from the mailboxes
            Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, __builtin_bit_cast(bf16x8, g0), Y, 0, 0, 0);
            Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, __builtin_bit_cast(bf16x8, g1), Y, 0, 0, 0);
            if (IH == 1) {
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2, __builtin_bit_cast(bf16x8, m0), Y, 0, 0, 0);
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x3, __builtin_bit_cast(bf16x8, m1), Y, 0, 0, 0);
            }
            // Y^T[p, i]: element r of this lane is channel 8(r/4) + 4q + r%4 of
            // token i.  Through this wave's own LDS tile to token-major rows, then
            // 16 bytes per lane with four lanes per 64-byte row of y.
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<uint2 *>(&ys[i][8 * a + 4 * q]) =
                    make_uint2(pack2(Y[4 * a], Y[4 * a + 1]), pack2(Y[4 * a + 2], Y[4 * a + 3]));
#if !SSM_DEFER_Y
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // same wave: LDS executes in order
            flush_y(t);
#endif
        }
        SSM_TRACE(1);
    });
#if SSM_DEFER_Y
    flush_y(t_prev);  // the last tile; the loop's final barrier has ordered its staging writes
#endif
}

// ---------------------------------------------------------------- state update of tile k, NS x 32 state indices
template <int SQ, int NS>
__device__ __forceinline__ void role_state(const Ctx &c, Lds &L, int lane)
{
    // S^T tiles: rows n = 32 (NS SQ + nb) + 8(r/4) + 4(lane/32) + r%4, column p = lane%32
    const int p = lane & 31, q = lane >> 5;
    f32x16 S[NS];
#pragma unroll
    for (int nb = 0; nb < NS; ++nb) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int n0 = 32 * (NS * SQ + nb) + 8 * a + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c.init)
                v = load_state4(c.init, ((size_t)c.h * c.P + c.pbase + p) * kN + n0, c.state_type);
            S[nb][4 * a + 0] = v.x;
            S[nb][4 * a + 1] = v.y;
            S[nb][4 * a + 2] = v.z;
            S[nb][4 * a + 3] = v.w;
            store_state_copy(L, 1, p, n0, v.x, v.y, v.z, v.w);
        }
    }
    // transpose reads, natural token order: group g4 covers row/column block
    // g4&1 and tokens 8(g4>>1) + 0..7 of each 16-token k-step
    const int g4 = lane >> 4;
    const int tr_row = 8 * (g4 >> 1) + ((lane & 15) >> 2);
    const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
#if SSM_WAVE_PRIO
    __builtin_amdgcn_s_setprio(1);
#endif
    SSM_TRACE_DECL
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        SSM_TRACE(2);
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 1) % 3;  // == s % 3 for s >= 0
        if (s >= 0) {
            const SsmTile t = tile_at(c, s);
            const bf16_t *px = &L.Xs[s & 1][tr_row][tr_col];
            bf16x8 fx[4], fb[NS][4];
#if SSM_XS_SPLIT
            const bf16_t *pl = &L.Xl[s & 1][tr_row][tr_col];
            bf16x8 fl[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                fl[ks] = lds_frag_tr(pl + 16 * ks * LDX, pl + (16 * ks + 4) * LDX);
#endif
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                fx[ks] = lds_frag_tr(px + 16 * ks * LDX, px + (16 * ks + 4) * LDX);
#pragma unroll
                for (int nb = 0; nb < NS; ++nb) {
                    const bf16_t *pb = &L.Bs[s & 1][tr_row][32 * (NS * SQ + nb) + tr_col];
                    fb[nb][ks] = lds_frag_tr(pb + 16 * ks * LDBS, pb + (16 * ks + 4) * LDBS);
                }
            }
            const float dl = L.tab[b].ei[kQ - 1];  // padded tokens have dt = 0, so this is e^{l_len}
#pragma unroll
            for (int nb = 0; nb < NS; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    S[nb][r] *= dl;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int nb = 0; nb < NS; ++nb)
                    S[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[nb][ks], fx[ks], S[nb], 0, 0, 0);
#if SSM_XS_SPLIT
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int nb = 0; nb < NS; ++nb)
                    S[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[nb][ks], fl[ks], S[nb], 0, 0, 0);
#endif
            // bf16 copy for the next tile's S.C product; checkpoint
#pragma unroll
            for (int nb = 0; nb < NS; ++nb)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int n0 = 32 * (NS * SQ + nb) + 8 * a + 4 * q;
                    store_state_copy(L, s & 1, p, n0, S[nb][4 * a], S[nb][4 * a + 1], S[nb][4 * a + 2], S[nb][4 * a + 3]);
                }
            if (t.ckpt_slot >= 0) {
#pragma unroll
                for (int nb = 0; nb < NS; ++nb) {
                    const size_t idx = (((size_t)t.ckpt_slot * c.H + c.h) * c.P + c.pbase + p) * kN +
                                       32 * (NS * SQ + nb) + 4 * q;
#pragma unroll
                    for (int a = 0; a < 4; ++a)
                        store_state4(c.state_out, idx + 8 * a, S[nb][4 * a], S[nb][4 * a + 1], S[nb][4 * a + 2],
                                     S[nb][4 * a + 3], c.state_type);
                }
            }
        }
        SSM_TRACE(1);
    });
}

__device__ __forceinline__ void role_idle(const Ctx &c)
{
    pipe_loop(c.n_tiles, [&](int, auto) {});
}

// Raw score blocks of every (tile, group): Gm^T[j, i] = B_j . C_i for keys j and
// queries i of one 64-token tile, without decay or mask.  One workgroup of
// three waves per (tile, group), one 32 x 32 block per wave (block 0: keys and
// queries 0..31, block 1: keys and queries 32..63, block 2: keys 0..31, queries
// 32..63).  Rows past the end of a partial tile count as zero.  The MFMA
// operands are read straight from device memory (16 bytes per lane); this
// kernel moves a few percent of the scan's bytes, so coalescing is not worth
// a trip through LDS here.
__global__ __launch_bounds__(64 * kScoreBlocksPerTile) void ssm_cb_kernel(
    const bf16_t *__restrict__ Bg, const bf16_t *__restrict__ Cg, const SsmTile *__restrict__ tiles,
    float *__restrict__ cb, int G, int n_tiles)
{
    const int tile = blockIdx.x / G, g = blockIdx.x % G;
    if (tile >= n_tiles)
        return;
    const SsmTile t = tiles[tile];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = lane & 31, q = lane >> 5;
    const int jrow = (w == 1 ? 32 : 0) + i;  // key token of this lane's B row
    const int irow = (w == 0 ? 0 : 32) + i;  // query token of this lane's C row
    const bf16x8 z = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
    bf16x8 fa[8], fc[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        fa[ks] = z;
        fc[ks] = z;
    }
    if (jrow < t.len) {
        const bf16_t *pb = Bg + ((size_t)(t.tok0 + jrow) * G + g) * kN + 8 * q;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            fa[ks] = *reinterpret_cast<const bf16x8 *>(pb + 16 * ks);
    }
    if (irow < t.len) {
        const bf16_t *pc = Cg + ((size_t)(t.tok0 + irow) * G + g) * kN + 8 * q;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            fc[ks] = *reinterpret_cast<const bf16x8 *>(pc + 16 * ks);
    }
    f32x16 acc = zero16();
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks], fc[ks], acc, 0, 0, 0);
#if SSM_CB_BF16
    uint4 *dst = reinterpret_cast<uint4 *>(cb) + ((size_t)blockIdx.x * kScoreBlocksPerTile + w) * 128 + lane;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
        dst[hf * 64] = make_uint4(pack2(acc[8 * hf + 0], acc[8 * hf + 1]), pack2(acc[8 * hf + 2], acc[8 * hf + 3]),
                                  pack2(acc[8 * hf + 4], acc[8 * hf + 5]), pack2(acc[8 * hf + 6], acc[8 * hf + 7]));
#else
    float *dst = cb + ((size_t)blockIdx.x * kScoreBlocksPerTile + w) * 1024 + 4 * lane;
#pragma unroll
    for (int a = 0; a < 4; ++a)
        *reinterpret_cast<float4 *>(dst + a * 256) =
            make_float4(acc[4 * a], acc[4 * a + 1], acc[4 * a + 2], acc[4 * a + 3]);
#endif
}

// Pointers are separate __restrict__ parameters (not a struct) so that the
// compiler may read the read-only tables with scalar loads.
__global__ __launch_bounds__(kThreads) void ssm_scan_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dt, const float *__restrict__ A_,
    const bf16_t *__restrict__ Bg, const bf16_t *__restrict__ Cg, const float *__restrict__ D_,
    bf16_t *__restrict__ y, void *__restrict__ state_out, const float *__restrict__ cb,
    const void *const *__restrict__ init_ptrs, const SsmTile *__restrict__ tiles, const SsmSeq *__restrict__ seqs,
    int H, int P, int G, int p_split, int wg_per_xcd, int n_wg, int state_type)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    Lds &L = *reinterpret_cast<Lds *>(lds_raw);

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that
    // consecutive logical ids (same head, then same group) share an XCD's L2.
    const int wg = (blockIdx.x & 7) * wg_per_xcd + (blockIdx.x >> 3);
    if (wg >= n_wg)
        return;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    Ctx c;
    c.x = x;
    c.dt = dt;
    c.Bg = Bg;
    c.Cg = Cg;
    c.y = y;
    c.state_out = state_out;
    c.state_type = state_type;
    c.cb = cb;
    c.tiles = tiles;
    c.H = H;
    c.P = P;
    c.G = G;
    const int ps = wg % p_split;
    c.h = (wg / p_split) % H;
    const int seq = wg / (p_split * H);
    c.g = c.h / (H / G);
    c.pbase = ps * kPW;
    c.Ah = A_[c.h];
    c.Dh = D_[c.h];
    c.init = init_ptrs ? init_ptrs[seq] : nullptr;
    const SsmSeq sq = seqs[seq];
    c.tile_begin = sq.tile_begin;
    c.n_tiles = sq.tile_end - sq.tile_begin;
    if (c.n_tiles <= 0)
        return;  // empty sequence: the whole workgroup leaves before any barrier

    // Every role runs the same number of barriers: n_tiles + 2 pipeline steps.
    // SIMD 0: output 0, scores 0, C 0;  SIMD 1: output 1, scores 1, C 1;
    // SIMD 2: state 0, B 0, x 0;        SIMD 3: state 1, B 1, x 1
    switch (w) {
    case 0: role_output<0>(c, L, lane); break;
    case 1: role_output<1>(c, L, lane); break;
    case 2: role_state<0, 2>(c, L, lane); break;
    case 3: role_state<1, 2>(c, L, lane); break;
    case 4: role_scores<0>(c, L, lane); break;
    case 5: role_scores<1>(c, L, lane); break;
    case 6: role_load_bc<false, 0>(c, L, lane); break;
    case 7: role_load_bc<false, 1>(c, L, lane); break;
    case 8: role_load_bc<true, 0>(c, L, lane); break;
    case 9: role_load_bc<true, 1>(c, L, lane); break;
    case 10: role_load_x<0>(c, L, lane); break;
    case 11: role_load_x<1>(c, L, lane); break;
    default: role_idle(c); break;
    }
}

}  // namespace

// Bytes of workspace (256-byte aligned device memory) the candidate needs for a plan.
size_t scan_mfma_next_workspace_bytes(const ssm_plan *plan)
{
    return plan->tiles.size() * (size_t)plan->shape.ngroups * kScoreBlocksPerTile * kScoreBlockBytes;
}

// `state_type`: storage of the initial states and of the checkpoints in args.state_out (0 fp32, 1 fp16, 2 bf16).
hipError_t launch_scan_mfma_next(const ssm_plan *plan, const ScanArgs &args, void *workspace, hipStream_t stream,
                                 int state_type)
{
    if (state_type < 0 || state_type > 2)
        return hipErrorInvalidValue;
    float *cb = static_cast<float *>(workspace);
    static bool attr_set = false;
    const size_t lds = sizeof(Lds);
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ssm_scan_mfma_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    const int n_wg = plan->n_workgroups;
    const int per_xcd = (n_wg + 7) / 8;
    const int n_tiles = (int)plan->tiles.size();
    if (n_tiles == 0 || n_wg == 0)
        return hipSuccess;
    hipLaunchKernelGGL(ssm_cb_kernel, dim3((unsigned)n_tiles * (unsigned)args.G), dim3(64 * kScoreBlocksPerTile), 0, stream,
                       static_cast<const bf16_t *>(args.B), static_cast<const bf16_t *>(args.C), args.tiles, cb,
                       args.G, n_tiles);
    hipLaunchKernelGGL(ssm_scan_mfma_kernel, dim3((unsigned)(per_xcd * 8)), dim3(kThreads), lds, stream,
                       static_cast<const bf16_t *>(args.x), static_cast<const bf16_t *>(args.dt), args.A,
                       static_cast<const bf16_t *>(args.B), static_cast<const bf16_t *>(args.C), args.D,
                       static_cast<bf16_t *>(args.y), static_cast<void *>(args.state_out), cb,
                       reinterpret_cast<const void *const *>(args.init_ptrs), args.tiles, args.seqs, args.H, args.P,
                       args.G, args.p_split, per_xcd, n_wg, state_type);
    return hipGetLastError();
}
