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
// The 8 waves of a workgroup are specialised and form a software pipeline
// over tiles with ONE workgroup barrier per tile.  In pipeline step k:
//
//   waves 4,5,7  loaders: write tile k+2 into LDS (B; C; dt prefix sums, the
//                per-token factor tables, x raw and decay-weighted) from
//                registers filled by coalesced global loads one step earlier
//   wave  6      off-diagonal score block (queries 32..63, keys 0..31) of
//                tile k+1, handed over through a per-lane LDS mailbox that
//                already holds the consumer's MFMA operand
//   waves 0,1    token half 0 / 1.  For tile k: S.C with the C fragments and
//                Gm.x with the masked diagonal score block this wave kept in
//                registers from the step before, y staged through LDS and
//                stored with coalesced writes.  For tile k+1: C fragments from
//                LDS, diagonal score block, masking.
//   waves 2,3    tile k: state update for 64 state indices each, bf16 copy of
//                the new state for tile k+1, checkpoint stores
//
// Every global access is laid out so that four neighbouring lanes touch one
// 64-byte segment; MFMA operand layouts are produced from LDS, never from
// global memory directly.
#include <type_traits>

#include "device_utils.h"


namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 512;             // 8 waves
constexpr int kQ = kMfmaTileTokens;  // 64 tokens per tile
constexpr int kN = 128;              // d_state
constexpr int kPW = 32;              // channels per workgroup
constexpr int LDB = kN + 16;         // row stride (elements) of the B and state tiles
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
};

struct Lds {
    bf16_t Bs[3][kQ][LDB];        // B tile, token major
    bf16_t Cs[2][kQ][LDB];        // C tile, token major
    bf16_t Xr[3][kQ][LDX];        // x as loaded, token major
    bf16_t Xs[3][kQ][LDX];        // e^{l_q-l_j} dt_j x_j, token major
    bf16_t Ss[2][kPW][LDB];       // bf16 copy of the running state, channel major
    uint4 M10[2][64][2];          // off-diagonal score block as the consumer lane's two MFMA operands
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

// What every role needs to know; all members are wave-uniform.
struct Ctx {
    const bf16_t *__restrict__ x;
    const bf16_t *__restrict__ dt;
    const bf16_t *__restrict__ Bg;
    const bf16_t *__restrict__ Cg;
    bf16_t *__restrict__ y;
    float *__restrict__ state_out;
    const SsmTile *__restrict__ tiles;
    const float *init;  // this sequence's initial state or nullptr
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

// Mask and decay a diagonal 32x32 score block held as Gm^T accumulators
// (element r of lane (i = lane%32, q = lane/32) is row j = 8(r/4) + 4q + r%4),
// add D on the diagonal, and pack it as the two bf16 operands of the Gm.x MFMAs.
__device__ __forceinline__ void mask_diag(const f32x16 &acc, const Tables &tb, int off, int i, int q, float Dh,
                                          uint4 &g0, uint4 &g1)
{
    const float ell2_i = tb.ell2[off + i];
    float v[16];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const float4 c4 = *reinterpret_cast<const float4 *>(&tb.cj[off + 8 * a + 4 * q]);
        const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int jl = 8 * a + 4 * q + r;
            float g = jl <= i ? acc[4 * a + r] * exp2_fast(ell2_i - cc[r]) : 0.f;
            if (jl == i)
                g += Dh;
            v[4 * a + r] = g;
        }
    }
    g0 = make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
    g1 = make_uint4(pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
}

// ---------------------------------------------------------------- loaders
// One 64 x 128 bf16 tile (B or C) per step: 16 coalesced 16-byte loads per
// lane (16 lanes per token row), written to LDS one step after they were
// issued and two tiles ahead of the consumers.
template <bool IS_C>
__device__ __forceinline__ void role_load_bc(const Ctx &c, Lds &L, int lane)
{
    uint4 r[16];
    const bf16_t *src = IS_C ? c.Cg : c.Bg;
    const int row_l = lane >> 4, col = 8 * (lane & 15);
    auto issue = [&](const SsmTile &t) {
        const bf16_t *p = src + (((size_t)t.tok0 + row_l) * c.G + c.g) * kN + col;
        const size_t step = (size_t)4 * c.G * kN;
        if (t.len == kQ) {  // full tile: no predication
#pragma unroll
            for (int kk = 0; kk < 16; ++kk)
                r[kk] = *reinterpret_cast<const uint4 *>(p + kk * step);
        } else {
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                r[kk] = make_uint4(0, 0, 0, 0);
                if (row_l + 4 * kk < t.len)
                    r[kk] = *reinterpret_cast<const uint4 *>(p + kk * step);
            }
        }
    };
    issue(tile_at(c, 0));
    SsmTile dpf = tile_at(c, 1);
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        constexpr int u = decltype(U)::value;  // == (s + 2) % 3: LDS buffer of tile k in a ring of three
        const int k = s + 2;
        if (k < c.n_tiles) {
            bf16_t(*dst)[LDB] = IS_C ? L.Cs[k & 1] : L.Bs[u];
#pragma unroll
            for (int kk = 0; kk < 16; ++kk)
                *reinterpret_cast<uint4 *>(&dst[row_l + 4 * kk][col]) = r[kk];
            if (k + 1 < c.n_tiles)
                issue(dpf);
            dpf = tile_at(c, k + 2);
        }
    });
}

// dt prefix sums, the per-token factor tables and the two x tiles.
__device__ __forceinline__ void role_load_x(const Ctx &c, Lds &L, int lane)
{
    uint32_t dt_raw = 0;
    uint4 xr[4];
    auto issue = [&](const SsmTile &t) {
        const bf16_t *px = c.x + (((size_t)t.tok0 + (lane >> 2)) * c.H + c.h) * c.P + c.pbase + 8 * (lane & 3);
        const size_t xstep = (size_t)16 * c.H * c.P;
        dt_raw = 0;
        if (lane < t.len)
            dt_raw = c.dt[((size_t)t.tok0 + lane) * c.H + c.h];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            xr[kk] = make_uint4(0, 0, 0, 0);
            if ((lane >> 2) + 16 * kk < t.len)
                xr[kk] = *reinterpret_cast<const uint4 *>(px + kk * xstep);
        }
    };
    issue(tile_at(c, 0));
    SsmTile dpf = tile_at(c, 1);
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        constexpr int u = decltype(U)::value;  // == (s + 2) % 3
        const int k = s + 2;
        if (k < c.n_tiles) {
            Tables &tb = L.tab[u];
            const float dtj = __uint_as_float(dt_raw << 16);
            const float ell2 = wave_inclusive_sum(dtj * c.Ah) * kLog2e;
            const float last = read_lane(ell2, 63), e31 = read_lane(ell2, 31);
            const float wj = exp2_fast(last - ell2) * dtj;  // weight of token `lane` in the state update
            tb.ell2[lane] = ell2;
            tb.cj[lane] = ell2 - __builtin_amdgcn_logf(dtj);
            tb.ei[lane] = exp2_fast(ell2);
            if (lane >= 32)
                tb.ri[lane - 32] = exp2_fast(ell2 - e31);
            else
                tb.cf[lane] = exp2_fast(e31 - ell2) * dtj;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int tok = (lane >> 2) + 16 * kk;
                const float wt = __shfl(wj, tok, 64);
                const uint4 xq = xr[kk];
                *reinterpret_cast<uint4 *>(&L.Xr[u][tok][8 * (lane & 3)]) = xq;
                const uint32_t xv[4] = {xq.x, xq.y, xq.z, xq.w};
                uint32_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = pack2(wt * __uint_as_float(xv[e] << 16), wt * __uint_as_float(xv[e] & 0xffff0000u));
                *reinterpret_cast<uint4 *>(&L.Xs[u][tok][8 * (lane & 3)]) = make_uint4(o[0], o[1], o[2], o[3]);
            }
            if (k + 1 < c.n_tiles)
                issue(dpf);
            dpf = tile_at(c, k + 2);
        }
    });
}

// ---------------------------------------------------------------- off-diagonal scores of tile k+1
// Gm^T[j, i] for keys j in 0..31 and queries i in 32..63: every entry is
// unmasked and the decay factorises as e^{l_i-l_31} * e^{l_31-l_j} dt_j, both
// factors <= 1.  Accumulator element r of lane (i = lane%32, q = lane/32) is key
// j = 8(r/4) + 4q + r%4; the consumer's MFMA takes exactly these values as its
// operand when its other operand lists tokens in the same order, so the packed
// block is mailed lane to lane.
__device__ __forceinline__ void role_offdiag(const Ctx &c, Lds &L, int lane)
{
    const int i = lane & 31, q = lane >> 5;
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 2) % 3;  // == (s + 1) % 3
        const int k = s + 1;
        if (k >= 0 && k < c.n_tiles) {
            const Tables &tb = L.tab[b];
            const bf16_t *pa = &L.Bs[b][i][8 * q];
            const bf16_t *pc = &L.Cs[k & 1][32 + i][8 * q];
            bf16x8 fa[8], fc[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                fa[ks] = lds_frag(pa + 16 * ks);
                fc[ks] = lds_frag(pc + 16 * ks);
            }
            const float ri = tb.ri[i];
            float4 c4[4];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                c4[a] = *reinterpret_cast<const float4 *>(&tb.cf[8 * a + 4 * q]);
            f32x16 acc = zero16();
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks], fc[ks], acc, 0, 0, 0);
            float v[16];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                v[4 * a + 0] = acc[4 * a + 0] * (ri * c4[a].x);
                v[4 * a + 1] = acc[4 * a + 1] * (ri * c4[a].y);
                v[4 * a + 2] = acc[4 * a + 2] * (ri * c4[a].z);
                v[4 * a + 3] = acc[4 * a + 3] * (ri * c4[a].w);
            }
            L.M10[k & 1][lane][0] =
                make_uint4(pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7]));
            L.M10[k & 1][lane][1] =
                make_uint4(pack2(v[8], v[9]), pack2(v[10], v[11]), pack2(v[12], v[13]), pack2(v[14], v[15]));
        }
    });
}

// ---------------------------------------------------------------- token half IH: outputs of tile k, scores of tile k+1
template <int IH>
__device__ __forceinline__ void role_half(const Ctx &c, Lds &L, int lane)
{
    const int i = lane & 31, q = lane >> 5;
    // transpose-read addressing: lane group g4 = lane/16 covers channel block
    // g4&1; tokens come in the order 8(e/4) + 4q + e%4, as in the scores
    const int g4 = lane >> 4;
    const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
    const int tr_row = 4 * (g4 >> 1) + ((lane & 15) >> 2);
    // carried from the scores part of one step to the outputs part of the next
    bf16x8 cf[8];       // C fragments of this half
    uint4 g0, g1;       // masked diagonal score block as two MFMA operands
    g0 = g1 = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        cf[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 1) % 3;   // == s % 3 for s >= 0
        constexpr int bn = (u + 2) % 3;  // == (s + 1) % 3
        // ---- LDS reads of both parts, issued before anything waits for them ----
        bf16x8 fs[8], x0, x1, x2, x3;
        uint4 m0, m1;
        float ei = 0.f;
        if (s >= 0) {
            const bf16_t *ps = &L.Ss[(s + 1) & 1][i][8 * q];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                fs[ks] = lds_frag(ps + 16 * ks);
            const bf16_t *px = &L.Xr[b][32 * IH + tr_row][tr_col];
            x0 = lds_frag_tr(px, px + 8 * LDX);
            x1 = lds_frag_tr(px + 16 * LDX, px + 24 * LDX);
            if (IH == 1) {
                const bf16_t *px0 = &L.Xr[b][tr_row][tr_col];
                x2 = lds_frag_tr(px0, px0 + 8 * LDX);
                x3 = lds_frag_tr(px0 + 16 * LDX, px0 + 24 * LDX);
                m0 = L.M10[s & 1][lane][0];
                m1 = L.M10[s & 1][lane][1];
            }
            ei = L.tab[b].ei[32 * IH + i];
        }
        bf16x8 cn[8], fb[8];
        const bool have_next = s + 1 < c.n_tiles;
        if (have_next) {
            const bf16_t *pc = &L.Cs[(s + 1) & 1][32 * IH + i][8 * q];
            const bf16_t *pb = &L.Bs[bn][32 * IH + i][8 * q];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                cn[ks] = lds_frag(pc + 16 * ks);
                fb[ks] = lds_frag(pb + 16 * ks);
            }
        }
        // Two independent MFMA chains back to back: first the diagonal score
        // block of tile s+1, then S.C of tile s.  The vector-ALU masking of the
        // first overlaps the matrix work of the second.
        f32x16 acc = zero16(), Y = zero16();
        if (have_next) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks], cn[ks], acc, 0, 0, 0);
        }
        if (s >= 0) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fs[ks], cf[ks], Y, 0, 0, 0);
        }
        uint4 gn0 = make_uint4(0, 0, 0, 0), gn1 = gn0;
        if (have_next)
            mask_diag(acc, L.tab[bn], 32 * IH, i, q, c.Dh, gn0, gn1);
        // ---- outputs of tile s ----
        if (s >= 0) {
            const SsmTile t = tile_at(c, s);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                Y[r] *= ei;
            Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, __builtin_bit_cast(bf16x8, g0), Y, 0, 0, 0);
            Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, __builtin_bit_cast(bf16x8, g1), Y, 0, 0, 0);
            if (IH == 1) {
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x2, __builtin_bit_cast(bf16x8, m0), Y, 0, 0, 0);
                Y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x3, __builtin_bit_cast(bf16x8, m1), Y, 0, 0, 0);
            }
            // Y^T[p, i]: element r of this lane is channel 8(r/4) + 4q + r%4 of
            // token i.  Through this wave's own LDS tile to token-major rows, then
            // 16 bytes per lane with four lanes per 64-byte row of y.
            bf16_t(*ys)[LDY] = L.Ys[IH];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<uint2 *>(&ys[i][8 * a + 4 * q]) =
                    make_uint2(pack2(Y[4 * a], Y[4 * a + 1]), pack2(Y[4 * a + 2], Y[4 * a + 3]));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // same wave: LDS executes in order
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int tok = (lane >> 2) + 16 * m;
                const uint4 o = *reinterpret_cast<const uint4 *>(&ys[tok][8 * (lane & 3)]);
                if (32 * IH + tok < t.len)
                    *reinterpret_cast<uint4 *>(c.y + (((size_t)t.tok0 + 32 * IH + tok) * c.H + c.h) * c.P + c.pbase +
                                               8 * (lane & 3)) = o;
            }
        }
        // the scores part hands its C fragments and masked block to the next step
        if (have_next) {
            g0 = gn0;
            g1 = gn1;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                cf[ks] = cn[ks];
        }
    });
}

// ---------------------------------------------------------------- state update of tile k, 64 state indices
__device__ __forceinline__ void role_state(const Ctx &c, Lds &L, int lane, int sw)
{
    // S^T tiles: rows n = 64sw + 32t + 8(r/4) + 4(lane/32) + r%4, column p = lane%32
    const int p = lane & 31, q = lane >> 5;
    f32x16 S[2];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int n0 = 64 * sw + 32 * t2 + 8 * a + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c.init)
                v = *reinterpret_cast<const float4 *>(c.init + ((size_t)c.h * c.P + c.pbase + p) * kN + n0);
            S[t2][4 * a + 0] = v.x;
            S[t2][4 * a + 1] = v.y;
            S[t2][4 * a + 2] = v.z;
            S[t2][4 * a + 3] = v.w;
            *reinterpret_cast<uint2 *>(&L.Ss[1][p][n0]) = make_uint2(pack2(v.x, v.y), pack2(v.z, v.w));
        }
    // transpose reads, natural token order: group g4 covers row/column block
    // g4&1 and tokens 8(g4>>1) + 0..7 of each 16-token k-step
    const int g4 = lane >> 4;
    const int tr_row = 8 * (g4 >> 1) + ((lane & 15) >> 2);
    const int tr_col = 16 * (g4 & 1) + 4 * (lane & 3);
    pipe_loop(c.n_tiles, [&](int s, auto U) {
        constexpr int u = decltype(U)::value;
        constexpr int b = (u + 1) % 3;  // == s % 3 for s >= 0
        if (s >= 0) {
            const SsmTile t = tile_at(c, s);
            const float dl = L.tab[b].ei[kQ - 1];  // padded tokens have dt = 0, so this is e^{l_len}
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                S[0][r] *= dl;
                S[1][r] *= dl;
            }
            const bf16_t *pb = &L.Bs[b][tr_row][64 * sw + tr_col];
            const bf16_t *px = &L.Xs[b][tr_row][tr_col];
            bf16x8 fx[4], f0[4], f1[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                fx[ks] = lds_frag_tr(px + 16 * ks * LDX, px + (16 * ks + 4) * LDX);
                f0[ks] = lds_frag_tr(pb + 16 * ks * LDB, pb + (16 * ks + 4) * LDB);
                f1[ks] = lds_frag_tr(pb + 16 * ks * LDB + 32, pb + (16 * ks + 4) * LDB + 32);
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0[ks], fx[ks], S[0], 0, 0, 0);
                S[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[ks], fx[ks], S[1], 0, 0, 0);
            }
            // bf16 copy for the next tile's S.C product; checkpoint
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int n0 = 64 * sw + 32 * t2 + 8 * a + 4 * q;
                    *reinterpret_cast<uint2 *>(&L.Ss[s & 1][p][n0]) =
                        make_uint2(pack2(S[t2][4 * a], S[t2][4 * a + 1]), pack2(S[t2][4 * a + 2], S[t2][4 * a + 3]));
                    if (t.ckpt_slot >= 0)
                        *reinterpret_cast<float4 *>(c.state_out +
                                                    (((size_t)t.ckpt_slot * c.H + c.h) * c.P + c.pbase + p) * kN + n0) =
                            make_float4(S[t2][4 * a], S[t2][4 * a + 1], S[t2][4 * a + 2], S[t2][4 * a + 3]);
                }
        }
    });
}

// Pointers are separate __restrict__ parameters (not a struct) so that the
// compiler may read the read-only tables with scalar loads.
__global__ __launch_bounds__(kThreads) void ssm_scan_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ dt, const float *__restrict__ A_,
    const bf16_t *__restrict__ Bg, const bf16_t *__restrict__ Cg, const float *__restrict__ D_,
    bf16_t *__restrict__ y, float *__restrict__ state_out, const float *const *__restrict__ init_ptrs,
    const SsmTile *__restrict__ tiles, const SsmSeq *__restrict__ seqs, int H, int P, int G, int p_split,
    int wg_per_xcd, int n_wg)
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
    switch (w) {
    case 0: role_half<0>(c, L, lane); break;
    case 1: role_half<1>(c, L, lane); break;
    case 2: role_state(c, L, lane, 0); break;
    case 3: role_state(c, L, lane, 1); break;
    case 4: role_load_bc<false>(c, L, lane); break;
    case 5: role_load_bc<true>(c, L, lane); break;
    case 6: role_offdiag(c, L, lane); break;
    default: role_load_x(c, L, lane); break;
    }
}

}  // namespace

hipError_t launch_scan_mfma(const ssm_plan *plan, const ScanArgs &args, void *, hipStream_t stream)
{
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
    hipLaunchKernelGGL(ssm_scan_mfma_kernel, dim3((unsigned)(per_xcd * 8)), dim3(kThreads), lds, stream,
                       static_cast<const bf16_t *>(args.x), static_cast<const bf16_t *>(args.dt), args.A,
                       static_cast<const bf16_t *>(args.B), static_cast<const bf16_t *>(args.C), args.D,
                       static_cast<bf16_t *>(args.y), static_cast<float *>(args.state_out),
                       reinterpret_cast<const float *const *>(args.init_ptrs), args.tiles, args.seqs,
                       args.H, args.P, args.G, args.p_split, per_xcd, n_wg);
    return hipGetLastError();
}
