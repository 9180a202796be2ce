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
// accumulation; bf16 rounding touches only MFMA operands (Gm, the decay-
// weighted x, the copy of S used for S.C).  Decay exponents, accumulators and
// checkpoints are fp32.
//
// The 8 waves of a workgroup form a two-stage pipeline.  While the four
// "front" waves stage tile m into LDS and turn it into masked scores, the four
// "back" waves consume tile m-1: outputs first, then the state update.  Two
// workgroup barriers per tile separate the stages; all tile buffers are double
// buffered.  Products are computed transposed (Gm^T, Y^T, S^T) so every lane
// holds 4 consecutive elements along the destination's fastest axis, and the
// token-major B and x tiles are fed to the state update through the LDS
// transpose reads of gfx950.
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
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kThreads = 512;
constexpr int kQ = kMfmaTileTokens;  // 64 tokens per tile
constexpr int kN = 128;              // d_state
constexpr int kPW = 32;              // channels per workgroup
constexpr int LDN = kN + 8;          // row stride (elements) of the B, C and state tiles
constexpr int LDG = kQ + 8;          // row stride of the score tile
constexpr int LDX = kPW;             // row stride of the x tiles (unpadded on purpose)
constexpr float kLog2e = 1.4426950408889634f;

struct TileBuf {
    bf16_t Bs[kQ][LDN];  // B tile, token major
    bf16_t Cs[kQ][LDN];  // C tile, token major
    bf16_t Xs[kQ][LDX];  // e^{l_q-l_j} dt_j x_j, token major
    bf16_t Xr[kQ][LDX];  // x as loaded, token major
    bf16_t Gm[kQ][LDG];  // masked scores, row i, column j
    float ei[kQ];        // e^{l_i}
};

struct Lds {
    TileBuf buf[2];
    bf16_t Ss[kPW][LDN];  // bf16 copy of the running state, channel major
    float ell2[kQ];       // l_i * log2(e)
    float cj[kQ];         // l_j * log2(e) - log2(dt_j)
    float cfac[3][kQ];    // column factors of the off-diagonal score blocks, row blocks 1..3
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

// 8 k-values of a transposed operand: rows r0..r0+7 of a token-major tile
__device__ __forceinline__ bf16x8 lds_frag_tr(const bf16_t *p, int row_stride)
{
    const s16x4 lo = lds_tr4(p), hi = lds_tr4(p + 4 * row_stride);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also
// wait for every outstanding global load, i.e. for the prefetch of the next
// tile, on each of the two barriers of a tile.  Global memory written by this
// kernel is never read back by it, so LDS ordering is all the stages need.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP row shifts and the
// two row broadcasts (no LDS round trips).
#define SSM_DPP(old, v, ctrl, row_mask, bound)                                                      \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, (float)(old)),     \
                                                          __builtin_bit_cast(int, (float)(v)), (ctrl), \
                                                          (row_mask), 0xF, (bound)))
__device__ __forceinline__ float wave_inclusive_sum(float v)
{
    v += SSM_DPP(0.f, v, 0x111, 0xF, true);  // row_shr:1
    v += SSM_DPP(0.f, v, 0x112, 0xF, true);  // row_shr:2
    v += SSM_DPP(0.f, v, 0x114, 0xF, true);  // row_shr:4
    v += SSM_DPP(0.f, v, 0x118, 0xF, true);  // row_shr:8
    v += SSM_DPP(0.f, v, 0x142, 0xA, false); // row_bcast:15 into rows 1 and 3
    v += SSM_DPP(0.f, v, 0x143, 0xC, false); // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ float read_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

struct TileRegs {
    uint4 x;     // 8 channels of one token
    uint4 b[4];  // 4 x (one token row, 8 state indices) of B
    uint4 c[4];
    uint32_t dt; // lane j of every front wave: bf16 bits of dt of token j
};

// Score blocks (16x16, jb <= ib) of each front wave, one byte per block: jb in
// the low nibble, ib in the high one.  Waves 0 and 1 take three blocks, waves 2
// and 3 two; immediates rather than a table so that no memory read is needed.
__device__ __forceinline__ uint32_t score_blocks(int w)
{
    return w == 0 ? 0x201000u : w == 1 ? 0x323130u : w == 2 ? 0x2111u : 0x3322u;
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

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const bool front = w < 4;
    const int ps = wg % p_split;
    const int h = (wg / p_split) % H;
    const int seq = wg / (p_split * H);
    const int g = h / (H / G);
    const int pbase = ps * kPW;
    const float Ah = A_[h];
    const float Dh = D_[h];

    // front waves: staging roles (ft = 0..255)
    const int ft = tid & 255;
    const int x_tok = ft >> 2, x_p0 = (ft & 3) * 8;
    const int b_row = ft >> 4, b_n0 = (ft & 15) * 8;
    // back waves: wave kw owns state rows n = 32kw + 8(r/4) + 4(lane/32) + r%4, column p = lane%32
    const int kw = w & 3;
    const int s_p = lane & 31;
    const int s_nb = 32 * kw + 4 * (lane >> 5);

    f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (!front) {
        const float *init = init_ptrs ? init_ptrs[seq] : nullptr;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            const int n0 = s_nb + 8 * q4;
            if (init)
                v = *reinterpret_cast<const float4 *>(init + ((size_t)h * P + pbase + s_p) * kN + n0);
            S[4 * q4 + 0] = v.x;
            S[4 * q4 + 1] = v.y;
            S[4 * q4 + 2] = v.z;
            S[4 * q4 + 3] = v.w;
            *reinterpret_cast<uint2 *>(&L.Ss[s_p][n0]) = make_uint2(pack2(v.x, v.y), pack2(v.z, v.w));
        }
    } else {
        // score blocks above the diagonal are read as part of 32-wide k-steps but never written
        uint32_t *gz0 = reinterpret_cast<uint32_t *>(&L.buf[0].Gm[0][0]);
        uint32_t *gz1 = reinterpret_cast<uint32_t *>(&L.buf[1].Gm[0][0]);
        for (int i = ft; i < kQ * LDG / 2; i += 256) {
            gz0[i] = 0u;
            gz1[i] = 0u;
        }
    }

    const SsmSeq sq = seqs[seq];
    const int n_tiles = sq.tile_end - sq.tile_begin;
    if (n_tiles <= 0)
        return;  // empty sequence: the whole workgroup leaves before any barrier

    auto load_tile = [&](const SsmTile &t, TileRegs &r) {
        const size_t tok0 = (size_t)t.tok0;
        const uint4 z = make_uint4(0, 0, 0, 0);
        // (plain ifs: a select between a global address and a zero temporary
        // would turn these into flat loads through scratch)
        r.x = z;
        if (x_tok < t.len)
            r.x = *reinterpret_cast<const uint4 *>(x + ((tok0 + x_tok) * H + h) * P + pbase + x_p0);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = b_row + 16 * k;
            const size_t off = ((tok0 + row) * G + g) * kN + b_n0;
            r.b[k] = z;
            r.c[k] = z;
            if (row < t.len) {
                r.b[k] = *reinterpret_cast<const uint4 *>(Bg + off);
                r.c[k] = *reinterpret_cast<const uint4 *>(Cg + off);
            }
        }
        r.dt = 0u;  // converted where it is used, so that nothing here waits for the loads
        if (lane < t.len)
            r.dt = dt[(tok0 + lane) * H + h];
    };

    // Tile descriptors travel through a short register pipeline (tile s-1, s,
    // s+1, and s+2 in flight), read with scalar loads two steps ahead of use.
    // (Indices past the end are clamped: those descriptors are never used.)
    auto tile_at = [&](int k) -> SsmTile {
        const int kk = k < n_tiles ? k : n_tiles - 1;
        return tiles[__builtin_amdgcn_readfirstlane(sq.tile_begin + kk)];
    };
    SsmTile tb = tile_at(0);      // tile s-1 (back waves; unused in step 0)
    SsmTile t_cur = tile_at(0);   // tile s
    SsmTile t_nxt = tile_at(1);   // tile s+1

    TileRegs R;
    if (front)
        load_tile(t_cur, R);
    __syncthreads();
    SSM_TRACE_DECL

    for (int s = 0; s <= n_tiles; ++s) {
        TileBuf &Tf = L.buf[s & 1];        // tile s, produced by the front waves
        TileBuf &Tb = L.buf[(s & 1) ^ 1];  // tile s-1, consumed by the back waves
        const SsmTile t_nn = tile_at(s + 2);

        // ================= phase 1 =================
        if (front) {
            if (s < n_tiles) {
                // decay exponents: inclusive scan of dt*A over the 64 lanes (lane = token)
                const float dtj = __uint_as_float(R.dt << 16);
                const float ell = wave_inclusive_sum(dtj * Ah);
                SSM_TRACE(5);
                const float ell2 = ell * kLog2e;
                const float ell2_last = read_lane(ell2, 63);
                const float wj = exp2_fast(ell2_last - ell2) * dtj;  // weight of token `lane` in the state update
                const float w_tok = __shfl(wj, x_tok, 64);

                // x tile: raw copy and decay-weighted copy, both token major
                *reinterpret_cast<uint4 *>(&Tf.Xr[x_tok][x_p0]) = R.x;
                {
                    const uint32_t xv[4] = {R.x.x, R.x.y, R.x.z, R.x.w};
                    uint32_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(xv[e] << 16);
                        const float hi = __uint_as_float(xv[e] & 0xffff0000u);
                        o[e] = pack2(w_tok * lo, w_tok * hi);
                    }
                    *reinterpret_cast<uint4 *>(&Tf.Xs[x_tok][x_p0]) = make_uint4(o[0], o[1], o[2], o[3]);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int row = b_row + 16 * k;
                    *reinterpret_cast<uint4 *>(&Tf.Bs[row][b_n0]) = R.b[k];
                    *reinterpret_cast<uint4 *>(&Tf.Cs[row][b_n0]) = R.c[k];
                }
                // per-token factors, spread over the four front waves
                if (w == 0) {
                    L.ell2[lane] = ell2;
                    L.cj[lane] = ell2 - __builtin_amdgcn_logf(dtj);
                    Tf.ei[lane] = exp2_fast(ell2);
                } else {
                    const float ref = read_lane(ell2, 16 * w - 1);  // end of row block w-1
                    L.cfac[w - 1][lane] = lane < 16 * w ? exp2_fast(ref - ell2) * dtj : 0.f;
                }
                SSM_TRACE(6);
                // next tile's global loads fly while this one is turned into scores
                if (s + 1 < n_tiles)
                    load_tile(t_nxt, R);
            }
        } else if (s >= 1) {
            // ---- outputs of tile s-1: Y^T[p, i], tokens i = 16kw + lane%16, two 16-channel blocks ----
            const int i = 16 * kw + (lane & 15);
            const int kq = 8 * (lane >> 4);
            f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 fb = lds_frag(&Tb.Cs[i][32 * ks + kq]);
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    acc[pb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        lds_frag(&L.Ss[16 * pb + (lane & 15)][32 * ks + kq]), fb, acc[pb], 0, 0, 0);
            }
            const float ei = Tb.ei[i];
            acc[0] *= ei;
            acc[1] *= ei;
            // intra-tile term; columns j > i are masked, so later 32-token halves can be skipped
            const int nks = kw >= 2 ? 2 : 1;
            // transposed x operand: this lane's group reads tokens 32ks + 8(lane/16) + {0..7}
            const bf16_t *xt = &Tb.Xr[kq + ((lane & 15) >> 2)][4 * (lane & 3)];
            for (int ks = 0; ks < nks; ++ks) {
                const bf16x8 fb = lds_frag(&Tb.Gm[i][32 * ks + kq]);
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    acc[pb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        lds_frag_tr(xt + 32 * ks * LDX + 16 * pb, LDX), fb, acc[pb], 0, 0, 0);
            }
            if (i < tb.len) {
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    const int p0 = 16 * pb + 4 * (lane >> 4);
                    const uint2 xr = *reinterpret_cast<const uint2 *>(&Tb.Xr[i][p0]);
                    const float x0 = __uint_as_float(xr.x << 16), x1 = __uint_as_float(xr.x & 0xffff0000u);
                    const float x2 = __uint_as_float(xr.y << 16), x3 = __uint_as_float(xr.y & 0xffff0000u);
                    const uint2 o = make_uint2(pack2(acc[pb][0] + Dh * x0, acc[pb][1] + Dh * x1),
                                               pack2(acc[pb][2] + Dh * x2, acc[pb][3] + Dh * x3));
                    *reinterpret_cast<uint2 *>(y + (((size_t)tb.tok0 + i) * H + h) * P + pbase + p0) = o;
                }
            }
        }
        SSM_TRACE(1);
        lds_barrier();
        SSM_TRACE(2);

        // ================= phase 2 =================
        if (front) {
            if (s < n_tiles) {
                // ---- Gm^T = mask(B C^T o decay): 16x16 blocks (jb <= ib), 2-3 per wave ----
                const int cnt = w < 2 ? 3 : 2;
                const uint32_t blocks = score_blocks(w);
                for (int t = 0; t < cnt; ++t) {
                    const int jb = (blocks >> (8 * t)) & 3, ib = (blocks >> (8 * t + 4)) & 3;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    const bf16_t *pa = &Tf.Bs[16 * jb + (lane & 15)][8 * (lane >> 4)];
                    const bf16_t *pb = &Tf.Cs[16 * ib + (lane & 15)][8 * (lane >> 4)];
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds_frag(pa + 32 * ks), lds_frag(pb + 32 * ks),
                                                                      acc, 0, 0, 0);
                    const int i = 16 * ib + (lane & 15);
                    const int j0 = 16 * jb + 4 * (lane >> 4);
                    const float ell2_i = L.ell2[i];
                    float v[4];
                    if (jb == ib) {
                        const float4 c4 = *reinterpret_cast<const float4 *>(&L.cj[j0]);
                        const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            v[r] = j0 + r <= i ? acc[r] * exp2_fast(ell2_i - cc[r]) : 0.f;
                    } else {
                        const float ri = exp2_fast(ell2_i - L.ell2[16 * ib - 1]);
                        const float4 c4 = *reinterpret_cast<const float4 *>(&L.cfac[ib - 1][j0]);
                        v[0] = acc[0] * (ri * c4.x);
                        v[1] = acc[1] * (ri * c4.y);
                        v[2] = acc[2] * (ri * c4.z);
                        v[3] = acc[3] * (ri * c4.w);
                    }
                    *reinterpret_cast<uint2 *>(&Tf.Gm[i][j0]) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
                }
            }
        } else if (s >= 1) {
            // ---- state: S^T <- e^{l_q} S^T + B^T (w x); 32 state indices per wave, all 32 channels ----
            const float dl = Tb.ei[kQ - 1];  // padded tokens have dt = 0, so this is e^{l_len}
#pragma unroll
            for (int r = 0; r < 16; ++r)
                S[r] *= dl;
            // transpose reads: lane group g4 = lane/16 covers 16 rows/columns (g4%2) and 8 tokens (g4/2)
            const int g4 = lane >> 4;
            const int trow = 8 * (g4 >> 1) + ((lane & 15) >> 2);
            const bf16_t *pa = &Tb.Bs[trow][32 * kw + 16 * (g4 & 1) + 4 * (lane & 3)];
            const bf16_t *pb = &Tb.Xs[trow][16 * (g4 & 1) + 4 * (lane & 3)];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_tr(pa + 16 * ks * LDN, LDN),
                                                            lds_frag_tr(pb + 16 * ks * LDX, LDX), S, 0, 0, 0);
            // publish the new state for the next tile's S.C product; checkpoint
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int n0 = s_nb + 8 * q4;
                *reinterpret_cast<uint2 *>(&L.Ss[s_p][n0]) =
                    make_uint2(pack2(S[4 * q4], S[4 * q4 + 1]), pack2(S[4 * q4 + 2], S[4 * q4 + 3]));
                if (tb.ckpt_slot >= 0)
                    *reinterpret_cast<float4 *>(state_out +
                                                (((size_t)tb.ckpt_slot * H + h) * P + pbase + s_p) * kN + n0) =
                        make_float4(S[4 * q4], S[4 * q4 + 1], S[4 * q4 + 2], S[4 * q4 + 3]);
            }
        }
        SSM_TRACE(3);
        lds_barrier();
        SSM_TRACE(4);
        tb = t_cur;
        t_cur = t_nxt;
        t_nxt = t_nn;
    }
}

}  // namespace

hipError_t launch_scan_mfma(const ssm_plan *plan, const ScanArgs &args, hipStream_t stream)
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
                       static_cast<bf16_t *>(args.y), args.state_out, args.init_ptrs, args.tiles, args.seqs,
                       args.H, args.P, args.G, args.p_split, per_xcd, n_wg);
    return hipGetLastError();
}
