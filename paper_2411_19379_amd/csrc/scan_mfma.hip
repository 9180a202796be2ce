// bf16 MFMA scan kernel for gfx950: d_state 128, headdim a multiple of 32,
// bf16 x/dt/B/C/y, fp32 A/D/state.
//
// One workgroup (4 waves) owns one (sequence, head, 32-channel slice) and
// walks the sequence's tiles in order; the slice's [32,128] state stays in
// MFMA accumulators from the first token to the last, so states reach device
// memory only as requested checkpoints.  Per tile of q <= 64 tokens starting
// after token s, with l_i = A * sum_{k<=i} dt_k inside the tile:
//
//   Gm[i,j] = (C_i.B_j) e^{l_i-l_j}      for j <= i, else 0     (masked score)
//   y_i     = e^{l_i} (S_s C_i) + sum_j Gm[i,j] (dt_j x_j) + D x_i
//   S_e     = e^{l_q} S_s + sum_j (e^{l_q-l_j} dt_j x_j) B_j^T
//
// All three contractions run on the matrix cores with bf16 operands and fp32
// accumulation; bf16 rounding touches only MFMA operands (x scaled by dt or
// by the decay weight, Gm, and the copy of S used for S.C).  Decay exponents,
// accumulators and checkpoints are fp32.
//
// Products are computed transposed (Gm^T, Y^T, S^T) so that every lane ends
// up with 4 consecutive elements along the destination's fastest axis.
#include "device_utils.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;
constexpr int kQ = kMfmaTileTokens;  // 64 tokens per tile
constexpr int kN = 128;              // d_state
constexpr int kPW = 32;              // channels per workgroup
constexpr int LDN = kN + 8;          // row stride (elements) of [*][128] bf16 tiles
constexpr int LDT = kQ + 8;          // row stride of [*][64] bf16 tiles
constexpr int LDX = kPW + 8;         // row stride of the raw x tile

struct Lds {
    bf16_t Bs[kQ][LDN];    // B tile, token major
    bf16_t Cs[kQ][LDN];    // C tile, token major
    bf16_t BT[kN][LDT];    // B tile, state-index major
    bf16_t XsT[kPW][LDT];  // e^{l_q-l_j} dt_j x_j, channel major
    bf16_t XdT[kPW][LDT];  // dt_j x_j, channel major
    bf16_t Xr[kQ][LDX];    // x tile as loaded
    bf16_t Gm[kQ][LDT];    // masked scores, row i, column j
    bf16_t Ss[kPW][LDN];   // bf16 copy of the running state, channel major
    float ell[kQ];
};

__device__ __forceinline__ bf16x8 lds_frag(const bf16_t *p)
{
    return *reinterpret_cast<const bf16x8 *>(p);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

struct TileRegs {
    uint4 x;      // 8 channels of one token
    uint4 b[4];   // 4 x (one token row, 8 state indices) of B
    uint4 c[4];
    float dt;     // lane j of every wave: dt of token j
};

__global__ __launch_bounds__(kThreads) void ssm_scan_mfma_kernel(ScanArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    Lds &L = *reinterpret_cast<Lds *>(lds_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int H = a.H, P = a.P, G = a.G;
    const int ps = blockIdx.x % a.p_split;
    const int h = (blockIdx.x / a.p_split) % H;
    const int seq = blockIdx.x / (a.p_split * H);
    const int g = h / (H / G);
    const int pbase = ps * kPW;

    const bf16_t *x = static_cast<const bf16_t *>(a.x);
    const bf16_t *dt = static_cast<const bf16_t *>(a.dt);
    const bf16_t *Bg = static_cast<const bf16_t *>(a.B);
    const bf16_t *Cg = static_cast<const bf16_t *>(a.C);
    bf16_t *y = static_cast<bf16_t *>(a.y);
    const float Ah = a.A[h];
    const float Dh = a.D[h];

    // staging roles
    const int x_tok = tid >> 2, x_p0 = (tid & 3) * 8;
    const int b_row = tid >> 4, b_n0 = (tid & 15) * 8;

    // S^T accumulator tile of this wave: rows n = 32w + 8(r/4) + 4(lane/32) + r%4, column p = lane%32
    const int s_p = lane & 31;
    const int s_nb = 32 * w + 4 * (lane >> 5);
    f32x16 S;
    {
        const float *init = a.init_ptrs ? a.init_ptrs[seq] : nullptr;
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
            uint2 pk = make_uint2(pack2(v.x, v.y), pack2(v.z, v.w));
            *reinterpret_cast<uint2 *>(&L.Ss[s_p][n0]) = pk;
        }
    }

    const SsmSeq sq = a.seqs[seq];

    auto load_tile = [&](const SsmTile &t, TileRegs &r) {
        const size_t tok0 = (size_t)t.tok0;
        const uint4 z = make_uint4(0, 0, 0, 0);
        r.x = x_tok < t.len
                  ? *reinterpret_cast<const uint4 *>(x + ((tok0 + x_tok) * H + h) * P + pbase + x_p0)
                  : z;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int row = b_row + 16 * k;
            const size_t off = ((tok0 + row) * G + g) * kN + b_n0;
            r.b[k] = row < t.len ? *reinterpret_cast<const uint4 *>(Bg + off) : z;
            r.c[k] = row < t.len ? *reinterpret_cast<const uint4 *>(Cg + off) : z;
        }
        r.dt = lane < t.len ? bf16_to_f32(dt[(tok0 + lane) * H + h]) : 0.f;
    };

    TileRegs R;
    SsmTile t = sq.tile_begin < sq.tile_end ? a.tiles[sq.tile_begin] : SsmTile{0, 0, -1, 0};
    if (sq.tile_begin < sq.tile_end)
        load_tile(t, R);

    for (int ti = sq.tile_begin; ti < sq.tile_end; ++ti) {
        const int len = t.len;
        const size_t tok0 = (size_t)t.tok0;
        const int slot = t.ckpt_slot;

        // ---- decay exponents: inclusive scan of dt*A over the 64 lanes (every wave) ----
        float ell = R.dt * Ah;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float up = __shfl_up(ell, d, 64);
            if (lane >= d)
                ell += up;
        }
        const float ell_last = __shfl(ell, 63, 64);
        if (w == 0)
            L.ell[lane] = ell;

        // ---- stage the tile into LDS ----
        {
            const float dt_tok = __shfl(R.dt, x_tok, 64);
            const float ell_tok = __shfl(ell, x_tok, 64);
            const float w_tok = __expf(ell_last - ell_tok) * dt_tok;
            const uint32_t xv[4] = {R.x.x, R.x.y, R.x.z, R.x.w};
            *reinterpret_cast<uint4 *>(&L.Xr[x_tok][x_p0]) = R.x;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = bf16_to_f32((bf16_t)(xv[e >> 1] >> (16 * (e & 1))));
                L.XdT[x_p0 + e][x_tok] = f32_to_bf16(dt_tok * v);
                L.XsT[x_p0 + e][x_tok] = f32_to_bf16(w_tok * v);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int row = b_row + 16 * k;
                *reinterpret_cast<uint4 *>(&L.Bs[row][b_n0]) = R.b[k];
                *reinterpret_cast<uint4 *>(&L.Cs[row][b_n0]) = R.c[k];
                const uint32_t bv[4] = {R.b[k].x, R.b[k].y, R.b[k].z, R.b[k].w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    L.BT[b_n0 + e][row] = (bf16_t)(bv[e >> 1] >> (16 * (e & 1)));
            }
        }
        __syncthreads();

        // next tile's global loads fly while this tile is computed
        SsmTile tn = t;
        if (ti + 1 < sq.tile_end) {
            tn = a.tiles[ti + 1];
            load_tile(tn, R);
        }

        // ---- Gm^T = mask(B C^T o decay): three 32x32 tiles on waves 0..2 ----
        if (w < 3) {
            const int jb = w == 2 ? 1 : 0, ib = w == 0 ? 0 : 1;
            f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            const bf16_t *pa = &L.Bs[32 * jb + (lane & 31)][8 * (lane >> 5)];
            const bf16_t *pb = &L.Cs[32 * ib + (lane & 31)][8 * (lane >> 5)];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(pa + 16 * ks), lds_frag(pb + 16 * ks),
                                                              acc, 0, 0, 0);
            const int i = 32 * ib + (lane & 31);
            const float ell_i = L.ell[i];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int j0 = 32 * jb + 8 * q4 + 4 * (lane >> 5);
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = j0 + r;
                    v[r] = j <= i ? acc[4 * q4 + r] * __expf(ell_i - L.ell[j]) : 0.f;
                }
                *reinterpret_cast<uint2 *>(&L.Gm[i][j0]) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
            }
        }

        // ---- state: S^T <- e^{l_q} S^T + B^T (w x), one 32-row tile of state indices per wave ----
        {
            const float dl = __expf(ell_last);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                S[r] *= dl;
            const bf16_t *pa = &L.BT[32 * w + (lane & 31)][8 * (lane >> 5)];
            const bf16_t *pb = &L.XsT[lane & 31][8 * (lane >> 5)];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(pa + 16 * ks), lds_frag(pb + 16 * ks),
                                                            S, 0, 0, 0);
        }
        __syncthreads();

        // ---- outputs: Y^T[p, i] for the 16 tokens i = 16w + lane%16, two 16-channel blocks ----
        {
            const int i = 16 * w + (lane & 15);
            const int kq = 8 * (lane >> 4);
            f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
            // S_s C_i with the state as it was before this tile
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 fb = lds_frag(&L.Cs[i][32 * ks + kq]);
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    acc[pb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        lds_frag(&L.Ss[16 * pb + (lane & 15)][32 * ks + kq]), fb, acc[pb], 0, 0, 0);
            }
            const float ei = __expf(L.ell[i]);
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
                acc[pb] *= ei;
            // intra-tile term; columns j > i are masked, so later 32-token halves can be skipped
            const int nks = w >= 2 ? 2 : 1;
            for (int ks = 0; ks < nks; ++ks) {
                const bf16x8 fb = lds_frag(&L.Gm[i][32 * ks + kq]);
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
                    acc[pb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        lds_frag(&L.XdT[16 * pb + (lane & 15)][32 * ks + kq]), fb, acc[pb], 0, 0, 0);
            }
            if (i < len) {
#pragma unroll
                for (int pb = 0; pb < 2; ++pb) {
                    const int p0 = 16 * pb + 4 * (lane >> 4);
                    const uint2 xr = *reinterpret_cast<const uint2 *>(&L.Xr[i][p0]);
                    const float x0 = bf16_to_f32((bf16_t)(xr.x & 0xffff)), x1 = bf16_to_f32((bf16_t)(xr.x >> 16));
                    const float x2 = bf16_to_f32((bf16_t)(xr.y & 0xffff)), x3 = bf16_to_f32((bf16_t)(xr.y >> 16));
                    const uint2 o = make_uint2(pack2(acc[pb][0] + Dh * x0, acc[pb][1] + Dh * x1),
                                               pack2(acc[pb][2] + Dh * x2, acc[pb][3] + Dh * x3));
                    *reinterpret_cast<uint2 *>(y + ((tok0 + i) * H + h) * P + pbase + p0) = o;
                }
            }
        }
        __syncthreads();

        // ---- publish the new state for the next tile's S.C product; checkpoint ----
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int n0 = s_nb + 8 * q4;
            *reinterpret_cast<uint2 *>(&L.Ss[s_p][n0]) =
                make_uint2(pack2(S[4 * q4], S[4 * q4 + 1]), pack2(S[4 * q4 + 2], S[4 * q4 + 3]));
            if (slot >= 0)
                *reinterpret_cast<float4 *>(a.state_out + (((size_t)slot * H + h) * P + pbase + s_p) * kN + n0) =
                    make_float4(S[4 * q4], S[4 * q4 + 1], S[4 * q4 + 2], S[4 * q4 + 3]);
        }
        t = tn;
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
    hipLaunchKernelGGL(ssm_scan_mfma_kernel, dim3((unsigned)plan->n_workgroups), dim3(kThreads), lds,
                       stream, args);
    return hipGetLastError();
}
