// fp32 vector-ALU scan kernel: any head shape that fits, f32 or bf16 storage,
// all arithmetic in fp32 (decay exponents summed in fp64).  It is the path of
// the fp32 mode and of shapes the MFMA kernel does not cover.
//
// One workgroup owns one (sequence, head) pair and walks the sequence's tiles
// in order, the [P,N] state living in registers (and mirrored in LDS for the
// C.S products).  Per tile of q <= 16 tokens starting after token s, with
// l_i = A * sum_{k<=i} dt_k inside the tile:
//
//   y_i  = e^{l_i} (S_s C_i) + sum_{j<=i} (C_i.B_j) e^{l_i-l_j} dt_j x_j + D x_i
//   S_e  = e^{l_q} S_s + sum_j e^{l_q-l_j} dt_j x_j B_j^T
//
// which is the token recurrence of ssm_prefill.h unrolled over the tile.
#include "device_utils.h"

namespace {

constexpr int kThreads = 256;
constexpr int kQ = kValuTileTokens;

template <typename IO, int EPT>
__global__ __launch_bounds__(kThreads) void ssm_scan_valu_kernel(ScanArgs a)
{
    const int tid = threadIdx.x;
    const int H = a.H, P = a.P, N = a.N, G = a.G;
    const int seq = blockIdx.x / H;
    const int h = blockIdx.x % H;
    const int g = h / (H / G);
    const int PN = P * N;
    const int NP1 = N + 1;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    double *ell = reinterpret_cast<double *>(lds_raw);            // [q] inclusive sums of dt*A
    float *S_lds = reinterpret_cast<float *>(ell + kQ);           // [P][N+1]
    float *xs = S_lds + (size_t)P * NP1;                          // [q][P]
    float *Bs = xs + kQ * P;                                      // [q][N]
    float *Cs = Bs + kQ * N;                                      // [q][N]
    float *Gm = Cs + kQ * N;                                      // [q][q] masked scores
    float *dts = Gm + kQ * kQ;                                    // [q]
    float *wj = dts + kQ;                                         // [q] e^{l_last-l_j} dt_j
    float *ei = wj + kQ;                                          // [q] e^{l_i}

    const IO *x = static_cast<const IO *>(a.x);
    const IO *dt = static_cast<const IO *>(a.dt);
    const IO *Bg = static_cast<const IO *>(a.B);
    const IO *Cg = static_cast<const IO *>(a.C);
    IO *y = static_cast<IO *>(a.y);
    const float Ah = a.A[h];
    const float Dh = a.D[h];

    // running state: element e = tid + k*256 of this head's [P,N] block
    float acc[EPT];
    const void *init = a.init_ptrs ? a.init_ptrs[seq] : nullptr;
    const int st = a.state_dtype;
#pragma unroll
    for (int k = 0; k < EPT; ++k) {
        const int e = tid + k * kThreads;
        float v = 0.f;
        if (e < PN) {
            if (init)
                v = state_load(init, (size_t)h * PN + e, st);
            S_lds[(e / N) * NP1 + (e % N)] = v;
        }
        acc[k] = v;
    }

    const SsmSeq sq = a.seqs[seq];
    for (int ti = sq.tile_begin; ti < sq.tile_end; ++ti) {
        const SsmTile t = a.tiles[ti];
        const int len = t.len;
        const size_t tok0 = (size_t)t.tok0;

        if (tid < kQ)
            dts[tid] = tid < len ? IoTraits<IO>::load(dt + (tok0 + tid) * H + h) : 0.f;
        for (int idx = tid; idx < kQ * P; idx += kThreads) {
            const int i = idx / P, p = idx % P;
            xs[idx] = i < len ? IoTraits<IO>::load(x + ((tok0 + i) * H + h) * P + p) : 0.f;
        }
        for (int idx = tid; idx < kQ * N; idx += kThreads) {
            const int i = idx / N, n = idx % N;
            const size_t off = ((tok0 + i) * G + g) * N + n;
            Bs[idx] = i < len ? IoTraits<IO>::load(Bg + off) : 0.f;
            Cs[idx] = i < len ? IoTraits<IO>::load(Cg + off) : 0.f;
        }
        __syncthreads();

        if (tid < kQ) {
            double s = 0.0;
            for (int k = 0; k <= tid; ++k)
                s += (double)dts[k] * (double)Ah;
            ell[tid] = s;
        }
        __syncthreads();
        if (tid < kQ) {
            wj[tid] = tid < len ? expf((float)(ell[len - 1] - ell[tid])) * dts[tid] : 0.f;
            ei[tid] = expf((float)ell[tid]);
        }
        // masked, decayed scores: one (i, j) pair per thread
        {
            const int i = tid / kQ, j = tid % kQ;
            float v = 0.f;
            if (j <= i && i < len) {
                float dot = 0.f;
                for (int n = 0; n < N; ++n)
                    dot += Cs[i * N + n] * Bs[j * N + n];
                v = dot * expf((float)(ell[i] - ell[j])) * dts[j];
            }
            Gm[tid] = v;
        }
        __syncthreads();

        // outputs of the tile
        for (int idx = tid; idx < len * P; idx += kThreads) {
            const int i = idx / P, p = idx % P;
            float inter = 0.f;
            const float *Sp = S_lds + p * NP1;
            for (int n = 0; n < N; ++n)
                inter += Cs[i * N + n] * Sp[n];
            float intra = 0.f;
            for (int j = 0; j <= i; ++j)
                intra += Gm[i * kQ + j] * xs[j * P + p];
            const float v = ei[i] * inter + intra + Dh * xs[idx];
            IoTraits<IO>::store(y + ((tok0 + i) * H + h) * P + p, v);
        }
        __syncthreads();

        // state after the tile
        const float dlast = ei[len - 1];
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const int e = tid + k * kThreads;
            if (e < PN) {
                const int p = e / N, n = e % N;
                float s = dlast * acc[k];
                for (int j = 0; j < len; ++j)
                    s += (wj[j] * xs[j * P + p]) * Bs[j * N + n];
                acc[k] = s;
                S_lds[p * NP1 + n] = s;
                if (t.ckpt_slot >= 0)
                    state_store(a.state_out, ((size_t)t.ckpt_slot * H + h) * PN + e, s, st);
            }
        }
        __syncthreads();
    }
}

template <typename IO>
hipError_t launch_ept(int ept, dim3 grid, size_t lds, hipStream_t stream, const ScanArgs &args)
{
#define SSM_LAUNCH(E)                                                                     \
    hipLaunchKernelGGL((ssm_scan_valu_kernel<IO, E>), grid, dim3(kThreads), lds, stream, args); \
    break;
    switch (ept) {
    case 1: SSM_LAUNCH(1)
    case 2: SSM_LAUNCH(2)
    case 4: SSM_LAUNCH(4)
    case 8: SSM_LAUNCH(8)
    case 16: SSM_LAUNCH(16)
    default: SSM_LAUNCH(32)
    }
#undef SSM_LAUNCH
    return hipGetLastError();
}

}  // namespace

size_t ssm_valu_lds_bytes(int P, int N);

hipError_t launch_scan_valu(const ssm_plan *plan, const ScanArgs &args, hipStream_t stream)
{
    const int PN = args.P * args.N;
    int ept = 1;
    while (ept * kThreads < PN)
        ept *= 2;
    const dim3 grid((unsigned)plan->n_workgroups);
    const size_t lds = ssm_valu_lds_bytes(args.P, args.N);
    if (plan->shape.io_dtype == SSM_DT_F32)
        return launch_ept<float>(ept, grid, lds, stream, args);
    return launch_ept<bf16_t>(ept, grid, lds, stream, args);
}
