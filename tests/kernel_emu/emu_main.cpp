// Driver of the CPU emulation of the scan kernels (test infrastructure only): reads a problem file, builds the plan
// with the library's own plan code, runs the CPU-compiled scan kernel on fibers and writes y and the checkpoint
// states.  Every buffer a kernel sees is an exact-size allocation flush against an inaccessible page.
//   emu_main <in.bin> <out.bin> [order: 0 forward | 1 reverse | n>=2 shuffle seed] [end|start] [drop_barrier]
//   "end"/"start": which end of each buffer touches the inaccessible page (overruns / underruns fault)
//   drop_barrier: ordinal of one workgroup barrier that is made not to wait (self-test of the race check; -1: none)
//   a 6th argument "advance" runs the roll-forward kernel instead of the scan: every sequence's state (its initial
//   state, or zeros) is advanced in place, and the output holds y and then one state per sequence;
//   a 7th argument f16 or bf16 keeps cached states in that type (converted from and to fp32 around the run)
//   with EMU_WIDE set in the environment the matrix-core scan runs in its 64-channel variant
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "device_utils.h"

namespace emu {
void set_order_mode(int m);
void set_drop_barrier(long n);
long switches();
}  // namespace emu

#include "emu_host.h"

int main(int argc, char **argv)
{
    if (argc < 3) {
        fprintf(stderr, "usage: emu_main in.bin out.bin [order] [end|start] [drop_barrier]\n");
        return 2;
    }
    emu::set_order_mode(argc > 3 ? atoi(argv[3]) : 0);
    const bool end_aligned = !(argc > 4 && argv[4][0] == 's');
    if (argc > 5)
        emu::set_drop_barrier(atol(argv[5]));
    const bool advance = argc > 6 && strcmp(argv[6], "advance") == 0;
    // storage type of cached states for the candidate kernels: argv[7] = f16 | bf16 (default fp32)
    const int st_type = argc > 7 ? (strcmp(argv[7], "f16") == 0 ? 1 : strcmp(argv[7], "bf16") == 0 ? 2 : 0) : 0;
    const size_t st_esz = st_type == 0 ? 4 : 2;
    auto to_state = [&](void *dst, size_t e, float v) {
        if (st_type == 0)
            static_cast<float *>(dst)[e] = v;
        else if (st_type == 1)
            static_cast<_Float16 *>(dst)[e] = (_Float16)v;
        else
            static_cast<bf16_t *>(dst)[e] = f32_to_bf16(v);
    };
    auto from_state = [&](const void *src, size_t e) {
        return st_type == 0   ? static_cast<const float *>(src)[e]
               : st_type == 1 ? (float)static_cast<const _Float16 *>(src)[e]
                              : bf16_to_f32(static_cast<const bf16_t *>(src)[e]);
    };
    FILE *f = fopen(argv[1], "rb");
    if (!f) {
        perror(argv[1]);
        return 2;
    }
    int32_t hdr[10];
    read_vec(f, hdr, 10);
    if (hdr[0] != 0x53534d31) {
        fprintf(stderr, "bad magic\n");
        return 2;
    }
    const int io = hdr[1], T = hdr[2], H = hdr[3], P = hdr[4], N = hdr[5], G = hdr[6], chunk = hdr[7], batch = hdr[8],
              n_ckpt = hdr[9];
    const size_t esz = io == 0 ? 4 : 2;
    std::vector<int32_t> cu(batch + 1), cu_ck(batch + 1), ck(n_ckpt > 0 ? n_ckpt : 1), has_init(batch);
    read_vec(f, cu.data(), batch + 1);
    read_vec(f, cu_ck.data(), batch + 1);
    read_vec(f, ck.data(), n_ckpt);
    read_vec(f, has_init.data(), batch);
    const size_t nx = (size_t)T * H * P, ndt = (size_t)T * H, nb = (size_t)T * G * N, nst = (size_t)H * P * N;
    void *x = guarded(nx * esz, end_aligned), *dt = guarded(ndt * esz, end_aligned), *B = guarded(nb * esz, end_aligned),
         *C = guarded(nb * esz, end_aligned);
    float *A = static_cast<float *>(guarded(H * 4, end_aligned)), *D = static_cast<float *>(guarded(H * 4, end_aligned));
    read_vec(f, static_cast<unsigned char *>(x), nx * esz);
    read_vec(f, static_cast<unsigned char *>(dt), ndt * esz);
    read_vec(f, static_cast<unsigned char *>(B), nb * esz);
    read_vec(f, static_cast<unsigned char *>(C), nb * esz);
    read_vec(f, A, H);
    read_vec(f, D, H);
    const float **init = static_cast<const float **>(guarded(sizeof(float *) * (batch ? batch : 1), end_aligned));
    bool any_init = false;
    for (int b = 0; b < batch; ++b) {
        init[b] = nullptr;
        if (has_init[b]) {
            float *s = static_cast<float *>(guarded(nst * 4, end_aligned));
            read_vec(f, s, nst);
            init[b] = s;
            any_init = true;
        }
    }
    fclose(f);

    ssm_shape_t shape;
    shape.nheads = H, shape.headdim = P, shape.d_state = N, shape.ngroups = G, shape.chunk = chunk, shape.io_dtype = io;
    shape.state_dtype = st_type;
    ssm_plan_t *plan = nullptr;
    int rc = ssm_plan_create(&shape, batch, cu.data(), cu_ck.data(), ck.data(), &plan);
    if (rc != 0) {
        fprintf(stderr, "ssm_plan_create: %d %s\n", rc, ssm_last_error());
        return 2;
    }
    if (getenv("EMU_WIDE") && plan->path == SSM_PATH_MFMA_BF16 && P % kMfmaWideChannels == 0) {
        // the 64-channel variant of the matrix-core scan, which the plan itself picks only for grids that fill a GPU
        ssm_plan_build_stretches(plan, 1, 0);
    }
    if (const char *sp = getenv("EMU_SPLIT")) {
        // "K:min": sequences cut into up to K stretches of at least `min` tiles (the plan itself cuts only long
        // sequences of batches that would leave a GPU idle)
        int kk = 2, min_tiles = 1;
        sscanf(sp, "%d:%d", &kk, &min_tiles);
        if (plan->path == SSM_PATH_MFMA_BF16 && P % kMfmaWideChannels == 0) {
            int active = 0;
            for (int b = 0; b < batch; ++b)
                active += cu[b + 1] > cu[b];
            ssm_plan_build_stretches(plan, (int64_t)active * H * (P / kMfmaWideChannels) * kk, min_tiles);
            fprintf(stderr, "stretches: %zu, carry slots: %d\n", plan->scan_seqs.size(), plan->n_carry);
        }
    }
    const size_t nt = plan->tiles.size();
    SsmTile *tiles = static_cast<SsmTile *>(guarded(sizeof(SsmTile) * (nt ? nt : 1), end_aligned));
    SsmSeq *seqs = static_cast<SsmSeq *>(guarded(sizeof(SsmSeq) * (batch ? batch : 1), end_aligned));
    memcpy(tiles, plan->tiles.data(), sizeof(SsmTile) * nt);
    memcpy(seqs, plan->seqs.data(), sizeof(SsmSeq) * batch);
    const size_t nss = plan->scan_seqs.size();
    SsmScanSeq *scan_seqs = static_cast<SsmScanSeq *>(guarded(sizeof(SsmScanSeq) * (nss ? nss : 1), end_aligned));
    memcpy(scan_seqs, plan->scan_seqs.data(), sizeof(SsmScanSeq) * nss);

    void *y = guarded((nx ? nx : 1) * esz, end_aligned);
    float *st = static_cast<float *>(guarded((size_t)(n_ckpt ? n_ckpt : 1) * nst * 4, end_aligned));
    memset(y, 0xFF, nx * esz);                       // NaN patterns: every output must be overwritten
    memset(st, 0xFF, (size_t)n_ckpt * nst * 4);

    ScanArgs args;
    args.x = x, args.dt = dt, args.A = A, args.B = B, args.C = C, args.D = D, args.y = y, args.state_out = st;
    args.init_ptrs = any_init ? reinterpret_cast<const void *const *>(init) : nullptr;
    args.tiles = tiles, args.seqs = seqs, args.scan_seqs = scan_seqs;
    args.H = H, args.P = P, args.N = N, args.G = G, args.p_split = plan->p_split;
    args.state_dtype = st_type;
    if (advance) {
        void **sp = static_cast<void **>(guarded(sizeof(void *) * (batch ? batch : 1), end_aligned));
        for (int b = 0; b < batch; ++b) {
            sp[b] = guarded(nst * st_esz, end_aligned);
            for (size_t e = 0; e < nst; ++e)
                to_state(sp[b], e, init[b] ? init[b][e] : 0.f);
        }
        if (launch_state_advance(plan, args, sp, nullptr) != hipSuccess) {
            fprintf(stderr, "launch_state_advance failed\n");
            return 2;
        }
        f = fopen(argv[2], "wb");
        fwrite(y, esz, nx, f);
        std::vector<float> back(nst);
        for (int b = 0; b < batch; ++b) {
            for (size_t e = 0; e < nst; ++e)
                back[e] = from_state(sp[b], e);
            fwrite(back.data(), 4, nst, f);
        }
        fclose(f);
        printf("emu ok: advance, %d sequences, %ld fiber switches\n", batch, emu::switches());
        return 0;
    }
    if (plan->n_workgroups > 0 && T > 0) {
        size_t ws_bytes = 0;
        ssm_plan_workspace_bytes(plan, &ws_bytes);
        void *ws = guarded(ws_bytes ? ws_bytes : 16, end_aligned);
        memset(ws, 0xFF, ws_bytes);
        void *st_red = nullptr;
        if (st_type != 0) {
            // cached states in the reduced type: convert the initial ones, give the kernel a checkpoint buffer of
            // that type, and convert the checkpoints back to fp32 for the output file
            for (int b = 0; b < batch; ++b)
                if (init[b]) {
                    void *conv = guarded(nst * st_esz, end_aligned);
                    for (size_t k = 0; k < nst; ++k)
                        to_state(conv, k, init[b][k]);
                    init[b] = static_cast<const float *>(conv);
                }
            const size_t nck = (size_t)(n_ckpt ? n_ckpt : 1) * nst;
            st_red = guarded(nck * st_esz, end_aligned);
            memset(st_red, 0xFF, nck * st_esz);
            args.state_out = st_red;
        }
        const hipError_t e = plan->path == SSM_PATH_MFMA_BF16 ? launch_scan_mfma(plan, args, ws, nullptr)
                                                              : launch_scan_valu(plan, args, nullptr);
        if (e != hipSuccess) {
            fprintf(stderr, "launch failed\n");
            return 2;
        }
        if (st_red)
            for (size_t k = 0; k < (size_t)n_ckpt * nst; ++k)
                st[k] = from_state(st_red, k);
    }
    f = fopen(argv[2], "wb");
    fwrite(y, esz, nx, f);
    fwrite(st, 4, (size_t)n_ckpt * nst, f);
    fclose(f);
    printf("emu ok: path %d, %d workgroups, %zu tiles, %ld fiber switches\n", plan->path, plan->n_workgroups, nt,
           emu::switches());
    return 0;
}
