// Driver of the CPU emulation for the convolution kernel (test infrastructure only): reads a problem file, builds
// the scan's plan for the layer shape (the convolution walks the same tile table), runs the CPU-compiled kernel on
// fibers and writes the outputs and the checkpointed states.  Buffers are guarded as in emu_main.cpp.
//   emu_conv_main <in.bin> <out.bin> [order] [end|start]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#include "device_utils.h"
#include "emu_host.h"

namespace emu {
void set_order_mode(int m);
long switches();
}  // namespace emu

int main(int argc, char **argv)
{
    if (argc < 3) {
        fprintf(stderr, "usage: emu_conv_main in.bin out.bin [order] [end|start]\n");
        return 2;
    }
    emu::set_order_mode(argc > 3 ? atoi(argv[3]) : 0);
    const bool end_aligned = !(argc > 4 && argv[4][0] == 's');
    FILE *f = fopen(argv[1], "rb");
    if (!f) {
        perror(argv[1]);
        return 2;
    }
    int32_t hdr[13];
    read_vec(f, hdr, 13);
    if (hdr[0] != 0x434f4e56) {
        fprintf(stderr, "bad magic\n");
        return 2;
    }
    const int io = hdr[1], T = hdr[2], H = hdr[3], P = hdr[4], N = hdr[5], G = hdr[6], chunk = hdr[7], batch = hdr[8],
              n_ckpt = hdr[9], K = hdr[10], act = hdr[11], has_bias = hdr[12];
    const int Cch = H * P + 2 * G * N;  // x, B and C of a Mamba2-style layer pass through the convolution together
    const size_t esz = io == 0 ? 4 : 2;
    std::vector<int32_t> cu(batch + 1), cu_ck(batch + 1), ck(n_ckpt > 0 ? n_ckpt : 1), has_init(batch);
    read_vec(f, cu.data(), batch + 1);
    read_vec(f, cu_ck.data(), batch + 1);
    read_vec(f, ck.data(), n_ckpt);
    read_vec(f, has_init.data(), batch);
    const size_t nin = (size_t)T * Cch, nst = (size_t)Cch * K;
    void *in = guarded((nin ? nin : 1) * esz, end_aligned);
    float *w = static_cast<float *>(guarded(nst * 4, end_aligned));
    float *bias = has_bias ? static_cast<float *>(guarded((size_t)Cch * 4, end_aligned)) : nullptr;
    read_vec(f, static_cast<unsigned char *>(in), nin * esz);
    read_vec(f, w, nst);
    if (bias)
        read_vec(f, bias, Cch);
    const void **init = static_cast<const void **>(guarded(sizeof(void *) * (batch ? batch : 1), end_aligned));
    bool any_init = false;
    for (int b = 0; b < batch; ++b) {
        init[b] = nullptr;
        if (has_init[b]) {
            void *s = guarded(nst * esz, end_aligned);
            read_vec(f, static_cast<unsigned char *>(s), nst * esz);
            init[b] = s;
            any_init = true;
        }
    }
    fclose(f);

    ssm_shape_t shape;
    shape.nheads = H, shape.headdim = P, shape.d_state = N, shape.ngroups = G, shape.chunk = chunk, shape.io_dtype = io;
    shape.state_dtype = SSM_ST_F32;
    ssm_plan_t *plan = nullptr;
    int rc = ssm_plan_create(&shape, batch, cu.data(), cu_ck.data(), ck.data(), &plan);
    if (rc != 0) {
        fprintf(stderr, "ssm_plan_create: %d %s\n", rc, ssm_last_error());
        return 2;
    }
    const size_t nt = plan->tiles.size();
    SsmTile *tiles = static_cast<SsmTile *>(guarded(sizeof(SsmTile) * (nt ? nt : 1), end_aligned));
    SsmSeq *seqs = static_cast<SsmSeq *>(guarded(sizeof(SsmSeq) * (batch ? batch : 1), end_aligned));
    memcpy(tiles, plan->tiles.data(), sizeof(SsmTile) * nt);
    memcpy(seqs, plan->seqs.data(), sizeof(SsmSeq) * batch);

    void *out = guarded((nin ? nin : 1) * esz, end_aligned);
    void *st = guarded((size_t)(n_ckpt ? n_ckpt : 1) * nst * esz, end_aligned);
    memset(out, 0xFF, nin * esz);  // NaN patterns: every output must be overwritten
    memset(st, 0xFF, (size_t)n_ckpt * nst * esz);
    if (launch_conv1d_prefill(plan, tiles, seqs, Cch, K, in, w, bias, any_init ? init : nullptr, out, st, act, nullptr) !=
        hipSuccess) {
        fprintf(stderr, "launch_conv1d_prefill failed\n");
        return 2;
    }
    f = fopen(argv[2], "wb");
    fwrite(out, esz, nin, f);
    fwrite(st, esz, (size_t)n_ckpt * nst, f);
    fclose(f);
    printf("emu ok: conv, %d channels, %zu tiles, %ld fiber switches\n", Cch, nt, emu::switches());
    return 0;
}
