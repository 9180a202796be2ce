// Spot check of the matrix-core scan at full problem sizes on the emulator (test infrastructure only): only the
// workgroups of the first two heads and of the last head run (in the scan, in the kernel in front of it, and in the
// kernels behind it that handle sequences cut into stretches), every buffer is guarded, and the outputs for those
// heads are compared with a plain fp64 recurrence computed here.  Inputs are drawn only where those workgroups read them.   emu_big <T> <ckpt_every> [H P G]
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "device_utils.h"
#include "emu_host.h"
namespace emu { void set_order_mode(int m); void set_block_filter(bool (*)(int, unsigned)); long switches(); }

static int gH, gP, gG, g_psplit, g_items, g_prep_parts = 1, g_fix_groups = 1, g_launches_before_fix = 2;
static std::vector<int> g_heads;  // heads whose workgroups run
static bool has_head(int h) { for (int x : g_heads) if (x == h) return true; return false; }
static bool filter(int launch, unsigned b)
{
    if (launch == 0) {  // the kernel in front of the scan, one or four blocks per (tile, group): keep the groups of the selected heads
        const int g = (b / g_prep_parts) % gG;  // block = ((tile * G) + g) * parts + part
        for (int h : g_heads) if (h / (gH / gG) == g) return true;
        return false;
    }
    if (launch == 1) {  // the scan: item = ((rank of the stretch) * H + head) * slices + slice
        const int item = ssm_launch_item(b, g_items);
        return item >= 0 && has_head((item / g_psplit) % gH);
    }
    if (launch < g_launches_before_fix)  // completing the carried states: block = slot * H + head
        return has_head(b % gH);
    // adding the carried states' contribution: block = ((slot * H + head) * slices + slice) * groups + group
    return has_head((b / g_fix_groups / (gP / 64)) % gH);
}
static uint32_t hash32(uint64_t x) { x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL; x ^= x >> 33; return (uint32_t)x; }
static float unif(uint64_t k) { return (hash32(k) >> 8) * (1.0f / 16777216.0f); }

int main(int argc, char **argv)
{
    const int T = argc > 1 ? atoi(argv[1]) : 4096, every = argc > 2 ? atoi(argv[2]) : 4096;
    const int H = argc > 3 ? atoi(argv[3]) : 128, P = argc > 4 ? atoi(argv[4]) : 64, G = argc > 5 ? atoi(argv[5]) : 8, N = 128;
    gH = H; gP = P; gG = G;
    ssm_shape_t sh = {H, P, N, G, 256, SSM_DT_BF16, SSM_ST_F32};
    std::vector<int32_t> ck; for (int p = every; p <= T; p += every) ck.push_back(p);
    int32_t cu[2] = {0, T}, cuck[2] = {0, (int32_t)ck.size()};
    ssm_plan_t *plan; if (ssm_plan_create(&sh, 1, cu, cuck, ck.data(), &plan)) { printf("plan: %s\n", ssm_last_error()); return 1; }
    g_psplit = plan->p_split; g_items = plan->n_items;
    g_prep_parts = (long long)plan->tiles.size() * G < kMfmaPrepSplitBelow ? 4 : 1;
    {   // groups of 8 tiles for a stretch's first 96 tiles, of 32 beyond
        const int m = plan->max_later_tiles;
        g_fix_groups = m <= 96 ? (m + 7) / 8 : 12 + (m - 96 + 31) / 32;
        if (g_fix_groups < 1) g_fix_groups = 1;
    }
    g_launches_before_fix = plan->carry_chains ? 3 : 2;
    g_heads = {0, 1, H - 1};
    const size_t nx = (size_t)T * H * P, nb = (size_t)T * G * N, ndt = (size_t)T * H, nst = (size_t)H * P * N;
    printf("T=%d tiles=%zu wgs=%d stretches=%zu ckpts=%zu; x %.2f GB\n", T, plan->tiles.size(), plan->n_workgroups,
           plan->scan_seqs.size(), ck.size(), nx * 2 / 1e9);
    bf16_t *x = (bf16_t *)guarded(nx * 2, true), *y = (bf16_t *)guarded(nx * 2, true), *B = (bf16_t *)guarded(nb * 2, true),
           *C = (bf16_t *)guarded(nb * 2, true), *dt = (bf16_t *)guarded(ndt * 2, true);
    float *A = (float *)guarded(H * 4, true), *D = (float *)guarded(H * 4, true);
    float *st = (float *)guarded((ck.size() ? ck.size() : 1) * nst * 4, true);
    // inputs only where the selected workgroups read them (the rest stays zero: untouched pages cost nothing)
    std::vector<int> heads = g_heads, groups;
    for (int h : heads) groups.push_back(h / (H / G));
    for (int h = 0; h < H; ++h) { A[h] = -expf(unif(7000 + h) * logf(16.f)); D[h] = unif(8000 + h) * 2 - 1; }
    for (int t = 0; t < T; ++t) {
        for (int h : heads) {
            dt[(size_t)t * H + h] = f32_to_bf16(expf(logf(1e-3f) + unif(1e9 + (uint64_t)t * H + h) * logf(100.f)));
            for (int p = 0; p < P; ++p) x[((size_t)t * H + h) * P + p] = f32_to_bf16((unif(2e9 + ((uint64_t)t * H + h) * P + p) * 2 - 1) * 1.7f);
        }
        for (int g : groups) for (int n = 0; n < N; ++n) {
            B[((size_t)t * G + g) * N + n] = f32_to_bf16((unif(3e12 + ((uint64_t)t * G + g) * N + n) * 2 - 1) * 0.15f);
            C[((size_t)t * G + g) * N + n] = f32_to_bf16((unif(4e12 + ((uint64_t)t * G + g) * N + n) * 2 - 1) * 0.15f);
        }
    }
    SsmTile *tiles = (SsmTile *)guarded(plan->tiles.size() * sizeof(SsmTile), true);
    SsmSeq *seqs = (SsmSeq *)guarded(sizeof(SsmSeq), true);
    memcpy(tiles, plan->tiles.data(), plan->tiles.size() * sizeof(SsmTile)); memcpy(seqs, plan->seqs.data(), sizeof(SsmSeq));
    SsmScanSeq *scan_seqs = (SsmScanSeq *)guarded(plan->scan_seqs.size() * sizeof(SsmScanSeq), true);
    memcpy(scan_seqs, plan->scan_seqs.data(), plan->scan_seqs.size() * sizeof(SsmScanSeq));
    ScanArgs a; a.x = x; a.dt = dt; a.A = A; a.B = B; a.C = C; a.D = D; a.y = y; a.state_out = st; a.init_ptrs = nullptr;
    a.tiles = tiles; a.seqs = seqs; a.scan_seqs = scan_seqs; a.H = H; a.P = P; a.N = N; a.G = G; a.p_split = plan->p_split; a.state_dtype = SSM_ST_F32;
    emu::set_order_mode(1); emu::set_block_filter(filter);
    size_t ws_bytes = 0; ssm_plan_workspace_bytes(plan, &ws_bytes);
    void *ws = guarded(ws_bytes ? ws_bytes : 16, true);
    if (launch_scan_mfma(plan, a, ws, nullptr) != hipSuccess) { printf("launch failed\n"); return 1; }
    printf("emulated the workgroups of %zu heads, %ld fiber switches\n", g_heads.size(), emu::switches());
    double worst_y = 0, worst_s = 0;
    const int NP = 32;  // channels checked per head: the first 32 of its last slice
    for (int h : g_heads) {
        const int ps = g_psplit - 1, g = h / (H / G), p0 = ps * (P / g_psplit);
        std::vector<double> S(32 * (size_t)N, 0.0), ref((size_t)T * 32);
        double rms = 0; size_t k = 0; double es = 0, srms = 0; std::vector<double> sref;
        for (int t = 0; t < T; ++t) {
            const double d = bf16_to_f32(dt[(size_t)t * H + h]), dec = exp(d * A[h]);
            for (int p = 0; p < 32; ++p) {
                const double xv = bf16_to_f32(x[((size_t)t * H + h) * P + p0 + p]); double acc = 0;
                for (int n = 0; n < N; ++n) { double &s = S[(size_t)p * N + n]; s = dec * s + d * xv * bf16_to_f32(B[((size_t)t * G + g) * N + n]); acc += bf16_to_f32(C[((size_t)t * G + g) * N + n]) * s; }
                ref[(size_t)t * 32 + p] = acc + D[h] * xv; rms += ref[(size_t)t * 32 + p] * ref[(size_t)t * 32 + p];
            }
            if (k < ck.size() && t + 1 == ck[k]) {
                double r2 = 0; for (double v : S) r2 += v * v; r2 = sqrt(r2 / S.size());
                for (int p = 0; p < 32; ++p) for (int n = 0; n < N; ++n) {
                    const double got = st[((k * H + h) * P + p0 + p) * (size_t)N + n], want = S[(size_t)p * N + n];
                    const double e = fabs(got - want) / fmax(fabs(want), r2); if (!(e <= es)) es = e; }
                ++k;
            }
        }
        rms = sqrt(rms / ((double)T * 32)); double ey = 0;
        for (int t = 0; t < T; ++t) for (int p = 0; p < 32; ++p) { const double r = ref[(size_t)t * 32 + p], gq = bf16_to_f32(y[((size_t)t * H + h) * P + p0 + p]);
            const double e = fabs(gq - r) / fmax(fabs(r), rms); if (!(e <= ey)) ey = e; }
        printf("head %d, channels %d..%d: y err %.3e, state err %.3e over %zu checkpoints\n", h, p0, p0 + NP - 1, ey, es, k);
        if (!(ey <= worst_y)) worst_y = ey; if (!(es <= worst_s)) worst_s = es;
    }
    printf(worst_y <= 2e-2 && worst_s <= 2e-2 ? "BIG CHECK OK\n" : "BIG CHECK FAILED\n");
    return 0;
}
