// Fiber runtime of the CPU emulation of the scan kernels.  TEST INFRASTRUCTURE ONLY: nothing in the library or its
// Python package builds, loads or calls this; the product runs on the GPU or fails.
//
// One fiber per lane.  The 64 lanes of a wave meet at every cross-lane operation (matrix-core products, LDS
// transpose reads, DPP shifts, lane reads), where the operation is evaluated for the whole wave from the operand
// layouts of gfx950; the waves of a workgroup meet at barriers.  Between two barriers the waves run one after
// another, whole, in an order the caller chooses (forward, reverse, seeded shuffle): a kernel whose LDS traffic is
// ordered by its barriers alone gives bit-identical results in every order, a kernel with a read/write or
// write/write race between two waves does not.  LDS starts filled with NaN patterns and sits, like every global
// buffer of the driver, flush against an inaccessible page, so an access out of bounds faults on the spot.
//
// Operand layouts (checked against the hardware with small probes):
//   mfma_f32_32x32x16_bf16  A: lane l holds row l%32, k = 8(l/32)+e;  B: lane l holds column l%32, same k;
//                           C/D: lane l, element r: column l%32, row 8(r/4) + 4(l/32) + r%4
//   mfma_f32_16x16x32_bf16  A: row l%16, k = 8(l/16)+e;  C/D: column l%16, row 4(l/16)+r
//   ds_read_tr16_b64        per 16 lanes: lane i receives as element e the 16-bit element i%4 of the 8 bytes that
//                           lane 4e + i/4 of the group points at
// Products are accumulated in double and rounded once; the matrix cores round differently in the last bits.
#include <hip/hip_runtime.h>
#include <sys/mman.h>
#include <ucontext.h>
#include <unistd.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

namespace emu {
namespace {
enum St { RUN, W_WAVE, W_BARRIER, DONE };
enum Op { OP_NONE, OP_SYNC, OP_MFMA32, OP_MFMA32H, OP_MFMA16, OP_TR, OP_DPP, OP_READLANE, OP_READFIRST, OP_SHFL, OP_YIELD };

struct Coll {
    int op = OP_NONE, line = 0;
    const void *a = nullptr, *b = nullptr, *c = nullptr;
    void *res = nullptr;
    int i0 = 0, i1 = 0, i2 = 0, i3 = 0, i4 = 0, i5 = 0;
};

struct Lane {
    ucontext_t ctx;
    void *stack = nullptr;
    Idx tid{0, 0, 0};
    Idx bid{0, 0, 0};              // the workgroup this lane belongs to
    unsigned char *lds = nullptr;  // and that workgroup's LDS
    St st = RUN;
    Coll k;
    int barrier_line = 0;
    long barriers = 0;  // barriers this lane has reached
};

constexpr size_t kStack = 256 * 1024;
std::vector<Lane> lanes;
Lane *cur = nullptr;
ucontext_t sched_ctx;
bool g_cooperative = false;  // run all workgroups of a launch at once (kernels whose workgroups wait for each other)
void (*g_fn)(void *) = nullptr;
void *g_arg = nullptr;
int g_order_mode = 0;  // 0 forward, 1 reverse, >=2 shuffle with this seed
long g_drop_barrier = -1;  // self-test of the checker: the barrier with this ordinal does not wait
long g_switches = 0;
bool (*g_block_filter)(int, unsigned) = nullptr;  // optional: which blocks of which launch to run
int g_launch_index = 0;

[[noreturn]] void die(const char *msg, int a = 0, int b = 0)
{
    fprintf(stderr, "EMU ERROR: %s (%d, %d) block %u\n", msg, a, b, cur ? cur->bid.x : 0u);
    fflush(stderr);
    _exit(3);
}

void yield_to_sched()
{
    ++g_switches;
    swapcontext(&cur->ctx, &sched_ctx);
}

void trampoline()
{
    g_fn(g_arg);
    cur->st = DONE;
    swapcontext(&cur->ctx, &sched_ctx);
    die("resumed a finished lane");
}

float bf(__bf16 v)
{
    uint16_t u;
    memcpy(&u, &v, 2);
    return __uint_as_float((uint32_t)u << 16);
}

// executes the collective all 64 lanes of wave `w` are waiting on
void run_collective(Lane *L)
{
    const Coll &k0 = L[0].k;
    for (int l = 1; l < 64; ++l)
        if (L[l].k.op != k0.op || L[l].k.line != k0.line)
            die("lanes of a wave wait on different cross-lane operations", k0.line, L[l].k.line);
    switch (k0.op) {
    case OP_SYNC: break;
    case OP_MFMA32:
    case OP_MFMA32H: {
        // A: lane l holds row l%32, k = 8(l/32)+e.  B: lane l holds column l%32, same k.
        // C/D: lane l, element r: column l%32, row 8(r/4) + 4(l/32) + r%4.  Same layouts for bf16 and fp16 operands.
        static double acc[32][32];
        for (int i = 0; i < 32; ++i)
            for (int j = 0; j < 32; ++j)
                acc[i][j] = 0.0;
        float A[32][16], B[16][32];
        for (int l = 0; l < 64; ++l) {
            if (k0.op == OP_MFMA32H) {
                const f16x8 a = *static_cast<const f16x8 *>(L[l].k.a), b = *static_cast<const f16x8 *>(L[l].k.b);
                for (int e = 0; e < 8; ++e) {
                    A[l % 32][8 * (l / 32) + e] = (float)a[e];
                    B[8 * (l / 32) + e][l % 32] = (float)b[e];
                }
                continue;
            }
            const bf16x8 a = *static_cast<const bf16x8 *>(L[l].k.a), b = *static_cast<const bf16x8 *>(L[l].k.b);
            for (int e = 0; e < 8; ++e) {
                A[l % 32][8 * (l / 32) + e] = bf(a[e]);
                B[8 * (l / 32) + e][l % 32] = bf(b[e]);
            }
        }
        for (int i = 0; i < 32; ++i)
            for (int kk = 0; kk < 16; ++kk)
                for (int j = 0; j < 32; ++j)
                    acc[i][j] += (double)A[i][kk] * (double)B[kk][j];
        for (int l = 0; l < 64; ++l) {
            const f32x16 c = *static_cast<const f32x16 *>(L[l].k.c);
            f32x16 d;
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r / 4) + 4 * (l / 32) + r % 4, col = l % 32;
                d[r] = (float)(acc[row][col] + (double)c[r]);
            }
            *static_cast<f32x16 *>(L[l].k.res) = d;
        }
        break;
    }
    case OP_MFMA16: {
        // A: lane l holds row l%16, k = 8(l/16)+e.  C/D: lane l, element r: column l%16, row 4(l/16) + r.
        double acc[16][16] = {};
        float A[16][32], B[32][16];
        for (int l = 0; l < 64; ++l) {
            const bf16x8 a = *static_cast<const bf16x8 *>(L[l].k.a), b = *static_cast<const bf16x8 *>(L[l].k.b);
            for (int e = 0; e < 8; ++e) {
                A[l % 16][8 * (l / 16) + e] = bf(a[e]);
                B[8 * (l / 16) + e][l % 16] = bf(b[e]);
            }
        }
        for (int i = 0; i < 16; ++i)
            for (int kk = 0; kk < 32; ++kk)
                for (int j = 0; j < 16; ++j)
                    acc[i][j] += (double)A[i][kk] * (double)B[kk][j];
        for (int l = 0; l < 64; ++l) {
            const f32x4 c = *static_cast<const f32x4 *>(L[l].k.c);
            f32x4 d;
            for (int r = 0; r < 4; ++r)
                d[r] = (float)(acc[4 * (l / 16) + r][l % 16] + (double)c[r]);
            *static_cast<f32x4 *>(L[l].k.res) = d;
        }
        break;
    }
    case OP_TR: {
        // per group of 16 lanes: lane i receives, as element e, the 16-bit element i%4 of the 8 bytes that lane
        // 4e + i/4 of the group points at
        for (int l = 0; l < 64; ++l) {
            const int g = l / 16, i = l % 16;
            s16x4 out;
            for (int e = 0; e < 4; ++e) {
                const unsigned char *src = static_cast<const unsigned char *>(L[16 * g + 4 * e + i / 4].k.a);
                short v;
                memcpy(&v, src + 2 * (i % 4), 2);
                out[e] = v;
            }
            *static_cast<s16x4 *>(L[l].k.res) = out;
        }
        break;
    }
    case OP_DPP: {
        const int ctrl = k0.i2, row_mask = k0.i3, bank_mask = k0.i4, bound = k0.i5;
        for (int l = 1; l < 64; ++l)
            if (L[l].k.i2 != ctrl || L[l].k.i3 != row_mask || L[l].k.i4 != bank_mask || L[l].k.i5 != bound)
                die("DPP controls differ between lanes", k0.line);
        for (int l = 0; l < 64; ++l) {
            const int row = l / 16, pos = l % 16, bank = pos / 4;
            int out = L[l].k.i0;  // old
            const bool enabled = ((row_mask >> row) & 1) && ((bank_mask >> bank) & 1);
            if (enabled) {
                int src = -1;
                bool valid = true;
                if (ctrl >= 0x111 && ctrl <= 0x11F) {  // row_shr:n
                    const int n = ctrl - 0x110;
                    if (pos >= n)
                        src = l - n;
                    else
                        valid = false;
                } else if (ctrl == 0x142) {  // row_bcast:15: lane 15 of each row to the next row
                    if (row >= 1)
                        src = 16 * (row - 1) + 15;
                    else
                        valid = false;
                } else if (ctrl == 0x143) {  // row_bcast:31: lane 31 to rows 2 and 3
                    if (row >= 2)
                        src = 31;
                    else
                        valid = false;
                } else {
                    die("DPP control not emulated", ctrl);
                }
                if (valid)
                    out = L[src].k.i1;
                else if (bound)
                    out = 0;
            }
            *static_cast<int *>(L[l].k.res) = out;
        }
        break;
    }
    case OP_READLANE:
        for (int l = 1; l < 64; ++l)
            if (L[l].k.i1 != k0.i1)
                die("readlane index differs between lanes", k0.line);
        if (k0.i1 < 0 || k0.i1 > 63)
            die("readlane index out of range", k0.i1);
        for (int l = 0; l < 64; ++l)
            *static_cast<int *>(L[l].k.res) = L[k0.i1].k.i0;
        break;
    case OP_READFIRST:
        for (int l = 0; l < 64; ++l)
            *static_cast<int *>(L[l].k.res) = L[0].k.i0;
        break;
    case OP_SHFL: {
        int vals[64];
        for (int l = 0; l < 64; ++l)
            vals[l] = L[l].k.i0;
        for (int l = 0; l < 64; ++l)
            *static_cast<int *>(L[l].k.res) = vals[L[l].k.i1 & 63];
        break;
    }
    default: die("unknown collective", k0.op);
    }
    for (int l = 0; l < 64; ++l) {
        L[l].k.op = OP_NONE;
        L[l].st = RUN;
    }
}

// run one wave until all its lanes sit at a barrier, are done, or have yielded (a spin-wait gives the other waves a
// turn); returns true in the last case
bool run_wave(int lane0, int w, int n_lanes)
{
    Lane *L = &lanes[lane0 + 64 * w];
    const int nl = std::min(64, n_lanes - 64 * w);
    for (;;) {
        bool progressed = false;
        for (int l = 0; l < nl; ++l) {
            if (L[l].st != RUN)
                continue;
            cur = &L[l];
            swapcontext(&sched_ctx, &cur->ctx);
            progressed = true;
        }
        int n_wave = 0, n_bar = 0, n_done = 0;
        for (int l = 0; l < nl; ++l) {
            n_wave += L[l].st == W_WAVE;
            n_bar += L[l].st == W_BARRIER;
            n_done += L[l].st == DONE;
        }
        if (n_wave == nl) {
            if (nl != 64)
                die("cross-lane operation in a partial wave");
            if (L[0].k.op == OP_YIELD) {
                for (int l = 1; l < 64; ++l)
                    if (L[l].k.op != OP_YIELD)
                        die("lanes of a wave wait on different cross-lane operations", L[0].k.line, L[l].k.line);
                for (int l = 0; l < 64; ++l) {
                    L[l].k.op = OP_NONE;
                    L[l].st = RUN;
                }
                return true;
            }
            run_collective(L);
            continue;
        }
        if (n_wave != 0)
            die("some lanes of a wave wait on a cross-lane operation while others sit at a barrier or are done",
                L[0].k.line, w);
        if (n_bar + n_done == nl) {
            if (n_bar != 0 && n_done != 0)
                die("some lanes of a wave are done while others wait at a barrier", w);
            return false;
        }
        if (!progressed)
            die("wave makes no progress", w);
    }
}

// Runs a set of workgroups to completion, all of them resident at once (one workgroup in the ordinary case).  The
// waves of all of them take turns in the chosen order; a barrier releases the lanes of its own workgroup only.
void run_blocks(const std::vector<unsigned> &ids, dim3 grid, dim3 block, size_t lds_bytes)
{
    const int n_per = (int)(block.x * block.y * block.z);
    const int waves_per = (n_per + 63) / 64;
    const int n_blocks = (int)ids.size();
    // LDS of each workgroup: exactly lds_bytes, flush against an inaccessible page, filled with NaN patterns
    const size_t page = 4096, span = (lds_bytes + page - 1) / page * page;
    std::vector<unsigned char *> maps(n_blocks);
    lanes.assign((size_t)n_blocks * n_per, Lane());
    for (int bi = 0; bi < n_blocks; ++bi) {
        unsigned char *m = static_cast<unsigned char *>(
            mmap(nullptr, span + 2 * page, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0));
        if (m == MAP_FAILED)
            die("mmap of LDS failed");
        mprotect(m, page, PROT_NONE);
        mprotect(m + page + span, page, PROT_NONE);
        maps[bi] = m;
        unsigned char *lds = m + page + span - ((lds_bytes + 15) / 16 * 16);
        memset(lds, 0xFF, (lds_bytes + 15) / 16 * 16);
        const unsigned b = ids[bi];
        for (int t = 0; t < n_per; ++t) {
            Lane &ln = lanes[(size_t)bi * n_per + t];
            ln.stack = mmap(nullptr, kStack, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
            if (ln.stack == MAP_FAILED)
                die("mmap of a lane stack failed");
            ln.tid = Idx{(unsigned)t % block.x, ((unsigned)t / block.x) % block.y, (unsigned)t / (block.x * block.y)};
            ln.bid = Idx{b % grid.x, (b / grid.x) % grid.y, b / (grid.x * grid.y)};
            ln.lds = lds;
            getcontext(&ln.ctx);
            ln.ctx.uc_stack.ss_sp = ln.stack;
            ln.ctx.uc_stack.ss_size = kStack;
            ln.ctx.uc_link = nullptr;
            makecontext(&ln.ctx, trampoline, 0);
        }
    }
    const int n_waves = n_blocks * waves_per;
    std::vector<int> order(n_waves);
    std::mt19937 rng((unsigned)g_order_mode * 7919u + ids[0] % grid.x);
    long yield_passes = 0;
    for (;;) {
        for (int w = 0; w < n_waves; ++w)
            order[w] = g_order_mode == 1 ? n_waves - 1 - w : w;
        if (g_order_mode >= 2)
            std::shuffle(order.begin(), order.end(), rng);
        bool yielded = false;
        for (int w : order)
            yielded = run_wave((w / waves_per) * n_per, w % waves_per, n_per) || yielded;
        // barriers, workgroup by workgroup
        bool released = false, any_waiting = false;
        for (int bi = 0; bi < n_blocks; ++bi) {
            int n_bar = 0, n_done = 0, n_other = 0;
            for (int t = 0; t < n_per; ++t) {
                const St st = lanes[(size_t)bi * n_per + t].st;
                n_bar += st == W_BARRIER;
                n_done += st == DONE;
                n_other += st != W_BARRIER && st != DONE;
            }
            if (n_bar == 0)
                continue;
            any_waiting = true;
            if (n_other != 0)
                continue;  // some of its waves have only yielded: they get there in a later pass
            if (n_done != 0) {
                cur = &lanes[(size_t)bi * n_per];
                die("barrier reached by only part of the workgroup: the rest has exited (a hang on the GPU)", n_bar, n_done);
            }
            for (int t = 0; t < n_per; ++t)
                lanes[(size_t)bi * n_per + t].st = RUN;
            released = true;
        }
        if (yielded || released) {  // a wave is spinning on something another wave will write, or a barrier opened
            if (yielded && ++yield_passes > 50000000L)
                die("waves keep yielding: a spin-wait that nothing ends (a hang on the GPU)");
            continue;
        }
        if (any_waiting)
            die("waves wait at a barrier that cannot open");
        break;  // every lane is done
    }
    for (Lane &ln : lanes)
        munmap(ln.stack, kStack);
    lanes.clear();
    cur = nullptr;
    for (unsigned char *m : maps)
        munmap(m, span + 2 * page);
}
}  // namespace

Idx &thread_idx() { return cur->tid; }
Idx &block_idx() { return cur->bid; }
unsigned char *lds_base() { return cur->lds; }
void set_cooperative(bool on) { g_cooperative = on; }
void set_order_mode(int m) { g_order_mode = m; }
// Run only the blocks for which filter(launch ordinal, linear block index) is true (for spot checks of large grids).
void set_block_filter(bool (*filter)(int, unsigned)) { g_block_filter = filter; }
long switches() { return g_switches; }

void buffer_range_fault(uint32_t off, uint32_t n, uint32_t bytes, int line)
{
    fprintf(stderr, "emu: buffer access of %u bytes at offset %u beyond a descriptor of %u bytes (source line %d)\n", n,
            off, bytes, line);
    abort();
}

void set_drop_barrier(long n) { g_drop_barrier = n; }

void barrier(int line)
{
    if (cur->barriers++ == g_drop_barrier)
        return;
    cur->st = W_BARRIER;
    cur->barrier_line = line;
    yield_to_sched();
}

static void collective(int op, int line)
{
    cur->k.op = op;
    cur->k.line = line;
    cur->st = W_WAVE;
    yield_to_sched();
}

void wave_sync(int line) { collective(OP_SYNC, line); }
void wave_yield(int line) { collective(OP_YIELD, line); }

f32x16 mfma_32x32x16_bf16(bf16x8 a, bf16x8 b, f32x16 c, int line)
{
    f32x16 res;
    cur->k.a = &a, cur->k.b = &b, cur->k.c = &c, cur->k.res = &res;
    collective(OP_MFMA32, line);
    return res;
}

f32x16 mfma_32x32x16_f16(f16x8 a, f16x8 b, f32x16 c, int line)
{
    f32x16 res;
    cur->k.a = &a, cur->k.b = &b, cur->k.c = &c, cur->k.res = &res;
    collective(OP_MFMA32H, line);
    return res;
}

f32x4 mfma_16x16x32_bf16(bf16x8 a, bf16x8 b, f32x4 c, int line)
{
    f32x4 res;
    cur->k.a = &a, cur->k.b = &b, cur->k.c = &c, cur->k.res = &res;
    collective(OP_MFMA16, line);
    return res;
}

s16x4 ds_read_tr16_b64(const void *p, int line)
{
    s16x4 res;
    const unsigned char *q = static_cast<const unsigned char *>(p);
    if (((uintptr_t)q & 7) != 0)
        die("transpose read address not 8-byte aligned", line);
    cur->k.a = q, cur->k.res = &res;
    collective(OP_TR, line);
    return res;
}

int update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl, int line)
{
    int res;
    cur->k.i0 = old, cur->k.i1 = src, cur->k.i2 = ctrl, cur->k.i3 = row_mask, cur->k.i4 = bank_mask,
    cur->k.i5 = bound_ctrl, cur->k.res = &res;
    collective(OP_DPP, line);
    return res;
}

int readlane(int v, int lane, int line)
{
    int res;
    cur->k.i0 = v, cur->k.i1 = lane, cur->k.res = &res;
    collective(OP_READLANE, line);
    return res;
}

int readfirstlane(int v, int line)
{
    int res;
    cur->k.i0 = v, cur->k.res = &res;
    collective(OP_READFIRST, line);
    return res;
}

int shfl(int v, int src_lane, int line)
{
    int res;
    cur->k.i0 = v, cur->k.i1 = src_lane, cur->k.res = &res;
    collective(OP_SHFL, line);
    return res;
}

void launch_impl(dim3 grid, dim3 block, size_t lds_bytes, void (*fn)(void *), void *arg)
{
    g_fn = fn;
    g_arg = arg;
    const int launch = g_launch_index++;
    std::vector<unsigned> ids;
    for (unsigned b = 0; b < grid.x * grid.y * grid.z; ++b)
        if (!g_block_filter || g_block_filter(launch, b))
            ids.push_back(b);
    if (ids.empty())
        return;
    if (g_cooperative) {
        run_blocks(ids, grid, block, lds_bytes);  // all workgroups resident at once
        return;
    }
    for (unsigned b : ids)
        run_blocks(std::vector<unsigned>{b}, grid, block, lds_bytes);
}
}  // namespace emu
