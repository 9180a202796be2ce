// Self-test of the emulator's cooperative mode (test infrastructure only): a kernel whose workgroups wait for each
// other.  Workgroup b spins until a word in "device" memory says b, adds its contribution and passes b + 1 on; with
// the waves taken in reverse order the last workgroup runs first, so the launch only ends if all workgroups are
// resident together and a spinning wave gives the others a turn.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

namespace emu {
void set_order_mode(int m);
void set_cooperative(bool on);
}

__global__ void relay_kernel(volatile int *turn, int *sum)
{
    const int b = blockIdx.x;
    int polls = 0;
    while (__builtin_amdgcn_readfirstlane(*turn) != b) {
        if (++polls > 1000000)
            return;  // bounded, like every wait of the product kernels
        __builtin_amdgcn_s_sleep(1);
    }
    __syncthreads();  // a barrier per workgroup, while other workgroups are elsewhere
    if (threadIdx.x == 0) {
        *sum = *sum * 3 + b;  // order-dependent on purpose
        *turn = b + 1;
    }
}

int main(int argc, char **argv)
{
    emu::set_order_mode(argc > 1 ? atoi(argv[1]) : 1);
    emu::set_cooperative(true);
    int turn = 0, sum = 0;
    const int n = 5;
    hipLaunchKernelGGL(relay_kernel, dim3(n), dim3(128), 0, nullptr, &turn, &sum);
    int want = 0;
    for (int b = 0; b < n; ++b)
        want = want * 3 + b;
    printf(turn == n && sum == want ? "COOP OK\n" : "COOP FAILED (turn %d, sum %d, want %d)\n", turn, sum, want);
    return turn == n && sum == want ? 0 : 1;
}
