// Host helpers shared by the emulation drivers (test infrastructure only).
#pragma once
#include <sys/mman.h>

#include <cstdio>
#include <cstdlib>

// exact-size allocation flush against an inaccessible page: any overrun faults at once
static void *guarded(size_t bytes, bool end_aligned)
{
    const size_t page = 4096, span = (bytes + page - 1) / page * page + page;
    unsigned char *m =
        static_cast<unsigned char *>(mmap(nullptr, span + 2 * page, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0));
    if (m == MAP_FAILED) {
        perror("mmap");
        exit(2);
    }
    mprotect(m, page, PROT_NONE);
    mprotect(m + page + span, page, PROT_NONE);
    if (!end_aligned)
        return m + page;
    return m + page + span - (bytes + 15) / 16 * 16;  // 16-byte alignment as device allocations have at least
}

template <typename T> static void read_vec(FILE *f, T *dst, size_t n)
{
    if (n && fread(dst, sizeof(T), n, f) != n) {
        fprintf(stderr, "short read\n");
        exit(2);
    }
}


// The launchers ask the library for the profiling event of the calling thread; the emulation has none.
void *ssm_profile_event(int) { return nullptr; }
