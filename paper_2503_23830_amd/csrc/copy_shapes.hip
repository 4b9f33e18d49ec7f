// Copy-shape microbenchmark: which launch shape moves a large contiguous buffer fastest on this
// machine.  Context for the design of the pack kernel (the rearrangement's row movement, Sec. 5.2.1,
// is a pure copy): persistent workgroups with several accesses in flight per lane, against one-shot
// workgroups whose lanes issue a single 16-byte load and store, with and without the two table
// lookups the pack kernel makes in front of its load.  Not part of liborch.so.
//   usage: copy_shapes [GiB per buffer, default 16]   (prints one line per shape; hipEvent timing)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

template <bool NT>
__device__ __forceinline__ u32x4 ld(const char *p)
{
    return NT ? __builtin_nontemporal_load((const u32x4 *)p) : *(const u32x4 *)p;
}
template <bool NT>
__device__ __forceinline__ void st(char *p, u32x4 v)
{
    if (NT) __builtin_nontemporal_store(v, (u32x4 *)p);
    else *(u32x4 *)p = v;
}

// PER accesses in flight per lane over a chunk of 256 * PER * 16 bytes; PERSIST: a fixed grid walks
// the chunks, else one workgroup per chunk
template <int PER, bool NT, bool PERSIST>
__global__ __launch_bounds__(256) void copy_chunks(const char *__restrict__ src, char *__restrict__ dst, int64_t total)
{
    constexpr int64_t CB = 256 * PER * 16;
    const int64_t nchunks = (total + CB - 1) / CB;
    for (int64_t c = blockIdx.x; c < nchunks; c += PERSIST ? gridDim.x : nchunks) {
        const int64_t x0 = c * CB + (int64_t)threadIdx.x * 16;
        u32x4 val[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (x0 + (int64_t)u * 4096 < total) val[u] = ld<NT>(src + x0 + (int64_t)u * 4096);
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (x0 + (int64_t)u * 4096 < total) st<NT>(dst + x0 + (int64_t)u * 4096, val[u]);
    }
}

// one access per lane, one-shot, workgroups of BS threads
template <int BS, bool NT>
__global__ __launch_bounds__(BS) void copy_one(const char *__restrict__ src, char *__restrict__ dst, int64_t total)
{
    const int64_t x = ((int64_t)blockIdx.x * BS + threadIdx.x) * 16;
    if (x < total) st<NT>(dst + x, ld<NT>(src + x));
}

// the same after two dependent scalar lookups (granule table, then segment fields)
template <int BS>
__global__ __launch_bounds__(BS) void copy_one_lookup(const char *__restrict__ src, char *__restrict__ dst,
                                                      const int32_t *__restrict__ gtab, const int64_t *__restrict__ seg_pos,
                                                      const int64_t *__restrict__ seg_src, const int64_t *__restrict__ seg_dst,
                                                      const int64_t *__restrict__ hdr)
{
    if (!hdr[0]) return;
    const int64_t cb = (int64_t)blockIdx.x * BS * 16;
    if (cb >= hdr[1]) return;
    int64_t p = gtab[cb >> hdr[2]];
    while (seg_pos[p + 1] <= cb) ++p;
    const int64_t x = cb + (int64_t)threadIdx.x * 16;
    if (x < seg_pos[p + 1])
        st<true>(dst + (seg_dst[p] - seg_pos[p]) + x, ld<true>(src + (seg_src[p] - seg_pos[p]) + x));
}

int main(int argc, char **argv)
{
    const int64_t gib = argc > 1 ? atoll(argv[1]) : 16;
    if (gib < 1 || gib > 32) {   // one-shot grids must stay below 2^32 threads
        printf("buffer size must be 1..32 GiB\n");
        return 1;
    }
    const int64_t total = gib << 30;
    char *a, *b;
    CK(hipMalloc(&a, total));
    CK(hipMalloc(&b, total));
    CK(hipMemset(a, 1, total));
    CK(hipMemset(b, 2, total));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    auto run = [&](const char *name, auto launch) {
        for (int i = 0; i < 2; ++i) launch();
        (void)hipEventRecord(e0);
        for (int i = 0; i < 5; ++i) launch();
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        ms /= 5;
        const hipError_t le = hipGetLastError();
        printf("%-72s %8.3f ms  %5.2f TB/s %s\n", name, ms, 2.0 * total / ms / 1e9, le == hipSuccess ? "" : hipGetErrorString(le));
        fflush(stdout);
    };
    // segments of total / 4096 bytes, granules of 1 MiB
    const int nseg = 4096;
    const int64_t segb = total / nseg;
    std::vector<int64_t> pos(nseg + 1), hdrh = {1, total, 20};
    for (int i = 0; i <= nseg; ++i) pos[i] = segb * i;
    std::vector<int32_t> gt(total >> 20);
    for (size_t g = 0; g < gt.size(); ++g) gt[g] = (int32_t)(((int64_t)g << 20) / segb);
    int32_t *dgt;
    int64_t *dpos, *dhdr;
    CK(hipMalloc(&dgt, gt.size() * 4));
    CK(hipMalloc(&dpos, pos.size() * 8));
    CK(hipMalloc(&dhdr, 24));
    CK(hipMemcpy(dgt, gt.data(), gt.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(dpos, pos.data(), pos.size() * 8, hipMemcpyHostToDevice));
    CK(hipMemcpy(dhdr, hdrh.data(), 24, hipMemcpyHostToDevice));

#define PERSIST(PER, NT, GRID) \
    run("persistent, " #PER " accesses per lane, non-temporal=" #NT ", " #GRID " workgroups", [&] { hipLaunchKernelGGL((copy_chunks<PER, NT, true>), dim3(GRID), dim3(256), 0, 0, a, b, total); })
#define ONESHOT(PER, NT) \
    run("one-shot, " #PER " accesses per lane, non-temporal=" #NT, [&] { hipLaunchKernelGGL((copy_chunks<PER, NT, false>), dim3((unsigned)(total / (4096 * PER))), dim3(256), 0, 0, a, b, total); })
#define ONE(BS, NT) \
    run("one-shot, 1 access per lane, " #BS "-thread workgroups, non-temporal=" #NT, [&] { hipLaunchKernelGGL((copy_one<BS, NT>), dim3((unsigned)(total / (16 * BS))), dim3(BS), 0, 0, a, b, total); })
#define ONE_LOOKUP(BS) \
    run("one-shot, 1 access per lane, " #BS "-thread workgroups, non-temporal, 2 lookups", [&] { hipLaunchKernelGGL((copy_one_lookup<BS>), dim3((unsigned)(total / (16 * BS))), dim3(BS), 0, 0, a, b, dgt, dpos, dpos, dpos, dhdr); })
    PERSIST(8, true, 2048);
    PERSIST(8, false, 2048);
    PERSIST(4, false, 4096);
    PERSIST(2, false, 8192);
    ONESHOT(8, false);
    ONESHOT(4, false);
    ONESHOT(4, true);
    ONESHOT(2, false);
    ONE(256, false);
    ONE(256, true);
    ONE(64, false);
    ONE(64, true);
    ONE(1024, false);
    ONE_LOOKUP(256);
    ONE_LOOKUP(64);
    return 0;
}
