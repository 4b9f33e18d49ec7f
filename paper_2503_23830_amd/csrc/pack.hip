// orch_pack: the row movement of the All-to-All Batch Communicator (OrchMLLM
// Sec. 5.2.1) on one device.  A sequence's rows are contiguous both in the
// source (sequences concatenated in original order) and in the destination
// (instance-major, push order), so the rearrangement is n contiguous segment
// copies.  The destination is cut into fixed-size byte chunks; a persistent grid
// walks the chunks, finds the segment(s) under each chunk by binary search in a
// small segment table and streams 16 bytes per lane.  Pure HBM traffic:
// 2 * row_bytes per row, no arithmetic.
#include "common.h"

namespace orch {
namespace {

struct PackHdr {
    int64_t nseg;        // segments in the table
    int64_t total_rows;  // destination rows covered by the chosen instances
    int32_t ok;          // 0 -> the copy kernel must not touch memory
    int32_t pad;
};

struct PackWs {
    PackHdr *hdr;
    int64_t *src_cu;   // [n+1] exclusive prefix of lengths, original order
    int64_t *seg_dst;  // [n+1] destination row of segment p (relative), [nseg] = total
    int64_t *seg_src;  // [n]   source row of segment p
};

size_t carve(PackWs &w, void *ws, int32_t n)
{
    size_t nn = (size_t)(n > 0 ? n : 0) + 1;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.hdr = (PackHdr *)take(sizeof(PackHdr));
    w.src_cu = (int64_t *)take(nn * 8);
    w.seg_dst = (int64_t *)take(nn * 8);
    w.seg_src = (int64_t *)take(nn * 8);
    return off;
}

constexpr int kPrepThreads = 1024;

// One workgroup: prefix-sum the lengths (source row of every sequence), then
// build the segment table of the chosen instances and validate every segment
// against the buffer sizes the caller stated.
__global__ __launch_bounds__(kPrepThreads) void pack_prep_kernel(
    const int32_t *__restrict__ lengths, int32_t n, int32_t D, int64_t T, int64_t packed_rows,
    const int32_t *__restrict__ inst, const int32_t *__restrict__ order,
    const int32_t *__restrict__ seq_off, const int64_t *__restrict__ tok_off,
    const int32_t *__restrict__ cu_seqlens, int32_t *dev_status, int32_t inst_begin,
    int32_t inst_end, PackHdr *hdr, int64_t *src_cu, int64_t *seg_dst, int64_t *seg_src)
{
    __shared__ int64_t part[kPrepThreads];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = (dev_status[0] != 0);
    const int64_t per = ((int64_t)n + kPrepThreads - 1) / kPrepThreads;
    const int64_t b0 = min((int64_t)n, per * tid), b1 = min((int64_t)n, b0 + per);
    int64_t sum = 0;
    int bad = 0;
    for (int64_t s = b0; s < b1; ++s) {
        int32_t L = lengths[s];
        if (L < 0) { bad = 1; L = 0; }
        sum += L;
    }
    part[tid] = sum;
    __syncthreads();
    for (int m = 1; m < kPrepThreads; m <<= 1) {  // inclusive scan over threads
        int64_t o = tid >= m ? part[tid - m] : 0;
        __syncthreads();
        part[tid] += o;
        __syncthreads();
    }
    int64_t run = part[tid] - sum;
    for (int64_t s = b0; s < b1; ++s) {
        src_cu[s] = run;
        run += lengths[s] > 0 ? lengths[s] : 0;
    }
    if (tid == kPrepThreads - 1) src_cu[n] = part[tid];
    if (part[kPrepThreads - 1] != T) bad = 1;
    __syncthreads();

    const int32_t p0 = seq_off[inst_begin], p1 = seq_off[inst_end];
    const int64_t row0 = tok_off[inst_begin], rows = tok_off[inst_end] - row0;
    if (p0 < 0 || p1 < p0 || p1 > n || rows < 0 || rows > packed_rows) bad = 1;
    if (!bad) {
        for (int64_t p = p0 + tid; p < p1; p += kPrepThreads) {
            const int32_t s = order[p];
            if (s < 0 || s >= n) { bad = 1; continue; }
            const int32_t i = inst[s];
            if (i < inst_begin || i >= inst_end) { bad = 1; continue; }
            const int64_t L = lengths[s];
            const int64_t dst = tok_off[i] - row0 + cu_seqlens[p + i];
            const int64_t src = src_cu[s];
            if (L < 0 || dst < 0 || dst + L > rows || src + L > T) bad = 1;
            seg_dst[p - p0] = dst;
            seg_src[p - p0] = src;
        }
    }
    if (bad) atomicOr(&s_bad, 1);
    __syncthreads();
    if (tid == 0) {
        const int ok = !s_bad;
        hdr->nseg = ok ? (int64_t)(p1 - p0) : 0;
        hdr->total_rows = ok ? rows : 0;
        hdr->ok = ok;
        if (ok) seg_dst[p1 - p0] = rows;
        else dev_status[0] = (int32_t)ORCH_EDATA;
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kCopyThreads = 256;
constexpr int kPer = 8;  // accesses in flight per lane

// last p in [lo, hi] with seg_dst[p] * row_bytes <= x
__device__ __forceinline__ int64_t seg_of(const int64_t *__restrict__ seg_dst, int64_t lo, int64_t hi,
                                          int64_t row_bytes, int64_t x)
{
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (seg_dst[mid] * row_bytes <= x) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <typename V>
__global__ __launch_bounds__(kCopyThreads) void pack_copy_kernel(
    const char *__restrict__ src, char *__restrict__ dst, const PackHdr *__restrict__ hdr,
    const int64_t *__restrict__ seg_dst, const int64_t *__restrict__ seg_src, int64_t row_bytes)
{
    if (!hdr->ok) return;
    constexpr int64_t VB = sizeof(V);
    constexpr int64_t CB = (int64_t)kCopyThreads * kPer * VB;
    const int64_t total = hdr->total_rows * row_bytes;
    const int64_t nseg = hdr->nseg;
    if (nseg <= 0 || total <= 0) return;
    const int64_t nchunks = (total + CB - 1) / CB;
    for (int64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const int64_t cb = c * CB, ce = min(cb + CB, total);
        const int64_t plo = seg_of(seg_dst, 0, nseg - 1, row_bytes, cb);
        const int64_t phi = seg_of(seg_dst, plo, nseg - 1, row_bytes, ce - 1);
        // usually one segment covers the whole chunk; otherwise walk the pieces
        for (int64_t p = plo; p <= phi; ++p) {
            const int64_t a = max(cb, seg_dst[p] * row_bytes), b = min(ce, seg_dst[p + 1] * row_bytes);
            if (a >= b) continue;
            const char *sp = src + (seg_src[p] - seg_dst[p]) * row_bytes;
            for (int64_t x0 = a + (int64_t)threadIdx.x * VB; x0 < b; x0 += CB) {
                V val[kPer];
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    const int64_t x = x0 + (int64_t)u * kCopyThreads * VB;
                    if (x < b) val[u] = __builtin_nontemporal_load((const V *)(sp + x));
                }
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    const int64_t x = x0 + (int64_t)u * kCopyThreads * VB;
                    if (x < b) __builtin_nontemporal_store(val[u], (V *)(dst + x));
                }
            }
        }
    }
}

}  // namespace

size_t pack_ws_bytes(int32_t n, int32_t D)
{
    (void)D;
    PackWs w;
    return carve(w, nullptr, n);
}

int launch_pack(const void *tokens, void *packed, const int32_t *lengths, int32_t n, int32_t D,
                int64_t T, int32_t H, int64_t packed_rows, orch_assignment a, int32_t inst_begin,
                int32_t inst_end, void *ws, size_t ws_bytes, hipStream_t stream)
{
    PackWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_pack: workspace %zu < %zu bytes", ws_bytes, need);
    const int64_t row_bytes = (int64_t)H * 2;

    hipLaunchKernelGGL(pack_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, lengths, n, D, T,
                       packed_rows, a.inst, a.order, a.seq_off, a.tok_off, a.cu_seqlens, a.dev_status,
                       inst_begin, inst_end, w.hdr, w.src_cu, w.seg_dst, w.seg_src);

    const int64_t max_bytes = (packed_rows < T ? packed_rows : T) * row_bytes;
    if (max_bytes > 0) {
        // widest access that divides the row size and both base addresses
        const uintptr_t mis = (uintptr_t)tokens | (uintptr_t)packed | (uintptr_t)row_bytes;
        int vb = 16;
        while (mis & (uintptr_t)(vb - 1)) vb >>= 1;
        const int64_t cb = (int64_t)kCopyThreads * kPer * vb;
        int64_t nchunks = (max_bytes + cb - 1) / cb;
        const int grid = (int)(nchunks < 256 * 8 ? nchunks : 256 * 8);
        const char *s = (const char *)tokens;
        char *d = (char *)packed;
        if (vb == 16)
            hipLaunchKernelGGL(pack_copy_kernel<u32x4>, dim3(grid), dim3(kCopyThreads), 0, stream, s, d,
                               w.hdr, w.seg_dst, w.seg_src, row_bytes);
        else if (vb == 8)
            hipLaunchKernelGGL(pack_copy_kernel<u32x2>, dim3(grid), dim3(kCopyThreads), 0, stream, s, d,
                               w.hdr, w.seg_dst, w.seg_src, row_bytes);
        else if (vb == 4)
            hipLaunchKernelGGL(pack_copy_kernel<uint32_t>, dim3(grid), dim3(kCopyThreads), 0, stream, s, d,
                               w.hdr, w.seg_dst, w.seg_src, row_bytes);
        else
            hipLaunchKernelGGL(pack_copy_kernel<uint16_t>, dim3(grid), dim3(kCopyThreads), 0, stream, s, d,
                               w.hdr, w.seg_dst, w.seg_src, row_bytes);
    }
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
