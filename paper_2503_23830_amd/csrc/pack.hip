// orch_pack: the row movement of the All-to-All Batch Communicator (OrchMLLM
// Sec. 5.2.1) on one device.  A sequence's rows are contiguous both in the
// source (sequences concatenated in original order) and in the destination
// (instance-major, push order), so the rearrangement is n contiguous segment
// copies.  The copied bytes are cut into 1 KB pieces, one per wavefront of a
// one-shot grid: the wavefront finds its segment through a coarse table (granule ->
// first segment under it) and a short walk, issues ONE 16-byte load and one store per
// lane and ends.  Millions of short-lived wavefronts sweeping the buffers in address
// order measured 20 % more HBM throughput here than a persistent grid with eight
// accesses in flight per lane.  Pure HBM traffic: 2 * row_bytes per row, no arithmetic.
//
// orch_pack_composed: the rearrangement composition of Sec. 5.3.  The source rows lie
// in an encoder phase's packed order and go straight to their place inside the
// interleaved sequences of the LLM-phase assignment, so every example is still one
// contiguous segment copy; only the segment table differs (source start from the
// encoder assignment, destination start shifted by the modality's offset inside the
// sequence).  Segments no longer tile the destination, so the copy kernel cuts the
// COPIED bytes (a running prefix over segment lengths) into chunks instead.
#include <algorithm>

#include "common.h"

namespace orch {
namespace {

struct alignas(32) PackHdr {
    int64_t nseg;        // segments in the table
    int64_t total_rows;  // rows the copy kernel moves
    int32_t ok;          // 0 -> the copy kernel must not touch memory
    int32_t gshift;      // granule g of the coarse table covers copied bytes [g << gshift, (g + 1) << gshift)
};

// coarse table: at most this many granules (of at least 1 MiB) over the copied bytes
constexpr int kGranules = 65536;

struct PackWs {
    PackHdr *hdr;
    int64_t *src_cu;   // [n+1] exclusive prefix of lengths, original order
    int64_t *seg_dst;  // [n+1] destination row of segment p (relative), [nseg] = total
    int64_t *seg_src;  // [n]   source row of segment p
    int32_t *gtab;     // [kGranules] segment that holds the first copied byte of a granule
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
    w.gtab = (int32_t *)take((size_t)kGranules * 4);
    return off;
}

struct ComposeWs {
    PackHdr *hdr;
    int64_t *src_start;  // [n]   first source row of example s
    int64_t *seg_pos;    // [n+1] exclusive prefix of segment lengths (rows), [nseg] = total
    int64_t *seg_dst;    // [n]   destination row of segment p (relative)
    int64_t *seg_src;    // [n]   source row of segment p
    int32_t *gtab;       // [kGranules]
};

size_t carve(ComposeWs &w, void *ws, int32_t n)
{
    size_t nn = (size_t)(n > 0 ? n : 0) + 1;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.hdr = (PackHdr *)take(sizeof(PackHdr));
    w.src_start = (int64_t *)take(nn * 8);
    w.seg_pos = (int64_t *)take(nn * 8);
    w.seg_dst = (int64_t *)take(nn * 8);
    w.seg_src = (int64_t *)take(nn * 8);
    w.gtab = (int32_t *)take((size_t)kGranules * 4);
    return off;
}

// orch_pack_composed_pieces: several segments per example (P pieces in all)
struct PiecesWs {
    PackHdr *hdr;
    int64_t *src_start;  // [n]     first source row of example s
    int64_t *piece_pre;  // [P+1]   exclusive prefix of piece lengths (rows), piece order
    int64_t *seg_base;   // [n+1]   first segment of the q-th chosen destination position
    int64_t *seg_pos;    // [P+1]   exclusive prefix of segment lengths (rows), [nseg] = total
    int64_t *seg_dst;    // [P]     destination row of segment (relative)
    int64_t *seg_src;    // [P]     source row of segment
    int32_t *gtab;       // [kGranules]
};

size_t carve(PiecesWs &w, void *ws, int32_t n, int32_t P)
{
    size_t nn = (size_t)(n > 0 ? n : 0) + 1, pp = (size_t)(P > 0 ? P : 0) + 1;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.hdr = (PackHdr *)take(sizeof(PackHdr));
    w.src_start = (int64_t *)take(nn * 8);
    w.piece_pre = (int64_t *)take(pp * 8);
    w.seg_base = (int64_t *)take(nn * 8);
    w.seg_pos = (int64_t *)take(pp * 8);
    w.seg_dst = (int64_t *)take(pp * 8);
    w.seg_src = (int64_t *)take(pp * 8);
    w.gtab = (int32_t *)take((size_t)kGranules * 4);
    return off;
}

constexpr int kPrepThreads = 1024;

// Inclusive scan of one value per thread over the workgroup; returns this thread's
// inclusive sum, total in part[kPrepThreads - 1].
__device__ __forceinline__ int64_t block_scan(int64_t *part, int tid, int64_t v)
{
    part[tid] = v;
    __syncthreads();
    for (int m = 1; m < kPrepThreads; m <<= 1) {
        int64_t o = tid >= m ? part[tid - m] : 0;
        __syncthreads();
        part[tid] += o;
        __syncthreads();
    }
    return part[tid];
}

// Last step of every prep kernel, all threads, after the header and the running sums are
// written: the coarse table of the copy kernel.  Granules are 2^gshift copied bytes, at least
// 1 MiB and few enough to fit the table; gtab[g] = the segment that holds byte g << gshift.  The
// non-empty segments partition the copied bytes, so every segment writes the entries of the
// granules that start inside it: nseg + granules steps in all, no searches.
__device__ void build_gtab(PackHdr *hdr, const int64_t *seg_pos, int64_t row_bytes, int32_t *gtab, int tid)
{
    __syncthreads();
    const int64_t nseg = hdr->nseg;
    const int64_t total = hdr->total_rows * row_bytes;
    if (!hdr->ok || nseg <= 0 || total <= 0) return;
    int gshift = 20;
    while (((total - 1) >> gshift) >= kGranules) ++gshift;
    if (tid == 0) hdr->gshift = gshift;
    const int64_t gmask = ((int64_t)1 << gshift) - 1;
    for (int64_t p = tid; p < nseg; p += kPrepThreads) {
        const int64_t b0 = seg_pos[p] * row_bytes, b1 = seg_pos[p + 1] * row_bytes;
        // granules g with b0 <= g << gshift < b1
        for (int64_t g = (b0 + gmask) >> gshift; (g << gshift) < b1; ++g) gtab[g] = (int32_t)p;
    }
}

// One workgroup: prefix-sum the lengths (source row of every sequence), then
// build the segment table of the chosen instances and validate every segment
// against the buffer sizes the caller stated.
__global__ __launch_bounds__(kPrepThreads) void pack_prep_kernel(
    const int32_t *__restrict__ lengths, int32_t n, int32_t D, int64_t T, int64_t packed_rows,
    const int32_t *__restrict__ inst, const int32_t *__restrict__ order,
    const int32_t *__restrict__ seq_off, const int64_t *__restrict__ tok_off,
    const int32_t *__restrict__ cu_seqlens, int32_t *dev_status, int32_t inst_begin,
    int32_t inst_end, PackHdr *hdr, int64_t *src_cu, int64_t *seg_dst, int64_t *seg_src,
    int64_t row_bytes, int32_t *gtab)
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
            // segments tile the destination: each must be exactly as long as its sequence
            if (L < 0 || dst < 0 || dst + L > rows || src + L > T || cu_seqlens[p + i + 1] - cu_seqlens[p + i] != L) bad = 1;
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
    build_gtab(hdr, seg_dst, row_bytes, gtab, tid);
}

// The source and destination sides of a composition, as the kernel needs them.
struct ComposeSide {
    const int32_t *inst, *order, *seq_off, *cu;
    const int64_t *tok_off;
    const int32_t *status;
    int32_t D;
};

// One workgroup.  (1) first source row of every example: from the encoder
// assignment (position p of its order holds example order[p]; its rows start at
// tok_off[i] + cu_i[j]), or the running sum of sub_len when the source is in
// original order; (2) one segment per example of the chosen destination instances,
// validated against both buffers and against the interleaved sequence it must fit
// in; (3) the running sum of segment lengths the copy kernel chunks over.
__global__ __launch_bounds__(kPrepThreads) void compose_prep_kernel(
    const int32_t *__restrict__ sub_len, const int32_t *__restrict__ sub_off, int32_t n,
    int64_t src_rows, int64_t packed_rows, int has_src, ComposeSide e, ComposeSide m,
    int32_t *dev_status, int32_t inst_begin, int32_t inst_end, PackHdr *hdr, int64_t *src_start,
    int64_t *seg_pos, int64_t *seg_dst, int64_t *seg_src, int64_t row_bytes, int32_t *gtab)
{
    __shared__ int64_t part[kPrepThreads];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = (m.status[0] != 0) || (has_src && e.status[0] != 0);
    int bad = 0;

    if (has_src) {
        for (int64_t s = tid; s < n; s += kPrepThreads) src_start[s] = -1;
        __syncthreads();
        const int32_t pe = e.seq_off[e.D];
        if (pe != n) bad = 1;
        else
            for (int64_t p = tid; p < n; p += kPrepThreads) {
                const int32_t s = e.order[p];
                if (s < 0 || s >= n) { bad = 1; continue; }
                const int32_t i = e.inst[s];
                if (i < 0 || i >= e.D) { bad = 1; continue; }
                if (p < e.seq_off[i] || p >= e.seq_off[i + 1]) { bad = 1; continue; }
                const int64_t c0 = e.cu[p + i], c1 = e.cu[p + i + 1];
                const int64_t start = e.tok_off[i] + c0;
                if (c1 - c0 < sub_len[s] || c0 < 0 || start < 0) { bad = 1; continue; }
                src_start[s] = start;
            }
    } else {
        const int64_t per = ((int64_t)n + kPrepThreads - 1) / kPrepThreads;
        const int64_t b0 = min((int64_t)n, per * tid), b1 = min((int64_t)n, b0 + per);
        int64_t sum = 0;
        for (int64_t s = b0; s < b1; ++s) {
            int32_t L = sub_len[s];
            if (L < 0) { bad = 1; L = 0; }
            sum += L;
        }
        int64_t run = block_scan(part, tid, sum) - sum;
        for (int64_t s = b0; s < b1; ++s) {
            src_start[s] = run;
            run += sub_len[s] > 0 ? sub_len[s] : 0;
        }
        if (part[kPrepThreads - 1] > src_rows) bad = 1;
    }
    __syncthreads();

    const int32_t p0 = m.seq_off[inst_begin], p1 = m.seq_off[inst_end];
    const int64_t row0 = m.tok_off[inst_begin], rows = m.tok_off[inst_end] - row0;
    if (p0 < 0 || p1 < p0 || p1 > n || rows < 0 || rows > packed_rows) bad = 1;
    const int64_t nseg = bad ? 0 : p1 - p0;
    const int64_t per = (nseg + kPrepThreads - 1) / kPrepThreads;
    const int64_t b0 = min(nseg, per * tid), b1 = min(nseg, b0 + per);
    int64_t sum = 0;
    for (int64_t q = b0; q < b1; ++q) {
        const int64_t p = p0 + q;
        seg_dst[q] = 0;
        seg_src[q] = 0;
        const int32_t s = m.order[p];
        if (s < 0 || s >= n) { bad = 1; continue; }
        const int32_t i = m.inst[s];
        if (i < inst_begin || i >= inst_end) { bad = 1; continue; }
        if (p < m.seq_off[i] || p >= m.seq_off[i + 1]) { bad = 1; continue; }
        const int64_t c0 = m.cu[p + i], seq_len = (int64_t)m.cu[p + i + 1] - c0;
        const int64_t L = sub_len[s], off = sub_off[s];
        const int64_t dst = m.tok_off[i] - row0 + c0 + off;
        const int64_t src = src_start[s];
        if (L < 0 || off < 0 || c0 < 0 || off + L > seq_len || dst < 0 || dst + L > rows || src < 0 ||
            src + L > src_rows) { bad = 1; continue; }
        seg_dst[q] = dst;
        seg_src[q] = src;
        sum += L;
    }
    if (bad) atomicOr(&s_bad, 1);
    int64_t run = block_scan(part, tid, sum) - sum;
    const int ok = !s_bad;  // every atomicOr above precedes the barriers inside block_scan
    if (ok)
        for (int64_t q = b0; q < b1; ++q) {
            seg_pos[q] = run;
            run += sub_len[m.order[p0 + q]];
        }
    if (tid == 0) {
        hdr->nseg = ok ? nseg : 0;
        hdr->total_rows = ok ? part[kPrepThreads - 1] : 0;
        hdr->ok = ok;
        if (ok) seg_pos[nseg] = part[kPrepThreads - 1];
        else dev_status[0] = (int32_t)ORCH_EDATA;
    }
    build_gtab(hdr, seg_pos, row_bytes, gtab, tid);
}

// One workgroup, the composition with several pieces per example (Sec. 6, subsequence assembly).
// (1) running sum of the piece lengths, which gives every example's row count of this modality
// and the place of every piece inside the example's run; (2) first source row of every example,
// from the encoder assignment or, for an original-order source, from that running sum; (3) one
// segment per piece of the examples on the chosen destination instances, in destination order,
// validated against both buffers, the interleaved sequence and the piece before it; (4) the
// running sum of segment lengths the copy kernel chunks over.
__global__ __launch_bounds__(kPrepThreads) void compose_pieces_prep_kernel(
    const int32_t *__restrict__ piece_ptr, const int32_t *__restrict__ piece_off,
    const int32_t *__restrict__ piece_len, int32_t n, int32_t P, int64_t src_rows, int64_t packed_rows,
    int has_src, ComposeSide e, ComposeSide m, int32_t *dev_status, int32_t inst_begin, int32_t inst_end,
    PackHdr *hdr, int64_t *src_start, int64_t *piece_pre, int64_t *seg_base, int64_t *seg_pos,
    int64_t *seg_dst, int64_t *seg_src, int64_t row_bytes, int32_t *gtab)
{
    __shared__ int64_t part[kPrepThreads];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = (m.status[0] != 0) || (has_src && e.status[0] != 0);
    int bad = 0;
    if (piece_ptr[0] != 0 || piece_ptr[n] != P) bad = 1;

    // (1) piece_pre
    {
        const int64_t per = ((int64_t)P + kPrepThreads - 1) / kPrepThreads;
        const int64_t b0 = min((int64_t)P, per * tid), b1 = min((int64_t)P, b0 + per);
        int64_t sum = 0;
        for (int64_t p = b0; p < b1; ++p) {
            const int32_t L = piece_len[p];
            if (L < 0 || piece_off[p] < 0) { bad = 1; continue; }
            sum += L;
        }
        int64_t run = block_scan(part, tid, sum) - sum;
        for (int64_t p = b0; p < b1; ++p) {
            piece_pre[p] = run;
            run += piece_len[p] > 0 ? piece_len[p] : 0;
        }
        if (tid == kPrepThreads - 1) piece_pre[P] = part[tid];
        if (part[kPrepThreads - 1] > src_rows) bad = 1;
    }
    __syncthreads();
    // a usable piece_ptr: non-decreasing inside [0, P]
    for (int64_t s = tid; s < n; s += kPrepThreads) {
        const int32_t a = piece_ptr[s], b = piece_ptr[s + 1];
        if (a < 0 || b < a || b > P) bad = 1;
    }
    if (bad) atomicOr(&s_bad, 1);
    __syncthreads();
    if (s_bad) {   // nothing below may index with a broken piece_ptr
        if (tid == 0) {
            hdr->nseg = 0;
            hdr->total_rows = 0;
            hdr->ok = 0;
            dev_status[0] = (int32_t)ORCH_EDATA;
        }
        return;
    }

    // (2) src_start
    if (has_src) {
        for (int64_t s = tid; s < n; s += kPrepThreads) src_start[s] = -1;
        __syncthreads();
        const int32_t pe = e.seq_off[e.D];
        if (pe != n) bad = 1;
        else
            for (int64_t p = tid; p < n; p += kPrepThreads) {
                const int32_t s = e.order[p];
                if (s < 0 || s >= n) { bad = 1; continue; }
                const int32_t i = e.inst[s];
                if (i < 0 || i >= e.D) { bad = 1; continue; }
                if (p < e.seq_off[i] || p >= e.seq_off[i + 1]) { bad = 1; continue; }
                const int64_t c0 = e.cu[p + i], c1 = e.cu[p + i + 1];
                const int64_t start = e.tok_off[i] + c0;
                const int64_t rows = piece_pre[piece_ptr[s + 1]] - piece_pre[piece_ptr[s]];
                if (c1 - c0 < rows || c0 < 0 || start < 0) { bad = 1; continue; }
                src_start[s] = start;
            }
    } else {
        for (int64_t s = tid; s < n; s += kPrepThreads) src_start[s] = piece_pre[piece_ptr[s]];
    }
    __syncthreads();

    // (3) segments of the chosen destination positions
    const int32_t p0 = m.seq_off[inst_begin], p1 = m.seq_off[inst_end];
    const int64_t row0 = m.tok_off[inst_begin], rows = m.tok_off[inst_end] - row0;
    if (p0 < 0 || p1 < p0 || p1 > n || rows < 0 || rows > packed_rows) bad = 1;
    const int64_t npos = bad ? 0 : p1 - p0;
    const int64_t per = (npos + kPrepThreads - 1) / kPrepThreads;
    const int64_t b0 = min(npos, per * tid), b1 = min(npos, b0 + per);
    int64_t cnt = 0;
    for (int64_t q = b0; q < b1; ++q) {
        const int32_t s = m.order[p0 + q];
        if (s < 0 || s >= n) { bad = 1; continue; }
        cnt += piece_ptr[s + 1] - piece_ptr[s];
    }
    if (bad) atomicOr(&s_bad, 1);
    int64_t base = block_scan(part, tid, cnt) - cnt;
    const int64_t nseg = part[kPrepThreads - 1];
    __syncthreads();   // part[] is reused below
    if (s_bad || nseg > P) bad = 1;
    if (!bad) {
        for (int64_t q = b0; q < b1; ++q) {
            const int64_t p = p0 + q;
            const int32_t s = m.order[p];
            const int32_t i = m.inst[s];
            const int32_t t0 = piece_ptr[s], t1 = piece_ptr[s + 1];
            seg_base[q] = base;
            if (i < inst_begin || i >= inst_end || p < m.seq_off[i] || p >= m.seq_off[i + 1]) {
                bad = 1;
                for (int32_t t = t0; t < t1; ++t) { seg_pos[base + (t - t0)] = 0; seg_dst[base + (t - t0)] = 0; seg_src[base + (t - t0)] = 0; }
                base += t1 - t0;
                continue;
            }
            const int64_t c0 = m.cu[p + i], seq_len = (int64_t)m.cu[p + i + 1] - c0;
            const int64_t dst0 = m.tok_off[i] - row0 + c0, src0 = src_start[s] - piece_pre[t0];
            int64_t prev_end = 0;
            for (int32_t t = t0; t < t1; ++t) {
                const int64_t L = piece_len[t], off = piece_off[t];
                const int64_t dst = dst0 + off, src = src0 + piece_pre[t];
                // pieces of an example ascend without overlap and stay inside its sequence
                if (off < prev_end || off + L > seq_len || c0 < 0 || dst < 0 || dst + L > rows || src < 0 ||
                    src + L > src_rows) bad = 1;
                prev_end = off + L;
                seg_pos[base] = L;   // length for now; the running sum follows
                seg_dst[base] = dst;
                seg_src[base] = src;
                ++base;
            }
        }
    }
    if (bad) atomicOr(&s_bad, 1);
    __syncthreads();
    const int ok = !s_bad;
    // (4) running sum of segment lengths, in place
    {
        const int64_t ns = ok ? nseg : 0;
        const int64_t per2 = (ns + kPrepThreads - 1) / kPrepThreads;
        const int64_t c0 = min(ns, per2 * tid), c1 = min(ns, c0 + per2);
        int64_t sum = 0;
        for (int64_t x = c0; x < c1; ++x) sum += seg_pos[x];
        int64_t run = block_scan(part, tid, sum) - sum;
        for (int64_t x = c0; x < c1; ++x) {
            const int64_t L = seg_pos[x];
            seg_pos[x] = run;
            run += L;
        }
        if (tid == 0) {
            hdr->nseg = ns;
            hdr->total_rows = ok ? part[kPrepThreads - 1] : 0;
            hdr->ok = ok;
            if (ok) seg_pos[ns] = part[kPrepThreads - 1];
            else dev_status[0] = (int32_t)ORCH_EDATA;
        }
    }
    build_gtab(hdr, seg_pos, row_bytes, gtab, tid);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kCopyThreads = 64;   // one wavefront per workgroup
// Workgroups per launch: grid size times workgroup size must stay below 2^32 threads (a larger
// launch is cut short without an error); bigger copies take several launches.
constexpr int64_t kCopyGrid = 1ll << 25;

// Pieces are cut in the space of copied bytes: segment p covers [seg_pos[p], seg_pos[p+1])
// rows of it, read from row seg_src[p] and written to row seg_dst[p].  For the plain pack the
// segments tile the destination and the caller passes seg_pos = seg_dst.  A workgroup is one
// wavefront and moves piece number piece0 + blockIdx.x, 64 accesses: granule table -> first
// segment, a short walk to the segment that holds the piece's first byte, one load and one
// store per lane.
template <typename V>
__global__ __launch_bounds__(kCopyThreads) void pack_copy_kernel(
    const char *__restrict__ src, char *__restrict__ dst, const PackHdr *__restrict__ hdr,
    const int64_t *__restrict__ seg_pos, const int64_t *__restrict__ seg_dst,
    const int64_t *__restrict__ seg_src, const int32_t *__restrict__ gtab, int64_t row_bytes, int64_t piece0)
{
    // a wavefront lives for one load and one store, so the chain of dependent scalar loads in
    // front of them is kept short: header (one load), granule table, the four fields of the
    // first segment together; anything else (a walk over short segments, a piece that straddles
    // segments) is off the common path
    PackHdr h = *hdr;
    asm volatile("" : "+s"(h.nseg), "+s"(h.total_rows), "+s"(h.ok), "+s"(h.gshift));   // one load, up front
    constexpr int64_t VB = sizeof(V);
    constexpr int64_t CB = (int64_t)kCopyThreads * VB;
    const int64_t total = h.total_rows * row_bytes;
    const int64_t cb = (piece0 + blockIdx.x) * CB;
    if (!h.ok || h.nseg <= 0 || cb >= total) return;
    const int64_t ce = min(cb + CB, total);
    const int64_t g = cb >> h.gshift;
    int64_t p = gtab[g];
    int64_t pos = seg_pos[p], nxt = seg_pos[p + 1], srow = seg_src[p], drow = seg_dst[p];
    // (the four loads are issued here, together: the empty statement keeps the compiler from
    // moving them behind the branches below)
    asm volatile("" : "+s"(pos), "+s"(nxt), "+s"(srow), "+s"(drow));
    // the segment of any byte of this piece lies in [p, last]: bisect there when a walk is needed,
    // so that runs of short or empty segments cost a logarithm, not their count
    int64_t last = h.nseg - 1;
    if (nxt * row_bytes <= cb) {   // uniform: the segment that holds the piece's first byte
        if (((g + 1) << h.gshift) < total) last = gtab[g + 1];
        int64_t lo = p + 1, hi = last;   // last q with seg_pos[q] * row_bytes <= cb
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) >> 1;
            if (seg_pos[mid] * row_bytes <= cb) lo = mid;
            else hi = mid - 1;
        }
        p = lo;
        pos = seg_pos[p];
        nxt = seg_pos[p + 1];
        srow = seg_src[p];
        drow = seg_dst[p];
    }
    const int64_t x = cb + (int64_t)threadIdx.x * VB;
    if (x >= ce) return;
    if (nxt * row_bytes < ce) {    // the piece straddles segments: a lane finds its own
        if (last == h.nseg - 1 && (((cb + CB - 1) >> h.gshift) + 1) << h.gshift < total)
            last = gtab[((cb + CB - 1) >> h.gshift) + 1];
        int64_t lo = p, hi = last;   // last q with seg_pos[q] * row_bytes <= x  (x < total)
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) >> 1;
            if (seg_pos[mid] * row_bytes <= x) lo = mid;
            else hi = mid - 1;
        }
        const int64_t qpos = seg_pos[lo];
        const V val = __builtin_nontemporal_load((const V *)(src + (seg_src[lo] - qpos) * row_bytes + x));
        __builtin_nontemporal_store(val, (V *)(dst + (seg_dst[lo] - qpos) * row_bytes + x));
        return;
    }
    const V val = __builtin_nontemporal_load((const V *)(src + (srow - pos) * row_bytes + x));
    __builtin_nontemporal_store(val, (V *)(dst + (drow - pos) * row_bytes + x));
}

// Copy kernel over at most max_bytes copied bytes, with the widest access that divides
// the row size and both base addresses.
void launch_copy(const void *src, void *dst, int64_t max_bytes, int64_t row_bytes, const PackHdr *hdr,
                 const int64_t *seg_pos, const int64_t *seg_dst, const int64_t *seg_src, const int32_t *gtab,
                 hipStream_t stream)
{
    if (max_bytes <= 0) return;
    const uintptr_t mis = (uintptr_t)src | (uintptr_t)dst | (uintptr_t)row_bytes;
    int vb = 16;
    while (mis & (uintptr_t)(vb - 1)) vb >>= 1;
    const int64_t cb = (int64_t)kCopyThreads * vb;
    const int64_t npieces = (max_bytes + cb - 1) / cb;
    const char *s = (const char *)src;
    char *d = (char *)dst;
    for (int64_t p0 = 0; p0 < npieces; p0 += kCopyGrid) {
        const dim3 grid((unsigned)std::min<int64_t>(kCopyGrid, npieces - p0));
        if (vb == 16)
            hipLaunchKernelGGL(pack_copy_kernel<u32x4>, grid, dim3(kCopyThreads), 0, stream, s, d, hdr, seg_pos,
                               seg_dst, seg_src, gtab, row_bytes, p0);
        else if (vb == 8)
            hipLaunchKernelGGL(pack_copy_kernel<u32x2>, grid, dim3(kCopyThreads), 0, stream, s, d, hdr, seg_pos,
                               seg_dst, seg_src, gtab, row_bytes, p0);
        else if (vb == 4)
            hipLaunchKernelGGL(pack_copy_kernel<uint32_t>, grid, dim3(kCopyThreads), 0, stream, s, d, hdr, seg_pos,
                               seg_dst, seg_src, gtab, row_bytes, p0);
        else
            hipLaunchKernelGGL(pack_copy_kernel<uint16_t>, grid, dim3(kCopyThreads), 0, stream, s, d, hdr, seg_pos,
                               seg_dst, seg_src, gtab, row_bytes, p0);
    }
}

// Communication-volume matrix (Sec. 5.2.2, first loop of the node-wise rearrangement
// algorithm): V[from][to] += length, and per source instance the tokens that leave its node.
__global__ void comm_clear_kernel(unsigned long long *V, int64_t cells, unsigned long long *inter, int32_t D_src)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < cells) V[e] = 0;
    if (inter && e < D_src) inter[e] = 0;
}

__global__ void comm_volume_kernel(const int32_t *__restrict__ lengths, int32_t n, int32_t D_src,
                                   const int32_t *__restrict__ from, int32_t D_dst,
                                   const int32_t *__restrict__ inst, unsigned long long *V, int32_t c,
                                   unsigned long long *inter, int32_t *dev_status)
{
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    const int32_t L = lengths[s], to = inst[s];
    const int32_t f = from ? from[s] : (int32_t)((s * D_src) / n);
    if (L < 0 || f < 0 || f >= D_src || to < 0 || to >= D_dst) {
        // several threads may find an error: an atomic store of the one value they all write
        __hip_atomic_store(dev_status, (int32_t)ORCH_EDATA, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (L == 0) return;
    atomicAdd(&V[(int64_t)f * D_dst + to], (unsigned long long)L);
    if (inter && c > 0 && to / c != f / c) atomicAdd(&inter[f], (unsigned long long)L);
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
                       inst_begin, inst_end, w.hdr, w.src_cu, w.seg_dst, w.seg_src, row_bytes, w.gtab);

    launch_copy(tokens, packed, (packed_rows < T ? packed_rows : T) * row_bytes, row_bytes, w.hdr,
                w.seg_dst, w.seg_dst, w.seg_src, w.gtab, stream);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

size_t pack_composed_ws_bytes(int32_t n)
{
    ComposeWs w;
    return carve(w, nullptr, n);
}

int launch_pack_composed(const void *enc_rows, void *packed, const int32_t *sub_len,
                         const int32_t *sub_off, int32_t n, int32_t D_src, const orch_assignment *src,
                         int32_t D_dst, orch_assignment dst, int64_t src_rows, int32_t H,
                         int64_t packed_rows, int32_t inst_begin, int32_t inst_end, void *ws,
                         size_t ws_bytes, hipStream_t stream)
{
    ComposeWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_pack_composed: workspace %zu < %zu bytes", ws_bytes, need);
    const int64_t row_bytes = (int64_t)H * 2;
    ComposeSide e{}, m{dst.inst, dst.order, dst.seq_off, dst.cu_seqlens, dst.tok_off, dst.dev_status, D_dst};
    if (src) e = ComposeSide{src->inst, src->order, src->seq_off, src->cu_seqlens, src->tok_off, src->dev_status, D_src};
    hipLaunchKernelGGL(compose_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, sub_len, sub_off, n,
                       src_rows, packed_rows, src ? 1 : 0, e, m, dst.dev_status, inst_begin, inst_end, w.hdr,
                       w.src_start, w.seg_pos, w.seg_dst, w.seg_src, row_bytes, w.gtab);
    launch_copy(enc_rows, packed, (packed_rows < src_rows ? packed_rows : src_rows) * row_bytes, row_bytes,
                w.hdr, w.seg_pos, w.seg_dst, w.seg_src, w.gtab, stream);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

size_t pack_composed_pieces_ws_bytes(int32_t n, int32_t P)
{
    PiecesWs w;
    return carve(w, nullptr, n, P);
}

int launch_pack_composed_pieces(const void *enc_rows, void *packed, const int32_t *piece_ptr,
                                const int32_t *piece_off, const int32_t *piece_len, int32_t n, int32_t P,
                                int32_t D_src, const orch_assignment *src, int32_t D_dst, orch_assignment dst,
                                int64_t src_rows, int32_t H, int64_t packed_rows, int32_t inst_begin,
                                int32_t inst_end, void *ws, size_t ws_bytes, hipStream_t stream)
{
    PiecesWs w;
    size_t need = carve(w, ws, n, P);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_pack_composed_pieces: workspace %zu < %zu bytes", ws_bytes, need);
    const int64_t row_bytes = (int64_t)H * 2;
    ComposeSide e{}, m{dst.inst, dst.order, dst.seq_off, dst.cu_seqlens, dst.tok_off, dst.dev_status, D_dst};
    if (src) e = ComposeSide{src->inst, src->order, src->seq_off, src->cu_seqlens, src->tok_off, src->dev_status, D_src};
    hipLaunchKernelGGL(compose_pieces_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, piece_ptr, piece_off,
                       piece_len, n, P, src_rows, packed_rows, src ? 1 : 0, e, m, dst.dev_status, inst_begin,
                       inst_end, w.hdr, w.src_start, w.piece_pre, w.seg_base, w.seg_pos, w.seg_dst, w.seg_src,
                       row_bytes, w.gtab);
    launch_copy(enc_rows, packed, (packed_rows < src_rows ? packed_rows : src_rows) * row_bytes, row_bytes,
                w.hdr, w.seg_pos, w.seg_dst, w.seg_src, w.gtab, stream);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

int launch_comm_volume(const int32_t *lengths, int32_t n, int32_t D_src, const int32_t *from, int32_t D_dst,
                       orch_assignment dst, uint64_t *V, int32_t node, uint64_t *inter, hipStream_t stream)
{
    const int64_t cells = (int64_t)D_src * D_dst;
    const int64_t clear = cells > D_src ? cells : D_src;
    hipLaunchKernelGGL(comm_clear_kernel, dim3((unsigned)((clear + 255) / 256)), dim3(256), 0, stream,
                       (unsigned long long *)V, cells, (unsigned long long *)inter, D_src);
    if (n > 0)
        hipLaunchKernelGGL(comm_volume_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, lengths, n, D_src, from,
                           D_dst, dst.inst, (unsigned long long *)V, node, (unsigned long long *)inter,
                           dst.dev_status);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
