// orch_balance: Eq. 2's per-sequence cost, Algorithm 1 (sort descending, then
// longest-first greedy onto the least-loaded instance) and the packed layout.
// (Sec. 5.1; the layout is Sec. 7's: sequences concatenated along the token axis, unpadded.)
//
// orch_balance_padded: Algorithm 2 (the same sort, ascending, then the bound search
// and the padded layout in one kernel; see padded_split_kernel).
//
// orch_balance_tolerance: Appendix A's third algorithm (the same sort by length, then
// greedy_tolerance_kernel, the same layout kernel).
//
// orch_balance, three launches on the caller's stream:
//   cost_sort_kernel   one 1024-thread workgroup: cost keys, then a stable LSD
//                      radix sort (8-bit digits, only as many passes as the
//                      largest key needs) of (~cost, index) pairs
//   greedy_kernel      one workgroup of four wavefronts (both forms of the loop in one
//                      launch; a flag from the sort kernel picks one).  Wave 0 runs the serial
//                      loop (in rounds of up to D items where the loads allow) and
//                      does nothing but choose the receiving instance; it publishes
//                      the choices per sorted position.  Waves 1-3 trail it, taking
//                      64-position chunks in turn, and make (instance, rank within
//                      instance, first token) per sequence, so that bookkeeping
//                      never sits on the dependent chain.
//   layout_kernel      n threads: scatter sequence ids and segment starts
// n <= 32768 keys is latency-bound work, so everything is arranged to keep the
// dependent chain short rather than to stream memory.
#include <mutex>

#include "common.h"

namespace orch {
namespace {

constexpr int kSortThreads = 1024;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kRadix = 256;

struct BalanceWs {
    uint64_t *csorted, *keyA, *keyB;  // csorted[t]: cost of the t-th sequence in descending order
    uint32_t *idxA, *idxB;
    int32_t *sorted, *rank, *start;
    int32_t *ipos;   // ipos[t]: instance chosen for sorted position t
    int32_t *flags;  // [0]: 1 when every load fits the packed (load << 12 | instance) key
                     // [1]: 1 when the sum of all keys is below 2^32
};

size_t carve(BalanceWs &w, void *ws, int32_t n)
{
    size_t nn = align_up((size_t)(n > 0 ? n : 1), 64);
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.csorted = (uint64_t *)take(nn * 8);
    w.keyA = (uint64_t *)take(nn * 8);
    w.keyB = (uint64_t *)take(nn * 8);
    w.idxA = (uint32_t *)take(nn * 4);
    w.idxB = (uint32_t *)take(nn * 4);
    w.sorted = (int32_t *)take(nn * 4);
    w.rank = (int32_t *)take(nn * 4);
    w.start = (int32_t *)take(nn * 4);
    w.ipos = (int32_t *)take(nn * 4);
    w.flags = (int32_t *)take(64);
    return off;
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t x, int m)
{
    return (uint64_t)__shfl_xor((unsigned long long)x, m);
}

// ---------------------------------------------------------------------------
// cost + stable radix sort, one workgroup
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kSortThreads) void cost_sort_kernel(
    const int32_t *__restrict__ lengths, int32_t n, uint64_t a, uint64_t b, int ascending,
    uint64_t *csorted, uint64_t *keyA, uint64_t *keyB, uint32_t *idxA, uint32_t *idxB,
    int32_t *sorted, int32_t *flags, int32_t *dev_status)
{
    __shared__ uint32_t hist[kSortWaves][kRadix];
    __shared__ uint32_t dig_base[kRadix];
    __shared__ uint64_t red_or[kSortWaves], red_sum[kSortWaves];
    __shared__ int red_err[kSortWaves];
    __shared__ int s_passes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Eq. 2, no-padding branch, per sequence: c = a*l^2 + b*l, exact in u64.
    uint64_t my_or = 0, my_sum = 0;
    int err = 0;
    for (int64_t i = tid; i < n; i += kSortThreads) {
        int32_t L = lengths[i];
        uint64_t c = 0;
        if (L < 0) {
            err = 1;
        } else {
            uint64_t l = (uint64_t)L, l2 = l * l;
            uint64_t t1 = a * l2, t2 = b * l;
            c = t1 + t2;
            bool bad = __umul64hi(a, l2) != 0 || __umul64hi(b, l) != 0 || c < t1 || (c >> 63);
            if (bad) { err = 1; c = 0; }
        }
        keyA[i] = ascending ? c : ~c;  // ascending on ~c == descending on c
        idxA[i] = (uint32_t)i;
        my_or |= c;
        my_sum += c;
        if (my_sum >> 63) { err = 1; my_sum = 0; }
    }
    for (int m = 32; m >= 1; m >>= 1) {
        my_or |= shfl_xor_u64(my_or, m);
        uint64_t o = shfl_xor_u64(my_sum, m);
        my_sum += o;
        if (my_sum >> 63) { err = 1; my_sum = (1ull << 63) - 1; }
        err |= __shfl_xor(err, m);
    }
    if (lane == 0) { red_or[wave] = my_or; red_sum[wave] = my_sum; red_err[wave] = err; }
    __syncthreads();
    if (tid == 0) {
        uint64_t o = 0, s = 0;
        int e = 0;
        for (int w = 0; w < kSortWaves; ++w) {
            o |= red_or[w];
            s += red_sum[w];
            if (s >> 63) { e = 1; s = (1ull << 63) - 1; }
            e |= red_err[w];
        }
        dev_status[0] = e ? (int32_t)ORCH_EDATA : (int32_t)ORCH_OK;
        flags[0] = (!e && s < (1ull << 51)) ? 1 : 0;  // no instance load can exceed the total
        flags[1] = (!e && s < (1ull << 32)) ? 1 : 0;  // every partial sum of keys fits 32 bits
        int nbits = o ? 64 - __clzll((long long)o) : 0;
        s_passes = (nbits + 7) / 8;
    }
    __syncthreads();
    const int passes = s_passes;

    // each wave owns a contiguous chunk (multiple of 64 keys)
    int64_t chunk = ((int64_t)n + kSortWaves - 1) / kSortWaves;
    chunk = (chunk + 63) / 64 * 64;
    const int64_t wbeg = min((int64_t)n, chunk * wave), wend = min((int64_t)n, chunk * (wave + 1));
    volatile uint32_t *hw = hist[wave];

    uint64_t *ksrc = keyA, *kdst = keyB;
    uint32_t *isrc = idxA, *idst = idxB;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&hist[0][0])[i] = 0;
        __syncthreads();
        for (int64_t i = wbeg + lane; i < wend; i += 64)
            atomicAdd(&hist[wave][(ksrc[i] >> shift) & 255], 1u);
        __syncthreads();
        // per digit: exclusive prefix over waves, digit totals
        if (tid < kRadix) {
            uint32_t run = 0;
            for (int w = 0; w < kSortWaves; ++w) {
                uint32_t t = hist[w][tid];
                hist[w][tid] = run;
                run += t;
            }
            dig_base[tid] = run;
        }
        __syncthreads();
        if (wave == 0) {  // exclusive scan of the 256 digit totals
            uint32_t t0 = dig_base[4 * lane], t1 = dig_base[4 * lane + 1], t2 = dig_base[4 * lane + 2],
                     t3 = dig_base[4 * lane + 3];
            uint32_t tot = t0 + t1 + t2 + t3, inc = tot;
            for (int m = 1; m < 64; m <<= 1) {
                uint32_t o = __shfl_up(inc, m);
                if (lane >= m) inc += o;
            }
            uint32_t ex = inc - tot;
            dig_base[4 * lane] = ex;
            dig_base[4 * lane + 1] = ex + t0;
            dig_base[4 * lane + 2] = ex + t0 + t1;
            dig_base[4 * lane + 3] = ex + t0 + t1 + t2;
        }
        __syncthreads();
        for (int i = tid; i < kSortWaves * kRadix; i += kSortThreads) (&hist[0][0])[i] += dig_base[i & 255];
        __syncthreads();
        // stable scatter: batches of 64 keys in order; lanes with the same digit
        // are ranked by lane id
        for (int64_t i0 = wbeg; i0 < wend; i0 += 64) {
            const int64_t i = i0 + lane;
            const bool valid = i < wend;
            uint64_t key = 0;
            uint32_t idx = 0;
            if (valid) { key = ksrc[i]; idx = isrc[i]; }
            const uint32_t dg = (uint32_t)(key >> shift) & 255u;
            uint64_t peers = __ballot(valid);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool on = (dg >> bit) & 1u;
                const uint64_t bm = __ballot(on);
                peers &= on ? bm : ~bm;
            }
            const uint32_t rank = __popcll(peers & ((1ull << lane) - 1ull));
            const uint32_t cnt = __popcll(peers);
            uint32_t base = 0;
            if (valid) base = hw[dg];
            __builtin_amdgcn_wave_barrier();
            if (valid && rank == cnt - 1) hw[dg] = base + cnt;
            __builtin_amdgcn_wave_barrier();
            if (valid) { kdst[base + rank] = key; idst[base + rank] = idx; }
        }
        __syncthreads();
        uint64_t *tk = ksrc; ksrc = kdst; kdst = tk;
        uint32_t *ti = isrc; isrc = idst; idst = ti;
    }
    for (int64_t i = tid; i < n; i += kSortThreads) {
        sorted[i] = (int32_t)isrc[i];
        csorted[i] = ascending ? ksrc[i] : ~ksrc[i];
    }
}

// ---------------------------------------------------------------------------
// wave-wide unsigned minimum (DPP row shifts + row broadcasts), result uniform
// ---------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_min_step(uint64_t x)
{
    uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    uint32_t olo = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, ROW_MASK, 0xf, false);
    uint32_t ohi = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, ROW_MASK, 0xf, false);
    uint64_t o = ((uint64_t)ohi << 32) | olo;
    return o < x ? o : x;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t x)
{
    x = dpp_min_step<0x111, 0xf>(x);  // row_shr:1
    x = dpp_min_step<0x112, 0xf>(x);  // row_shr:2
    x = dpp_min_step<0x114, 0xf>(x);  // row_shr:4
    x = dpp_min_step<0x118, 0xf>(x);  // row_shr:8  -> lane 15 of each row holds the row minimum
    x = dpp_min_step<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
    x = dpp_min_step<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3 -> lane 63 holds the minimum
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, 63);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), 63);
    return ((uint64_t)hi << 32) | lo;
}

// 32-bit wave minimum, result uniform.  Each stage is one v_min_u32 with a DPP source operand
// (lanes whose DPP source does not exist keep their value); a VALU result needs two wait
// states before a DPP read of it.  The n-step loops that use this are bound by the number of
// dependent instructions per step, so the fused form matters.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x)
{
    uint32_t r;
    asm volatile(
        "s_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"
        "v_min_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\ts_nop 1\n\t"
        "v_readlane_b32 %1, %0, 63\n\t"
        "s_nop 3"
        : "+v"(x), "=s"(r));
    return r;
}

__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int j)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, j);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), j);
    return ((uint64_t)hi << 32) | lo;
}

// Closing work shared by the greedy kernels: instance i's sequence count and
// token total become seq_off / tok_off and the last cu_seqlens entry.
// `per` consecutive instances per lane, held in LDS arrays.  One wavefront.
__device__ void finish_layout(const uint32_t *cnt, const unsigned long long *tok, int D, int32_t *seq_off,
                              int64_t *tok_off, int32_t *cu_seqlens, int32_t *dev_status)
{
    const int lane = threadIdx.x & 63;
    const int per = (D + 63) / 64;
    const int b0 = min(D, lane * per), b1 = min(D, b0 + per);
    uint32_t csum = 0;
    uint64_t tsum = 0;
    int err = 0;
    for (int i = b0; i < b1; ++i) {
        csum += cnt[i];
        tsum += tok[i];
        if (tok[i] > 0x7fffffffull) err = 1;
    }
    uint32_t cinc = csum;
    uint64_t tinc = tsum;
    for (int m = 1; m < 64; m <<= 1) {
        uint32_t oc = __shfl_up(cinc, m);
        uint64_t ot = (uint64_t)__shfl_up((unsigned long long)tinc, m);
        if (lane >= m) { cinc += oc; tinc += ot; }
    }
    uint32_t c = cinc - csum;
    uint64_t t = tinc - tsum;
    for (int i = b0; i < b1; ++i) {
        seq_off[i] = (int32_t)c;
        tok_off[i] = (int64_t)t;
        c += cnt[i];
        t += tok[i];
        cu_seqlens[c + i] = (int32_t)tok[i];  // entry cnt_i of instance i's slice
        if (i == D - 1) { seq_off[D] = (int32_t)c; tok_off[D] = (int64_t)t; }
    }
    if (__any(err) && lane == 0) dev_status[0] = (int32_t)ORCH_EDATA;
}

// ---------------------------------------------------------------------------
// The two halves of a greedy workgroup talk through `ipos` (global, one entry
// per sorted position) and a chunk counter in LDS.  The chooser never waits
// for the bookkeeper, and the bookkeeper only waits for chunks the chooser is
// certain to publish, so both always run to the end.
// ---------------------------------------------------------------------------
struct ChoiceLog {
    int32_t *ipos;
    int *progress;   // LDS: number of sorted positions whose choice is published
    int32_t rec;     // lane j: instance chosen at step j of the current chunk
};

__device__ __forceinline__ void log_choice(ChoiceLog &g, int lane, int j, int32_t instance)
{
    g.rec = lane == j ? instance : g.rec;
}

__device__ __forceinline__ void publish_upto(int *progress, int64_t done)
{
    // release: the ipos stores before this are visible to the workgroup before the counter moves
    __hip_atomic_store(progress, (int)done, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ void publish_chunk(ChoiceLog &g, int64_t t0, int32_t n, int lane, int chunk)
{
    (void)chunk;
    if (t0 + lane < n) g.ipos[t0 + lane] = g.rec;
    publish_upto(g.progress, min((int64_t)n, t0 + 64));
}

// Waves 1..kBookWaves.  Chunks of 64 sorted positions are dealt round-robin to
// the bookkeeping waves.  For its chunk a wave waits until the choices are
// published, counts for every lane the earlier lanes of the same instance
// (lane order = assignment order) and their tokens, then takes its turn (chunks
// in order, `booked` is the baton) to add the running per-instance count and
// token total kept in LDS.  Only that last part is serial across waves.
constexpr int kBookWaves = 3;
constexpr int kGreedyThreads = 64 * (1 + kBookWaves);

struct BookState {
    int *progress;   // LDS: sorted positions published by the choosing wave
    int *booked;     // LDS: chunks whose running totals are updated
    uint32_t *cnt;   // LDS [D]: sequences per instance so far
    unsigned long long *tok;  // LDS [D]: tokens per instance so far
};

__device__ void bookkeep_wave(const int32_t *ipos, const int32_t *__restrict__ sorted,
                              const int32_t *__restrict__ lengths, int32_t n, int32_t D, int lane,
                              int wid, BookState b, int32_t *inst, int32_t *rank, int32_t *start,
                              int32_t *dev_status)
{
    int bad = 0;
    for (int64_t q = wid; q * 64 < n; q += kBookWaves) {
        const int64_t t0 = q * 64;
        const bool valid = t0 + lane < n;
        int32_t s = 0, l = 0;
        if (valid) { s = sorted[t0 + lane]; l = lengths[s]; }
        const int need = (int)min((int64_t)n, t0 + 64);
        while (__hip_atomic_load(b.progress, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need)
            __builtin_amdgcn_s_sleep(2);
        int32_t g = valid ? ipos[t0 + lane] : -1 - lane;  // idle lanes match nobody
        if (valid && (uint32_t)g >= (uint32_t)D) { g = 0; bad = 1; }  // never index outside the tables
        uint32_t before_c = 0;
        uint64_t before_l = 0;
        // all 64 lanes every time (idle lanes match nobody), in unrolled blocks so that the
        // cross-lane reads of a block are in flight together
        for (int j0 = 0; j0 < 64; j0 += 16) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int j = j0 + u;
                const int32_t gj = __builtin_amdgcn_readlane(g, j);
                const uint64_t lj = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(l, j);
                const bool bef = gj == g && j < lane;
                before_c += bef ? 1u : 0u;
                before_l += bef ? lj : 0ull;
            }
        }
        while (__hip_atomic_load(b.booked, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (int)q)
            __builtin_amdgcn_s_sleep(1);
        uint32_t bc = 0;
        uint64_t bt = 0;
        if (valid) {
            bc = b.cnt[g];
            bt = b.tok[g];
            // the last lane of an instance carries the largest values: the maximum is its update
            atomicMax(&b.cnt[g], bc + before_c + 1u);
            atomicMax(&b.tok[g], (unsigned long long)(bt + before_l + (uint64_t)(uint32_t)l));
        }
        __hip_atomic_store(b.booked, (int)q + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (valid) {
            inst[s] = g;
            rank[s] = (int32_t)(bc + before_c);
            start[s] = (int32_t)(bt + before_l);
        }
    }
    if (bad) dev_status[0] = (int32_t)ORCH_EDATA;
}


#define ORCH_GREEDY_PARAMS                                                                          \
    const uint64_t *__restrict__ csorted, const int32_t *__restrict__ sorted,                       \
        const int32_t *__restrict__ lengths, int32_t n, int32_t D, int32_t *ipos, int32_t *inst,    \
        int32_t *rank, int32_t *start, uint64_t *loads, int32_t *seq_off, int64_t *tok_off,         \
        int32_t *cu_seqlens, const int32_t *flags, int32_t *dev_status

// ---------------------------------------------------------------------------
// Algorithm 1, lines 2-7, general form: instance loads in registers, lane l
// owns instances l*K .. l*K+K-1, so "lowest lane, then lowest k" is the lowest
// instance index among equal loads.  A step is a 64-lane min-reduction.
// ---------------------------------------------------------------------------
template <int K>
__device__ __forceinline__ void greedy_reg_body(ORCH_GREEDY_PARAMS, uint32_t *s_cnt, unsigned long long *s_tok,
                                                int &s_progress, int &s_booked)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    for (int i = threadIdx.x; i < 64 * K; i += kGreedyThreads) { s_cnt[i] = 0; s_tok[i] = 0; }
    if (threadIdx.x == 0) { s_progress = 0; s_booked = 0; }
    __syncthreads();
    if (wave >= 1) {
        bookkeep_wave(ipos, sorted, lengths, n, D, lane, wave - 1, BookState{&s_progress, &s_booked, s_cnt, s_tok},
                      inst, rank, start, dev_status);
    } else {
        uint64_t load[K];
#pragma unroll
        for (int k = 0; k < K; ++k) load[k] = (lane * K + k < D) ? 0ull : ~0ull;
        ChoiceLog log{ipos, &s_progress, 0};
        uint64_t c_cur = lane < n ? csorted[lane] : 0;
        int chunk = 0;
        for (int64_t t0 = 0; t0 < n; t0 += 64, ++chunk) {
            const uint64_t c_nxt = (t0 + 64 + lane < n) ? csorted[t0 + 64 + lane] : 0;
            const int m = (int)min((int64_t)64, (int64_t)n - t0);
            for (int j = 0; j < m; ++j) {
                const uint64_t c = readlane_u64(c_cur, j);
                uint64_t lm = load[0];
#pragma unroll
                for (int k = 1; k < K; ++k) lm = load[k] < lm ? load[k] : lm;
                const uint64_t g = wave_min_u64(lm);
                const uint64_t ball = __ballot(lm == g);
                const int win = __ffsll((unsigned long long)ball) - 1;
                int kk = K - 1;
#pragma unroll
                for (int k = K - 2; k >= 0; --k) kk = (load[k] == g) ? k : kk;
                if (lane == win) {
#pragma unroll
                    for (int k = 0; k < K; ++k)
                        if (k == kk) load[k] += c;
                }
                log_choice(log, lane, j, __builtin_amdgcn_readlane(lane * K + kk, win));
            }
            publish_chunk(log, t0, n, lane, chunk);
            c_cur = c_nxt;
        }
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (lane * K + k < D) loads[lane * K + k] = load[k];
    }
    __syncthreads();
    if (wave == 0) finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
}

// ---------------------------------------------------------------------------
// Algorithm 1, lines 2-7, fast form.  When every load fits in 51 bits the pair
// (load, instance) packs into one u64 key, load << 12 | instance, whose order
// is exactly "smaller load first, lower instance on ties".  The D keys are
// kept SORTED across the wavefront (element e in register e/64, lane e%64).
//
// Rounds instead of steps.  With sorted keys k_0 < k_1 < ... and the next
// items c_0 >= c_1 >= ..., the sequential loop gives item i to element i for
// as long as k_i is still below every key produced so far in the round:
//     k_i < min(k_0 + c_0, ..., k_{i-1} + c_{i-1})            (*)
// An exclusive prefix minimum over the tentative keys k_e + c_e tests (*) for
// all elements at once; the first m' items (the longest prefix on which it
// holds, at least 1) are then assigned together and the keys are put back in
// order, either by m' single insertions or, for a long prefix, by a rank sort
// (every key counts the keys below it; keys are distinct).  The assignment is
// the one the item-by-item loop makes: (*) is exactly its choice rule.
// On balanced workloads a round hands one item to every instance.
// ---------------------------------------------------------------------------
// Lane i receives x from lane i + 1; lane 63, which has no source, receives `fill`.
__device__ __forceinline__ uint64_t wave_shl1_u64(uint64_t x, uint64_t fill)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)fill, (int)(uint32_t)x, 0x130, 0xf,
                                                        0xf, false);  // wave_shl:1
    uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(fill >> 32),
                                                        (int)(uint32_t)(x >> 32), 0x130, 0xf, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}

// Lane i receives x from lane i - 1; lane 0 receives `fill`.
__device__ __forceinline__ uint64_t wave_shr1_u64(uint64_t x, uint64_t fill)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)fill, (int)(uint32_t)x, 0x138, 0xf,
                                                        0xf, false);  // wave_shr:1
    uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(fill >> 32),
                                                        (int)(uint32_t)(x >> 32), 0x138, 0xf, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}

// Inclusive prefix minimum across the 64 lanes (the reduction above, before
// its final broadcast, is a scan: lane i ends with min(x_0..x_i)).
__device__ __forceinline__ uint64_t wave_prefix_min_u64(uint64_t x)
{
    x = dpp_min_step<0x111, 0xf>(x);
    x = dpp_min_step<0x112, 0xf>(x);
    x = dpp_min_step<0x114, 0xf>(x);
    x = dpp_min_step<0x118, 0xf>(x);
    x = dpp_min_step<0x142, 0xa>(x);
    x = dpp_min_step<0x143, 0xc>(x);
    return x;
}

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


constexpr int kRing = 4096;         // LDS window over the sorted costs, entries (power of two)
constexpr int kRefillChunks = 16;   // 64-entry chunks fetched per refill

template <int K>
__device__ __forceinline__ void greedy_sorted_body(ORCH_GREEDY_PARAMS, uint32_t *s_cnt, unsigned long long *s_tok,
                                                   int &s_progress, int &s_booked)
{
    __shared__ uint64_t s_perm[64 * K];   // rank-sort scatter, then loads by instance
    __shared__ uint64_t s_ring[kRing];    // (cost << 12) of sorted positions [.., filled)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    for (int i = threadIdx.x; i < 64 * K; i += kGreedyThreads) { s_cnt[i] = 0; s_tok[i] = 0; }
    if (threadIdx.x == 0) { s_progress = 0; s_booked = 0; }
    __syncthreads();
    if (wave >= 1) {
        bookkeep_wave(ipos, sorted, lengths, n, D, lane, wave - 1, BookState{&s_progress, &s_booked, s_cnt, s_tok},
                      inst, rank, start, dev_status);
    } else {
        uint64_t key[K];  // sorted position 64r + lane
#pragma unroll
        for (int r = 0; r < K; ++r) {
            const int e = 64 * r + lane;
            key[r] = e < D ? (uint64_t)e : ~0ull;
        }
        // one insertion costs about 10 + 12K instructions, a rank sort D(2 + 2K)
        const int seq_limit = min(64, D * (2 + 2 * K) / (10 + 12 * K));
        int64_t j = 0, filled = 0;  // items consumed; items staged in the ring (multiple of 64)

        // one sequential step: the new key of element 0 moves up to its place
        auto insert = [&](uint64_t c) {
            const uint64_t k0 = readlane_u64(key[0], 0);
            const uint64_t nk = k0 + c;
            // sh = the keys moved down one place; with p = number of keys other than key_0
            // below nk:  e < p <=> sh_e < nk,  e == p <=> key_e < nk <= sh_e.
            // Registers whose first key is already above nk are left alone.
            bool settled = false;
#pragma unroll
            for (int r = 0; r < K; ++r) {
                if (!settled) {
                    const uint64_t fill = (r + 1 < K) ? readlane_u64(key[(r + 1 < K) ? r + 1 : r], 0) : ~0ull;
                    const uint64_t sh = wave_shl1_u64(key[r], fill);
                    key[r] = sh < nk ? sh : (key[r] < nk ? nk : key[r]);
                    settled = nk < fill;
                }
            }
        };

        while (j < n) {
            const int m = (int)min((int64_t)D, (int64_t)n - j);
            if (filled < j + m) {
                // the ring holds [j, filled): top it up by as many chunks as fit and exist
                const int room = (int)((kRing - (filled - j)) / 64);
                const int want = (int)(((int64_t)n - filled + 63) / 64);
                const int G = min(min(room, want), kRefillChunks);
                uint64_t v[kRefillChunks];
#pragma unroll
                for (int g = 0; g < kRefillChunks; ++g) {
                    // clamped, unconditional: all the loads are in flight together
                    const int64_t pos = min(filled + 64 * g + lane, (int64_t)n - 1);
                    v[g] = csorted[pos];
                }
#pragma unroll
                for (int g = 0; g < kRefillChunks; ++g)
                    if (g < G) s_ring[(filled + 64 * g + lane) & (kRing - 1)] = v[g] << 12;
                filled += 64 * G;
                wave_lds_fence();
            }
            uint64_t c[K], nk[K];
#pragma unroll
            for (int r = 0; r < K; ++r) {
                const int e = 64 * r + lane;
                c[r] = e < m ? s_ring[(j + e) & (kRing - 1)] : 0;
                nk[r] = key[r] + c[r];
            }
            const int32_t idx0 = (int32_t)((uint32_t)readlane_u64(key[0], 0) & 4095u);
            if (readlane_u64(c[0], 0) == 0) {
                // costs are sorted: every remaining item is free, the minimum never moves
                for (int64_t t = j + lane; t < n; t += 64) ipos[t] = idx0;
                j = n;
                publish_upto(&s_progress, j);
                break;
            }
            // longest prefix on which (*) holds
            int mp = m;
            {
                uint64_t carry = ~0ull;  // smallest tentative key of the registers before r
                bool found = false;
#pragma unroll
                for (int r = 0; r < K; ++r) {
                    if (64 * r < m && !found) {
                        const int e = 64 * r + lane;
                        const uint64_t inc = wave_prefix_min_u64(e < m ? nk[r] : ~0ull);
                        uint64_t exc = wave_shr1_u64(inc, ~0ull);
                        exc = carry < exc ? carry : exc;
                        const uint64_t bad = __ballot(e < m && !(key[r] < exc));
                        if (bad) { mp = 64 * r + (__ffsll((unsigned long long)bad) - 1); found = true; }
                        const uint64_t tot = readlane_u64(inc, 63);
                        carry = tot < carry ? tot : carry;
                    }
                }
            }
            // the first mp items go to elements 0..mp-1, in that order
#pragma unroll
            for (int r = 0; r < K; ++r) {
                const int e = 64 * r + lane;
                if (e < mp) ipos[j + e] = (int32_t)((uint32_t)key[r] & 4095u);
            }
            if (mp <= seq_limit) {
                for (int i = 0; i < mp; ++i) insert(readlane_u64(c[0], i));
            } else {
                uint32_t below[K];
#pragma unroll
                for (int r = 0; r < K; ++r) {
                    if (64 * r + lane < mp) key[r] = nk[r];
                    below[r] = 0;
                }
#pragma unroll
                for (int rp = 0; rp < K; ++rp) {
                    // blocks of 16 lanes, unrolled: the cross-lane reads of a block are in
                    // flight together; padding keys (~0) are below nothing
                    const int cnt = min(64, D - 64 * rp);
                    for (int l0 = 0; l0 < cnt; l0 += 16) {
#pragma unroll
                        for (int u = 0; u < 16; ++u) {
                            const uint64_t s = readlane_u64(key[rp], l0 + u);
#pragma unroll
                            for (int r = 0; r < K; ++r) below[r] += (s < key[r]) ? 1u : 0u;
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < K; ++r)
                    if (64 * r + lane < D) s_perm[below[r]] = key[r];
                wave_lds_fence();
#pragma unroll
                for (int r = 0; r < K; ++r)
                    if (64 * r + lane < D) key[r] = s_perm[64 * r + lane];
                wave_lds_fence();
            }
            j += mp;
            publish_upto(&s_progress, j);
        }
#pragma unroll
        for (int r = 0; r < K; ++r)
            if (key[r] != ~0ull) s_perm[key[r] & 4095u] = key[r] >> 12;  // back to instance order
    }
    __syncthreads();
    if (wave == 0) {
        for (int i = lane; i < D; i += 64) loads[i] = s_perm[i];
        finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
    }
}

// One entry for both register forms: the sort kernel's flag (every load fits the packed
// (load << 12 | instance) key) picks the body on the device, so a call enqueues one launch.
#define ORCH_GREEDY_NAMES                                                                           \
    csorted, sorted, lengths, n, D, ipos, inst, rank, start, loads, seq_off, tok_off, cu_seqlens,   \
        flags, dev_status
template <int K>
__global__ __launch_bounds__(kGreedyThreads) void greedy_kernel(ORCH_GREEDY_PARAMS)
{
    __shared__ uint32_t s_cnt[64 * K];
    __shared__ unsigned long long s_tok[64 * K];
    __shared__ int s_progress, s_booked;
    if (flags[0] == 1) greedy_sorted_body<K>(ORCH_GREEDY_NAMES, s_cnt, s_tok, s_progress, s_booked);
    else greedy_reg_body<K>(ORCH_GREEDY_NAMES, s_cnt, s_tok, s_progress, s_booked);
}

// Same loop for D beyond what registers hold: per-instance loads in LDS,
// instance i lives at lane i%64, slot i/64.  Two reductions per step: the
// minimal load, then the minimal instance index among lanes that hold it.
constexpr int kMaxInstances = 4096;

__global__ __launch_bounds__(kGreedyThreads) void greedy_lds_kernel(ORCH_GREEDY_PARAMS)
{
    (void)flags;
    __shared__ uint64_t s_load[kMaxInstances];
    __shared__ unsigned long long s_tok[kMaxInstances];
    __shared__ uint32_t s_cnt[kMaxInstances];
    __shared__ int s_progress, s_booked;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int K = (D + 63) / 64;
    for (int i = threadIdx.x; i < K * 64; i += kGreedyThreads) {
        s_load[i] = i < D ? 0ull : ~0ull;
        s_tok[i] = 0;
        s_cnt[i] = 0;
    }
    if (threadIdx.x == 0) { s_progress = 0; s_booked = 0; }
    __syncthreads();
    if (wave >= 1) {
        bookkeep_wave(ipos, sorted, lengths, n, D, lane, wave - 1, BookState{&s_progress, &s_booked, s_cnt, s_tok},
                      inst, rank, start, dev_status);
    } else {
        ChoiceLog log{ipos, &s_progress, 0};
        int chunk = 0;
        for (int64_t t0 = 0; t0 < n; t0 += 64, ++chunk) {
            const uint64_t c_cur = (t0 + lane < n) ? csorted[t0 + lane] : 0;
            const int m = (int)min((int64_t)64, (int64_t)n - t0);
            for (int j = 0; j < m; ++j) {
                const uint64_t c = readlane_u64(c_cur, j);
                uint64_t lm = ~0ull;
                uint32_t li = 0xffffffffu;
                for (int k = 0; k < K; ++k) {
                    const uint64_t v = s_load[k * 64 + lane];
                    if (v < lm) { lm = v; li = (uint32_t)(k * 64 + lane); }
                }
                const uint64_t g = wave_min_u64(lm);
                const uint64_t cand = (lm == g) ? (uint64_t)li : ~0ull;
                const uint32_t bi = (uint32_t)wave_min_u64(cand);
                if (lane == (int)(bi & 63u)) s_load[bi] += c;
                log_choice(log, lane, j, (int32_t)bi);
                // one wave owns s_load: order the update before the next scan
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            publish_chunk(log, t0, n, lane, chunk);
        }
        for (int i = lane; i < D; i += 64) loads[i] = s_load[i];
    }
    __syncthreads();
    if (wave == 0) finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
}

// ---------------------------------------------------------------------------
// The appendix's third algorithm: Algorithm 1 whose "lightest batch" is, among the
// batches with a length sum less than (smallest length sum) + max(v, 1), the one with
// the smallest sum of squared lengths (lowest index on ties).  Same workgroup shape as
// greedy_reg_kernel: wave 0 chooses, the other waves turn choices into the layout.
// The n steps depend on one another and one wavefront issues about one instruction per
// 5 clocks, so a step costs what its instruction count says.  Two forms:
//   * general (64-bit length sums): three 64-lane reductions per step: smallest sum,
//     smallest squares inside the window, lowest lane holding it;
//   * all lengths together < 2^32 and the longest < 2^30 (so the squares of all sequences
//     together stay below 2^62): 32-bit sums; the smallest sum is kept from step to step
//     and recomputed only when the instance that held it wins; the squares are compared by
//     their leading 31 bits (one 32-bit reduction whose result lands in every lane, no
//     scalar round trip), and only when two candidates agree in those bits does the step
//     fall back to the exact 64-bit comparison.
// ---------------------------------------------------------------------------

// Smallest x over the wavefront (HALF: over lanes 0..31), delivered to every one of those
// lanes: four butterfly stages inside the rows of 16 lanes (each one v_min_u32 with a DPP
// operand; a VALU result needs two wait states before a DPP read of it), then the rows are
// combined by the row / half swaps.
template <bool HALF>
__device__ __forceinline__ uint32_t lanes_min_u32(uint32_t x)
{
    uint32_t r, t;   // every lane of a quad has a partner, so the first stage may write a fresh register
    if (HALF)
        asm volatile(
            "s_nop 1\n\t"
            "v_min_u32_dpp %0, %2, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_e32 %1, %0\n\ts_nop 1\n\t"
            "v_permlane16_swap_b32_e32 %0, %1\n\t"   // rows 0|1 (and 2|3)
            "v_min_u32_e32 %0, %0, %1"
            : "=&v"(r), "=&v"(t)
            : "v"(x));
    else
        asm volatile(
            "s_nop 1\n\t"
            "v_min_u32_dpp %0, %2, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
            "v_min_u32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_e32 %1, %0\n\ts_nop 1\n\t"
            "v_permlane16_swap_b32_e32 %0, %1\n\t"   // rows 0|1 and 2|3
            "v_min_u32_e32 %0, %0, %1\n\t"
            "v_mov_b32_e32 %1, %0\n\ts_nop 1\n\t"
            "v_permlane32_swap_b32_e32 %0, %1\n\t"   // lanes 0..31 | 32..63
            "v_min_u32_e32 %0, %0, %1"
            : "=&v"(r), "=&v"(t)
            : "v"(x));
    return r;
}

#define ORCH_TOL_PARAMS                                                                                           \
    const uint64_t *__restrict__ csorted, const int32_t *__restrict__ sorted, const int32_t *__restrict__ lengths, \
        int32_t n, int32_t D, uint64_t window, uint64_t a, uint64_t b, int32_t *ipos, int32_t *inst,              \
        int32_t *rank, int32_t *start, uint64_t *loads, int32_t *seq_off, int64_t *tok_off,                       \
        int32_t *cu_seqlens, const int32_t *flags, int32_t *dev_status

// the choosing wavefront, general form
template <int K>
__device__ __forceinline__ void tolerance_choose64(const uint64_t *__restrict__ csorted, int32_t n, int32_t D,
                                                   uint64_t window, uint64_t a, uint64_t b, int32_t *ipos,
                                                   uint64_t *loads, int32_t *dev_status, int *progress, int lane)
{
    // lane l owns instances l*K .. l*K+K-1; slots past D never enter a window
    uint64_t sum[K], sq[K];
#pragma unroll
    for (int k = 0; k < K; ++k) { sum[k] = (lane * K + k < D) ? 0ull : ~0ull; sq[k] = 0; }
    int err = 0;
    ChoiceLog log{ipos, progress, 0};
    uint64_t c_cur = lane < n ? csorted[lane] : 0;
    int chunk = 0;
    for (int64_t t0 = 0; t0 < n; t0 += 64, ++chunk) {
        const uint64_t c_nxt = (t0 + 64 + lane < n) ? csorted[t0 + 64 + lane] : 0;
        const int m = (int)min((int64_t)64, (int64_t)n - t0);
        for (int j = 0; j < m; ++j) {
            const uint64_t c = readlane_u64(c_cur, j);  // the length
            uint64_t lm = sum[0];
#pragma unroll
            for (int k = 1; k < K; ++k) lm = sum[k] < lm ? sum[k] : lm;
            const uint64_t least = wave_min_u64(lm);
            uint64_t lq = ~0ull;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const bool in = sum[k] != ~0ull && sum[k] - least < window;
                lq = (in && sq[k] < lq) ? sq[k] : lq;
            }
            const uint64_t q = wave_min_u64(lq);  // < 2^63: some real instance holds `least`
            const uint64_t ball = __ballot(lq == q);
            const int win = __ffsll((unsigned long long)ball) - 1;
            int kk = K - 1;
#pragma unroll
            for (int k = K - 2; k >= 0; --k)
                kk = (sum[k] != ~0ull && sum[k] - least < window && sq[k] == q) ? k : kk;
            if (lane == win) {
#pragma unroll
                for (int k = 0; k < K; ++k)
                    if (k == kk) {
                        sum[k] += c;
                        sq[k] += c * c;
                        if (sq[k] >> 63) { err = 1; sq[k] = 0; }
                    }
            }
            log_choice(log, lane, j, __builtin_amdgcn_readlane(lane * K + kk, win));
        }
        publish_chunk(log, t0, n, lane, chunk);
        c_cur = c_nxt;
    }
    // Eq. 2, no-padding branch per instance: a * sum of squares + b * length sum
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (lane * K + k < D) {
            const uint64_t t1 = a * sq[k], t2 = b * sum[k], load = t1 + t2;
            if (__umul64hi(a, sq[k]) != 0 || __umul64hi(b, sum[k]) != 0 || load < t1 || (load >> 63)) err = 1;
            loads[lane * K + k] = load;
        }
    if (__any(err) && lane == 0) dev_status[0] = (int32_t)ORCH_EDATA;
}

// the choosing wavefront when all lengths together are < 2^32 and their squares together are
// sq_total < 2^62.  HALF: only lanes 0..31 call it (and are the active ones throughout).
template <int K, bool HALF>
__device__ __forceinline__ void tolerance_choose32(const uint64_t *__restrict__ csorted, int32_t n, int32_t D,
                                                   uint64_t window, uint64_t a, uint64_t b, uint64_t sq_total,
                                                   int32_t *ipos, uint64_t *loads, int32_t *dev_status,
                                                   int *progress, int lane)
{
    static_assert(!HALF || K == 1, "32 lanes hold one instance each");
    constexpr int W = HALF ? 32 : 64;   // lanes at work = steps per published chunk
    const uint32_t win32 = window > 0xffffffffull ? 0xffffffffu : (uint32_t)window;
    // leading bits of a sum of squares: (sq >> shift) < 2^31 for every sq <= sq_total
    const int bits = 64 - __clzll((unsigned long long)(sq_total | 1));
    const uint32_t shift = bits > 31 ? (uint32_t)(bits - 31) : 0u;   // <= 31
    // slots past D: every bit of the length sum, the squares and their leading bits set, so they
    // never hold the smallest sum and never equal the smallest leading bits inside the window
    uint32_t sum[K], top[K];
    uint64_t sq[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const bool real = lane * K + k < D;
        sum[k] = real ? 0u : 0xffffffffu;
        top[k] = real ? 0u : 0xffffffffu;
        sq[k] = real ? 0ull : ~0ull;
    }
    uint32_t least = 0;   // smallest length sum, in every lane
    const uint64_t all_lanes = __builtin_amdgcn_read_exec();
    ChoiceLog log{ipos, progress, 0};
    uint32_t c_cur = lane < n ? (uint32_t)csorted[lane] : 0;
    for (int64_t t0 = 0; t0 < n; t0 += W) {
        const uint32_t c_nxt = (t0 + W + lane < n) ? (uint32_t)csorted[t0 + W + lane] : 0;
        const int m = (int)min((int64_t)W, (int64_t)n - t0);
        for (int j = 0; j < m; ++j) {
            const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)c_cur, j);  // the length
            // leading bits of this lane's smallest squares inside the window (2^32 - 1: none inside)
            uint32_t kx[K];
            uint32_t key = 0xffffffffu;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                kx[k] = (sum[k] - least < win32) ? top[k] : 0xffffffffu;
                key = kx[k] < key ? kx[k] : key;
            }
            const uint32_t kmin = lanes_min_u32<HALF>(key);   // < 2^31: the holder of `least` is inside
            uint64_t ball = __builtin_amdgcn_ballot_w64(key == kmin);
            bool unique = __builtin_popcountll(ball) == 1;
            if (K > 1 && unique) {   // one lane; one slot of it?
                int hits = 0;
#pragma unroll
                for (int k = 0; k < K; ++k) hits += kx[k] == kmin ? 1 : 0;
                unique = __builtin_amdgcn_ballot_w64(hits > 1) == 0;
            }
            int win = __builtin_ctzll(ball), kk = 0;
            if (K > 1) {
#pragma unroll
                for (int k = K - 1; k >= 0; --k) kk = kx[k] == kmin ? k : kk;
            }
            if (__builtin_expect(!unique, 0)) {
                // several candidates agree in the leading bits: the exact comparison among them,
                // lowest instance on ties (high words, then low words among the lanes that hold the
                // smallest high word)
                uint64_t lq = ~0ull;
#pragma unroll
                for (int k = 0; k < K; ++k) lq = (kx[k] == kmin && sq[k] < lq) ? sq[k] : lq;
                const uint32_t lh = (uint32_t)(lq >> 32), ll = (uint32_t)lq;
                const uint32_t qh = lanes_min_u32<HALF>(lh);
                const uint32_t ql = lanes_min_u32<HALF>(lh == qh ? ll : 0xffffffffu);
                ball = __builtin_amdgcn_ballot_w64(lh == qh && ll == ql);
                win = __builtin_ctzll(ball);
                ball = 1ull << win;
                if (K > 1) {
#pragma unroll
                    for (int k = K - 1; k >= 0; --k) kk = (kx[k] == kmin && sq[k] == lq) ? k : kk;
                }
            }
            if (K > 1) kk = __builtin_amdgcn_readlane(kk, win);
            // the winner's update; did it hold the smallest sum?  exec = the winner's lane for three
            // instructions (restored before the statement ends); the slot is uniform
            uint64_t was_least = 0;
#pragma unroll
            for (int k = 0; k < K; ++k)
                if (K == 1 || kk == k) {
                    uint64_t carry;
                    asm volatile(
                        "s_mov_b64 exec, %[m]\n\t"
                        "v_cmp_eq_u32_e64 %[wl], %[sum], %[least]\n\t"
                        "v_add_u32_e32 %[sum], %[c], %[sum]\n\t"
                        "v_mad_u64_u32 %[sq], %[cy], %[c], %[c], %[sq]\n\t"
                        "s_mov_b64 exec, %[all]"
                        : [sum] "+v"(sum[k]), [sq] "+v"(sq[k]), [wl] "=&s"(was_least), [cy] "=&s"(carry)
                        : [m] "s"(ball), [c] "s"(c), [least] "v"(least), [all] "s"(all_lanes));
                    top[k] = __builtin_amdgcn_alignbit((uint32_t)(sq[k] >> 32), (uint32_t)sq[k], shift);
                }
            if (__builtin_expect(was_least != 0, 0)) {
                uint32_t lm = sum[0];
#pragma unroll
                for (int k = 1; k < K; ++k) lm = sum[k] < lm ? sum[k] : lm;
                least = lanes_min_u32<HALF>(lm);
            }
            log_choice(log, lane, j, win * K + kk);
        }
        if (t0 + lane < n) ipos[t0 + lane] = log.rec;
        publish_upto(progress, min((int64_t)n, t0 + W));
        c_cur = c_nxt;
    }
    // Eq. 2, no-padding branch per instance (the squares cannot pass 2^62 here)
    int err = 0;
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (lane * K + k < D) {
            const uint64_t t1 = a * sq[k], t2 = b * (uint64_t)sum[k], load = t1 + t2;
            if (__umul64hi(a, sq[k]) != 0 || __umul64hi(b, (uint64_t)sum[k]) != 0 || load < t1 || (load >> 63)) err = 1;
            loads[lane * K + k] = load;
        }
    if (__any(err) && lane == 0) dev_status[0] = (int32_t)ORCH_EDATA;
}

// HALF: K == 1 and D <= 32 (the instances sit in lanes 0..31)
template <int K, bool HALF>
__global__ __launch_bounds__(kGreedyThreads) void greedy_tolerance_kernel(ORCH_TOL_PARAMS)
{
    __shared__ uint32_t s_cnt[64 * K];
    __shared__ unsigned long long s_tok[64 * K];
    __shared__ unsigned long long s_sq[kGreedyThreads / 64];
    __shared__ int s_progress, s_booked;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    for (int i = threadIdx.x; i < 64 * K; i += kGreedyThreads) { s_cnt[i] = 0; s_tok[i] = 0; }
    if (threadIdx.x == 0) { s_progress = 0; s_booked = 0; }
    // flags[1]: all lengths together < 2^32.  The keys are the lengths, longest first: with the
    // longest < 2^30 the squares of all sequences together are < 2^62 and summed here.
    const bool narrow = flags[1] != 0 && n > 0 && csorted[0] < (1ull << 30);
    if (narrow) {
        uint64_t part = 0;
        for (int64_t i = threadIdx.x; i < n; i += kGreedyThreads) { const uint64_t c = csorted[i]; part += c * c; }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o);
        if (lane == 0) s_sq[wave] = part;
    }
    __syncthreads();
    if (wave >= 1) {
        bookkeep_wave(ipos, sorted, lengths, n, D, lane, wave - 1, BookState{&s_progress, &s_booked, s_cnt, s_tok},
                      inst, rank, start, dev_status);
    } else if (narrow) {
        uint64_t sq_total = 0;
        for (int w = 0; w < kGreedyThreads / 64; ++w) sq_total += s_sq[w];
        if (!HALF || lane < 32)
            tolerance_choose32<K, HALF>(csorted, n, D, window, a, b, sq_total, ipos, loads, dev_status, &s_progress, lane);
    } else {
        tolerance_choose64<K>(csorted, n, D, window, a, b, ipos, loads, dev_status, &s_progress, lane);
    }
    __syncthreads();
    if (wave == 0) finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
}
#undef ORCH_TOL_PARAMS

// ---------------------------------------------------------------------------
// Algorithm 2 (Sec. 5.1, balancing for batches with paddings)
// ---------------------------------------------------------------------------
// The sequences arrive sorted ascending by length.  For a bound b on the padded
// batch length (count * longest), the algorithm's batch-counting helper cuts the list greedily: a batch
// that starts at position p always takes p and then extends while
// (q - p + 1) * len[q] <= b.  That product never decreases with q, so the end of a
// batch is found by bisection instead of a walk, and one evaluation of the bound
// costs at most (D + 1) bisections.  The number of batches never grows with b, so
// the smallest b that needs at most D batches is well defined; the listing finds it
// by binary search, here 1024 candidate bounds are tried per round (one per thread),
// which reaches the same value in log_1025 instead of log_2 of the range rounds.
constexpr int kPadThreads = 1024;
constexpr int kPadLdsKeys = 32768;  // sorted lengths kept in LDS up to this n

template <bool LDS>
struct SortedLen {
    const uint32_t *lds;
    const uint64_t *glob;
    __device__ __forceinline__ uint64_t operator()(int t) const { return LDS ? (uint64_t)lds[t] : glob[t]; }
};

// Last position of the batch that starts at p under bound b.  A batch never holds more
// sequences than the one before it (if it held k + 1, then (k + 1) * len[p + k] <= b, but the
// previous batch of k stopped because (k + 1) * (a length no longer than that) > b), so the
// answer lies in [p, p + kprev - 1] and usually at its top: probe there first, then gallop
// down, then bisect what is left.  kprev = n for the first batch (plain bisection).
template <bool LDS>
__device__ __forceinline__ int batch_end(const SortedLen<LDS> &len, int p, int n, uint64_t b, int kprev)
{
    int lo = p, hi = n - 1;
    if (kprev < n) {
        hi = min(hi, p + kprev - 1);
        if (hi == p || (uint64_t)(hi - p + 1) * len(hi) <= b) return hi;
        int rej = hi;  // rejected
        for (int step = 1;; step <<= 1) {
            const int q = rej - step;
            if (q <= p) break;
            if ((uint64_t)(q - p + 1) * len(q) <= b) { lo = q; break; }
            rej = q;
        }
        hi = rej - 1;
    }
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((uint64_t)(mid - p + 1) * len(mid) <= b) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

template <bool LDS>
__device__ __forceinline__ bool at_most_D_batches(const SortedLen<LDS> &len, int n, int D, uint64_t b)
{
    int p = 0, cnt = 0, k = n;
    while (p < n) {
        if (++cnt > D) return false;
        const int e = batch_end(len, p, n, b, k);
        k = e - p + 1;
        p = e + 1;
    }
    return true;
}

template <bool LDS>
__global__ __launch_bounds__(kPadThreads) void padded_split_kernel(
    const uint64_t *__restrict__ csorted, const int32_t *__restrict__ sorted, int32_t n, int32_t D,
    uint64_t a, uint64_t b, int32_t *inst, int32_t *order, int32_t *seq_off, int64_t *tok_off,
    int32_t *cu_seqlens, uint64_t *loads, unsigned long long *bound_out, int32_t *dev_status)
{
    __shared__ uint32_t s_len[LDS ? kPadLdsKeys : 1];
    __shared__ int32_t s_bstart[kMaxInstances + 1];  // first sorted position of batch i; n past the last
    __shared__ unsigned long long s_scan[kPadThreads];
    __shared__ unsigned long long s_left, s_right;
    __shared__ int s_first, s_err;

    const int tid = threadIdx.x;
    if (LDS)
        for (int t = tid; t < n; t += kPadThreads) s_len[t] = (uint32_t)csorted[t];
    const SortedLen<LDS> len{s_len, csorted};
    if (tid == 0) {
        s_err = 0;
        // as printed: left = the shortest length; right = longest * (n / d + 1), which every
        // batch of floor(n/d) + 1 sequences satisfies, so it needs at most d batches
        s_left = n > 0 ? csorted[0] : 0;
        s_right = n > 0 ? csorted[n - 1] * ((uint64_t)(n / D) + 1) : 0;
    }
    __syncthreads();

    for (;;) {
        const uint64_t left = s_left, right = s_right;
        if (left >= right) break;
        const uint64_t span = right - left;
        const bool dense = span <= (uint64_t)kPadThreads;  // every remaining bound gets a thread
        const uint64_t step = span / (kPadThreads + 1);
        const uint64_t cand = dense ? left + tid : left + step * (uint64_t)(tid + 1);
        const bool valid = !dense || (uint64_t)tid < span;
        if (tid == 0) s_first = kPadThreads;
        __syncthreads();
        if (valid && at_most_D_batches(len, n, D, cand)) atomicMin(&s_first, tid);
        __syncthreads();
        if (tid == 0) {
            const int t = s_first;
            if (dense) {
                s_left = s_right = t < kPadThreads ? left + t : right;
            } else if (t < kPadThreads) {
                s_right = left + step * (uint64_t)(t + 1);
                if (t > 0) s_left = left + step * (uint64_t)t + 1;
            } else {
                s_left = left + step * (uint64_t)kPadThreads + 1;
            }
        }
        __syncthreads();
    }
    const uint64_t bound = s_left;

    // the batches at the final bound
    if (tid == 0) {
        int p = 0, k = 0, cnt = n;
        while (p < n && k < D) {
            s_bstart[k++] = p;
            const int e = batch_end(len, p, n, bound, cnt);
            cnt = e - p + 1;
            p = e + 1;
        }
        if (p < n) s_err = 1;  // cannot happen for a feasible bound; keeps every index in range
        for (; k <= D; ++k) s_bstart[k] = n;
        if (bound_out) bound_out[0] = bound;
    }
    __syncthreads();

    // per instance: count, longest, padded rows, Eq. 2 padding branch
    // a * L^2 / cnt + b * L with L = cnt * max  ==  cnt * (a * max^2 + b * max)
    const int per = (D + kPadThreads - 1) / kPadThreads;
    const int i0 = min(D, per * tid), i1 = min(D, i0 + per);
    unsigned long long rows_sum = 0;
    int err = 0;
    for (int i = i0; i < i1; ++i) {
        const int c = s_bstart[i + 1] - s_bstart[i];
        const uint64_t mx = c ? len(s_bstart[i + 1] - 1) : 0;
        const uint64_t rows = (uint64_t)c * mx;
        if (rows > 0x7fffffffull) err = 1;
        const uint64_t mx2 = mx * mx, t1 = a * mx2, t2 = b * mx, per_seq = t1 + t2;
        const uint64_t load = per_seq * (uint64_t)c;
        if (__umul64hi(a, mx2) != 0 || __umul64hi(b, mx) != 0 || per_seq < t1 ||
            __umul64hi(per_seq, (uint64_t)c) != 0 || (load >> 63))
            err = 1;
        loads[i] = load;
        seq_off[i] = s_bstart[i];
        cu_seqlens[s_bstart[i + 1] + i] = (int32_t)rows;  // the slice's last entry: cnt * max (0 when empty)
        rows_sum += rows;
    }
    s_scan[tid] = rows_sum;
    __syncthreads();
    for (int m = 1; m < kPadThreads; m <<= 1) {
        const unsigned long long o = tid >= m ? s_scan[tid - m] : 0;
        __syncthreads();
        s_scan[tid] += o;
        __syncthreads();
    }
    unsigned long long run = s_scan[tid] - rows_sum;
    for (int i = i0; i < i1; ++i) {
        tok_off[i] = (int64_t)run;
        const int c = s_bstart[i + 1] - s_bstart[i];
        run += (uint64_t)c * (c ? len(s_bstart[i + 1] - 1) : 0);
    }
    if (tid == kPadThreads - 1) {
        tok_off[D] = (int64_t)s_scan[tid];
        seq_off[D] = n;
    }
    if (err) atomicOr(&s_err, 1);

    // per sorted position: its batch (bisection over the batch starts), slot j * max
    for (int t = tid; t < n; t += kPadThreads) {
        int lo = 0, hi = D - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_bstart[mid] <= t) lo = mid;
            else hi = mid - 1;
        }
        const int i = lo;
        const int32_t s = sorted[t];
        const uint64_t mx = len(s_bstart[i + 1] - 1);
        inst[s] = i;
        order[t] = s;
        cu_seqlens[t + i] = (int32_t)((uint64_t)(t - s_bstart[i]) * mx);
    }
    __syncthreads();
    if (tid == 0 && s_err) dev_status[0] = (int32_t)ORCH_EDATA;
}

__global__ void layout_kernel(const int32_t *__restrict__ inst, const int32_t *__restrict__ rank,
                              const int32_t *__restrict__ start, const int32_t *__restrict__ seq_off,
                              int32_t n, int32_t *order, int32_t *cu_seqlens)
{
    const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    const int32_t i = inst[s];
    const int32_t p = seq_off[i] + rank[s];
    order[p] = (int32_t)s;
    cu_seqlens[p + i] = start[s];  // instance i's slice begins at seq_off[i] + i
}

}  // namespace

size_t balance_ws_bytes(int32_t n, int32_t D)
{
    (void)D;
    BalanceWs w;
    return carve(w, nullptr, n);
}

int launch_balance(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                   orch_assignment out, void *ws, size_t ws_bytes, hipStream_t stream, void *const *stage_events)
{
    BalanceWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_balance: workspace %zu < %zu bytes", ws_bytes, need);
    // optional: the caller's events, recorded before the sort, after it, after the greedy and
    // after the layout kernel (how the bench splits the call into its stages)
    auto mark = [&](int i) {
        if (stage_events && stage_events[i]) (void)hipEventRecord((hipEvent_t)stage_events[i], stream);
    };

    mark(0);
    hipLaunchKernelGGL(cost_sort_kernel, dim3(1), dim3(kSortThreads), 0, stream, lengths, n, phase.a,
                       phase.b, 0, w.csorted, w.keyA, w.keyB, w.idxA, w.idxB, w.sorted, w.flags, out.dev_status);
    mark(1);
#define ORCH_GREEDY_ARGS                                                                        \
    w.csorted, w.sorted, lengths, n, D, w.ipos, out.inst, w.rank, w.start, out.loads,           \
        out.seq_off, out.tok_off, out.cu_seqlens, w.flags, out.dev_status
    // the flag written by the sort kernel decides on the device which form of the greedy runs
#define ORCH_GREEDY_BOTH(K_) \
    hipLaunchKernelGGL(greedy_kernel<K_>, dim3(1), dim3(kGreedyThreads), 0, stream, ORCH_GREEDY_ARGS)
    if (D <= 64) ORCH_GREEDY_BOTH(1);
    else if (D <= 128) ORCH_GREEDY_BOTH(2);
    else if (D <= 256) ORCH_GREEDY_BOTH(4);
    else if (D <= 512) ORCH_GREEDY_BOTH(8);
    else if (D <= 1024) ORCH_GREEDY_BOTH(16);
    else hipLaunchKernelGGL(greedy_lds_kernel, dim3(1), dim3(kGreedyThreads), 0, stream, ORCH_GREEDY_ARGS);
#undef ORCH_GREEDY_BOTH
#undef ORCH_GREEDY_ARGS
    mark(2);
    if (n > 0)
        hipLaunchKernelGGL(layout_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, out.inst, w.rank,
                           w.start, out.seq_off, n, out.order, out.cu_seqlens);
    mark(3);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

// ---------------------------------------------------------------------------
// orch_balance_static: orch_balance with its workspace in a file-scope device
// array, for callers that cannot allocate (HIP graph capture, tight serving
// loops).  The array's name is only a host-side handle; its device address is
// looked up once per device and that address is what the kernels receive.
// ---------------------------------------------------------------------------
constexpr int32_t kStaticMaxN = 65536;
constexpr size_t kStaticBytes = (size_t)kStaticMaxN * 48 + 16 * 256;   // carve(kStaticMaxN) fits
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kStaticMaxDevices = 64;
static void *g_scratch_ptr[kStaticMaxDevices];   // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

int32_t balance_static_max_n() { return kStaticMaxN; }

int launch_balance_static(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                          orch_assignment out, hipStream_t stream)
{
    if (n > kStaticMaxN)
        ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_static: n = %d exceeds the built-in scratch (%d sequences)", n,
                  kStaticMaxN);
    int dev = -1;
    ORCH_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices)
        ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_static: device %d outside [0, %d)", dev, kStaticMaxDevices);
    void *ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            ORCH_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p) ORCH_FAIL(ORCH_EHIP, "orch_balance_static: no device address for the scratch array");
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    BalanceWs w;
    if (carve(w, nullptr, n) > kStaticBytes)
        ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_static: n = %d needs more than %zu bytes", n, kStaticBytes);
    // every word of the workspace that a kernel reads was written earlier in the same call
    // (the sort kernel writes flags, keys and order; the greedy writes ipos, rank and start
    // before the layout kernel reads them), so nothing has to be cleared between calls
    return launch_balance(lengths, n, D, phase, out, ptr, kStaticBytes, stream, nullptr);
}

int launch_balance_padded(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                          orch_assignment out, uint64_t *bound, void *ws, size_t ws_bytes,
                          hipStream_t stream)
{
    BalanceWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_balance_padded: workspace %zu < %zu bytes", ws_bytes, need);
    // Algorithm 2 sorts by length: key = 0 * l^2 + 1 * l, ascending, ties by index
    hipLaunchKernelGGL(cost_sort_kernel, dim3(1), dim3(kSortThreads), 0, stream, lengths, n, (uint64_t)0,
                       (uint64_t)1, 1, w.csorted, w.keyA, w.keyB, w.idxA, w.idxB, w.sorted, w.flags,
                       out.dev_status);
    if (n <= kPadLdsKeys)
        hipLaunchKernelGGL(padded_split_kernel<true>, dim3(1), dim3(kPadThreads), 0, stream, w.csorted,
                           w.sorted, n, D, phase.a, phase.b, out.inst, out.order, out.seq_off, out.tok_off,
                           out.cu_seqlens, out.loads, (unsigned long long *)bound, out.dev_status);
    else
        hipLaunchKernelGGL(padded_split_kernel<false>, dim3(1), dim3(kPadThreads), 0, stream, w.csorted,
                           w.sorted, n, D, phase.a, phase.b, out.inst, out.order, out.seq_off, out.tok_off,
                           out.cu_seqlens, out.loads, (unsigned long long *)bound, out.dev_status);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

int launch_balance_tolerance(const int32_t *lengths, int32_t n, int32_t D, uint64_t v, orch_phase phase,
                             orch_assignment out, void *ws, size_t ws_bytes, hipStream_t stream)
{
    BalanceWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_balance_tolerance: workspace %zu < %zu bytes", ws_bytes, need);
    // sorted by length, descending, ties by index: key = 0 * l^2 + 1 * l
    hipLaunchKernelGGL(cost_sort_kernel, dim3(1), dim3(kSortThreads), 0, stream, lengths, n, (uint64_t)0,
                       (uint64_t)1, 0, w.csorted, w.keyA, w.keyB, w.idxA, w.idxB, w.sorted, w.flags,
                       out.dev_status);
    const uint64_t window = v > 1 ? v : 1;
    // one launch; the flag written by the sort kernel decides on the device which form runs
#define ORCH_TOL(K_, HALF_)                                                                                 \
    hipLaunchKernelGGL((greedy_tolerance_kernel<K_, HALF_>), dim3(1), dim3(kGreedyThreads), 0, stream,      \
                       w.csorted, w.sorted, lengths, n, D, window, phase.a, phase.b, w.ipos, out.inst,     \
                       w.rank, w.start, out.loads, out.seq_off, out.tok_off, out.cu_seqlens, w.flags,      \
                       out.dev_status)
    if (D <= 32) ORCH_TOL(1, true);
    else if (D <= 64) ORCH_TOL(1, false);
    else if (D <= 128) ORCH_TOL(2, false);
    else if (D <= 256) ORCH_TOL(4, false);
    else if (D <= 512) ORCH_TOL(8, false);
    else if (D <= 1024) ORCH_TOL(16, false);
    else ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_tolerance: D = %d > 1024", D);
#undef ORCH_TOL
    if (n > 0)
        hipLaunchKernelGGL(layout_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, out.inst, w.rank,
                           w.start, out.seq_off, n, out.order, out.cu_seqlens);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
