// orch_balance: Eq. 2's per-sequence cost, Algorithm 1 (sort descending, then
// longest-first greedy onto the least-loaded instance) and the packed layout.
// (OrchMLLM Sec. 5.1; layout per Sec. 7 "batched along the sequence length".)
//
// Three launches on the caller's stream:
//   cost_sort_kernel   one 1024-thread workgroup: cost keys, then a stable LSD
//                      radix sort (8-bit digits, only as many passes as the
//                      largest key needs) of (~cost, index) pairs
//   greedy_*_kernel    one wavefront: the n-step serial loop; each step is a
//                      64-lane min-reduction over the instance loads with
//                      lowest-index tie-break
//   layout_kernel      n threads: scatter sequence ids and segment starts
// n <= 32768 keys is latency-bound work, so everything is arranged to keep the
// dependent chain short rather than to stream memory.
#include "common.h"

namespace orch {
namespace {

constexpr int kSortThreads = 1024;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kRadix = 256;

struct BalanceWs {
    uint64_t *cost, *keyA, *keyB;
    uint32_t *idxA, *idxB;
    int32_t *sorted, *rank, *start;
};

size_t carve(BalanceWs &w, void *ws, int32_t n)
{
    size_t nn = align_up((size_t)(n > 0 ? n : 1), 64);
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.cost = (uint64_t *)take(nn * 8);
    w.keyA = (uint64_t *)take(nn * 8);
    w.keyB = (uint64_t *)take(nn * 8);
    w.idxA = (uint32_t *)take(nn * 4);
    w.idxB = (uint32_t *)take(nn * 4);
    w.sorted = (int32_t *)take(nn * 4);
    w.rank = (int32_t *)take(nn * 4);
    w.start = (int32_t *)take(nn * 4);
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
    const int32_t *__restrict__ lengths, int32_t n, uint64_t a, uint64_t b, uint64_t *cost,
    uint64_t *keyA, uint64_t *keyB, uint32_t *idxA, uint32_t *idxB, int32_t *sorted,
    int32_t *dev_status)
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
        cost[i] = c;
        keyA[i] = ~c;  // ascending on ~c == descending on c
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
    for (int64_t i = tid; i < n; i += kSortThreads) sorted[i] = (int32_t)isrc[i];
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

__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int j)
{
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, j);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), j);
    return ((uint64_t)hi << 32) | lo;
}

// Closing work shared by both greedy kernels: instance i's sequence count and
// token total become seq_off / tok_off and the last cu_seqlens entry.
// `per` consecutive instances per lane, held in LDS arrays.
__device__ void finish_layout(const uint32_t *cnt, const uint64_t *tok, int D, int32_t *seq_off,
                              int64_t *tok_off, int32_t *cu_seqlens, int32_t *dev_status)
{
    const int lane = threadIdx.x;
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
// Algorithm 1, lines 2-7: one wavefront, instance loads in registers.
// Lane l owns instances l*K .. l*K+K-1, so "lowest lane, then lowest k" is the
// lowest instance index among equal loads.
// ---------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(64) void greedy_reg_kernel(
    const uint64_t *__restrict__ cost, const int32_t *__restrict__ sorted,
    const int32_t *__restrict__ lengths, int32_t n, int32_t D, int32_t *inst, int32_t *rank,
    int32_t *start, uint64_t *loads, int32_t *seq_off, int64_t *tok_off, int32_t *cu_seqlens,
    int32_t *dev_status)
{
    __shared__ uint32_t s_cnt[64 * K];
    __shared__ uint64_t s_tok[64 * K];
    const int lane = threadIdx.x;
    uint64_t load[K], tok[K];
    uint32_t cnt[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        load[k] = (lane * K + k < D) ? 0ull : ~0ull;
        tok[k] = 0;
        cnt[k] = 0;
    }
    int32_t s_cur = 0, l_cur = 0;
    uint64_t c_cur = 0;
    if (lane < n) { s_cur = sorted[lane]; c_cur = cost[s_cur]; l_cur = lengths[s_cur]; }
    for (int64_t t0 = 0; t0 < n; t0 += 64) {
        int32_t s_nxt = 0, l_nxt = 0;
        uint64_t c_nxt = 0;
        if (t0 + 64 + lane < n) {
            s_nxt = sorted[t0 + 64 + lane];
            c_nxt = cost[s_nxt];
            l_nxt = lengths[s_nxt];
        }
        const int m = (int)min((int64_t)64, (int64_t)n - t0);
        for (int j = 0; j < m; ++j) {
            const uint64_t c = readlane_u64(c_cur, j);
            const int32_t s = __builtin_amdgcn_readlane(s_cur, j);
            const int32_t l = __builtin_amdgcn_readlane(l_cur, j);
            uint64_t lm = load[0];
#pragma unroll
            for (int k = 1; k < K; ++k) lm = load[k] < lm ? load[k] : lm;
            const uint64_t g = wave_min_u64(lm);
            const uint64_t ball = __ballot(lm == g);
            const int win = __ffsll((unsigned long long)ball) - 1;
            if (lane == win) {
                int kk = K - 1;
#pragma unroll
                for (int k = K - 2; k >= 0; --k) kk = (load[k] == g) ? k : kk;
                uint32_t r = 0;
                uint64_t st = 0;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    if (k == kk) {
                        r = cnt[k];
                        st = tok[k];
                        load[k] += c;
                        cnt[k] += 1;
                        tok[k] += (uint64_t)(int64_t)l;
                    }
                }
                inst[s] = lane * K + kk;
                rank[s] = (int32_t)r;
                start[s] = (int32_t)st;
            }
        }
        s_cur = s_nxt; c_cur = c_nxt; l_cur = l_nxt;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int i = lane * K + k;
        s_cnt[i] = cnt[k];
        s_tok[i] = tok[k];
        if (i < D) loads[i] = load[k];
    }
    __syncthreads();
    finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
}

// Same loop for D beyond what registers hold: per-instance state in LDS,
// instance i lives at lane i%64, slot i/64.  Two reductions per step: the
// minimal load, then the minimal instance index among lanes that hold it.
constexpr int kMaxInstances = 4096;

__global__ __launch_bounds__(64) void greedy_lds_kernel(
    const uint64_t *__restrict__ cost, const int32_t *__restrict__ sorted,
    const int32_t *__restrict__ lengths, int32_t n, int32_t D, int32_t *inst, int32_t *rank,
    int32_t *start, uint64_t *loads, int32_t *seq_off, int64_t *tok_off, int32_t *cu_seqlens,
    int32_t *dev_status)
{
    __shared__ uint64_t s_load[kMaxInstances];
    __shared__ uint64_t s_tok[kMaxInstances];
    __shared__ uint32_t s_cnt[kMaxInstances];
    const int lane = threadIdx.x;
    const int K = (D + 63) / 64;
    for (int i = lane; i < K * 64; i += 64) {
        s_load[i] = i < D ? 0ull : ~0ull;
        s_tok[i] = 0;
        s_cnt[i] = 0;
    }
    __syncthreads();
    for (int64_t t0 = 0; t0 < n; t0 += 64) {
        int32_t s_cur = 0, l_cur = 0;
        uint64_t c_cur = 0;
        if (t0 + lane < n) { s_cur = sorted[t0 + lane]; c_cur = cost[s_cur]; l_cur = lengths[s_cur]; }
        const int m = (int)min((int64_t)64, (int64_t)n - t0);
        for (int j = 0; j < m; ++j) {
            const uint64_t c = readlane_u64(c_cur, j);
            const int32_t s = __builtin_amdgcn_readlane(s_cur, j);
            const int32_t l = __builtin_amdgcn_readlane(l_cur, j);
            uint64_t lm = ~0ull;
            uint32_t li = 0xffffffffu;
            for (int k = 0; k < K; ++k) {
                const uint64_t v = s_load[k * 64 + lane];
                if (v < lm) { lm = v; li = (uint32_t)(k * 64 + lane); }
            }
            const uint64_t g = wave_min_u64(lm);
            const uint64_t cand = (lm == g) ? (uint64_t)li : ~0ull;
            const uint32_t bi = (uint32_t)wave_min_u64(cand);
            if (lane == (int)(bi & 63u)) {
                inst[s] = (int32_t)bi;
                rank[s] = (int32_t)s_cnt[bi];
                start[s] = (int32_t)s_tok[bi];
                s_load[bi] += c;
                s_cnt[bi] += 1;
                s_tok[bi] += (uint64_t)(int64_t)l;
            }
            __syncthreads();  // single wave: orders the LDS update before the next scan
        }
    }
    for (int i = lane; i < D; i += 64) loads[i] = s_load[i];
    __syncthreads();
    finish_layout(s_cnt, s_tok, D, seq_off, tok_off, cu_seqlens, dev_status);
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
                   orch_assignment out, void *ws, size_t ws_bytes, hipStream_t stream)
{
    BalanceWs w;
    size_t need = carve(w, ws, n);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_balance: workspace %zu < %zu bytes", ws_bytes, need);

    hipLaunchKernelGGL(cost_sort_kernel, dim3(1), dim3(kSortThreads), 0, stream, lengths, n, phase.a,
                       phase.b, w.cost, w.keyA, w.keyB, w.idxA, w.idxB, w.sorted, out.dev_status);
#define ORCH_GREEDY_ARGS                                                                        \
    w.cost, w.sorted, lengths, n, D, out.inst, w.rank, w.start, out.loads, out.seq_off,         \
        out.tok_off, out.cu_seqlens, out.dev_status
    if (D <= 64) hipLaunchKernelGGL(greedy_reg_kernel<1>, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
    else if (D <= 128) hipLaunchKernelGGL(greedy_reg_kernel<2>, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
    else if (D <= 256) hipLaunchKernelGGL(greedy_reg_kernel<4>, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
    else if (D <= 512) hipLaunchKernelGGL(greedy_reg_kernel<8>, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
    else if (D <= 1024) hipLaunchKernelGGL(greedy_reg_kernel<16>, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
    else hipLaunchKernelGGL(greedy_lds_kernel, dim3(1), dim3(64), 0, stream, ORCH_GREEDY_ARGS);
#undef ORCH_GREEDY_ARGS
    if (n > 0)
        hipLaunchKernelGGL(layout_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, out.inst, w.rank,
                           w.start, out.seq_off, n, out.order, out.cu_seqlens);
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
