// orch_varlen_attn_bwd: backward of the padding-free attention (the back-propagation that
// mirrors the forward pass, OrchMLLM Sec. 5.3; the operator itself is the one of Sec. 7).
//
//   p_ij = exp(scale * q_i.k_j - lse_i)         dp_ij = dout_i . v_j
//   delta_i = dout_i . out_i  (= sum_j p_ij dp_ij)      ds_ij = p_ij (dp_ij - delta_i)
//   dq_i = scale * sum_j ds_ij k_j     dk_j = scale * sum_i ds_ij q_i     dv_j = sum_i p_ij dout_i
//
// Two or three launches after the tile table, no atomics, so the result is deterministic:
//   attn_bwd_dq_kernel     query-stationary, shaped like the forward kernel: a workgroup of 4
//                          wavefronts owns 128 query rows of one q-head, streams K/V tiles of
//                          64 keys through LDS, recomputes the transposed scores
//                          S^T = K Q^T and dP^T = V dout^T (a lane holds 16 keys of ONE query,
//                          so lse and delta are per-lane scalars), and accumulates
//                          dQ^T += K^T dS^T.  It also computes delta[h, i] (fp32) for its rows
//                          from the dout fragments it holds and writes it for the kernels below.
//   dK, dV                 key-stationary: a workgroup owns 128 keys of one kv-head (32 per
//                          wavefront, K or V fragments live in registers), loops over the q-heads
//                          of the group and over 64-row tiles of Q and dout, computes S = Q K^T
//                          and dP = dout V^T (a lane holds 16 queries of ONE key, which is the
//                          B-operand layout for contractions over queries) and accumulates
//                          dV^T += dout^T P and dK^T += Q^T dS.
//                          head_dim 128: attn_bwd_dkv_fused_kernel, 8 wavefronts, S computed once:
//                          four wavefronts make P and dV, four take P through LDS and make dK.
//                          head_dim 64: attn_bwd_dkv_kernel, launched once for dK and once for dV.
// The transposed A operands (K^T, Q^T, dout^T) are read with ds_read_b64_tr_b16 from the same
// row-major LDS tile that serves the first products; the tiles get into LDS by LDS-DMA (PairStage).
// Every product is v_mfma_f32_32x32x16_bf16 with fp32 accumulation; P and dS are rounded to
// bf16 before the second products, as P is in the forward pass.
#include <algorithm>
#include <type_traits>

#include "attn_tiles.h"
#include "common.h"

namespace orch {
namespace {

constexpr int kFragAhead = 1;   // LDS fragment reads run this many MFMAs ahead of their use
constexpr int kOwn = 128;       // rows a workgroup owns (queries for dq, keys for dk/dv)
constexpr int kPrepThreads = 1024;
constexpr float kLog2e = 1.4426950408889634f;

struct BwdHdr {
    int32_t total_tiles;
    int32_t ok;
};

// tile_off[t] = number of 128-row tiles in sequences before t; validates cu_seqlens (not
// non-decreasing inside [0, total_tokens], or a sequence longer than a nonzero max_seqlen: no
// tile is scheduled and dev_status, if given, receives ORCH_EDATA).
__global__ __launch_bounds__(kPrepThreads) void bwd_prep_kernel(const int32_t *__restrict__ cu, int32_t batch,
                                                               int32_t total_tokens, int32_t max_seqlen,
                                                               BwdHdr *hdr, int32_t *tile_off, int32_t *dev_status)
{
    __shared__ int32_t part[kPrepThreads];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    const int per = (batch + kPrepThreads - 1) / kPrepThreads;
    const int b0 = min(batch, per * tid), b1 = min(batch, b0 + per);
    int32_t sum = 0;
    int bad = 0;
    for (int t = b0; t < b1; ++t) {
        const int32_t lo = cu[t], hi = cu[t + 1];
        if (lo < 0 || hi < lo || hi > total_tokens || (max_seqlen > 0 && hi - lo > max_seqlen)) { bad = 1; continue; }
        sum += (hi - lo + kOwn - 1) / kOwn;
    }
    if (bad) atomicOr(&s_bad, 1);
    part[tid] = sum;
    __syncthreads();
    for (int m = 1; m < kPrepThreads; m <<= 1) {
        int32_t o = tid >= m ? part[tid - m] : 0;
        __syncthreads();
        part[tid] += o;
        __syncthreads();
    }
    int32_t run = part[tid] - sum;
    if (!s_bad)
        for (int t = b0; t < b1; ++t) {
            tile_off[t] = run;
            run += (cu[t + 1] - cu[t] + kOwn - 1) / kOwn;
        }
    if (tid == 0) {
        const int ok = !s_bad;
        hdr->ok = ok;
        hdr->total_tiles = ok ? part[kPrepThreads - 1] : 0;
        if (ok) tile_off[batch] = part[kPrepThreads - 1];
        if (dev_status) dev_status[0] = ok ? (int32_t)ORCH_OK : (int32_t)ORCH_EDATA;
    }
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// block -> (tile u, head).  With the kv-head count a multiple of 8 the kv-head is chosen by
// blockIdx % 8, i.e. by XCD, so the workgroups that stream the same rows share an L2.
__device__ __forceinline__ void block_to_tile(int bid, int heads, int Hkv, int group_of_heads, int &u, int &h)
{
    if ((Hkv & 7) == 0) {
        const int kvh = (bid & 7) + 8 * ((bid >> 3) % (Hkv >> 3));
        const int rest = bid / Hkv;
        h = kvh * group_of_heads + rest % group_of_heads;
        u = rest / group_of_heads;
    } else {
        h = bid % heads;
        u = bid / heads;
    }
}

// ---------------------------------------------------------------------------
// dQ: query-stationary
// ---------------------------------------------------------------------------
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint16_t *__restrict__ dout, const float *__restrict__ lse, const uint16_t *__restrict__ out,
    float *__restrict__ delta, uint16_t *__restrict__ dq, const int32_t *__restrict__ cu, const BwdHdr *__restrict__ hdr,
    const int32_t *__restrict__ tile_off, int32_t batch, int32_t total_tokens, int32_t Hq, int32_t Hkv,
    float scale, float scale_log2)
{
    using PS = PairStage<HD>;
    constexpr int NC = HD / 16, NDB = HD / 32;
    __shared__ __attribute__((aligned(1024))) char lds_raw[PS::BYTES];

    const int total_tiles = hdr->total_tiles;
    const int group = Hq / Hkv;
    int u, h;
    block_to_tile(blockIdx.x, Hq, Hkv, group, u, h);
    if (u >= total_tiles) return;
    const int g_kv = h / group;
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tile_off[mid] <= u) lo = mid; else hi = mid - 1;
    }
    const int row0 = cu[lo];
    const int L = cu[lo + 1] - row0;
    const int ntile_q = (L + kOwn - 1) / kOwn;
    const int q0 = (ntile_q - 1 - (u - tile_off[lo])) * kOwn;  // heaviest (last) tile first

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int qm = q0 + 32 * wave + l32;
    const int qm_c = qm < L ? qm : L - 1;

    // stationary B operands (column = this lane's query) and the per-query scalars
    bf16x8 qf[NC], dof[NC];
    {
        const uint16_t *qp = q + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
        const uint16_t *dp = dout + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            qf[c] = *(const bf16x8 *)(qp + 16 * c);
            dof[c] = *(const bf16x8 *)(dp + 16 * c);
        }
    }
    const float lse2 = lse[(size_t)h * total_tokens + row0 + qm_c] * kLog2e;
    // delta of this lane's query row = dout . out over the head dimension: the lane holds dout at
    // columns 16 c + 8 g + [0..7], its partner (lane ^ 32) the other half.  Every (row, head) belongs
    // to exactly one lane pair of this launch, which also writes it for the dK / dV kernels.
    float dlt = 0.f;
    {
        const uint16_t *op = out + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const u32x4 a = __builtin_bit_cast(u32x4, dof[c]);
            const u32x4 b = *(const u32x4 *)(op + 16 * c);
            dlt += bf16_lo(a.x) * bf16_lo(b.x) + bf16_hi(a.x) * bf16_hi(b.x) + bf16_lo(a.y) * bf16_lo(b.y) +
                   bf16_hi(a.y) * bf16_hi(b.y) + bf16_lo(a.z) * bf16_lo(b.z) + bf16_hi(a.z) * bf16_hi(b.z) +
                   bf16_lo(a.w) * bf16_lo(b.w) + bf16_hi(a.w) * bf16_hi(b.w);
        }
        dlt += __shfl_xor(dlt, 32);
        if (g == 0 && qm < L) delta[(size_t)h * total_tokens + row0 + qm] = dlt;
    }

    f32x16 acc[NDB];
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    const int kend = CAUSAL ? min(L, q0 + kOwn) : L;
    const int ntile_k = (kend + kT - 1) / kT;

    PS ps;
    ps.init((uint32_t)(uintptr_t)lds_raw, lane, wave);
    TileSrc src{k, v, row0, L, 0, Hkv, g_kv};
    ps.begin(src, 0);
    // the next tile's loads go out between this tile's MFMAs, one every kSlots / NLOAD slots (a slot
    // is a pair of first-product MFMAs or one MFMA of the last product)
    using Plan = typename PS::Plan;
    constexpr int kSlots = 4 * NC;
    bool has_next = false;
    auto dma_slot = [&](const Plan &pl, int i) {
        constexpr int every = kSlots / PS::NLOAD;
        if (i % every == 1 && has_next) PS::issue(pl, i / every);
    };
    // tile `it` lives in stage it % 2; the loop is unrolled by the two stages so that the stage
    // offset of every fragment read is an immediate
    auto tile_step = [&](auto stage_tag, int it) {
        constexpr int ST = decltype(stage_tag)::value;
        const int n0 = it * kT;
        ps.publish();
        has_next = it + 1 < ntile_k;
        if (has_next) src.m0 = n0 + kT;
        const Plan pl = ps.plan(src, ST ^ 1);
        if (CAUSAL && n0 > q0 + 32 * wave + 31) {  // this wavefront's rows see none of the tile
            if (has_next) {
#pragma unroll
                for (int kq_ = 0; kq_ < PS::NLOAD; ++kq_) PS::issue(pl, kq_);
            }
            return;
        }
        const uint32_t kb = ps.x_at(ST), vb = ps.y_at(ST);

        // per 32-key block: S^T = K Q^T and dP^T = V dout^T, then dS^T = P^T (dP^T - delta),
        // rounded to bf16 in the B-operand layout.  Fragment reads run PF steps ahead of the MFMAs
        // that use them (explicitly: left alone the compiler reuses one pair of fragment registers
        // and every MFMA waits out a full LDS latency); the fences keep that order.
        const bool need_mask = (n0 + kT > L) || (CAUSAL && n0 + kT - 1 > q0 + 32 * wave);
        constexpr int PF = kFragAhead;
        bf16x8 dsf[4];
        bf16x8 kq[PF + 1], vq[PF + 1], tq[PF + 1];
#pragma unroll
        for (int i = 0; i < PF; ++i) { kq[i] = ps.rd_row(kb, 0, i); vq[i] = ps.rd_row(vb, 0, i); }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            f32x16 sa, da;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sa[e] = 0.f; da[e] = 0.f; }
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int sn = NC * nb + c + PF;  // the step fetched now
                if (sn < 2 * NC) {
                    kq[sn % (PF + 1)] = ps.rd_row(kb, sn / NC, sn % NC);
                    vq[sn % (PF + 1)] = ps.rd_row(vb, sn / NC, sn % NC);
                } else {
                    tq[(sn - 2 * NC) % (PF + 1)] = ps.rd_tr(kb, sn - 2 * NC);  // K^T, from the same K tile
                }
                __builtin_amdgcn_sched_barrier(0);
                sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kq[(NC * nb + c) % (PF + 1)], qf[c], sa, 0, 0, 0);
                da = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[(NC * nb + c) % (PF + 1)], dof[c], da, 0, 0, 0);
                dma_slot(pl, NC * nb + c);
                __builtin_amdgcn_sched_barrier(0);
            }
            float d16[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) d16[e] = __builtin_amdgcn_exp2f(sa[e] * scale_log2 - lse2) * (da[e] - dlt);
            if (need_mask) {   // one wave-uniform branch around all the selects
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int n = n0 + 32 * nb + 8 * (e >> 2) + 4 * g + (e & 3);
                    const bool vis = n < L && (!CAUSAL || n <= qm);
                    d16[e] = vis ? d16[e] : 0.f;
                }
            }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                u32x4 pk;
                pk.x = pack_bf16(d16[8 * half + 0], d16[8 * half + 1]);
                pk.y = pack_bf16(d16[8 * half + 2], d16[8 * half + 3]);
                pk.z = pack_bf16(d16[8 * half + 4], d16[8 * half + 5]);
                pk.w = pack_bf16(d16[8 * half + 6], d16[8 * half + 7]);
                dsf[2 * nb + half] = __builtin_bit_cast(bf16x8, pk);
            }
        }
        // dQ^T += K^T dS^T, step j = 4 b + kk: keys 16 kk .. + 15 of the tile, head-dim columns 32 b .. + 31
#pragma unroll
        for (int j = 0; j < 4 * NDB; ++j) {
            if (j + PF < 4 * NDB) tq[(j + PF) % (PF + 1)] = ps.rd_tr(kb, j + PF);
            __builtin_amdgcn_sched_barrier(0);
            acc[j >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[j % (PF + 1)], dsf[j & 3], acc[j >> 2], 0, 0, 0);
            dma_slot(pl, 2 * NC + j);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int it = 0; it < ntile_k; it += 2) {
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < ntile_k) tile_step(std::integral_constant<int, 1>{}, it + 1);
    }

    if (qm < L) {
        uint16_t *op = dq + ((size_t)(row0 + qm) * Hq + h) * HD;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x2 w;
                w.x = pack_bf16(acc[b][4 * r] * scale, acc[b][4 * r + 1] * scale);
                w.y = pack_bf16(acc[b][4 * r + 2] * scale, acc[b][4 * r + 3] * scale);
                *(u32x2 *)(op + 32 * b + 8 * r + 4 * g) = w;
            }
    }
}

// ---------------------------------------------------------------------------
// dK, dV: key-stationary.  One kernel body, instantiated once per output (PART): holding
// both accumulators needs more than 256 registers per lane, which leaves one wavefront per
// SIMD and nothing to hide LDS and barrier latency behind; each half fits in 256, so two
// workgroups share a CU, at the price of recomputing S for the second output.
//   PART_DV: S -> P,          dV^T += dout^T P
//   PART_DK: S, dP -> dS,     dK^T += Q^T dS
// Both stream the Q and dout tiles of the group's q-heads; the transposed operand of the last
// product is read from the same row-major tile (Q for dK, dout for dV).
// ---------------------------------------------------------------------------
constexpr int PART_DV = 1, PART_DK = 2;

template <int HD, bool CAUSAL, int PART>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dkv_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint16_t *__restrict__ dout, const float *__restrict__ lse, const float *__restrict__ delta,
    uint16_t *__restrict__ dkv, const int32_t *__restrict__ cu, const BwdHdr *__restrict__ hdr,
    const int32_t *__restrict__ tile_off, int32_t batch, int32_t total_tokens, int32_t Hq, int32_t Hkv,
    float scale, float scale_log2)
{
    constexpr bool DK = PART == PART_DK;
    using PS = PairStage<HD>;
    constexpr int NC = HD / 16, NDB = HD / 32;
    __shared__ __attribute__((aligned(1024))) char lds_raw[PS::BYTES];
    __shared__ __attribute__((aligned(16))) float s_lse[2][kT];  // lse * log2(e) of the tile's rows, by step parity
    __shared__ __attribute__((aligned(16))) float s_dlt[2][kT];

    const int total_tiles = hdr->total_tiles;
    const int group = Hq / Hkv;
    int u, g_kv;
    block_to_tile(blockIdx.x, Hkv, Hkv, 1, u, g_kv);
    if (u >= total_tiles) return;
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tile_off[mid] <= u) lo = mid; else hi = mid - 1;
    }
    const int row0 = cu[lo];
    const int L = cu[lo + 1] - row0;
    const int k0 = (u - tile_off[lo]) * kOwn;  // under a causal mask the first key tile is the heaviest

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int n0w = k0 + 32 * wave;     // this wavefront's keys
    const int kn = n0w + l32;           // this lane's key (a column of S)
    const int kn_c = kn < L ? kn : L - 1;

    // stationary B operands (column = this lane's key)
    bf16x8 kfs[NC], vfs[DK ? NC : 1];
    {
        const uint16_t *kp = k + ((size_t)(row0 + kn_c) * Hkv + g_kv) * HD + 8 * g;
        const uint16_t *vp = v + ((size_t)(row0 + kn_c) * Hkv + g_kv) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            kfs[c] = *(const bf16x8 *)(kp + 16 * c);
            if (DK) vfs[c] = *(const bf16x8 *)(vp + 16 * c);
        }
    }
    f32x16 acc[NDB];
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    const int m_begin = CAUSAL ? (k0 / kT) * kT : 0;  // rows before the first key see none of them
    const int ntile_m = m_begin < L ? (L - m_begin + kT - 1) / kT : 0;
    const int steps = ntile_m * group;

    PS ps;
    ps.init((uint32_t)(uintptr_t)lds_raw, lane, wave);
    TileSrc src{q, dout, row0, L, m_begin, Hq, g_kv * group};
    float r_lse = 0.f, r_dlt = 0.f;
    // step st covers head g_kv * group + st / ntile_m, rows m_begin + 64 (st % ntile_m) ..
    auto start_step = [&](int st, int stage) {
        src.hd = g_kv * group + st / ntile_m;
        src.m0 = m_begin + (st % ntile_m) * kT;
        ps.begin_at(src, stage);
        if (tid < kT) {
            int m = src.m0 + tid;
            m = m < L ? m : L - 1;
            r_lse = lse[(size_t)src.hd * total_tokens + row0 + m] * kLog2e;
            if (DK) r_dlt = delta[(size_t)src.hd * total_tokens + row0 + m];
        }
    };
    auto store_stats = [&](int stage) {
        if (tid < kT) { s_lse[stage][tid] = r_lse; s_dlt[stage][tid] = r_dlt; }
    };
    if (steps > 0) {
        start_step(0, 0);
        store_stats(0);
    }
    // step st lives in stage st % 2; the loop is unrolled by the two stages so that the stage
    // offset of every fragment read is an immediate
    auto do_step = [&](auto stage_tag, int st) {
        constexpr int ST = decltype(stage_tag)::value;
        const int m0 = m_begin + (st % ntile_m) * kT;
        ps.publish();
        if (st + 1 < steps) start_step(st + 1, ST ^ 1);
        // rows of the tile that lie before this wavefront's keys see none of them
        if (!(CAUSAL && m0 + kT - 1 < n0w)) {
            const uint32_t qb = ps.x_at(ST), ob = ps.y_at(ST);
            const uint32_t xb = DK ? qb : ob;
            const float *lse_s = s_lse[ST], *dlt_s = s_dlt[ST];
            // only tiles that touch the end of the sequence or the diagonal have masked elements
            const bool need_mask = m0 + kT > L || n0w + 32 > L || (CAUSAL && n0w + 31 > m0);
            // Fragment reads run PF steps ahead of the MFMAs that use them; the fences keep that order.
            constexpr int PF = kFragAhead;
            bf16x8 bf[4];  // P (dV) or dS (dK) of the tile's 64 rows, B-operand layout
            bf16x8 qq[PF + 1], oq[DK ? PF + 1 : 1], tq[PF + 1];
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                qq[i] = ps.rd_row(qb, 0, i);
                if (DK) oq[i] = ps.rd_row(ob, 0, i);
            }
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                // S = Q K^T (and dP = dout V^T) for 32 rows x this wavefront's 32 keys
                f32x16 sa, da;
#pragma unroll
                for (int e = 0; e < 16; ++e) { sa[e] = 0.f; da[e] = 0.f; }
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int sn = NC * mb + c + PF;  // the step fetched now
                    if (sn < 2 * NC) {
                        qq[sn % (PF + 1)] = ps.rd_row(qb, sn / NC, sn % NC);
                        if (DK) oq[sn % (PF + 1)] = ps.rd_row(ob, sn / NC, sn % NC);
                    } else {
                        tq[(sn - 2 * NC) % (PF + 1)] = ps.rd_tr(xb, sn - 2 * NC);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qq[(NC * mb + c) % (PF + 1)], kfs[c], sa, 0, 0, 0);
                    if (DK) da = __builtin_amdgcn_mfma_f32_32x32x16_bf16(oq[(NC * mb + c) % (PF + 1)], vfs[c], da, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // register e of the accumulator is row 8 (e / 4) + 4 g + e % 4 of the block
                float x16[16];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const f32x4 l4 = *(const f32x4 *)(&lse_s[32 * mb + 8 * j + 4 * g]);
                    f32x4 t4 = {0.f, 0.f, 0.f, 0.f};
                    if (DK) t4 = *(const f32x4 *)(&dlt_s[32 * mb + 8 * j + 4 * g]);
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const int e = 4 * j + w;
                        const float p = __builtin_amdgcn_exp2f(sa[e] * scale_log2 - l4[w]);
                        x16[e] = DK ? p * (da[e] - t4[w]) : p;
                    }
                }
                if (need_mask) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int m = m0 + 32 * mb + 8 * (e >> 2) + 4 * g + (e & 3);
                        const bool vis = m < L && kn < L && (!CAUSAL || kn <= m);
                        x16[e] = vis ? x16[e] : 0.f;
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    u32x4 a;
                    a.x = pack_bf16(x16[8 * half + 0], x16[8 * half + 1]);
                    a.y = pack_bf16(x16[8 * half + 2], x16[8 * half + 3]);
                    a.z = pack_bf16(x16[8 * half + 4], x16[8 * half + 5]);
                    a.w = pack_bf16(x16[8 * half + 6], x16[8 * half + 7]);
                    bf[2 * mb + half] = __builtin_bit_cast(bf16x8, a);
                }
            }
            // dV^T += dout^T P  or  dK^T += Q^T dS  over the tile's 64 rows, step j = 4 b + t
#pragma unroll
            for (int j = 0; j < 4 * NDB; ++j) {
                if (j + PF < 4 * NDB) tq[(j + PF) % (PF + 1)] = ps.rd_tr(xb, j + PF);
                __builtin_amdgcn_sched_barrier(0);
                acc[j >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[j % (PF + 1)], bf[j & 3], acc[j >> 2], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the next step's row statistics: its slot was last read in the previous step
        if (st + 1 < steps) store_stats(ST ^ 1);
    };
    for (int st = 0; st < steps; st += 2) {
        do_step(std::integral_constant<int, 0>{}, st);
        if (st + 1 < steps) do_step(std::integral_constant<int, 1>{}, st + 1);
    }

    if (kn < L) {
        const float f = DK ? scale : 1.0f;
        uint16_t *op = dkv + ((size_t)(row0 + kn) * Hkv + g_kv) * HD;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x2 w;
                w.x = pack_bf16(acc[b][4 * r] * f, acc[b][4 * r + 1] * f);
                w.y = pack_bf16(acc[b][4 * r + 2] * f, acc[b][4 * r + 3] * f);
                *(u32x2 *)(op + 32 * b + 8 * r + 4 * g) = w;
            }
    }
}

// ---------------------------------------------------------------------------
// dK and dV in one pass: 8 wavefronts, two per 32-key block of the workgroup's 128 keys.
//   producer (wavefronts 0..3), tile t in step t:      S = Q K^T -> P (to LDS, bf16),  dV^T += dout^T P
//   consumer (wavefronts 4..7), tile t in step t + 1:  dP = dout V^T, dS = P (dP - delta),  dK^T += Q^T dS
// Each role holds one 64-register accumulator and one stationary operand, so both fit the 256
// registers that two wavefronts per SIMD allow (a SIMD runs one producer and one consumer), and S
// is computed once for both outputs: four products per (query, key) pair instead of five.  P
// crosses in the B-operand layout it is consumed in (16 bytes per lane and 16 rows); tiles, P and
// the row statistics live in three stages because the consumer runs one step behind.
// One workgroup barrier per step orders all of it.
// ---------------------------------------------------------------------------
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(2 * kThreads, 1) void attn_bwd_dkv_fused_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint16_t *__restrict__ dout, const float *__restrict__ lse, const float *__restrict__ delta,
    uint16_t *__restrict__ dk, uint16_t *__restrict__ dv, const int32_t *__restrict__ cu,
    const BwdHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t batch, int32_t total_tokens,
    int32_t Hq, int32_t Hkv, float scale, float scale_log2)
{
    using PS = PairStage<HD, 3, 8>;
    constexpr int NC = HD / 16, NDB = HD / 32;
    __shared__ __attribute__((aligned(1024))) char lds_raw[PS::BYTES];
    // P and the row statistics live in a slot per stage, like the tiles they belong to
    __shared__ __attribute__((aligned(16))) bf16x8 s_p[3][4][4][64];  // P: stage, key block, fragment, lane
    __shared__ __attribute__((aligned(16))) float s_lse[3][kT];        // lse * log2(e) of a tile's rows (read in its step)
    __shared__ __attribute__((aligned(16))) float s_dlt[3][kT];        // delta of a tile's rows (read one step later)

    const int total_tiles = hdr->total_tiles;
    const int group = Hq / Hkv;
    int u, g_kv;
    block_to_tile(blockIdx.x, Hkv, Hkv, 1, u, g_kv);
    if (u >= total_tiles) return;
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tile_off[mid] <= u) lo = mid; else hi = mid - 1;
    }
    const int row0 = cu[lo];
    const int L = cu[lo + 1] - row0;
    const int k0 = (u - tile_off[lo]) * kOwn;  // under a causal mask the first key tile is the heaviest

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kbw = wave & 3;            // 32-key block of this wavefront
    const bool consumer = wave >= 4;
    const int l32 = lane & 31, g = lane >> 5;
    const int n0w = k0 + 32 * kbw;
    const int kn = n0w + l32;            // this lane's key (a column of S and dP)
    const int kn_c = kn < L ? kn : L - 1;

    // stationary B operand (column = this lane's key): K for the producer, V for the consumer
    bf16x8 sf[NC];
    {
        const uint16_t *sp = (consumer ? v : k) + ((size_t)(row0 + kn_c) * Hkv + g_kv) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) sf[c] = *(const bf16x8 *)(sp + 16 * c);
    }
    f32x16 acc[NDB];
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    const int m_begin = CAUSAL ? (k0 / kT) * kT : 0;  // rows before the first key see none of them
    const int ntile_m = m_begin < L ? (L - m_begin + kT - 1) / kT : 0;
    const int steps = ntile_m * group;

    PS ps;
    ps.init((uint32_t)(uintptr_t)lds_raw, lane, wave);
    TileSrc src{q, dout, row0, L, m_begin, Hq, g_kv * group};
    float r_lse = 0.f, r_dlt = 0.f;
    // Steps walk the group's q-heads, and inside a head the 64-row tiles from m_begin on.  The
    // loop is unrolled by the three stages, so a step's stage is a constant and every fragment
    // read is a fixed lane address plus an immediate offset.
    int f_tile = 0;                 // tile index (inside its head) of the step fetched next
    // Moves on to the next step's tile (when there is one) and returns its loads; the caller
    // spreads them over its MFMAs.
    using Plan = typename PS::Plan;
    auto start_step = [&](auto stage_c, bool more) {
        constexpr int STG = decltype(stage_c)::value;
        if (more) {
            if (f_tile == ntile_m) { f_tile = 0; ++src.hd; }
            src.m0 = m_begin + f_tile * kT;
            ++f_tile;
        }
        if (tid < kT) {
            int m = src.m0 + tid;
            m = m < L ? m : L - 1;
            r_lse = lse[(size_t)src.hd * total_tokens + row0 + m] * kLog2e;
            r_dlt = delta[(size_t)src.hd * total_tokens + row0 + m];
        }
        return ps.plan(src, STG);
    };
    // load k of the plan goes out after MFMA 1 + k * (MFMAs per step / loads per step) of the step
    constexpr int kMfmaPerStep = 4 * NC;
    bool has_next = false;
    auto dma_slot = [&](const Plan &pl, int i) {
        constexpr int every = kMfmaPerStep / PS::NLOAD;
        if (i % every == 1 && has_next) PS::issue(pl, i / every);
    };
    auto store_stats = [&](auto stage_c) {
        constexpr int STG = decltype(stage_c)::value;
        if (tid < kT) { s_lse[STG][tid] = r_lse; s_dlt[STG][tid] = r_dlt; }
    };
    if (steps > 0) {
        const Plan pl = start_step(std::integral_constant<int, 0>{}, true);
#pragma unroll
        for (int k = 0; k < PS::NLOAD; ++k) PS::issue(pl, k);
        store_stats(std::integral_constant<int, 0>{});
    }
    constexpr int PF = kFragAhead;
    const int nloop = steps > 0 ? steps + 1 : 0;   // the consumer's last tile is done in one more step
    int w_tile = consumer ? -1 : 0;                // tile index (inside its head) this wavefront works on

    // dV^T += dout^T P (producer) or dK^T += Q^T dS (consumer) over the tile's 64 rows, step j = 4 b + t
    auto accumulate = [&](uint32_t xb, const bf16x8 (&bf)[4], bf16x8 (&tq)[PF + 1], const Plan &pl) {
#pragma unroll
        for (int j = 0; j < 4 * NDB; ++j) {
            if (j + PF < 4 * NDB) tq[(j + PF) % (PF + 1)] = ps.rd_tr(xb, j + PF);
            __builtin_amdgcn_sched_barrier(0);
            acc[j >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[j % (PF + 1)], bf[j & 3], acc[j >> 2], 0, 0, 0);
            dma_slot(pl, 2 * NC + j);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto step = [&](auto stage_c, int st) {
        constexpr int SA = decltype(stage_c)::value;   // stage of the tile fetched for step st (the producer's)
        constexpr int SB = (SA + 2) % 3;               // stage of the tile of step st - 1 (the consumer's)
        ps.publish();
        has_next = st + 1 < steps;
        const Plan pl = start_step(std::integral_constant<int, (SA + 1) % 3>{}, has_next);
        const int m0 = m_begin + w_tile * kT;
        const bool live = consumer ? st >= 1 : st < steps;
        // rows of the tile that lie before this wavefront's keys see none of them (both roles skip alike)
        if (live && !(CAUSAL && m0 + kT - 1 < n0w)) {
            bf16x8 bf[4];  // P (producer) or dS (consumer) of the tile's 64 rows, B-operand layout
            // one ring for row and transposed fragments: every run of MFMAs has an even length
            static_assert(PF == 1 && NC % 2 == 0, "the fragment ring alternates between two registers");
            bf16x8 fq[2];
            if (!consumer) {
                const uint32_t qb = ps.x_at(SA), ob = ps.y_at(SA);
                const float *lse_s = s_lse[SA];
                // only tiles that touch the end of the sequence or the diagonal have masked elements
                const bool need_mask = m0 + kT > L || n0w + 32 > L || (CAUSAL && n0w + 31 > m0);
#pragma unroll
                for (int i = 0; i < PF; ++i) fq[i] = ps.rd_row(qb, 0, i);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    f32x16 sa;
#pragma unroll
                    for (int e = 0; e < 16; ++e) sa[e] = 0.f;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int sn = NC * mb + c + PF;
                        if (sn < 2 * NC) fq[sn % (PF + 1)] = ps.rd_row(qb, sn / NC, sn % NC);
                        else fq[(sn - 2 * NC) % (PF + 1)] = ps.rd_tr(ob, sn - 2 * NC);
                        __builtin_amdgcn_sched_barrier(0);
                        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[(NC * mb + c) % (PF + 1)], sf[c], sa, 0, 0, 0);
                        dma_slot(pl, NC * mb + c);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // register e of the accumulator is row 8 (e / 4) + 4 g + e % 4 of the block
                    float x16[16];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const f32x4 l4 = *(const f32x4 *)(&lse_s[32 * mb + 8 * j + 4 * g]);
#pragma unroll
                        for (int w = 0; w < 4; ++w)
                            x16[4 * j + w] = __builtin_amdgcn_exp2f(sa[4 * j + w] * scale_log2 - l4[w]);
                    }
                    if (need_mask) {
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int m = m0 + 32 * mb + 8 * (e >> 2) + 4 * g + (e & 3);
                            const bool vis = m < L && kn < L && (!CAUSAL || kn <= m);
                            x16[e] = vis ? x16[e] : 0.f;
                        }
                    }
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        u32x4 a;
                        a.x = pack_bf16(x16[8 * half + 0], x16[8 * half + 1]);
                        a.y = pack_bf16(x16[8 * half + 2], x16[8 * half + 3]);
                        a.z = pack_bf16(x16[8 * half + 4], x16[8 * half + 5]);
                        a.w = pack_bf16(x16[8 * half + 6], x16[8 * half + 7]);
                        bf[2 * mb + half] = __builtin_bit_cast(bf16x8, a);
                        s_p[SA][kbw][2 * mb + half][lane] = bf[2 * mb + half];
                    }
                }
                accumulate(ob, bf, fq, pl);
            } else {
                const uint32_t qb = ps.x_at(SB), ob = ps.y_at(SB);
                const float *dlt_s = s_dlt[SB];
#pragma unroll
                for (int i = 0; i < PF; ++i) fq[i] = ps.rd_row(ob, 0, i);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    f32x16 da;
#pragma unroll
                    for (int e = 0; e < 16; ++e) da[e] = 0.f;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int sn = NC * mb + c + PF;
                        if (sn < 2 * NC) fq[sn % (PF + 1)] = ps.rd_row(ob, sn / NC, sn % NC);
                        else fq[(sn - 2 * NC) % (PF + 1)] = ps.rd_tr(qb, sn - 2 * NC);
                        __builtin_amdgcn_sched_barrier(0);
                        da = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[(NC * mb + c) % (PF + 1)], sf[c], da, 0, 0, 0);
                        dma_slot(pl, NC * mb + c);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const u32x4 pw = __builtin_bit_cast(u32x4, s_p[SB][kbw][2 * mb + half][lane]);
                        float d8[8];
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const f32x4 t4 = *(const f32x4 *)(&dlt_s[32 * mb + 8 * (2 * half + jj) + 4 * g]);
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                const int i = 4 * jj + w;                      // element of the fragment
                                const uint32_t pr = pw[i >> 1];
                                const float p = __uint_as_float((i & 1) ? (pr & 0xffff0000u) : (pr << 16));
                                d8[i] = p * (da[8 * half + i] - t4[w]);
                            }
                        }
                        u32x4 a;
                        a.x = pack_bf16(d8[0], d8[1]);
                        a.y = pack_bf16(d8[2], d8[3]);
                        a.z = pack_bf16(d8[4], d8[5]);
                        a.w = pack_bf16(d8[6], d8[7]);
                        bf[2 * mb + half] = __builtin_bit_cast(bf16x8, a);
                    }
                }
                accumulate(qb, bf, fq, pl);
            }
        } else if (has_next) {   // nothing to compute in this step: the loads still go out
#pragma unroll
            for (int k = 0; k < PS::NLOAD; ++k) PS::issue(pl, k);
        }
        if (++w_tile == ntile_m) w_tile = 0;
        // the next step's row statistics: their slots were last read before this step's barrier
        if (st + 1 < steps) store_stats(std::integral_constant<int, (SA + 1) % 3>{});
    };
    for (int st = 0; st < nloop; st += 3) {
        step(std::integral_constant<int, 0>{}, st);
        if (st + 1 < nloop) step(std::integral_constant<int, 1>{}, st + 1);
        if (st + 2 < nloop) step(std::integral_constant<int, 2>{}, st + 2);
    }

    if (kn < L) {
        const float f = consumer ? scale : 1.0f;
        uint16_t *op = (consumer ? dk : dv) + ((size_t)(row0 + kn) * Hkv + g_kv) * HD;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x2 w;
                w.x = pack_bf16(acc[b][4 * r] * f, acc[b][4 * r + 1] * f);
                w.y = pack_bf16(acc[b][4 * r + 2] * f, acc[b][4 * r + 3] * f);
                *(u32x2 *)(op + 32 * b + 8 * r + 4 * g) = w;
            }
    }
}

struct BwdWs {
    BwdHdr *hdr;
    int32_t *tile_off;
    float *delta;
};

size_t carve(BwdWs &w, void *ws, int32_t batch, int64_t total_tokens, int32_t Hq)
{
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes, 256); return r; };
    w.hdr = (BwdHdr *)take(sizeof(BwdHdr));
    w.tile_off = (int32_t *)take(((size_t)(batch > 0 ? batch : 0) + 1) * 4);
    w.delta = (float *)take((size_t)(total_tokens > 0 ? total_tokens : 0) * (size_t)Hq * 4 + 4);
    return off;
}

}  // namespace

size_t attn_bwd_ws_bytes(int32_t batch, int32_t total_tokens, int32_t Hq)
{
    BwdWs w;
    return carve(w, nullptr, batch, total_tokens, Hq);
}

int launch_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                    const void *dout, void *dq, void *dk, void *dv, const int32_t *cu_seqlens,
                    int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t Hq, int32_t Hkv, int32_t d,
                    float scale, int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes,
                    hipStream_t stream)
{
    BwdWs w;
    const size_t need = carve(w, ws, batch, total_tokens, Hq);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_varlen_attn_bwd: workspace %zu < %zu bytes", ws_bytes, need);
    hipLaunchKernelGGL(bwd_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, cu_seqlens, batch, total_tokens,
                       max_seqlen, w.hdr, w.tile_off, dev_status);
    int64_t max_tiles = (int64_t)total_tokens / kOwn + batch;
    if (max_seqlen > 0) max_tiles = std::min<int64_t>(max_tiles, (int64_t)batch * ((max_seqlen + kOwn - 1) / kOwn));
    // (a launch of 2^32 threads or more in all is cut short by the runtime without an error)
    if (max_tiles * Hq > 0x7fffffffLL || max_tiles * Hq * (2 * kThreads) > 0xffffffffLL)
        ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_bwd: %lld workgroups", (long long)(max_tiles * Hq));
    if (scale <= 0.f) scale = 1.0f / sqrtf((float)d);
    const float sl2 = scale * kLog2e;
    if (batch > 0 && total_tokens > 0) {
        const unsigned qgrid = (unsigned)(max_tiles * Hq), kgrid = (unsigned)(max_tiles * Hkv);
#define ORCH_BWD_COMMON (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (const uint16_t *)dout, lse, w.delta
#define ORCH_BWD_TAIL cu_seqlens, w.hdr, w.tile_off, batch, total_tokens, Hq, Hkv, scale, sl2
// head_dim 128 (long LLM-phase sequences): dK and dV from the fused producer/consumer kernel.
// head_dim 64 (encoder phases, sequences of a few hundred rows): one kernel per output; the fused
// kernel's extra step per (key tile, head) costs more there than the second S product.
#define ORCH_BWD_LAUNCH(HD_, C_)                                                                                  \
    do {                                                                                                          \
        hipLaunchKernelGGL((attn_bwd_dq_kernel<HD_, C_>), dim3(qgrid), dim3(kThreads), 0, stream,                 \
                           (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (const uint16_t *)dout, \
                           lse, (const uint16_t *)out, w.delta, (uint16_t *)dq, ORCH_BWD_TAIL);                   \
        if (HD_ == 128) {                                                                                         \
            hipLaunchKernelGGL((attn_bwd_dkv_fused_kernel<128, C_>), dim3(kgrid), dim3(2 * kThreads), 0, stream,  \
                               ORCH_BWD_COMMON, (uint16_t *)dk, (uint16_t *)dv, ORCH_BWD_TAIL);                   \
        } else {                                                                                                  \
            hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, C_, PART_DK>), dim3(kgrid), dim3(kThreads), 0, stream,    \
                               ORCH_BWD_COMMON, (uint16_t *)dk, ORCH_BWD_TAIL);                                   \
            hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, C_, PART_DV>), dim3(kgrid), dim3(kThreads), 0, stream,    \
                               ORCH_BWD_COMMON, (uint16_t *)dv, ORCH_BWD_TAIL);                                   \
        }                                                                                                         \
    } while (0)
        if (d == 128 && causal) ORCH_BWD_LAUNCH(128, true);
        else if (d == 128) ORCH_BWD_LAUNCH(128, false);
        else if (causal) ORCH_BWD_LAUNCH(64, true);
        else ORCH_BWD_LAUNCH(64, false);
#undef ORCH_BWD_LAUNCH
#undef ORCH_BWD_TAIL
#undef ORCH_BWD_COMMON
    }
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
