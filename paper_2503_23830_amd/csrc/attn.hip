// orch_varlen_attn_fwd: padding-free attention forward over sequences stored
// back to back (the batching the paper uses for every phase that runs without
// paddings, Sec. 7; the quadratic term of Eq. 2).
//
// One workgroup (4 wavefronts) owns 128*MB consecutive query rows of one
// sequence and one q-head; each wavefront owns MB blocks of 32 rows.  K/V tiles
// of BN = 64 keys are staged through LDS (V transposed on the way in) and shared
// by the four wavefronts; with MB = 2 every K/V fragment read from LDS feeds two
// MFMAs, which halves LDS traffic per FLOP.  The scores are computed transposed,
// S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in the accumulator layout every
// lane then holds 16 keys of ONE query, so the online-softmax statistics are
// per-lane scalars (one cross-lane exchange per tile), the probabilities are
// already in the B-operand layout of the second product O^T += V^T P^T, and
// rescaling O is a per-lane multiply.  The running maximum is only moved when a
// row's maximum grows by more than 2^8 (exact: the stale reference cancels in
// the final division), so O is rarely rescaled after the first tile.
#include <stdlib.h>

#include <type_traits>

#include "common.h"

namespace orch {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BN = 64;   // keys per LDS tile
constexpr int kThreads = 256;
constexpr int kPrepThreads = 1024;

struct AttnHdr {
    int32_t total_tiles;
    int32_t ok;
};

// tile_off[t] = number of BM-row query tiles in sequences before t.
__global__ __launch_bounds__(kPrepThreads) void attn_prep_kernel(const int32_t *__restrict__ cu,
                                                                int32_t batch, int32_t total_tokens,
                                                                int32_t BM, AttnHdr *hdr,
                                                                int32_t *tile_off, int32_t *dev_status)
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
        if (lo < 0 || hi < lo || hi > total_tokens) { bad = 1; continue; }
        sum += (hi - lo + BM - 1) / BM;
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
            run += (cu[t + 1] - cu[t] + BM - 1) / BM;
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


template <int HD, bool CAUSAL, int MB>
__global__ __launch_bounds__(kThreads, (MB * HD > 128 ? 1 : 2)) void attn_fwd_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,
    const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t batch,
    int32_t total_tokens, int32_t Hq, int32_t Hkv, float scale, float scale_log2)
{
    constexpr int BM = 128 * MB;  // query rows per workgroup
    constexpr int NBLK = 4 * MB;  // 32-row blocks per workgroup
    constexpr int KS = HD + 8;    // K tile row stride (elements): 16-byte rows land on distinct banks
    constexpr int VS = BN + 8;    // V^T tile row stride
    constexpr int NC = HD / 16;   // 16-wide chunks of the head dimension
    constexpr int NDB = HD / 32;  // 32-row blocks of O^T
    __shared__ __attribute__((aligned(16))) uint16_t Ks[BN * KS];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[HD * VS];

    const int total_tiles = hdr->total_tiles;
    const int group = Hq / Hkv;

    // block -> (query tile u, head h).  With Hkv a multiple of 8 the kv-head is
    // chosen by blockIdx % 8, i.e. by XCD, so the blocks that share a K/V stream
    // share an L2.
    int u, h;
    {
        const int bid = blockIdx.x;
        if ((Hkv & 7) == 0) {
            const int kvh = (bid & 7) + 8 * ((bid >> 3) % (Hkv >> 3));
            const int rest = bid / Hkv;
            h = kvh * group + rest % group;
            u = rest / group;
        } else {
            h = bid % Hq;
            u = bid / Hq;
        }
    }
    if (u >= total_tiles) return;
    const int g_kv = h / group;

    // sequence t with tile_off[t] <= u < tile_off[t+1]
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tile_off[mid] <= u) lo = mid; else hi = mid - 1;
    }
    const int seq = lo;
    const int row0 = cu[seq];
    const int L = cu[seq + 1] - row0;
    const int ntile_q = (L + BM - 1) / BM;
    const int qt = ntile_q - 1 - (u - tile_off[seq]);  // heaviest (last) tile first
    const int q0 = qt * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;

    // 32-row blocks of this wavefront.  Under a causal mask block b needs b+1
    // units of work near the diagonal, so wave w takes blocks w and NBLK-1-w:
    // every wavefront then carries the same amount.
    int blk[MB], qm[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        blk[mb] = (mb & 1) ? (NBLK - 1 - wave - 4 * (mb >> 1)) : (wave + 4 * (mb >> 1));
        qm[mb] = q0 + 32 * blk[mb] + l32;
    }

    // ---- Q fragments: B operand, column m = lane%32, k = 16c + 8g + [0..7]
    bf16x8 qf[MB][NC];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int qm_c = qm[mb] < L ? qm[mb] : L - 1;
        const uint16_t *qp = q + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[mb][c] = *(const bf16x8 *)(qp + 16 * c);
    }

    f32x16 acc_o[MB][NDB];
    float m_run[MB], l_run[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        m_run[mb] = -INFINITY;
        l_run[mb] = 0.f;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[mb][b][e] = 0.f;
    }
    // a row's reference maximum moves only when it grows by more than 2^8
    const float lazy_thr = 8.0f / scale_log2;

    const int kend = CAUSAL ? min(L, q0 + BM) : L;
    const int ntile_k = (kend + BN - 1) / BN;

    // ---- global -> register staging of one K/V tile
    constexpr int KROWS_PER_PASS = kThreads / (HD / 8);  // rows covered by 256 16-byte loads
    constexpr int KPASS = BN / KROWS_PER_PASS;
    constexpr int VBLK = (BN / 4) * (HD / 4) / kThreads;  // 4(key) x 4(dim) blocks per thread
    u32x4 kreg[KPASS];
    u32x2 vreg[VBLK][4];
    const int k_col = (tid % (HD / 8)) * 8, k_row = tid / (HD / 8);
    // V blocks: 8 adjacent lanes take 8 different key quads (so their transposed
    // 8-byte LDS writes fall on different banks), the next lane bits walk the
    // head dimension
    const int v_nq0 = tid & 7, v_dq = (tid >> 3) % (HD / 4), v_nqhi = (tid >> 3) / (HD / 4);
    static_assert(VBLK * (kThreads / 8 / (HD / 4)) * 8 == BN / 4, "V staging must cover the tile");

    auto load_tile = [&](int n0) {
#pragma unroll
        for (int p = 0; p < KPASS; ++p) {
            int n = n0 + p * KROWS_PER_PASS + k_row;
            n = n < L ? n : L - 1;
            kreg[p] = *(const u32x4 *)(k + ((size_t)(row0 + n) * Hkv + g_kv) * HD + k_col);
        }
#pragma unroll
        for (int b = 0; b < VBLK; ++b) {
            const int nq = v_nq0 + 8 * (v_nqhi + b * (kThreads / 8 / (HD / 4)));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int n = n0 + 4 * nq + j;
                n = n < L ? n : L - 1;
                vreg[b][j] = *(const u32x2 *)(v + ((size_t)(row0 + n) * Hkv + g_kv) * HD + 4 * v_dq);
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int p = 0; p < KPASS; ++p)
            *(u32x4 *)(&Ks[(p * KROWS_PER_PASS + k_row) * KS + k_col]) = kreg[p];
#pragma unroll
        for (int b = 0; b < VBLK; ++b) {
            const int nq = v_nq0 + 8 * (v_nqhi + b * (kThreads / 8 / (HD / 4)));
            // key n = 16t + 8u + 4g + w is stored at slot 16t + 8g + 4u + w, so the 8
            // keys a lane contracts in one MFMA are contiguous
            const int slot = 16 * (nq >> 2) + 8 * (nq & 1) + 4 * ((nq >> 1) & 1);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                const uint32_t a0 = (c & 2) ? vreg[b][0].y : vreg[b][0].x;
                const uint32_t a1 = (c & 2) ? vreg[b][1].y : vreg[b][1].x;
                const uint32_t a2 = (c & 2) ? vreg[b][2].y : vreg[b][2].x;
                const uint32_t a3 = (c & 2) ? vreg[b][3].y : vreg[b][3].x;
                u32x2 w;
                w.x = __builtin_amdgcn_perm(a1, a0, sel);
                w.y = __builtin_amdgcn_perm(a3, a2, sel);
                *(u32x2 *)(&Vt[(4 * v_dq + c) * VS + slot]) = w;
            }
        }
    };

    // One K/V tile for the row blocks mb >= MB0 of this wavefront (blocks below
    // MB0 lie entirely above the causal diagonal for this tile).
    auto compute_tile = [&](auto mb0_tag, int n0) {
        constexpr int MB0 = decltype(mb0_tag)::value;
        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 acc_s[MB][2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int mb = MB0; mb < MB; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_s[mb][nb][e] = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const bf16x8 kf = *(const bf16x8 *)(&Ks[(32 * nb + l32) * KS + 16 * c + 8 * g]);
#pragma unroll
                for (int mb = MB0; mb < MB; ++mb)
                    acc_s[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[mb][c], acc_s[mb][nb], 0, 0, 0);
            }
        }

        bf16x8 pf[MB][4];
        bool any_upd = false;
        float alpha[MB];
#pragma unroll
        for (int mb = MB0; mb < MB; ++mb) {
            // ---- mask (only tiles that touch the sequence end or the diagonal)
            const bool need_mask = (n0 + BN > L) || (CAUSAL && n0 + BN - 1 > q0 + 32 * blk[mb]);
            if (need_mask) {
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int n = n0 + 32 * nb + 8 * (e >> 2) + 4 * g + (e & 3);
                        const bool vis = n < L && (!CAUSAL || n <= qm[mb]);
                        if (!vis) acc_s[mb][nb][e] = -INFINITY;
                    }
            }
            // ---- online softmax, one query per lane (shared by lanes l and l^32)
            float tmax = acc_s[mb][0][0];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, acc_s[mb][nb][e]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const bool upd = tmax > m_run[mb] + lazy_thr;
            const float m_new = upd ? tmax : m_run[mb];
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[mb] = upd ? __builtin_amdgcn_exp2f((m_run[mb] - m_use) * scale_log2) : 1.0f;
            any_upd |= upd;
            m_run[mb] = m_new;
            const float mbias = m_use * scale_log2;
            float psum = 0.f;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(acc_s[mb][kk >> 1][8 * (kk & 1) + e] * scale_log2 - mbias);
                    psum += p[e];
                }
                u32x4 pk;
                pk.x = pack_bf16(p[0], p[1]);
                pk.y = pack_bf16(p[2], p[3]);
                pk.z = pack_bf16(p[4], p[5]);
                pk.w = pack_bf16(p[6], p[7]);
                pf[mb][kk] = __builtin_bit_cast(bf16x8, pk);
            }
            l_run[mb] = l_run[mb] * alpha[mb] + psum;
        }
        if (__any(any_upd)) {
#pragma unroll
            for (int mb = MB0; mb < MB; ++mb)
#pragma unroll
                for (int b = 0; b < NDB; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc_o[mb][b][e] *= alpha[mb];
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 vf = *(const bf16x8 *)(&Vt[(32 * b + l32) * VS + 16 * kk + 8 * g]);
#pragma unroll
                for (int mb = MB0; mb < MB; ++mb)
                    acc_o[mb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mb][kk], acc_o[mb][b], 0, 0, 0);
            }
    };

    load_tile(0);
    for (int it = 0; it < ntile_k; ++it) {
        const int n0 = it * BN;
        __syncthreads();
        store_tile();
        __syncthreads();
        if (it + 1 < ntile_k) load_tile(n0 + BN);

        // row blocks entirely above the diagonal have nothing to do in this tile;
        // blk[] ascends with mb, so the active ones are a suffix
        int first = 0;
        if (CAUSAL) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                if (n0 > q0 + 32 * blk[mb] + 31) first = mb + 1;
        }
        if (first == 0) compute_tile(std::integral_constant<int, 0>{}, n0);
        else if (MB > 1 && first == 1) compute_tile(std::integral_constant<int, (MB > 1 ? 1 : 0)>{}, n0);
    }

    // ---- epilogue
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float l_tot = l_run[mb] + __shfl_xor(l_run[mb], 32);
        const float inv = 1.f / l_tot;
        if (qm[mb] < L) {
            uint16_t *op = out + ((size_t)(row0 + qm[mb]) * Hq + h) * HD;
#pragma unroll
            for (int b = 0; b < NDB; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    u32x2 w;
                    w.x = pack_bf16(acc_o[mb][b][4 * r] * inv, acc_o[mb][b][4 * r + 1] * inv);
                    w.y = pack_bf16(acc_o[mb][b][4 * r + 2] * inv, acc_o[mb][b][4 * r + 3] * inv);
                    *(u32x2 *)(op + 32 * b + 8 * r + 4 * g) = w;
                }
            if (lse != nullptr && g == 0)
                lse[(size_t)h * total_tokens + row0 + qm[mb]] = m_run[mb] * scale + __logf(l_tot);
        }
    }
}


// ---------------------------------------------------------------------------
// Ping-pong variant: 8 wavefronts (two per SIMD) own 256 query rows, 32 each.
// The key sequence is walked in 32-key blocks b; a wavefront alternates
//     M(b): S^T = K_b Q^T  and  O^T += V_{b-1}^T P_{b-1}^T   (16 MFMAs, LDS reads)
//     V(b): online softmax of block b -> P_b                  (vector ALU),
//           plus its share of the global -> LDS staging
// with a workgroup barrier after every phase.  Wavefronts 4..7 run one phase
// behind wavefronts 0..3, so on every SIMD one wavefront is in its MFMA phase
// while the other is in its vector-ALU phase: the matrix cores and the vector
// ALU work at the same time without relying on instruction scheduling.
//
// K and V^T tiles (64 keys = two blocks) are double-buffered in LDS.  With
// phases numbered t (group 0: M(b) at 2b; group 1: M(b) at 2b+1), tile i's K is
// read during t in [4i, 4i+3] and its V during [4i+2, 4i+5]; every wavefront
// stores its share of K_{i+1} in V(2i) and of V_{i+1} in V(2i+1), which for both
// groups falls after the last read of the buffer being replaced and before the
// first read of the new tile.
// ---------------------------------------------------------------------------
constexpr int kPPThreads = 512;
#ifndef ORCH_DBG_NOSHIFT
#define ORCH_DBG_NOSHIFT 0
#endif
#ifndef ORCH_DBG_TIMING
#define ORCH_DBG_TIMING 0
#endif

// Workgroup barrier that orders LDS traffic only: LDS writes of this wavefront
// are complete before it, but global loads already in flight (the prefetch of a
// later tile) are NOT waited for, unlike __syncthreads().
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(kPPThreads) void attn_fwd_pp_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,
    const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t batch,
    int32_t total_tokens, int32_t Hq, int32_t Hkv, float scale, float scale_log2)
{
    constexpr int BM = 256;
    constexpr int KS = HD + 8;
    constexpr int VS = BN + 8;
    constexpr int NC = HD / 16;
    constexpr int NDB = HD / 32;
    constexpr int KTILE = BN * KS, VTILE = HD * VS;
    __shared__ __attribute__((aligned(16))) uint16_t Ks[2 * KTILE];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[2 * VTILE];

    const int total_tiles = hdr->total_tiles;
    const int group = Hq / Hkv;
    int u, h;
    {
        const int bid = blockIdx.x;
        if ((Hkv & 7) == 0) {
            const int kvh = (bid & 7) + 8 * ((bid >> 3) % (Hkv >> 3));
            const int rest = bid / Hkv;
            h = kvh * group + rest % group;
            u = rest / group;
        } else {
            h = bid % Hq;
            u = bid / Hq;
        }
    }
    if (u >= total_tiles) return;
    const int g_kv = h / group;
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tile_off[mid] <= u) lo = mid; else hi = mid - 1;
    }
    const int seq = lo;
    const int row0 = cu[seq];
    const int L = cu[seq + 1] - row0;
    const int ntile_q = (L + BM - 1) / BM;
    const int qt = ntile_q - 1 - (u - tile_off[seq]);
    const int q0 = qt * BM;

    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform values are kept in scalar registers so that per-wavefront
    // decisions become scalar branches
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int grp = ORCH_DBG_NOSHIFT ? 0 : (wave >> 2);  // 0: leading group, 1: one phase behind
    // waves w and w+4 share a SIMD; row blocks w and 7-w even out the causal work per SIMD
    const int rblk = wave < 4 ? wave : 11 - wave;
    const int qrow0 = q0 + 32 * rblk;
    const int qm = qrow0 + l32;

    bf16x8 qf[NC];
    {
        const int qm_c = qm < L ? qm : L - 1;
        const uint16_t *qp = q + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c] = *(const bf16x8 *)(qp + 16 * c);
    }
    f32x16 acc_o[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[d][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float lazy_thr = 8.0f / scale_log2;

    const int kend = CAUSAL ? min(L, q0 + BM) : L;
    const int ntile_k = (kend + BN - 1) / BN;               // tiles the workgroup stages
    const int nblk = 2 * ntile_k;                           // 32-key blocks every wavefront steps through
    const int kend_w = CAUSAL ? min(L, qrow0 + 32) : L;
    const int nblk_w = qrow0 < L ? (kend_w + 31) / 32 : 0;  // blocks this wavefront computes

    // ---- global -> register -> LDS staging (512 threads)
    constexpr int KLOADS = BN * (HD / 8) / kPPThreads;      // 16-byte K loads per thread
    constexpr int KROWS_PER_PASS = kPPThreads / (HD / 8);
    constexpr int VBLOCKS = (BN / 4) * (HD / 4);            // 4(key) x 4(dim) blocks per tile
    const bool v_active = VBLOCKS >= kPPThreads || tid < VBLOCKS;
    u32x4 kreg[KLOADS];
    u32x2 vreg[4];
    const int k_col = (tid % (HD / 8)) * 8, k_row = tid / (HD / 8);
    const int v_dq = (tid >> 3) % (HD / 4);
    const int v_nq = ((tid & 7) + 8 * ((tid >> 3) / (HD / 4))) & 15;
    const uint16_t *kbase = k + ((size_t)row0 * Hkv + g_kv) * HD + k_col;
    const uint16_t *vbase = v + ((size_t)row0 * Hkv + g_kv) * HD + 4 * v_dq;
    const size_t rstride = (size_t)Hkv * HD;
    const int v_slot = 16 * (v_nq >> 2) + 8 * (v_nq & 1) + 4 * ((v_nq >> 1) & 1);

    // tile indices past the end are clamped (the copy lands in a buffer nobody
    // reads again); rows past the sequence end repeat row L-1 and are masked later
    auto load_k = [&](int t) {
        t = t < ntile_k ? t : ntile_k - 1;
#pragma unroll
        for (int p = 0; p < KLOADS; ++p) {
            int n = t * BN + p * KROWS_PER_PASS + k_row;
            n = n < L ? n : L - 1;
            kreg[p] = *(const u32x4 *)(kbase + (size_t)n * rstride);
        }
    };
    auto load_v = [&](int t) {
        t = t < ntile_k ? t : ntile_k - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n = t * BN + 4 * v_nq + j;
            n = n < L ? n : L - 1;
            vreg[j] = *(const u32x2 *)(vbase + (size_t)n * rstride);
        }
    };
    auto store_k = [&](int buf) {
#pragma unroll
        for (int p = 0; p < KLOADS; ++p)
            *(u32x4 *)(&Ks[buf * KTILE + (p * KROWS_PER_PASS + k_row) * KS + k_col]) = kreg[p];
    };
    auto store_v = [&](int buf) {
        if (!v_active) return;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
            const uint32_t a0 = (c & 2) ? vreg[0].y : vreg[0].x;
            const uint32_t a1 = (c & 2) ? vreg[1].y : vreg[1].x;
            const uint32_t a2 = (c & 2) ? vreg[2].y : vreg[2].x;
            const uint32_t a3 = (c & 2) ? vreg[3].y : vreg[3].x;
            u32x2 w;
            w.x = __builtin_amdgcn_perm(a1, a0, sel);
            w.y = __builtin_amdgcn_perm(a3, a2, sel);
            *(u32x2 *)(&Vt[buf * VTILE + (4 * v_dq + c) * VS + v_slot]) = w;
        }
    };

    f32x16 S;      // scores of the current block
    bf16x8 P[2];   // its probabilities: two 16-key chunks (B operand of P V)
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) P[kk] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});

    // M phase of block b.  All 16 LDS fragment reads are issued back to back
    // (inline asm keeps them in this order and in flight together); each MFMA
    // then waits only until ITS fragment has arrived (LDS returns in order, so
    // "at most n reads outstanding" means the first 16-n are complete).
    const uint32_t lds_k0 = (uint32_t)(uintptr_t)(&Ks[0]) + 2u * (uint32_t)(l32 * KS + 8 * g);
    const uint32_t lds_v0 = (uint32_t)(uintptr_t)(&Vt[0]) + 2u * (uint32_t)(l32 * VS + 8 * g);
    // The phase is branch-free: a wavefront that does not need block b (beyond its
    // causal range) still runs the MFMAs -- it would otherwise idle at the barrier
    // -- on valid staged data, with P = 0 so that O is unchanged.
    // It is written as two asm blocks so that the order is exactly: all LDS reads,
    // then per MFMA "wait until my fragment is in, multiply".  The compiler does
    // not know these are MFMAs, so the hazards it would pad are padded by hand:
    // s_nop before the second block (vector-ALU write of P / O -> MFMA read) and
    // after it (MFMA write -> vector-ALU read).
    auto phase_m = [&](int b) {
        const int pb = b >= 1 ? b - 1 : 0;
        const uint32_t ka = lds_k0 + 2u * (uint32_t)(((b >> 1) & 1) * KTILE + 32 * (b & 1) * KS);
        const uint32_t va = lds_v0 + 2u * (uint32_t)(((pb >> 1) & 1) * VTILE + 32 * (pb & 1));
        if constexpr (HD == 128) {
            bf16x8 k0, k1, k2, k3, k4, k5, k6, k7, v0, v1, v2, v3, v4, v5, v6, v7;
            asm volatile(
                "ds_read_b128 %1, %17 offset:0\n\t"
                "ds_read_b128 %2, %17 offset:32\n\t"
                "ds_read_b128 %3, %17 offset:64\n\t"
                "ds_read_b128 %4, %17 offset:96\n\t"
                "ds_read_b128 %5, %17 offset:128\n\t"
                "ds_read_b128 %6, %17 offset:160\n\t"
                "ds_read_b128 %7, %17 offset:192\n\t"
                "ds_read_b128 %8, %17 offset:224\n\t"
                "ds_read_b128 %9, %18 offset:0\n\t"
                "ds_read_b128 %10, %18 offset:32\n\t"
                "ds_read_b128 %11, %18 offset:%27\n\t"
                "ds_read_b128 %12, %18 offset:%28\n\t"
                "ds_read_b128 %13, %18 offset:%29\n\t"
                "ds_read_b128 %14, %18 offset:%30\n\t"
                "ds_read_b128 %15, %18 offset:%31\n\t"
                "ds_read_b128 %16, %18 offset:%32\n\t"
                "s_waitcnt lgkmcnt(15)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %1, %19, 0\n\t"
                "s_waitcnt lgkmcnt(14)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %2, %20, %0\n\t"
                "s_waitcnt lgkmcnt(13)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %3, %21, %0\n\t"
                "s_waitcnt lgkmcnt(12)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %4, %22, %0\n\t"
                "s_waitcnt lgkmcnt(11)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %5, %23, %0\n\t"
                "s_waitcnt lgkmcnt(10)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %6, %24, %0\n\t"
                "s_waitcnt lgkmcnt(9)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %7, %25, %0\n\t"
                "s_waitcnt lgkmcnt(8)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %8, %26, %0\n\t"
                : "=&v"(S), "=&v"(k0), "=&v"(k1), "=&v"(k2), "=&v"(k3), "=&v"(k4), "=&v"(k5), "=&v"(k6),
                  "=&v"(k7), "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6),
                  "=&v"(v7)
                : "v"(ka), "v"(va), "v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]), "v"(qf[4]), "v"(qf[5]),
                  "v"(qf[6]), "v"(qf[7]), "n"(2 * 32 * VS), "n"(2 * 32 * VS + 32), "n"(4 * 32 * VS),
                  "n"(4 * 32 * VS + 32), "n"(6 * 32 * VS), "n"(6 * 32 * VS + 32)
                : "memory");
            asm volatile(
                "s_nop 7\n\t"
                "s_waitcnt lgkmcnt(7)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %4, %12, %0\n\t"
                "s_waitcnt lgkmcnt(6)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %5, %13, %0\n\t"
                "s_waitcnt lgkmcnt(5)\n\t"
                "v_mfma_f32_32x32x16_bf16 %1, %6, %12, %1\n\t"
                "s_waitcnt lgkmcnt(4)\n\t"
                "v_mfma_f32_32x32x16_bf16 %1, %7, %13, %1\n\t"
                "s_waitcnt lgkmcnt(3)\n\t"
                "v_mfma_f32_32x32x16_bf16 %2, %8, %12, %2\n\t"
                "s_waitcnt lgkmcnt(2)\n\t"
                "v_mfma_f32_32x32x16_bf16 %2, %9, %13, %2\n\t"
                "s_waitcnt lgkmcnt(1)\n\t"
                "v_mfma_f32_32x32x16_bf16 %3, %10, %12, %3\n\t"
                "s_waitcnt lgkmcnt(0)\n\t"
                "v_mfma_f32_32x32x16_bf16 %3, %11, %13, %3\n\t"
                "s_nop 15\n\t"
                : "+v"(acc_o[0]), "+v"(acc_o[1]), "+v"(acc_o[2]), "+v"(acc_o[3])
                : "v"(v0), "v"(v1), "v"(v2), "v"(v3), "v"(v4), "v"(v5), "v"(v6), "v"(v7), "v"(P[0]), "v"(P[1])
                : "memory");
        } else {
            bf16x8 k0, k1, k2, k3, v0, v1, v2, v3;
            asm volatile(
                "ds_read_b128 %1, %9 offset:0\n\t"
                "ds_read_b128 %2, %9 offset:32\n\t"
                "ds_read_b128 %3, %9 offset:64\n\t"
                "ds_read_b128 %4, %9 offset:96\n\t"
                "ds_read_b128 %5, %10 offset:0\n\t"
                "ds_read_b128 %6, %10 offset:32\n\t"
                "ds_read_b128 %7, %10 offset:%15\n\t"
                "ds_read_b128 %8, %10 offset:%16\n\t"
                "s_waitcnt lgkmcnt(7)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %1, %11, 0\n\t"
                "s_waitcnt lgkmcnt(6)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %2, %12, %0\n\t"
                "s_waitcnt lgkmcnt(5)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %3, %13, %0\n\t"
                "s_waitcnt lgkmcnt(4)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %4, %14, %0\n\t"
                : "=&v"(S), "=&v"(k0), "=&v"(k1), "=&v"(k2), "=&v"(k3), "=&v"(v0), "=&v"(v1), "=&v"(v2),
                  "=&v"(v3)
                : "v"(ka), "v"(va), "v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]), "n"(2 * 32 * VS),
                  "n"(2 * 32 * VS + 32)
                : "memory");
            asm volatile(
                "s_nop 7\n\t"
                "s_waitcnt lgkmcnt(3)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %2, %6, %0\n\t"
                "s_waitcnt lgkmcnt(2)\n\t"
                "v_mfma_f32_32x32x16_bf16 %0, %3, %7, %0\n\t"
                "s_waitcnt lgkmcnt(1)\n\t"
                "v_mfma_f32_32x32x16_bf16 %1, %4, %6, %1\n\t"
                "s_waitcnt lgkmcnt(0)\n\t"
                "v_mfma_f32_32x32x16_bf16 %1, %5, %7, %1\n\t"
                "s_nop 15\n\t"
                : "+v"(acc_o[0]), "+v"(acc_o[1])
                : "v"(v0), "v"(v1), "v"(v2), "v"(v3), "v"(P[0]), "v"(P[1])
                : "memory");
        }
    };
    // softmax of block b: S -> P, running statistics, rescale of O when the
    // reference maximum moves
    auto softmax = [&](bool masked, int b) {
        if (masked) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int n = 32 * b + 8 * (e >> 2) + 4 * g + (e & 3);
                const bool vis = n < L && (!CAUSAL || n <= qm);
                if (!vis) S[e] = -INFINITY;
            }
        }
        float tmax = S[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, S[e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const bool upd = tmax > m_run + lazy_thr;
        const float m_new = upd ? tmax : m_run;
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        if (__any(upd)) {
            const float alpha = upd ? __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2) : 1.0f;
            l_run *= alpha;
#pragma unroll
            for (int d = 0; d < NDB; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_o[d][e] *= alpha;
        }
        m_run = m_new;
        const float mbias = m_use * scale_log2;
        float psum = 0.f;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            u32x4 pk;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p0 = __builtin_amdgcn_exp2f(S[8 * kk + 2 * e] * scale_log2 - mbias);
                const float p1 = __builtin_amdgcn_exp2f(S[8 * kk + 2 * e + 1] * scale_log2 - mbias);
                psum += p0 + p1;
                pk[e] = pack_bf16(p0, p1);
            }
            P[kk] = __builtin_bit_cast(bf16x8, pk);
        }
        l_run += psum;
    };
    auto softmax_or_skip = [&](int b) {
        if (b < nblk_w) {
            const bool masked = (32 * b + 32 > L) || (CAUSAL && 32 * b + 31 > qrow0);
            softmax(masked, b);
        } else {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) P[kk] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
        }
    };
    // V phases of the two blocks of tile i.  The staging is written without any
    // parity test so that the prefetch registers have one definition per loop
    // trip: K_{i+1} replaces K_{i-1} in the even phase, V_{i+1} replaces V_{i-1}
    // in the odd one, and each new global load lands in the registers just stored.
    auto phase_v_even = [&](int i) {
        softmax_or_skip(2 * i);
        store_k((i + 1) & 1);
        asm volatile("" ::: "memory");
        load_k(i + 2);
    };
    auto phase_v_odd = [&](int i) {
        softmax_or_skip(2 * i + 1);
        store_v((i + 1) & 1);
        asm volatile("" ::: "memory");
        if (v_active) load_v(i + 2);
    };

    // ---- prologue: tile 0 into LDS, tile 1 into the staging registers
    load_k(0);
    if (v_active) load_v(0);
    store_k(0);
    store_v(0);
    load_k(1);
    if (v_active) load_v(1);
    lds_barrier();
    if (grp == 1) lds_barrier();   // the trailing group starts one phase late

#if ORCH_DBG_TIMING
    // debug build only: workgroup 0 of head 0 stamps the shader clock at every
    // phase boundary into the lse buffer (viewed as uint64[8 waves][1024])
    uint64_t *dbg = (uint64_t *)lse + (size_t)wave * 1024;
    int dbg_n = 0;
    const bool dbg_on = blockIdx.x == (unsigned)ORCH_DBG_TIMING - 1 && lane == 0 && lse != nullptr;
#define ORCH_STAMP() do { if (dbg_on && dbg_n < 1024) dbg[dbg_n++] = __builtin_amdgcn_s_memtime(); } while (0)
#else
#define ORCH_STAMP() do { } while (0)
#endif
    for (int i = 0; i < ntile_k; ++i) {
        ORCH_STAMP();
        phase_m(2 * i);
        ORCH_STAMP();
        lds_barrier();
        ORCH_STAMP();
        phase_v_even(i);
        ORCH_STAMP();
        lds_barrier();
        ORCH_STAMP();
        phase_m(2 * i + 1);
        ORCH_STAMP();
        lds_barrier();
        ORCH_STAMP();
        phase_v_odd(i);
        ORCH_STAMP();
        lds_barrier();
    }
    ORCH_STAMP();
    phase_m(nblk);                   // drain: P V of the last block
    if (grp == 0) lds_barrier();   // every wavefront passes the same number of barriers

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    if (qm < L) {
        uint16_t *op = out + ((size_t)(row0 + qm) * Hq + h) * HD;
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x2 w;
                w.x = pack_bf16(acc_o[d][4 * r] * inv, acc_o[d][4 * r + 1] * inv);
                w.y = pack_bf16(acc_o[d][4 * r + 2] * inv, acc_o[d][4 * r + 3] * inv);
                *(u32x2 *)(op + 32 * d + 8 * r + 4 * g) = w;
            }
        if (!ORCH_DBG_TIMING && lse != nullptr && g == 0)
            lse[(size_t)h * total_tokens + row0 + qm] = m_run * scale + __logf(l_tot);
    }
}

}  // namespace

size_t attn_ws_bytes(int32_t batch)
{
    return align_up(sizeof(AttnHdr), 256) + align_up(((size_t)(batch > 0 ? batch : 0) + 1) * 4, 256);
}

int launch_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens, int32_t Hq,
                int32_t Hkv, int32_t d, float scale, int32_t causal, void *ws, size_t ws_bytes,
                hipStream_t stream)
{
    const size_t need = attn_ws_bytes(batch);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_varlen_attn_fwd: workspace %zu < %zu bytes", ws_bytes, need);
    AttnHdr *hdr = (AttnHdr *)ws;
    int32_t *tile_off = (int32_t *)((char *)ws + align_up(sizeof(AttnHdr), 256));
    // Row blocks per wavefront: 2 halves LDS traffic per FLOP but runs one
    // wavefront per SIMD; 1 keeps two.  ORCH_ATTN_MB overrides for tuning runs.
    int MB = 1;
    bool pipe = true;
    if (const char *e = getenv("ORCH_ATTN_MB")) { MB = atoi(e) == 2 ? 2 : 1; pipe = false; }
    const int BM = pipe ? 256 : 128 * MB;
    hipLaunchKernelGGL(attn_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, cu_seqlens, batch,
                       total_tokens, BM, hdr, tile_off, (int32_t *)nullptr);
    const int64_t max_tiles = (int64_t)total_tokens / BM + batch;
    const int64_t grid = max_tiles * Hq;
    if (grid > 0x7fffffffLL) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_fwd: %lld workgroups", (long long)grid);
    if (scale <= 0.f) scale = 1.0f / sqrtf((float)d);
    const float sl2 = scale * 1.4426950408889634f;
    if (grid > 0 && batch > 0) {
#define ORCH_ATTN_ARGS                                                                          \
    (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)out, lse,        \
        cu_seqlens, hdr, tile_off, batch, total_tokens, Hq, Hkv, scale, sl2
#define ORCH_ATTN_LAUNCH(HD_, C_, MB_)                                                           \
    hipLaunchKernelGGL((attn_fwd_kernel<HD_, C_, MB_>), dim3((unsigned)grid), dim3(kThreads), 0, \
                       stream, ORCH_ATTN_ARGS)
#define ORCH_ATTN_LAUNCH_PIPE(HD_, C_)                                                           \
    hipLaunchKernelGGL((attn_fwd_pp_kernel<HD_, C_>), dim3((unsigned)grid), dim3(kPPThreads), 0, \
                       stream, ORCH_ATTN_ARGS)
        const int key = (d == 128 ? 4 : 0) | (causal ? 2 : 0) | (MB == 2 ? 1 : 0);
        if (pipe) {
            if (d == 128 && causal) ORCH_ATTN_LAUNCH_PIPE(128, true);
            else if (d == 128) ORCH_ATTN_LAUNCH_PIPE(128, false);
            else if (causal) ORCH_ATTN_LAUNCH_PIPE(64, true);
            else ORCH_ATTN_LAUNCH_PIPE(64, false);
        } else switch (key) {
        case 0: ORCH_ATTN_LAUNCH(64, false, 1); break;
        case 1: ORCH_ATTN_LAUNCH(64, false, 2); break;
        case 2: ORCH_ATTN_LAUNCH(64, true, 1); break;
        case 3: ORCH_ATTN_LAUNCH(64, true, 2); break;
        case 4: ORCH_ATTN_LAUNCH(128, false, 1); break;
        case 5: ORCH_ATTN_LAUNCH(128, false, 2); break;
        case 6: ORCH_ATTN_LAUNCH(128, true, 1); break;
        default: ORCH_ATTN_LAUNCH(128, true, 2); break;
        }
#undef ORCH_ATTN_LAUNCH
#undef ORCH_ATTN_LAUNCH_PIPE
#undef ORCH_ATTN_ARGS
    }
    set_attn_variant(pipe ? "mfma32x32x16_bm256_pingpong" : MB == 2 ? "mfma32x32x16_bm256_bn64" : "mfma32x32x16_bm128_bn64");
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
