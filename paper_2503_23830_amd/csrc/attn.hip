// orch_varlen_attn_fwd: padding-free attention forward over sequences stored
// back to back (the batching the paper uses for every phase that runs without
// paddings, Sec. 7; the quadratic term of Eq. 2).
//
// Common to both kernels below (head_dim 64: attn_fwd_kernel; head_dim 128:
// attn_fwd_il_kernel, described at its definition): the transposed score
// product, per-lane softmax statistics, and a softmax reference that is fixed in
// the launch every call makes and moves lazily in the rare redo pass.
//
// attn_fwd_kernel: one workgroup (4 wavefronts) owns 128*MB consecutive query rows
// of one sequence and one q-head; each wavefront owns MB blocks of 32 rows.  K/V tiles
// of BN = 64 keys go from global memory into LDS by LDS-DMA (row-major, swizzled; two
// stages, one barrier per tile, the tile loop unrolled by the stages so that fragment
// reads use immediate offsets) and are shared by the four wavefronts; the V^T operand
// of the second product is read from the row-major V tile with transpose reads.  With
// MB = 2 every K/V fragment read from LDS feeds two MFMAs, which halves LDS traffic per FLOP.  The scores are computed transposed,
// S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: in the accumulator layout every
// lane then holds 16 keys of ONE query, so the online-softmax statistics are
// per-lane scalars (one cross-lane exchange per tile), the probabilities are
// already in the B-operand layout of the second product O^T += V^T P^T, and
// rescaling O is a per-lane multiply.  In the moving-reference form the running
// maximum is only moved when a row's maximum grows by more than 2^8 (exact: the
// stale reference cancels in the final division), so O is rarely rescaled after the
// first tile.
#include <algorithm>
#include <type_traits>

#include "attn_tiles.h"
#include "common.h"

namespace orch {
namespace {

constexpr int BN = 64;   // keys per LDS tile
constexpr int kPrepThreads = 1024;

struct AttnHdr {
    int32_t total_tiles;
    int32_t ok;
    int32_t bm;   // query rows per tile the table was built for; a kernel built for another size does nothing
};

// Fixed softmax reference (the form of both kernels that normally runs): every probability of
// a row is taken against the row's maximum over its FIRST 32-key block, which never moves, so
// later blocks compute no maximum and O is never rescaled (the result is the same: the
// reference cancels in the final division, and fp32 carries probabilities up to 2^64 times the
// reference with the same relative precision).  A row whose sum of probabilities does not stay
// below 2^64 marks its (query tile, head) in `redo` and appends it to `redo_list`; the
// moving-reference form of the same code, launched right after with a small grid, walks
// that list (normally empty) and recomputes exactly the marked tiles.
constexpr float kRedoSum = 1.8446744e19f;   // 2^64

// tile_off[t] = number of BM-row query tiles in sequences before t.
// A cu_seqlens that is not non-decreasing inside [0, total_tokens], or a sequence longer than a
// nonzero max_seqlen (the launch was sized for that bound), is a data error: no tile is
// scheduled and dev_status, if given, receives ORCH_EDATA.
__global__ __launch_bounds__(kPrepThreads) void attn_prep_kernel(const int32_t *__restrict__ cu,
                                                                int32_t batch, int32_t total_tokens,
                                                                int32_t max_seqlen, int32_t BM, AttnHdr *hdr,
                                                                int32_t *tile_off, int32_t *dev_status,
                                                                int32_t *redo, int32_t *redo_list, int32_t Hq)
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
        hdr->bm = BM;
        hdr->total_tiles = ok ? part[kPrepThreads - 1] : 0;
        if (ok) tile_off[batch] = part[kPrepThreads - 1];
        if (dev_status) dev_status[0] = ok ? (int32_t)ORCH_OK : (int32_t)ORCH_EDATA;
    }
    // clear the redo marks of every (query tile, head) the attention kernels will visit
    if (redo != nullptr && !s_bad) {
        const int64_t marks = (int64_t)part[kPrepThreads - 1] * Hq;
        for (int64_t i = tid; i < marks; i += kPrepThreads) redo[i] = 0;
    }
    if (redo_list != nullptr && tid == 0) redo_list[0] = 0;   // number of listed tiles
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}


// One (query tile, head) of the grid, named by the workgroup number `bid` it has in the
// fixed-reference launch.  The moving-reference form is driven by the list of marked tiles.
template <int HD, bool CAUSAL, int MB, bool FIXED>
__device__ __forceinline__ void attn_tile(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,
    const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t *__restrict__ redo,
    int32_t *__restrict__ redo_list, int32_t batch, int32_t total_tokens, int32_t Hq, int32_t Hkv, float scale,
    float scale_log2, const int bid)
{
    constexpr int BM = 128 * MB;  // query rows per workgroup
    constexpr int NBLK = 4 * MB;  // 32-row blocks per workgroup
    constexpr int NC = HD / 16;   // 16-wide chunks of the head dimension
    constexpr int NDB = HD / 32;  // 32-row blocks of O^T
    using PS = PairStage<HD>;
    static_assert(BN == kT, "the staged tile pair is 64 keys deep");
    __shared__ __attribute__((aligned(1024))) char lds_raw[PS::BYTES];

    const int total_tiles = hdr->bm == BM ? hdr->total_tiles : 0;
    const int group = Hq / Hkv;

    // block -> (query tile u, head h).  With Hkv a multiple of 8 the kv-head is
    // chosen by blockIdx % 8, i.e. by XCD, so the blocks that share a K/V stream
    // share an L2.
    int u, h;
    {
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

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    PS ps;
    ps.init((uint32_t)(uintptr_t)lds_raw, lane, wave);

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

    // One K/V tile for the row blocks mb >= MB0 of this wavefront (blocks below
    // MB0 lie entirely above the causal diagonal for this tile).
    auto compute_tile = [&](auto mb0_tag, int n0, uint32_t kb, uint32_t vb) {
        constexpr int MB0 = decltype(mb0_tag)::value;
        const bool first = n0 == 0;   // fixed reference: taken here, from the first 32 keys
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
                const bf16x8 kf = ps.rd_row(kb, nb, c);
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
            float mbias;
            if (FIXED) {
                if (first) {   // key 0 is visible to every row, so the maximum is finite
                    float tmax = acc_s[mb][0][0];
#pragma unroll
                    for (int e = 1; e < 16; ++e) tmax = fmaxf(tmax, acc_s[mb][0][e]);
                    m_run[mb] = fmaxf(tmax, __shfl_xor(tmax, 32));
                }
                alpha[mb] = 1.0f;
                mbias = m_run[mb] * scale_log2;
            } else {
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
                mbias = m_use * scale_log2;
            }
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
            l_run[mb] = FIXED ? l_run[mb] + psum : l_run[mb] * alpha[mb] + psum;
        }
        if (!FIXED && __any(any_upd)) {
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
                const bf16x8 vf = ps.rd_tr(vb, 4 * b + kk);  // V^T: head-dim columns 32 b .. + 31, keys 16 kk .. + 15
#pragma unroll
                for (int mb = MB0; mb < MB; ++mb)
                    acc_o[mb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[mb][kk], acc_o[mb][b], 0, 0, 0);
            }
    };

    TileSrc src{k, v, row0, L, 0, Hkv, g_kv};
    ps.begin_at(src, 0);
    // tile `it` lives in stage it % 2; the loop is unrolled by the two stages so that the stage
    // offset of every fragment read is an immediate
    auto tile_step = [&](auto stage_tag, int it) {
        constexpr int ST = decltype(stage_tag)::value;
        const int n0 = it * BN;
        ps.publish();
        if (it + 1 < ntile_k) {
            src.m0 = n0 + BN;
            ps.begin_at(src, ST ^ 1);
        }
        // row blocks entirely above the diagonal have nothing to do in this tile;
        // blk[] ascends with mb, so the active ones are a suffix
        int first = 0;
        if (CAUSAL) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                if (n0 > q0 + 32 * blk[mb] + 31) first = mb + 1;
        }
        if (first == 0) compute_tile(std::integral_constant<int, 0>{}, n0, ps.x_at(ST), ps.y_at(ST));
        else if (MB > 1 && first == 1) compute_tile(std::integral_constant<int, (MB > 1 ? 1 : 0)>{}, n0, ps.x_at(ST), ps.y_at(ST));
    };
    for (int it = 0; it < ntile_k; it += 2) {
        tile_step(std::integral_constant<int, 0>{}, it);
        if (it + 1 < ntile_k) tile_step(std::integral_constant<int, 1>{}, it + 1);
    }

    // ---- epilogue
    bool bad = false;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float l_tot = l_run[mb] + __shfl_xor(l_run[mb], 32);
        const float inv = 1.f / l_tot;
        if (FIXED) bad |= !(l_tot < kRedoSum);   // rows past the end were computed on the clamped last row
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
    // a sum that did not stay below 2^64 (or is not a number): the moving-reference pass redoes the tile
    // (the first wavefront of the workgroup to find one appends the tile to the list)
    if (FIXED && __any(bad) && lane == 0 && atomicExch(&redo[u * Hq + h], 1) == 0)
        redo_list[1 + atomicAdd(&redo_list[0], 1)] = bid;
}

#define ORCH_ATTN_PARAMS                                                                                       \
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,            \
        uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,                   \
        const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t *__restrict__ redo,     \
        int32_t *__restrict__ redo_list, int32_t batch, int32_t total_tokens, int32_t Hq, int32_t Hkv,         \
        float scale, float scale_log2
#define ORCH_ATTN_NAMES q, k, v, out, lse, cu, hdr, tile_off, redo, redo_list, batch, total_tokens, Hq, Hkv, scale, scale_log2

// the launch every call makes: fixed reference, one workgroup per (query tile, head)
template <int HD, bool CAUSAL, int MB>
__global__ __launch_bounds__(kThreads, (MB * HD > 128 ? 1 : (MB * HD > 64 ? 2 : 4))) void attn_fwd_kernel(ORCH_ATTN_PARAMS)
{
    attn_tile<HD, CAUSAL, MB, true>(ORCH_ATTN_NAMES, (int)blockIdx.x);
}

// the moving-reference pass: a small grid walks the list of marked tiles (normally empty)
template <int HD, bool CAUSAL, int MB>
__global__ __launch_bounds__(kThreads, (MB * HD > 128 ? 1 : (MB * HD > 64 ? 2 : 4))) void attn_fwd_redo_kernel(ORCH_ATTN_PARAMS)
{
    const int count = redo_list[0];
    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        attn_tile<HD, CAUSAL, MB, false>(ORCH_ATTN_NAMES, redo_list[1 + item]);
        __syncthreads();   // the LDS stages are reused by the next tile
    }
}


// ---------------------------------------------------------------------------
// Interleaved variant (head_dim 128): 8 wavefronts (two per SIMD) own 32 query
// rows each.  No vector register ever stages K or V:
//   * K and V blocks (32 keys x 256 B) go from global memory straight into LDS
//     with 16-byte LDS-DMA loads.  A wave-wide load fills 1 KB of LDS in lane
//     order, so bank conflicts are avoided by choosing WHICH 16-byte chunk of a
//     row each lane fetches: row r keeps chunk c at slot c ^ swz(r).
//       K: swz = r & 15              (A-operand reads: 16 rows, same chunk)
//       V: swz = 4 (r & 3) + 2 ((r >> 2) & 1)   (transpose reads: 4 rows x 64 B)
//   * V is consumed by ds_read_b64_tr_b16, which hands a lane four keys of one
//     head-dim column from row-major [key][dim] storage: in a 16-lane block,
//     lane i receives element i%4 of the 8-byte words addressed by lanes
//     i/4, 4 + i/4, 8 + i/4, 12 + i/4.  Two such reads are the A operand of
//     O^T += V^T P^T for the keys a lane's P registers hold.
// Eight-stage rings of 32-key blocks for K and V (128 KB of LDS), block b in stage
// b % 8; the workgroup meets at a barrier every four blocks, and what an interval of
// four blocks reads was requested during the interval before it (see `block` below).
// The block loop is unrolled by the ring depth, so every fragment read is a fixed
// lane address plus an immediate offset.  The LDS-DMA unit is shared by the workgroup
// and a wavefront stalls at issue while it is busy, so a wavefront's loads are spread
// over the iterations that issue them, two per half.
//
// Each wavefront software-pipelines over 32-key blocks b.  Iteration b issues
//     half 1:  O^T   += V(b-1)^T P(b-1) 8 MFMAs | (moving reference only: row maxima
//                                                 of S(b)) exp of its keys 0..15
//     half 2:  S(b+1) = K(b+1) Q^T      8 MFMAs | exp of S(b), keys 16..31
// with the vector-ALU work cut into pieces that sit between consecutive MFMAs,
// so the matrix core and the vector ALU of a SIMD are busy at the same time
// within one instruction stream; the second wavefront of the SIMD fills what
// stalls remain.  P is single-buffered: its first chunk is rewritten in the
// second part of half 1, after the four MFMAs that read the old one, its second
// chunk in half 2.  LDS fragments are single-buffered in registers too: fragment j
// of K(b+1) is requested right after MFMA j of half 1 (its register was last read by
// MFMA j of the previous half 2), the fragments of V(b) likewise during half 2.
// Reference maximum: fixed (the row's maximum over block 0, taken in the prologue) in
// the launch every call makes; in the redo pass lazy (moves only on growth > 2^8), and
// the factor alpha_b that carries O and l from the reference of block b-1 to that of
// block b is applied at the end of iteration b: O has received P(b-1) V(b-1) and not
// yet P(b) V(b).
// ---------------------------------------------------------------------------
constexpr int kILThreads = 512;

#define ORCH_SB() __builtin_amdgcn_sched_barrier(0)

// FIXED: fixed softmax reference (see kRedoSum above); its row maximum over block 0 is taken in
// the prologue, so every block of the tile loop runs the same code without maxima.
// One (query tile, head) of the grid, named by the workgroup number `bid` it has in the
// fixed-reference launch.  The moving-reference form is driven by the list of marked tiles.
template <int HD, bool CAUSAL, bool FIXED>
__device__ __forceinline__ void attn_il_tile(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,
    const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t *__restrict__ redo,
    int32_t *__restrict__ redo_list, int32_t batch, int32_t total_tokens, int32_t Hq, int32_t Hkv, float scale,
    float scale_log2, const int bid)
{
    static_assert(HD == 128, "layout constants below assume 256-byte rows");
    constexpr int BM = 256;
    constexpr int NC = HD / 16;    // k-chunks of Q K^T
    constexpr int NDB = HD / 32;   // 32-row blocks of O^T
    constexpr int ROWB = HD * 2;   // bytes per key row
    constexpr int TILE_B = BN * ROWB;
    constexpr int KST = 4, VST = 4;   // ring depths (K is requested three tiles ahead, V two); the tile
                                      // loop is unrolled by the depth so that stage offsets are immediates
    __shared__ __attribute__((aligned(1024))) char lds_raw[(KST + VST) * TILE_B];
    const uint32_t lds_k = (uint32_t)(uintptr_t)lds_raw;
    const uint32_t lds_v = lds_k + KST * TILE_B;

    const int total_tiles = hdr->bm == BM ? hdr->total_tiles : 0;
    const int group = Hq / Hkv;
    int u, h;
    {
        if ((Hkv & 7) == 0) {   // kv-head chosen by XCD: blocks sharing K/V share an L2
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
    const int qt = ntile_q - 1 - (u - tile_off[seq]);  // heaviest (last) tile first
    const int q0 = qt * BM;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // waves w and w+4 share a SIMD; row blocks w and 7-w even out the causal work per SIMD
    const int rblk = wave < 4 ? wave : 11 - wave;
    const int qrow0 = q0 + 32 * rblk;
    const int qm = qrow0 + l32;

    const int kend = CAUSAL ? min(L, q0 + BM) : L;
    const int nblk_wg = (kend + 31) / 32;                   // 32-key blocks the workgroup stages
    const int kend_w = CAUSAL ? min(L, qrow0 + 32) : L;
    const int nblk_w = qrow0 < L ? (kend_w + 31) / 32 : 0;  // 32-key blocks this wavefront computes

    // ---- LDS-DMA: per 32-key block this wavefront fetches rows 4w..4w+3 of K and of V (one load
    // each); lane -> (row, slot), slot -> chunk by the swizzle.  Block b of either tensor lives in
    // ring stage b % 8 (8 KB per stage).
    constexpr int BLK_B = 32 * ROWB;
    constexpr int NSTG = 8;
    static_assert(KST * TILE_B == NSTG * BLK_B && VST * TILE_B == NSTG * BLK_B, "ring size");
    const uint32_t rstride_b = (uint32_t)Hkv * HD * 2;
    const char *kseq = (const char *)(k + ((size_t)row0 * Hkv + g_kv) * HD);
    const char *vseq = (const char *)(v + ((size_t)row0 * Hkv + g_kv) * HD);
    // per-lane byte offset of the 16 bytes this lane fetches, relative to the block's first row:
    // [0] for blocks inside the sequence, [1] for the last block this workgroup stages, whose rows
    // past the end repeat row L-1 (they are masked later)
    uint32_t dma_off[2][2];
    {
        const int lrem_last = L - 1 - (nblk_wg - 1) * 32;
        const int r = 4 * wave + (lane >> 4);
        const int slot = lane & 15;
#pragma unroll
        for (int is_v = 0; is_v < 2; ++is_v) {
            const int swz = is_v ? 4 * (r & 3) + 2 * ((r >> 2) & 1) : (r & 15);
            const uint32_t col = 16u * (uint32_t)(slot ^ swz);
            dma_off[0][is_v] = __umul24((uint32_t)r, rstride_b) + col;
            dma_off[1][is_v] = __umul24((uint32_t)min(r, lrem_last), rstride_b) + col;
        }
    }
    // One LDS-DMA load: 64 lanes x 16 bytes from block base `tb` (scalar) + per-lane offset into
    // 1 KB of LDS at `dst`.  Written as asm so that the compiler does not tie later LDS reads
    // (of other stages) to this load with a vmcnt(0); completion is waited for explicitly
    // before the barrier.  M0 = LDS destination of lane 0 (declared as clobbered).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // M0 is reserved; the clobber is deliberate
    auto dma_issue = [&](const char *tb, uint32_t off, uint32_t dst) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(dst), "v"(off), "s"(tb) : "memory", "m0");
    };
#pragma clang diagnostic pop
    struct DmaJob {
        const char *tb;     // first row of the block
        uint32_t off;       // this lane's offset
        uint32_t dst;       // this wavefront's 1 KB of the block's ring stage
    };
    auto dma_job = [&](int blk, bool is_v) {
        const int bc = blk < nblk_wg ? blk : nblk_wg - 1;   // past the end: repeat the last block
        const bool last = bc == nblk_wg - 1;
        DmaJob j;
        j.tb = (is_v ? vseq : kseq) + (size_t)bc * 32 * rstride_b;
        j.off = last ? dma_off[1][is_v] : dma_off[0][is_v];
        j.dst = (is_v ? lds_v : lds_k) + (uint32_t)(blk & (NSTG - 1)) * BLK_B + (uint32_t)wave * 1024u;
        return j;
    };
    auto dma_run = [&](const DmaJob &j) { dma_issue(j.tb, j.off, j.dst); };
    auto dma_block = [&](int blk, bool is_v) { dma_run(dma_job(blk, is_v)); };
    // the loads a wavefront issues during block b of an interval of four blocks (between two
    // workgroup barriers): everything the NEXT interval reads, requested in its first two blocks
    struct DmaSet {
        DmaJob j[4];
        bool on;   // the next interval exists
    };
    auto dma_set = [&](int b) {
        const int q = b & 3, i4 = b - q;   // block q of the interval that starts at block i4
        DmaSet s;
        s.on = i4 + 4 < nblk_wg;
        // interval I reads K blocks 4I+1 .. 4I+4 and V blocks 4I .. 4I+3
        s.j[0] = dma_job(i4 + 5 + 2 * q, false);
        s.j[1] = dma_job(i4 + 6 + 2 * q, false);
        s.j[2] = dma_job(i4 + 4 + 2 * q, true);
        s.j[3] = dma_job(i4 + 5 + 2 * q, true);
        return s;
    };

    // ---- per-lane LDS addresses of the fragments (stage 0, first 32-key block)
    // K, A operand of MFMA j: row l32, chunk (2j+g) ^ (l32 & 15)
    uint32_t kaddr[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) kaddr[j] = lds_k + (uint32_t)(l32 * ROWB + 16 * ((2 * j + g) ^ (l32 & 15)));
    // V, transpose read for O block db: this lane addresses key row 4g + j4 (j4 = (lane%16)/4) and
    // the 8 bytes of columns 32 db + 16 half + 4 a .. +3 (half = (lane/16)%2, a = lane%4).  The
    // swizzle of that row is 4 j4 + 2 g for every block and chunk.
    uint32_t vaddr[NDB];
    {
        const int j4 = (lane & 15) >> 2, a = lane & 3, half = (lane >> 4) & 1;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int c = (4 * db + 2 * half + (a >> 1)) ^ (4 * j4 + 2 * g);
            vaddr[db] = lds_v + (uint32_t)((4 * g + j4) * ROWB + 16 * c + 8 * (a & 1));
        }
    }

    // ---- Q fragments: B operand, column m = lane%32, k = 16c + 8g + [0..7]
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

    f32x16 S[2];     // scores of blocks b (current) and b+1 (next), by parity
    bf16x8 P[2];     // probabilities, two 16-key chunks: block b-1 until rewritten for block b
    bf16x8 kf[NC], vf[2 * NDB];
    float alpha = 1.f, mbias = 0.f, psum = 0.f;
    bool moved = false;

    auto lds_rd128 = [](uint32_t addr, int off) {
        return *(const __attribute__((address_space(3))) bf16x8 *)(uintptr_t)(addr + (uint32_t)off);
    };
    auto lds_rd_tr = [](uint32_t addr, int off) {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(addr + (uint32_t)off));
    };
    // fragment reads; `off` = stage * TILE_B + (row offset of the block in its tile) * ROWB, an immediate
    auto read_k1 = [&](int j, int off) { kf[j] = lds_rd128(kaddr[j], off); };
    auto read_k = [&](int off) {
#pragma unroll
        for (int j = 0; j < NC; ++j) read_k1(j, off);
    };
    // V fragments: chunk kk (16 keys), O block db: keys 16kk + 4g + [0..3] and 16kk + 8 + 4g + [0..3]
    auto read_v1 = [&](int db, int kk, int off) {
        const s16x4 lo4 = lds_rd_tr(vaddr[db], off + (16 * kk) * ROWB);
        const s16x4 hi4 = lds_rd_tr(vaddr[db], off + (16 * kk + 8) * ROWB);
        const s16x8 both = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        vf[2 * db + kk] = __builtin_bit_cast(bf16x8, both);
    };
    auto read_v = [&](int off) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) read_v1(db, kk, off);
    };
    // keys of block b beyond the sequence or above the diagonal get -inf
    auto mask_block = [&](f32x16 &Sx, int b) {
        const bool masked = (32 * b + 32 > L) || (CAUSAL && 32 * b + 31 > qrow0);
        if (masked) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int n = 32 * b + 8 * (e >> 2) + 4 * g + (e & 3);
                const bool vis = n < L && (!CAUSAL || n <= qm);
                if (!vis) Sx[e] = -INFINITY;
            }
        }
    };
    // Row maximum of a block and the (lazy) reference it is exponentiated against, in three
    // pieces that fit between MFMAs.  Trees, not chains: the instructions of a piece are
    // independent of one another, so the wavefront does not stall on its own results.
    // (maxima as instructions: the scores are never NaN here, so the canonicalising copies
    // the compiler adds around fmaxf are not wanted)
    auto vmax3 = [](float a, float b, float c) {
        float r;
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
        return r;
    };
    auto vmax2 = [](float a, float b) {
        float r;
        asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
        return r;
    };
    float tm[5];
    auto max_a = [&](const f32x16 &Sx) {
#pragma unroll
        for (int i = 0; i < 5; ++i) tm[i] = vmax3(Sx[3 * i], Sx[3 * i + 1], Sx[3 * i + 2]);
        asm volatile("" : "+v"(tm[0]), "+v"(tm[1]), "+v"(tm[2]), "+v"(tm[3]), "+v"(tm[4]));
    };
    auto max_b = [&](const f32x16 &Sx) {
        const float u0 = vmax3(tm[0], tm[1], tm[2]);
        const float u1 = vmax3(tm[3], tm[4], Sx[15]);
        float tmax = vmax2(u0, u1);
        {   // the other half of the row lives in lane ^ 32
            const uint32_t tb = __float_as_uint(tmax);
            const auto sw = __builtin_amdgcn_permlane32_swap(tb, tb, false, false);
            tmax = vmax2(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        asm volatile("" : "+v"(tmax));
        tm[0] = tmax;
    };
    auto max_c = [&]() {
        const float tmax = tm[0];
        const bool upd = FIXED || tmax > m_run + lazy_thr;   // FIXED: called once, for block 0
        const float m_new = upd ? tmax : m_run;
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        alpha = upd ? __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2) : 1.0f;
        moved = __any(upd);
        m_run = m_new;
        mbias = m_use * scale_log2;
        asm volatile("" : "+v"(mbias), "+v"(alpha));
    };
    // The 16 exponentials of the current block as a four-stage pipeline over "ticks" (one tick
    // per MFMA slot): element e enters at tick(e); A: x = S*c - m, B (next tick): p = 2^x,
    // C (tick after): sum += p, D (with C of the odd element): pack the pair to bf16 into P.
    // A tick's instructions belong to different elements, so none waits for another.  Elements
    // 0..7 enter two per tick (ticks 0..3), elements 8..15 one per tick (ticks 4..11); ticks 12
    // and 13 drain.  The empty asm pins a tick's results where the tick is written (between two
    // MFMAs): they must exist there, so the work cannot sink to where P is consumed.
    float xs[16], ps[16];
    auto tick_of = [](int e) { return e < 8 ? e / 2 : e - 4; };
    auto exp_tick = [&](const f32x16 &Sc, int t) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int te = tick_of(e);
            if (te == t) {   // A
                xs[e] = Sc[e] * scale_log2 - mbias;
                asm volatile("" : "+v"(xs[e]));
            }
            if (te + 1 == t) {   // B
                ps[e] = __builtin_amdgcn_exp2f(xs[e]);
                asm volatile("" : "+v"(ps[e]));
            }
            if (te + 2 == t) {   // C, and D for a completed pair
                psum += ps[e];
                if (e & 1) {
                    uint32_t pk = pack_bf16(ps[e - 1], ps[e]);
                    asm volatile("" : "+v"(pk), "+v"(psum));
                    u32x4 w = __builtin_bit_cast(u32x4, P[e >> 3]);
                    w[(e & 7) >> 1] = pk;
                    P[e >> 3] = __builtin_bit_cast(bf16x8, w);
                }
            }
        }
    };
    // Fixed reference: the same pipeline laid out EVENLY, one element entering per MFMA slot.  Slot
    // g = 0..15 of iteration b (half 1: g = j, half 2: g = 8 + j) holds stage A of element g - 2 of
    // block b, stage B of element g - 3 and stage C/D of element g - 4; the last elements of a
    // block run over into the next iteration: stage A of elements 14, 15 of block b-1 sits in its
    // slots 0, 1, their stage B in slots 1, 2 (element 13: slot 0), stage C/D of elements 12..15 in
    // slots 0..3.  Every slot then carries one fma, one exp2, one add and half a pack (24-28
    // vector-ALU cycles against the 32 of its MFMA) instead of 40-52 cycles in the first slots and
    // 8-28 in the last ones.  P's chunk 0 (elements 0..7) is complete by slot 12, its chunk 1 by
    // slot 3 of the next iteration: before the MFMAs that read them (slots 0..3 and 4..7 of half 1).
    // The row sum goes straight into l_run.
    auto even_items = [&](const f32x16 &Sx, int ea, int eb, int ec) {
        if (ea >= 0 && ea < 16) {   // A
            xs[ea] = Sx[ea] * scale_log2 - mbias;
            asm volatile("" : "+v"(xs[ea]));
        }
        if (eb >= 0 && eb < 16) {   // B
            ps[eb] = __builtin_amdgcn_exp2f(xs[eb]);
            asm volatile("" : "+v"(ps[eb]));
        }
        if (ec >= 0 && ec < 16) {   // C, and D for a completed pair
            l_run += ps[ec];
            if (ec & 1) {
                uint32_t pk = pack_bf16(ps[ec - 1], ps[ec]);
                asm volatile("" : "+v"(pk), "+v"(l_run));
                u32x4 w = __builtin_bit_cast(u32x4, P[ec >> 3]);
                w[(ec & 7) >> 1] = pk;
                P[ec >> 3] = __builtin_bit_cast(bf16x8, w);
            }
        }
    };
    auto even_tick = [&](const f32x16 &Sc, const f32x16 &Sp, int g) {
        even_items(Sc, g - 2, g - 3, g - 4);       // block b
        even_items(Sp, g + 14, g + 13, g + 12);    // block b-1 (slots 0..3 only)
    };
    auto mfma = [](const bf16x8 &a, const bf16x8 &b, const f32x16 &c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    };

    // one pipeline iteration for block b of parity PAR: S[PAR] holds S(b), P holds P(b-1),
    // vf holds V(b-1)
    // The LDS-DMA unit is shared by the workgroup and a wavefront stalls at issue while it is
    // busy, so the four loads of a block (blocks 0 and 1 of an interval have them) are spread
    // over the iteration: two in each half.
    auto body = [&](auto bs_c, int b, const DmaSet &ds) {
        constexpr int BS = decltype(bs_c)::value;   // ring stage of block b (= b % 8)
        constexpr int PAR = BS & 1;
        constexpr bool LOADS = (BS & 3) < 2;
        // A block's maximum is computed only with a moving reference (the fixed one comes from
        // block 0 in the prologue).  Without it the exponentials start two slots into half 1 (chunk
        // 0 of P is rewritten from tick 2 on, after MFMAs 0..3 have read it) and end with half 2.
        constexpr bool WITH_MAX = !FIXED;
        constexpr int T0 = WITH_MAX ? 4 : 2;        // half-1 slot of tick 0
        // ring stages of K(b+1) and V(b)
        constexpr int K_OFF = ((BS + 1) % NSTG) * BLK_B;
        constexpr int V_OFF = BS * BLK_B;
        f32x16 &Sc = S[PAR];
        f32x16 &Sn = S[PAR ^ 1];
        psum = 0.f;
        // ---- half 1: O^T += V(b-1)^T P(b-1); maxima of S(b); exp of keys 0..15
#pragma unroll
        for (int j = 0; j < 2 * NDB; ++j) {
            const int db = j % NDB, kk = j / NDB;
            acc_o[db] = mfma(vf[2 * db + kk], P[kk], acc_o[db]);
            ORCH_SB();
            // K(b+1), one fragment per slot (odd half of this tile, or even half of the next
            // one); the MFMA that last read kf[j] was issued in the previous half 2
            read_k1(j, K_OFF);
            ORCH_SB();
            if (j == 0) mask_block(Sc, b);
            if (WITH_MAX && j == 1) max_a(Sc);
            if (WITH_MAX && j == 2) max_b(Sc);
            if (WITH_MAX && j == 3) max_c();
            // chunk 0 of P is rewritten from tick 2 on: MFMAs 0..3 have read it by then
            if (FIXED) even_tick(Sc, Sn, j);   // Sn still holds S(b-1) during half 1
            else if (j >= T0) exp_tick(Sc, j - T0);
            if (LOADS && j == 2 && ds.on) dma_run(ds.j[0]);
            if (LOADS && j == 6 && ds.on) dma_run(ds.j[1]);
            ORCH_SB();
        }
        // ---- half 2: S(b+1) = K(b+1) Q^T; exp of keys 16..31
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            if (j == 0) {
                f32x16 z;
#pragma unroll
                for (int e = 0; e < 16; ++e) z[e] = 0.f;
                Sn = mfma(kf[0], qf[0], z);
            } else {
                Sn = mfma(kf[j], qf[j], Sn);
            }
            ORCH_SB();
            // V(b), the fragment that MFMA j of the next half 1 reads
            read_v1(j % NDB, j / NDB, V_OFF);
            ORCH_SB();
            if (FIXED) even_tick(Sc, Sc, 8 + j);   // (no element of block b-1 is left by now)
            else exp_tick(Sc, 8 - T0 + j);
            if (LOADS && j == 2 && ds.on) dma_run(ds.j[2]);
            if (LOADS && j == 6 && ds.on) dma_run(ds.j[3]);
            ORCH_SB();
        }
        if (WITH_MAX) {
            exp_tick(Sc, 12);
            exp_tick(Sc, 13);
        }
        if (FIXED) return;   // (the row sum went into l_run as it was formed)
        // ---- carry O and l to the reference of block b (rarely != 1), add this block's sum
        if (moved) {
#pragma unroll
            for (int d = 0; d < NDB; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_o[d][e] *= alpha;
        }
        l_run = l_run * alpha + psum;
    };

    // ---- prologue: what interval 0 reads (K blocks 0..4, V blocks 0..3); S(0); V(0) fragments
    // meet P = 0.  (Block indices past the end are clamped: the copy lands in a stage whose
    // contents are masked or never read.)
#pragma unroll
    for (int blk = 0; blk < 5; ++blk) dma_block(blk, false);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) dma_block(blk, true);
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wavefront's DMA has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) P[kk] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
    if (FIXED) {
        // "block -1", whose last pipeline stages sit in the first slots of iteration 0: all zeros
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            S[1][e] = -INFINITY;
            xs[e] = -INFINITY;
            ps[e] = 0.f;
        }
    }
    if (nblk_w > 0) {
        read_k(0);
        read_v(0);
        f32x16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        S[0] = mfma(kf[0], qf[0], z);
#pragma unroll
        for (int j = 1; j < NC; ++j) S[0] = mfma(kf[j], qf[j], S[0]);
        if (FIXED) {   // the row's reference: its maximum over block 0 (key 0 is visible to every row)
            // the maxima are asm statements, for which the compiler adds no MFMA-result wait
            // states: let the last product retire first (in the tile loop the distance is there
            // by construction)
            ORCH_SB();
            asm volatile("s_nop 15\n\ts_nop 15");
            ORCH_SB();
            mask_block(S[0], 0);
            max_a(S[0]);
            max_b(S[0]);
            max_c();
        }
    }
    // K block 0 is the one block that is read outside the interval scheme (just above), and the
    // last requests of interval 0 reuse its stage: every wavefront has it in registers (its
    // products are issued) before anybody goes on
    __builtin_amdgcn_s_barrier();

    // One 32-key block whose ring stage BS = b % 8 is a compile-time constant.  The workgroup
    // meets at a barrier every FOUR blocks: interval I (blocks 4I .. 4I+3) reads K blocks 4I+1 ..
    // 4I+4 (the scores run one block ahead) and V blocks 4I .. 4I+3, all requested during interval
    // I-1 and waited for (vmcnt(0)) before its barrier; its own requests, K blocks 4I+5 .. 4I+8
    // and V blocks 4I+4 .. 4I+7, replace K blocks 4I-3 .. 4I and V blocks 4I-4 .. 4I-1, which nobody
    // reads any more once everybody has passed that barrier.
    auto block = [&](auto bs_c, int b) {
        constexpr int BS = decltype(bs_c)::value;
        if ((BS & 3) == 0 && b > 0) {
            __builtin_amdgcn_s_waitcnt(0x0f70);
            __builtin_amdgcn_s_barrier();
        }
        const DmaSet ds = dma_set(b);
        if (b < nblk_w) {
            body(bs_c, b, ds);
        } else if ((BS & 3) < 2 && ds.on) {   // a wavefront past its causal range still feeds the ring
#pragma unroll
            for (int i = 0; i < 4; ++i) dma_run(ds.j[i]);
        }
    };
    for (int b0 = 0; b0 < nblk_wg; b0 += NSTG) {
        block(std::integral_constant<int, 0>{}, b0);
        if (b0 + 1 < nblk_wg) block(std::integral_constant<int, 1>{}, b0 + 1);
        if (b0 + 2 < nblk_wg) block(std::integral_constant<int, 2>{}, b0 + 2);
        if (b0 + 3 < nblk_wg) block(std::integral_constant<int, 3>{}, b0 + 3);
        if (b0 + 4 < nblk_wg) block(std::integral_constant<int, 4>{}, b0 + 4);
        if (b0 + 5 < nblk_wg) block(std::integral_constant<int, 5>{}, b0 + 5);
        if (b0 + 6 < nblk_wg) block(std::integral_constant<int, 6>{}, b0 + 6);
        if (b0 + 7 < nblk_wg) block(std::integral_constant<int, 7>{}, b0 + 7);
    }
    // ---- drain: O^T += V(B-1)^T P(B-1) for the wavefront's last block; both are in registers
    // (fixed reference: after the pipeline stages of its last elements, which no further
    // iteration carries)
    if (nblk_w > 0) {
        if (FIXED) {
            auto flush = [&](const f32x16 &Sl) {
#pragma unroll
                for (int g = 16; g < 20; ++g) even_items(Sl, g - 2, g - 3, g - 4);
            };
            if ((nblk_w - 1) & 1) flush(S[1]);
            else flush(S[0]);
        }
#pragma unroll
        for (int j = 0; j < 2 * NDB; ++j) {
            const int db = j % NDB, kk = j / NDB;
            acc_o[db] = mfma(vf[2 * db + kk], P[kk], acc_o[db]);
        }
    }

    // ---- epilogue
    float l_tot;
    {
        const uint32_t lb = __float_as_uint(l_run);
        const auto sw = __builtin_amdgcn_permlane32_swap(lb, lb, false, false);
        l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = 1.f / l_tot;
    if (FIXED) {
        // a sum that did not stay below 2^64 (or is not a number): the moving-reference pass redoes the tile
        // (the first wavefront of the workgroup to find one appends the tile to the list)
        if (__any(!(l_tot < kRedoSum)) && lane == 0 && atomicExch(&redo[u * Hq + h], 1) == 0)
            redo_list[1 + atomicAdd(&redo_list[0], 1)] = bid;
    }
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
        if (lse != nullptr && g == 0)
            lse[(size_t)h * total_tokens + row0 + qm] = m_run * scale + __logf(l_tot);
    }
}

#undef ORCH_SB

// the launch every call makes: fixed reference, one workgroup per (query tile, head)
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(kILThreads) void attn_fwd_il_kernel(ORCH_ATTN_PARAMS)
{
    attn_il_tile<HD, CAUSAL, true>(ORCH_ATTN_NAMES, (int)blockIdx.x);
}

// the moving-reference pass: a small grid walks the list of marked tiles (normally empty)
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(kILThreads) void attn_fwd_il_redo_kernel(ORCH_ATTN_PARAMS)
{
    const int count = redo_list[0];
    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        attn_il_tile<HD, CAUSAL, false>(ORCH_ATTN_NAMES, redo_list[1 + item]);
        __syncthreads();   // the LDS rings are reused by the next tile
    }
}
#undef ORCH_ATTN_PARAMS
#undef ORCH_ATTN_NAMES

}  // namespace

// workspace: header, tile_off[batch + 1], redo[(query tiles) * Hq] (one mark per workgroup),
// redo_list[1 + marks] (count, then the marked workgroup numbers)
static size_t attn_max_tiles(int32_t batch, int32_t total_tokens)
{
    return (size_t)(total_tokens > 0 ? total_tokens : 0) / 128 + (size_t)(batch > 0 ? batch : 0);
}

size_t attn_ws_bytes(int32_t batch, int32_t total_tokens, int32_t Hq)
{
    const size_t marks = attn_max_tiles(batch, total_tokens) * (size_t)(Hq > 0 ? Hq : 0);
    return align_up(sizeof(AttnHdr), 256) + align_up(((size_t)(batch > 0 ? batch : 0) + 1) * 4, 256) +
           align_up(marks * 4, 256) + align_up((marks + 1) * 4, 256);
}

int launch_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                int32_t Hq, int32_t Hkv, int32_t d, float scale, int32_t causal, int32_t *dev_status,
                void *ws, size_t ws_bytes, hipStream_t stream)
{
    const size_t need = attn_ws_bytes(batch, total_tokens, Hq);
    if (ws_bytes < need) ORCH_FAIL(ORCH_ENOSPC, "orch_varlen_attn_fwd: workspace %zu < %zu bytes", ws_bytes, need);
    AttnHdr *hdr = (AttnHdr *)ws;
    int32_t *tile_off = (int32_t *)((char *)ws + align_up(sizeof(AttnHdr), 256));
    int32_t *redo = (int32_t *)((char *)tile_off + align_up(((size_t)(batch > 0 ? batch : 0) + 1) * 4, 256));
    int32_t *redo_list = (int32_t *)((char *)redo + align_up(attn_max_tiles(batch, total_tokens) * (size_t)Hq * 4, 256));
    // head_dim 128: the 8-wavefront kernel with LDS-DMA staging and MFMA / vector-ALU work
    // interleaved in one instruction stream, first with a fixed softmax reference, then (same
    // grid; returns at once unless a tile was marked) with a moving one.  head_dim 64: half the
    // MFMA work per softmax, so the vector ALU dominates and the simpler 4-wavefront kernel with
    // one or two row blocks per wavefront is used.
    const bool il = d == 128;
    // Row blocks per wavefront of the head_dim-64 kernel launched below (the tile table the prep
    // kernel builds and the grid use the same rows per workgroup; a kernel built for another
    // size finds the mismatch in the header and does nothing).  Bidirectional (the encoder
    // phases: sequences of a few hundred rows): one block, 128-row tiles, four workgroups per CU,
    // whose phases overlap; measured 810 against 720-750 TFLOP/s (C2) and 616 against 543 (C3) for
    // two blocks.  Causal keeps two blocks (the diagonal balances over block pairs).
    const int mb64 = (!il && !causal) ? 1 : 2;
    const int BM = il ? 256 : 128 * mb64;   // query rows per workgroup
    hipLaunchKernelGGL(attn_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, cu_seqlens, batch,
                       total_tokens, max_seqlen, BM, hdr, tile_off, dev_status, redo, redo_list, Hq);
    // sum over sequences of ceil(L / BM) <= total / BM + batch, and <= batch * ceil(max_seqlen / BM)
    int64_t max_tiles = (int64_t)total_tokens / BM + batch;
    if (max_seqlen > 0) max_tiles = std::min<int64_t>(max_tiles, (int64_t)batch * ((max_seqlen + BM - 1) / BM));
    const int64_t grid = max_tiles * Hq;
    // (a launch of 2^32 threads or more in all is cut short by the runtime without an error)
    if (grid > 0x7fffffffLL || grid * (il ? kILThreads : kThreads) > 0xffffffffLL)
        ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_fwd: %lld workgroups", (long long)grid);
    if (scale <= 0.f) scale = 1.0f / sqrtf((float)d);
    const float sl2 = scale * 1.4426950408889634f;
    if (grid > 0 && batch > 0) {
#define ORCH_ATTN_HEAD (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)out, lse, cu_seqlens, hdr, tile_off
#define ORCH_ATTN_TAIL batch, total_tokens, Hq, Hkv, scale, sl2
        const dim3 g((unsigned)grid);
        // the redo pass: a small grid walks the list of marked tiles (launching the full grid of
        // 128 KB workgroups only to find nothing marked cost 130 us on C4)
        const dim3 gr((unsigned)std::min<int64_t>(grid, il ? 256 : 1024));
#define ORCH_ATTN_LAUNCH(FAST_, REDO_, THREADS_)                                                                      \
    do {                                                                                                              \
        hipLaunchKernelGGL((FAST_), g, dim3(THREADS_), 0, stream, ORCH_ATTN_HEAD, redo, redo_list, ORCH_ATTN_TAIL);  \
        hipLaunchKernelGGL((REDO_), gr, dim3(THREADS_), 0, stream, ORCH_ATTN_HEAD, redo, redo_list, ORCH_ATTN_TAIL); \
    } while (0)
        if (il && causal) ORCH_ATTN_LAUNCH((attn_fwd_il_kernel<128, true>), (attn_fwd_il_redo_kernel<128, true>), kILThreads);
        else if (il) ORCH_ATTN_LAUNCH((attn_fwd_il_kernel<128, false>), (attn_fwd_il_redo_kernel<128, false>), kILThreads);
        else if (mb64 == 1) ORCH_ATTN_LAUNCH((attn_fwd_kernel<64, false, 1>), (attn_fwd_redo_kernel<64, false, 1>), kThreads);
        else if (causal) ORCH_ATTN_LAUNCH((attn_fwd_kernel<64, true, 2>), (attn_fwd_redo_kernel<64, true, 2>), kThreads);
        else ORCH_ATTN_LAUNCH((attn_fwd_kernel<64, false, 2>), (attn_fwd_redo_kernel<64, false, 2>), kThreads);
#undef ORCH_ATTN_LAUNCH
#undef ORCH_ATTN_HEAD
#undef ORCH_ATTN_TAIL
    }
    set_attn_variant(il ? "mfma32x32x16_bm256_8wave_ldsdma_interleaved_fixedref"
                        : (mb64 == 1 ? "mfma32x32x16_bm128_4wave_ldsdma_fixedref" : "mfma32x32x16_bm256_4wave_ldsdma_fixedref"));
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
