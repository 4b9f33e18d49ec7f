// orch_varlen_attn_fwd: padding-free attention forward over sequences stored
// back to back (the batching the paper uses for every phase that runs without
// paddings, Sec. 7; the quadratic term of Eq. 2).
//
// One workgroup (4 wavefronts) owns BM = 128 consecutive query rows of one
// sequence and one q-head; each wavefront owns 32 of them.  K/V tiles of
// BN = 64 keys are staged through LDS (V transposed on the way in) and shared by
// the four wavefronts.  The scores are computed transposed, S^T = K Q^T, with
// v_mfma_f32_32x32x16_bf16: in the accumulator layout every lane then holds 16
// keys of ONE query, so the online-softmax statistics are per-lane scalars
// (one cross-lane exchange per tile), the probabilities are already in the
// B-operand layout of the second product O^T += V^T P^T, and rescaling O is a
// per-lane multiply.
#include "common.h"

namespace orch {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128;  // query rows per workgroup
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
                                                                AttnHdr *hdr, int32_t *tile_off,
                                                                int32_t *dev_status)
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

template <int HD, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    uint16_t *__restrict__ out, float *__restrict__ lse, const int32_t *__restrict__ cu,
    const AttnHdr *__restrict__ hdr, const int32_t *__restrict__ tile_off, int32_t batch,
    int32_t total_tokens, int32_t Hq, int32_t Hkv, float scale, float scale_log2)
{
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

    // ---- Q fragments: B operand, column m = lane%32, k = 16c + 8g + [0..7]
    const int qm = q0 + wave * 32 + l32;
    const int qm_c = qm < L ? qm : L - 1;
    bf16x8 qf[NC];
    {
        const uint16_t *qp = q + ((size_t)(row0 + qm_c) * Hq + h) * HD + 8 * g;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c] = *(const bf16x8 *)(qp + 16 * c);
    }

    f32x16 acc_o[NDB];
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[b][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int kend = CAUSAL ? min(L, q0 + BM) : L;
    const int ntile_k = (kend + BN - 1) / BN;

    // ---- global -> register staging of one K/V tile
    constexpr int KROWS_PER_PASS = kThreads / (HD / 8);  // rows covered by 256 16-byte loads
    constexpr int KPASS = BN / KROWS_PER_PASS;
    constexpr int VBLK = (BN / 4) * (HD / 4) / kThreads;  // 4x4 blocks per thread
    u32x4 kreg[KPASS];
    u32x2 vreg[VBLK][4];
    const int k_col = (tid % (HD / 8)) * 8, k_row = tid / (HD / 8);
    const int v_dq = tid % (HD / 4), v_nq0 = tid / (HD / 4);
    constexpr int V_NQ_STEP = kThreads / (HD / 4);

    auto load_tile = [&](int n0) {
#pragma unroll
        for (int p = 0; p < KPASS; ++p) {
            int n = n0 + p * KROWS_PER_PASS + k_row;
            n = n < L ? n : L - 1;
            kreg[p] = *(const u32x4 *)(k + ((size_t)(row0 + n) * Hkv + g_kv) * HD + k_col);
        }
#pragma unroll
        for (int b = 0; b < VBLK; ++b) {
            const int nq = v_nq0 + b * V_NQ_STEP;
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
            const int nq = v_nq0 + b * V_NQ_STEP;
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

    load_tile(0);
    for (int it = 0; it < ntile_k; ++it) {
        const int n0 = it * BN;
        __syncthreads();
        store_tile();
        __syncthreads();
        if (it + 1 < ntile_k) load_tile(n0 + BN);

        // ---- S^T = K Q^T : two 32-key blocks
        f32x16 acc_s[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_s[nb][e] = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const bf16x8 kf = *(const bf16x8 *)(&Ks[(32 * nb + l32) * KS + 16 * c + 8 * g]);
                acc_s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], acc_s[nb], 0, 0, 0);
            }
        }

        // ---- mask (only tiles that touch the sequence end or the diagonal)
        const bool need_mask = (n0 + BN > L) || (CAUSAL && n0 + BN - 1 > q0 + wave * 32);
        if (need_mask) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int n = n0 + 32 * nb + 8 * (e >> 2) + 4 * g + (e & 3);
                    const bool vis = n < L && (!CAUSAL || n <= qm);
                    if (!vis) acc_s[nb][e] = -INFINITY;
                }
        }

        // ---- online softmax, one query per lane (shared by lanes l and l^32)
        float tmax = acc_s[0][0];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, acc_s[nb][e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2);
        const float mb = m_use * scale_log2;
        float psum = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                p[e] = __builtin_amdgcn_exp2f(acc_s[kk >> 1][8 * (kk & 1) + e] * scale_log2 - mb);
                psum += p[e];
            }
            u32x4 pk;
            pk.x = pack_bf16(p[0], p[1]);
            pk.y = pack_bf16(p[2], p[3]);
            pk.z = pack_bf16(p[4], p[5]);
            pk.w = pack_bf16(p[6], p[7]);
            pf[kk] = __builtin_bit_cast(bf16x8, pk);
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[b][e] *= alpha;

        // ---- O^T += V^T P^T
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 vf = *(const bf16x8 *)(&Vt[(32 * b + l32) * VS + 16 * kk + 8 * g]);
                acc_o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kk], acc_o[b], 0, 0, 0);
            }
    }

    // ---- epilogue
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.f / l_tot;
    if (qm < L) {
        uint16_t *op = out + ((size_t)(row0 + qm) * Hq + h) * HD;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x2 w;
                w.x = pack_bf16(acc_o[b][4 * r] * inv, acc_o[b][4 * r + 1] * inv);
                w.y = pack_bf16(acc_o[b][4 * r + 2] * inv, acc_o[b][4 * r + 3] * inv);
                *(u32x2 *)(op + 32 * b + 8 * r + 4 * g) = w;
            }
        if (lse != nullptr && g == 0)
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
    hipLaunchKernelGGL(attn_prep_kernel, dim3(1), dim3(kPrepThreads), 0, stream, cu_seqlens, batch,
                       total_tokens, hdr, tile_off, (int32_t *)nullptr);
    const int64_t max_tiles = (int64_t)total_tokens / BM + batch;
    const int64_t grid = max_tiles * Hq;
    if (grid > 0x7fffffffLL) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_fwd: %lld workgroups", (long long)grid);
    if (scale <= 0.f) scale = 1.0f / sqrtf((float)d);
    const float sl2 = scale * 1.4426950408889634f;
    if (grid > 0 && batch > 0) {
#define ORCH_ATTN_ARGS                                                                          \
    (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)out, lse,        \
        cu_seqlens, hdr, tile_off, batch, total_tokens, Hq, Hkv, scale, sl2
        if (d == 128 && causal)
            hipLaunchKernelGGL((attn_fwd_kernel<128, true>), dim3((unsigned)grid), dim3(kThreads), 0, stream, ORCH_ATTN_ARGS);
        else if (d == 128)
            hipLaunchKernelGGL((attn_fwd_kernel<128, false>), dim3((unsigned)grid), dim3(kThreads), 0, stream, ORCH_ATTN_ARGS);
        else if (d == 64 && causal)
            hipLaunchKernelGGL((attn_fwd_kernel<64, true>), dim3((unsigned)grid), dim3(kThreads), 0, stream, ORCH_ATTN_ARGS);
        else
            hipLaunchKernelGGL((attn_fwd_kernel<64, false>), dim3((unsigned)grid), dim3(kThreads), 0, stream, ORCH_ATTN_ARGS);
#undef ORCH_ATTN_ARGS
    }
    set_attn_variant("mfma32x32x16_bm128_bn64");
    ORCH_HIP_CHECK(hipGetLastError());
    return ORCH_OK;
}

}  // namespace orch
