// Streamed LDS tiles of the attention kernels: LDS-DMA staging into a swizzled, unpadded layout and
// the MFMA fragment reads on it.  Shared by the backward kernels and the head_dim-64 forward kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace orch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// Transposed A-operand fragments (row M = a column of X, contraction over 16 rows of X) come from
// the ROW-MAJOR tile X[row][col] with two ds_read_b64_tr_b16: inside a block of 16 lanes, lane i
// receives element i % 4 of the 8-byte words addressed by lanes i / 4, 4 + i / 4, 8 + i / 4 and
// 12 + i / 4.  Lane (g, half, j4, a) = (lane / 32, (lane / 16) % 2, (lane % 16) / 4, lane % 4)
// addresses row 4 g + j4 and columns 16 half + 4 a .. + 3, so it receives rows 4 g .. 4 g + 3 of
// column 16 half + (lane % 16) = lane % 32; a second read 8 rows further completes the 8
// contraction slots of the lane (rows 4 g + w and 8 + 4 g + w: the rows its registers 0..7 of a
// 32x32 accumulator hold).  PairStage::rd_tr does this on the swizzled tile.

constexpr int kT = 64;        // rows of a streamed LDS tile
constexpr int kThreads = 256; // 4 wavefronts: the workgroup of every kernel here but the fused dK/dV one (8)

__device__ __forceinline__ bf16x8 lds_rd128(uint32_t addr)
{
    return *(const __attribute__((address_space(3))) bf16x8 *)(uintptr_t)addr;
}

// Where a pair of 64-row tiles comes from: rows [m0, m0 + 64) of the sequence that starts at
// row0 and has L rows, head hd of two [T, heads, HD] tensors (K and V, or Q and dout).
struct TileSrc {
    const uint16_t *px, *py;
    int row0, L, m0, heads, hd;
};

// The pair of streamed LDS tiles of a step (X: K or Q, Y: V or dout) and the fragment reads on
// them.  Rows go straight from global memory into LDS by LDS-DMA (no staging registers, no LDS
// store instructions); NST stages, one barrier per step.  Rows are unpadded; a slot swizzle keeps
// both read patterns (16-byte row reads for the first products, 8-byte transpose reads for the
// last one) free of bank conflicts.
// Slot swizzle of the LDS-DMA layout: row r keeps its 16-byte chunk c at slot c ^ swz(r).
// 256-byte rows (head_dim 128, 16 chunks, one row per 64 banks): swz = 4 (r % 4) + (r / 4) % 4.
// 128-byte rows (head_dim 64, 8 chunks, two rows per 64 banks): swz = 4 r1 + 2 r3 + r2 (bits of r).
// In both, 16 consecutive rows at one chunk land in 16 distinct 16-byte bank groups, and so do the
// 4 rows x 4 chunks that a half-wavefront reads in one transpose read.
template <int HD>
__device__ __forceinline__ int dma_swz(int r)
{
    if (HD == 128) return 4 * (r & 3) + ((r >> 2) & 3);
    return 4 * ((r >> 1) & 1) + 2 * ((r >> 3) & 1) + ((r >> 2) & 1);
}

// NST stages (a tile pair stays readable for NST - 1 steps after the one that fetched it);
// NWAVE wavefronts share the staging, each fetching kT / NWAVE rows of both tiles.
template <int HD, int NST = 2, int NWAVE = 4>
struct PairStage {
    static constexpr int ROWB = 2 * HD;
    static constexpr int TILE_B = kT * ROWB;
    static constexpr int BYTES = NST * 2 * TILE_B;
    static constexpr int CH = ROWB / 16;          // 16-byte chunks per row
    static constexpr int RPI = 1024 / ROWB;       // rows one DMA load moves (64 lanes x 16 bytes)
    static constexpr int WROWS = kT / NWAVE;      // rows of a tile one wavefront fetches
    static constexpr int NP = WROWS / RPI;        // loads per wavefront and tile
    static_assert(NP >= 1 && NP * RPI * NWAVE == kT, "the wavefronts' loads must tile the 64 rows");
    uint32_t base;
    uint32_t raddr[HD / 16];     // row reads: l32 * ROWB + 16 * ((2 c + g) ^ swz(l32))
    uint32_t taddr[2][HD / 32];  // transpose reads, rows 8 u + 4 g + j4, columns of block b
    uint32_t dcol[NP];           // DMA: byte column this lane fetches in load p
    int drow;                    // DMA: row of the tile this lane fetches in load 0 (load p: + RPI p)
    uint32_t ddst;               // DMA: LDS offset of this wavefront's first load inside a tile

    __device__ __forceinline__ void init(uint32_t lds_base, int lane, int wave)
    {
        base = lds_base;
        const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
        for (int c = 0; c < HD / 16; ++c) raddr[c] = (uint32_t)(l32 * ROWB + 16 * ((2 * c + g) ^ dma_swz<HD>(l32)));
        const int half = (lane >> 4) & 1, j4 = (lane & 15) >> 2, a = lane & 3;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int b = 0; b < HD / 32; ++b) {
                const int r = 8 * u + 4 * g + j4;
                taddr[u][b] = (uint32_t)(r * ROWB + 16 * ((4 * b + 2 * half + (a >> 1)) ^ dma_swz<HD>(r)) + 8 * (a & 1));
            }
        // a DMA load moves 64 lanes x 16 bytes = RPI rows into 1 KB of LDS in lane order; this
        // wavefront fetches rows WROWS wave .. + WROWS - 1 of the tile in NP loads
        drow = WROWS * wave + lane / CH;
#pragma unroll
        for (int p = 0; p < NP; ++p) dcol[p] = 16u * (uint32_t)((lane % CH) ^ dma_swz<HD>(drow + RPI * p));
        ddst = (uint32_t)(WROWS * wave * ROWB);
    }
    __device__ __forceinline__ uint32_t x_base(int it) const
    {
        return base + (uint32_t)((NST == 2 ? (it & 1) : (it % NST)) * 2 * TILE_B);
    }
    __device__ __forceinline__ uint32_t y_base(int it) const { return x_base(it) + TILE_B; }
    // the same by stage number (a constant in loops unrolled by NST)
    __device__ __forceinline__ uint32_t x_at(int stage) const { return base + (uint32_t)(stage * 2 * TILE_B); }
    __device__ __forceinline__ uint32_t y_at(int stage) const { return x_at(stage) + TILE_B; }
    __device__ __forceinline__ bf16x8 rd_row(uint32_t tile, int blk, int c) const
    {
        return lds_rd128(tile + raddr[c] + (uint32_t)(blk * 32 * ROWB));
    }
    __device__ __forceinline__ bf16x8 rd_tr(uint32_t tile, int j) const
    {
        const uint32_t o = tile + (uint32_t)(16 * (j & 3) * ROWB);
        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(o + taddr[0][j >> 2]));
        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(o + taddr[1][j >> 2]));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
    }
    // One LDS-DMA load: 64 lanes x 16 bytes from scalar base `tb` + per-lane byte offset into the
    // 1 KB of LDS that starts at `dst` (M0, declared as clobbered).  Written as asm so that the
    // compiler does not tie later LDS reads of the other stage to it; publish() waits for it.
    // (the compiler reserves M0 for its own LDS-DMA / indexed-register sequences and warns about
    // the clobber; declaring it is what makes it re-materialise M0 after this statement)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    static __device__ __forceinline__ void dma_issue(const char *tb, uint32_t off, uint32_t dst)
    {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off), "s"(tb)
                     : "memory", "m0");
    }
#pragma clang diagnostic pop
    static __device__ __forceinline__ const char *uniform_ptr(const void *ptr)
    {
        const uint64_t v = (uint64_t)(uintptr_t)ptr;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
        return (const char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
    }
    // The loads of one tile pair, ready to issue: 2 NP per wavefront.  The LDS-DMA unit is shared
    // by the workgroup and a wavefront stalls at issue while it is busy, so callers that can
    // spread issue(plan, k), k = 0 .. 2 NP - 1, over their MFMAs instead of issuing all at once.
    struct Plan {
        const char *tx, *ty;   // first row of the tiles (scalar)
        uint32_t dx;           // LDS address of this wavefront's first load in the X tile (scalar)
        uint32_t off[NP];      // this lane's byte offsets from tx / ty
    };
    static constexpr int NLOAD = 2 * NP;
    __device__ __forceinline__ Plan plan(const TileSrc &s, int stage) const
    {
        Plan p;
        const uint32_t rstride = (uint32_t)s.heads * HD * 2;
        const size_t e = ((size_t)(s.row0 + s.m0) * s.heads + s.hd) * HD;
        p.tx = uniform_ptr(s.px + e);
        p.ty = uniform_ptr(s.py + e);
        const int last = s.L - 1 - s.m0;  // rows past the end of the sequence repeat its last row (masked later)
        p.dx = (uint32_t)__builtin_amdgcn_readfirstlane((int)(x_at(stage) + ddst));
#pragma unroll
        for (int i = 0; i < NP; ++i) p.off[i] = (uint32_t)min(drow + RPI * i, last) * rstride + dcol[i];
        return p;
    }
    static __device__ __forceinline__ void issue(const Plan &p, int k)
    {
        const int i = k >> 1;
        if (k & 1) dma_issue(p.ty, p.off[i], p.dx + (uint32_t)(TILE_B + RPI * i * ROWB));
        else dma_issue(p.tx, p.off[i], p.dx + (uint32_t)(RPI * i * ROWB));
    }
    __device__ __forceinline__ void begin(const TileSrc &s, int it) { begin_at(s, NST == 2 ? (it & 1) : (it % NST)); }
    __device__ __forceinline__ void begin_at(const TileSrc &s, int stage)
    {
        const Plan p = plan(s, stage);
#pragma unroll
        for (int k = 0; k < NLOAD; ++k) issue(p, k);
    }
    __device__ __forceinline__ void publish()
    {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
};

}  // namespace orch
