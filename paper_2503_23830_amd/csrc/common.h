// Internal helpers shared by the HIP translation units of liborch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "orch.h"

namespace orch {

// Thread-local message behind orch_last_error().
void set_error(const char *fmt, ...);
void set_attn_variant(const char *name);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#define ORCH_FAIL(code, ...)            \
    do {                                \
        ::orch::set_error(__VA_ARGS__); \
        return (code);                  \
    } while (0)

#define ORCH_HIP_CHECK(expr)                                                        \
    do {                                                                            \
        hipError_t e_ = (expr);                                                     \
        if (e_ != hipSuccess) ORCH_FAIL(ORCH_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Launchers implemented per translation unit (host side).
int launch_balance(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                   orch_assignment out, void *ws, size_t ws_bytes, hipStream_t stream, void *const *stage_events);
int launch_balance_static(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                          orch_assignment out, hipStream_t stream);
int32_t balance_static_max_n();
int launch_balance_padded(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                          orch_assignment out, uint64_t *bound, void *ws, size_t ws_bytes,
                          hipStream_t stream);
int launch_balance_tolerance(const int32_t *lengths, int32_t n, int32_t D, uint64_t v, orch_phase phase,
                             orch_assignment out, void *ws, size_t ws_bytes, hipStream_t stream);
int launch_pack(const void *tokens, void *packed, const int32_t *lengths, int32_t n, int32_t D,
                int64_t T, int32_t H, int64_t packed_rows, orch_assignment a, int32_t inst_begin,
                int32_t inst_end, void *ws, size_t ws_bytes, hipStream_t stream);
int launch_pack_composed(const void *enc_rows, void *packed, const int32_t *sub_len,
                         const int32_t *sub_off, int32_t n, int32_t D_src, const orch_assignment *src,
                         int32_t D_dst, orch_assignment dst, int64_t src_rows, int32_t H,
                         int64_t packed_rows, int32_t inst_begin, int32_t inst_end, void *ws,
                         size_t ws_bytes, hipStream_t stream);
int launch_pack_composed_pieces(const void *enc_rows, void *packed, const int32_t *piece_ptr,
                                const int32_t *piece_off, const int32_t *piece_len, int32_t n, int32_t P,
                                int32_t D_src, const orch_assignment *src, int32_t D_dst, orch_assignment dst,
                                int64_t src_rows, int32_t H, int64_t packed_rows, int32_t inst_begin,
                                int32_t inst_end, void *ws, size_t ws_bytes, hipStream_t stream);
size_t pack_composed_pieces_ws_bytes(int32_t n, int32_t P);
int launch_comm_volume(const int32_t *lengths, int32_t n, int32_t D_src, const int32_t *from, int32_t D_dst,
                       orch_assignment dst, uint64_t *V, int32_t node, uint64_t *inter, hipStream_t stream);
int launch_attn(const void *q, const void *k, const void *v, void *out, float *lse,
                const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                int32_t Hq, int32_t Hkv, int32_t d, float scale, int32_t causal, int32_t *dev_status,
                void *ws, size_t ws_bytes, hipStream_t stream);
int launch_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                    const void *dout, void *dq, void *dk, void *dv, const int32_t *cu_seqlens,
                    int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t Hq, int32_t Hkv, int32_t d,
                    float scale, int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes,
                    hipStream_t stream);
size_t attn_bwd_ws_bytes(int32_t batch, int32_t total_tokens, int32_t Hq);
size_t balance_ws_bytes(int32_t n, int32_t D);
size_t pack_ws_bytes(int32_t n, int32_t D);
size_t pack_composed_ws_bytes(int32_t n);
size_t attn_ws_bytes(int32_t batch, int32_t total_tokens, int32_t Hq);

}  // namespace orch
