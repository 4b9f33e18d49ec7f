// The C ABI of liborch: argument validation, then the launchers.
#include <string.h>

#include "common.h"

namespace orch {

static thread_local char g_err[512] = "";
static thread_local char g_variant[128] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

void set_attn_variant(const char *name)
{
    strncpy(g_variant, name, sizeof g_variant - 1);
    g_variant[sizeof g_variant - 1] = 0;
}

static bool assignment_complete(const orch_assignment &a)
{
    return a.inst && a.order && a.seq_off && a.tok_off && a.cu_seqlens && a.loads && a.dev_status;
}

}  // namespace orch

using namespace orch;

extern "C" {

const char *orch_last_error(void) { return g_err; }
const char *orch_attn_variant(void) { return g_variant; }

size_t orch_balance_workspace(int32_t n, int32_t D) { return balance_ws_bytes(n, D); }
size_t orch_pack_workspace(int32_t n, int32_t D) { return pack_ws_bytes(n, D); }
size_t orch_pack_composed_workspace(int32_t n) { return pack_composed_ws_bytes(n); }
size_t orch_pack_composed_pieces_workspace(int32_t n, int32_t n_pieces) { return pack_composed_pieces_ws_bytes(n, n_pieces); }
size_t orch_varlen_attn_workspace(int32_t batch, int32_t total_tokens, int32_t Hq)
{
    return attn_ws_bytes(batch, total_tokens, Hq);
}
size_t orch_varlen_attn_bwd_workspace(int32_t batch, int32_t total_tokens, int32_t Hq)
{
    return attn_bwd_ws_bytes(batch, total_tokens, Hq);
}

int orch_balance(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase, orch_assignment out,
                 void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0) ORCH_FAIL(ORCH_EINVAL, "orch_balance: n = %d < 0", n);
    if (D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_balance: D = %d < 1", D);
    if (D > 4096) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance: D = %d > 4096", D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_balance: lengths is NULL");
    if (!assignment_complete(out)) ORCH_FAIL(ORCH_EINVAL, "orch_balance: an output pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_balance: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_balance: workspace not 256-byte aligned");
    return launch_balance(lengths, n, D, phase, out, ws, ws_bytes, (hipStream_t)stream, nullptr);
}

int orch_balance_stages(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase, orch_assignment out,
                        void *ws, size_t ws_bytes, void *stream, void *const *host_events)
{
    if (!host_events) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: host_events is NULL");
    if (n < 0) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: n = %d < 0", n);
    if (D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: D = %d < 1", D);
    if (D > 4096) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_stages: D = %d > 4096", D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: lengths is NULL");
    if (!assignment_complete(out)) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: an output pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_balance_stages: workspace not 256-byte aligned");
    return launch_balance(lengths, n, D, phase, out, ws, ws_bytes, (hipStream_t)stream, host_events);
}

int32_t orch_balance_static_max_n(void) { return balance_static_max_n(); }

int orch_balance_static(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase, orch_assignment out,
                        void *stream)
{
    if (n < 0) ORCH_FAIL(ORCH_EINVAL, "orch_balance_static: n = %d < 0", n);
    if (D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_balance_static: D = %d < 1", D);
    if (D > 4096) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_static: D = %d > 4096", D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_balance_static: lengths is NULL");
    if (!assignment_complete(out)) ORCH_FAIL(ORCH_EINVAL, "orch_balance_static: an output pointer is NULL");
    return launch_balance_static(lengths, n, D, phase, out, (hipStream_t)stream);
}

int orch_balance_padded(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase, orch_assignment out,
                        uint64_t *bound, void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: n = %d < 0", n);
    if (D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: D = %d < 1", D);
    if (D > 4096) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_padded: D = %d > 4096", D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: lengths is NULL");
    if (!assignment_complete(out)) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: an output pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_balance_padded: workspace not 256-byte aligned");
    return launch_balance_padded(lengths, n, D, phase, out, bound, ws, ws_bytes, (hipStream_t)stream);
}

int orch_balance_tolerance(const int32_t *lengths, int32_t n, int32_t D, uint64_t v, orch_phase phase,
                           orch_assignment out, void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: n = %d < 0", n);
    if (D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: D = %d < 1", D);
    if (D > 1024) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_balance_tolerance: D = %d > 1024", D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: lengths is NULL");
    if (!assignment_complete(out)) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: an output pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_balance_tolerance: workspace not 256-byte aligned");
    return launch_balance_tolerance(lengths, n, D, v, phase, out, ws, ws_bytes, (hipStream_t)stream);
}

int orch_pack(const void *tokens, void *packed, const int32_t *lengths, int32_t n, int32_t D, int64_t T,
              int32_t H, int64_t packed_rows, orch_assignment a, int32_t inst_begin, int32_t inst_end,
              void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0 || D < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack: n = %d, D = %d", n, D);
    if (T < 0 || packed_rows < 0) ORCH_FAIL(ORCH_EINVAL, "orch_pack: T = %lld, packed_rows = %lld", (long long)T, (long long)packed_rows);
    if (H < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack: H = %d < 1", H);
    if (inst_begin < 0 || inst_end > D || inst_begin > inst_end)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack: instance range [%d, %d) outside [0, %d]", inst_begin, inst_end, D);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_pack: lengths is NULL");
    if ((T > 0 && !tokens) || (packed_rows > 0 && !packed)) ORCH_FAIL(ORCH_EINVAL, "orch_pack: a row buffer is NULL");
    if (((uintptr_t)tokens | (uintptr_t)packed) & 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack: row buffers must be 2-byte aligned");
    if (!assignment_complete(a)) ORCH_FAIL(ORCH_EINVAL, "orch_pack: an assignment pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_pack: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_pack: workspace not 256-byte aligned");
    return launch_pack(tokens, packed, lengths, n, D, T, H, packed_rows, a, inst_begin, inst_end, ws,
                       ws_bytes, (hipStream_t)stream);
}

int orch_pack_composed(const void *enc_rows, void *packed, const int32_t *sub_len, const int32_t *sub_off,
                       int32_t n, int32_t D_src, const orch_assignment *src, int32_t D_dst,
                       orch_assignment dst, int64_t src_rows, int32_t H, int64_t packed_rows,
                       int32_t inst_begin, int32_t inst_end, void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0 || D_dst < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: n = %d, D_dst = %d", n, D_dst);
    if (src && D_src < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: D_src = %d < 1", D_src);
    if (src_rows < 0 || packed_rows < 0)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: src_rows = %lld, packed_rows = %lld", (long long)src_rows, (long long)packed_rows);
    if (H < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: H = %d < 1", H);
    if (inst_begin < 0 || inst_end > D_dst || inst_begin > inst_end)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: instance range [%d, %d) outside [0, %d]", inst_begin, inst_end, D_dst);
    if (n > 0 && (!sub_len || !sub_off)) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: sub_len or sub_off is NULL");
    if ((src_rows > 0 && !enc_rows) || (packed_rows > 0 && !packed)) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: a row buffer is NULL");
    if (((uintptr_t)enc_rows | (uintptr_t)packed) & 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: row buffers must be 2-byte aligned");
    if (!assignment_complete(dst) || (src && !assignment_complete(*src)))
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: an assignment pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed: workspace not 256-byte aligned");
    return launch_pack_composed(enc_rows, packed, sub_len, sub_off, n, D_src, src, D_dst, dst, src_rows, H,
                                packed_rows, inst_begin, inst_end, ws, ws_bytes, (hipStream_t)stream);
}

int orch_pack_composed_pieces(const void *enc_rows, void *packed, const int32_t *piece_ptr, const int32_t *piece_off,
                              const int32_t *piece_len, int32_t n, int32_t n_pieces, int32_t D_src,
                              const orch_assignment *src, int32_t D_dst, orch_assignment dst, int64_t src_rows,
                              int32_t H, int64_t packed_rows, int32_t inst_begin, int32_t inst_end, void *ws,
                              size_t ws_bytes, void *stream)
{
    if (n < 0 || n_pieces < 0 || D_dst < 1)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: n = %d, n_pieces = %d, D_dst = %d", n, n_pieces, D_dst);
    if (src && D_src < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: D_src = %d < 1", D_src);
    if (src_rows < 0 || packed_rows < 0)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: src_rows = %lld, packed_rows = %lld", (long long)src_rows, (long long)packed_rows);
    if (H < 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: H = %d < 1", H);
    if (inst_begin < 0 || inst_end > D_dst || inst_begin > inst_end)
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: instance range [%d, %d) outside [0, %d]", inst_begin, inst_end, D_dst);
    if (!piece_ptr) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: piece_ptr is NULL");
    if (n_pieces > 0 && (!piece_off || !piece_len)) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: piece_off or piece_len is NULL");
    if ((src_rows > 0 && !enc_rows) || (packed_rows > 0 && !packed)) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: a row buffer is NULL");
    if (((uintptr_t)enc_rows | (uintptr_t)packed) & 1) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: row buffers must be 2-byte aligned");
    if (!assignment_complete(dst) || (src && !assignment_complete(*src)))
        ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: an assignment pointer is NULL");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_pack_composed_pieces: workspace not 256-byte aligned");
    return launch_pack_composed_pieces(enc_rows, packed, piece_ptr, piece_off, piece_len, n, n_pieces, D_src, src,
                                       D_dst, dst, src_rows, H, packed_rows, inst_begin, inst_end, ws, ws_bytes,
                                       (hipStream_t)stream);
}

int orch_comm_volume(const int32_t *lengths, int32_t n, int32_t D_src, const int32_t *from, int32_t D_dst,
                     orch_assignment dst, uint64_t *V, int32_t node, uint64_t *inter, void *stream)
{
    if (n < 0 || D_src < 1 || D_dst < 1) ORCH_FAIL(ORCH_EINVAL, "orch_comm_volume: n = %d, D_src = %d, D_dst = %d", n, D_src, D_dst);
    if (node < 0) ORCH_FAIL(ORCH_EINVAL, "orch_comm_volume: node = %d < 0", node);
    if (n > 0 && !lengths) ORCH_FAIL(ORCH_EINVAL, "orch_comm_volume: lengths is NULL");
    if (!V) ORCH_FAIL(ORCH_EINVAL, "orch_comm_volume: V is NULL");
    if (!dst.inst || !dst.dev_status) ORCH_FAIL(ORCH_EINVAL, "orch_comm_volume: an assignment pointer is NULL");
    return launch_comm_volume(lengths, n, D_src, from, D_dst, dst, V, node, inter, (hipStream_t)stream);
}

int orch_varlen_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                         const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens,
                         int32_t max_seqlen, int32_t Hq, int32_t Hkv, int32_t d, float scale,
                         int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes, void *stream)
{
    if (batch < 0 || total_tokens < 0) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: batch = %d, total_tokens = %d", batch, total_tokens);
    if (max_seqlen < 0 || max_seqlen > total_tokens) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: max_seqlen = %d outside [0, %d]", max_seqlen, total_tokens);
    if (Hq < 1 || Hkv < 1 || Hq % Hkv) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: Hq = %d, Hkv = %d", Hq, Hkv);
    if (d != 64 && d != 128) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_fwd: head_dim %d (64 and 128 are built)", d);
    if (!cu_seqlens) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: cu_seqlens is NULL");
    if (total_tokens > 0 && (!q || !k || !v || !out)) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: q, k, v or out is NULL");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15)
        ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: q, k, v, out must be 16-byte aligned");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_fwd: workspace not 256-byte aligned");
    return launch_attn(q, k, v, out, lse, cu_seqlens, batch, total_tokens, max_seqlen, Hq, Hkv, d, scale, causal,
                       dev_status, ws, ws_bytes, (hipStream_t)stream);
}

int orch_varlen_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                         const void *dout, void *dq, void *dk, void *dv, const int32_t *cu_seqlens,
                         int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t Hq, int32_t Hkv,
                         int32_t d, float scale, int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes,
                         void *stream)
{
    if (batch < 0 || total_tokens < 0) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: batch = %d, total_tokens = %d", batch, total_tokens);
    if (max_seqlen < 0 || max_seqlen > total_tokens) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: max_seqlen = %d outside [0, %d]", max_seqlen, total_tokens);
    if (Hq < 1 || Hkv < 1 || Hq % Hkv) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: Hq = %d, Hkv = %d", Hq, Hkv);
    if (d != 64 && d != 128) ORCH_FAIL(ORCH_EUNSUPPORTED, "orch_varlen_attn_bwd: head_dim %d (64 and 128 are built)", d);
    if (!cu_seqlens) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: cu_seqlens is NULL");
    if (total_tokens > 0 && (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv))
        ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: a tensor pointer is NULL (lse from the forward pass is required)");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)dout | (uintptr_t)dq | (uintptr_t)dk | (uintptr_t)dv) & 15)
        ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: tensors must be 16-byte aligned");
    if (!ws) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: workspace is NULL");
    if ((uintptr_t)ws & 255) ORCH_FAIL(ORCH_EINVAL, "orch_varlen_attn_bwd: workspace not 256-byte aligned");
    return launch_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, cu_seqlens, batch, total_tokens, max_seqlen, Hq, Hkv,
                           d, scale, causal, dev_status, ws, ws_bytes, (hipStream_t)stream);
}

}  // extern "C"
