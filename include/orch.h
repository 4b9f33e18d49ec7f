/* liborch: the data-parallel hot path behind OrchMLLM's Batch Post-Balancing
 * Dispatcher, for one MI355X (gfx950).
 *
 *   orch_balance          Sec. 5.1: Eq. 2 (no-padding branch) as a per-sequence
 *                         cost, Algorithm 1 (sort descending, give each
 *                         sequence to the least-loaded new batch) and the
 *                         padding-free batch layout of Sec. 7.
 *   orch_balance_padded   Sec. 5.1, Algorithm 2: the policy for phases that batch with
 *                         paddings (ascending sort, smallest feasible bound on
 *                         count * longest, greedy contiguous cut).
 *   orch_balance_tolerance  Appendix A, third algorithm: longest-first greedy ordered by
 *                         length sums within a tolerance interval, else by squares.
 *   orch_pack             Sec. 5.2.1: the row movement of the All-to-All Batch
 *                         Communicator, performed on one device.
 *   orch_pack_composed    Sec. 5.3 (rearrangement composition): rows in an encoder
 *                         phase's packed order go straight into the LLM phase's
 *                         packed, interleaved sequences: one row pass, not two.
 *   orch_pack_composed_pieces  the same with several sub-sequences per example and modality
 *                         (Sec. 6, subsequence assembly).
 *   orch_comm_volume      Sec. 5.2.2: the communication-volume matrix V of a rearrangement.
 *   orch_varlen_attn_bwd  its backward (dq, dk, dv from dout, out and lse).
 *   orch_varlen_attn_fwd  the attention each instance then runs on its sequences,
 *                         concatenated without padding (Sec. 7); its
 *                         quadratic term is beta*sum(l^2) in Eq. 2.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with host_.
 *     The caller owns every buffer; the library allocates nothing and keeps no
 *     state between calls besides a thread-local error string.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is enqueued on it; no call synchronises with the host.
 *   - Return value: ORCH_OK or a negative orch_status.  Errors the host can see
 *     (bad sizes, null pointers, unsupported head_dim, small workspace) return
 *     before anything is launched.  Errors only the device can see (a negative
 *     length, cost overflow, a buffer too small for the rows an assignment
 *     implies) store ORCH_EDATA into `dev_status[0]`; the other outputs are
 *     then unspecified but no access leaves the caller's buffers.
 *   - Inputs are never written.  Workspaces need 256-byte alignment.
 */
#ifndef ORCH_H
#define ORCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ORCH_OK = 0,
    ORCH_EINVAL = -1,       /* bad argument */
    ORCH_ENOSPC = -2,       /* workspace too small */
    ORCH_EUNSUPPORTED = -3, /* head_dim / sizes outside what the kernels cover */
    ORCH_EHIP = -4,         /* a HIP runtime call failed */
    ORCH_EDATA = -5         /* data error found on the device (dev_status) */
} orch_status;

/* Per-sequence cost of a phase: cost(L) = a*L*L + b*L, exact in u64 (Eq. 2,
 * no-padding branch, a = beta, b = alpha).  a = 0, b = 1 balances token counts
 * (Algorithm 1 as printed).  Precondition: the sum of all costs is < 2^63. */
typedef struct {
    uint64_t a, b;
} orch_phase;

/* Outputs of orch_balance (device memory, caller-allocated). */
typedef struct {
    int32_t *inst;        /* [n]    instance that receives sequence s */
    int32_t *order;       /* [n]    sequence ids, instance-major; inside an
                                    instance in the order Algorithm 1 pushed them */
    int32_t *seq_off;     /* [D+1]  order[seq_off[i] .. seq_off[i+1]) is instance i */
    int64_t *tok_off;     /* [D+1]  first packed row of instance i */
    int32_t *cu_seqlens;  /* [n+D]  instance i's cumulative lengths: cnt_i+1
                                    entries starting at index seq_off[i]+i,
                                    first entry 0, rows local to the instance */
    uint64_t *loads;      /* [D]    summed cost per instance */
    int32_t *dev_status;  /* [1]    ORCH_OK or ORCH_EDATA, written by the device */
} orch_assignment;

/* Bytes of workspace orch_balance needs for n sequences and D instances. */
size_t orch_balance_workspace(int32_t n, int32_t D);

/* Sec. 5.1, Algorithm 1 with Eq. 2's per-sequence cost as the key.
 *   lengths[n]  int32, >= 0 (zero-length sequences are kept as empty segments)
 *   1 <= D <= 4096, n >= 0
 * Ties: equal costs keep ascending sequence index; among equally loaded
 * instances the lowest index receives the sequence. */
int orch_balance(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                 orch_assignment out, void *ws, size_t ws_bytes, void *stream);

/* orch_balance with the caller's events between its stages, for measurement: host_events is a
 * HOST array of four hipEvent_t handles (any of them may be NULL), recorded on `stream` before
 * the cost / sort kernel, after it, after the greedy kernel and after the layout kernel.
 * Everything else as orch_balance (Sec. 5.1, Algorithm 1). */
int orch_balance_stages(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                        orch_assignment out, void *ws, size_t ws_bytes, void *stream,
                        void *const *host_events);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): orch_balance with its workspace inside
 * the library, in a device array of fixed size (about 3 MB, held on every GPU the library
 * runs on until the process ends).  Same inputs, outputs, ties and device-side errors as
 * orch_balance; n above orch_balance_static_max_n() returns ORCH_EUNSUPPORTED before any
 * launch.  The call allocates nothing.  All calls on one GPU share the array: calls that
 * overlap on one GPU (different streams, or threads) race and must be serialised by the
 * caller; calls in stream order on one stream are safe. */
int orch_balance_static(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                        orch_assignment out, void *stream);

/* Largest n orch_balance_static accepts. */
int32_t orch_balance_static_max_n(void);

/* Sec. 5.1, Algorithm 2: the balancing for phases that batch
 * with paddings (the auditory encoder, Sec. 7), where a batch of cnt sequences costs
 * cnt * (its longest sequence) rows (Eq. 1, padding branch).  Sorts ascending by length
 * (ties: ascending index), finds the smallest bound b for which the greedy cut of that list
 * ("close the batch when (count + 1) * length > b") needs at most D batches, and returns the
 * batches at that bound; batch k is instance k, trailing instances may be empty.
 * The search range is [shortest length, longest length * (n / D + 1)].
 * Outputs, in the same structure as orch_balance:
 *   inst, seq_off   as there;  order = the ascending order
 *   cu_seqlens      instance i's slice holds j * max_i for j = 0..cnt_i (max_i = its longest
 *                   sequence): sequence j owns rows [j * max_i, (j + 1) * max_i) of the padded
 *                   batch, of which the first length rows are data
 *   tok_off         prefix sums of the padded batch lengths cnt_i * max_i
 *   loads[i]        Eq. 2, padding branch: a * L_i^2 / cnt_i + b * L_i with L_i = cnt_i * max_i,
 *                   i.e. cnt_i * (a * max_i^2 + b * max_i), exact u64
 *   bound[1]        device, may be NULL: the bound found
 * Rows are moved into that layout by orch_pack_composed (src = NULL for rows in original
 * order); orch_pack refuses such an assignment.  Uses orch_balance_workspace(n, D) bytes.
 * A padded batch of more than 2^31 - 1 rows or a cost >= 2^63 sets dev_status = ORCH_EDATA. */
int orch_balance_padded(const int32_t *lengths, int32_t n, int32_t D, orch_phase phase,
                        orch_assignment out, uint64_t *bound, void *ws, size_t ws_bytes, void *stream);

/* Appendix A, the third balancing algorithm: Algorithm 1 for models where the quadratic
 * term is not negligible (objective max_i L_i + lambda * sum_j l_ij^2).  Sequences are taken
 * longest first (ties: ascending index); each goes to the batch that the listing's comparator
 * CMP puts first.  CMP is not a strict weak order, so top() is fixed here by two passes:
 * m = the smallest length sum; among the batches whose length sum is below m + max(v, 1) the
 * one with the smallest sum of squared lengths receives the sequence, the lowest index on
 * ties.  v <= 1 is Algorithm 1 on lengths with squares as tie-break.
 *   v      tolerance interval, in tokens
 *   phase  only for loads[i] = a * (sum of squares) + b * (length sum)  (Eq. 2, no padding)
 * Outputs and layout as orch_balance.  1 <= D <= 1024.  Uses orch_balance_workspace(n, D) bytes.
 * A sum of squares or a load >= 2^63 sets dev_status = ORCH_EDATA. */
int orch_balance_tolerance(const int32_t *lengths, int32_t n, int32_t D, uint64_t v, orch_phase phase,
                           orch_assignment out, void *ws, size_t ws_bytes, void *stream);

/* Bytes of workspace orch_pack needs. */
size_t orch_pack_workspace(int32_t n, int32_t D);

/* Sec. 5.2.1 on one device: packed[tok_off[i]-tok_off[inst_begin] + cu_i[j] + r, :]
 * = tokens[src_cu[s] + r, :] for s the j-th sequence of instance i, 0 <= r < L_s,
 * inst_begin <= i < inst_end, where src_cu is the exclusive prefix sum of
 * lengths in original order (the source buffer holds the sequences
 * concatenated in original order).
 *   tokens  [T, H] 16-bit words, row-major; T = sum of lengths
 *   packed  [packed_rows, H]; packed_rows must cover the rows of the chosen
 *           instances, else dev_status is set and nothing past it is written
 *   a       the assignment orch_balance produced for these lengths (every segment exactly
 *           as long as its sequence: a padded assignment sets dev_status = ORCH_EDATA)
 * Rows are copied bit for bit. */
int orch_pack(const void *tokens, void *packed, const int32_t *lengths, int32_t n, int32_t D,
              int64_t T, int32_t H, int64_t packed_rows, orch_assignment a, int32_t inst_begin,
              int32_t inst_end, void *ws, size_t ws_bytes, void *stream);

/* Bytes of workspace orch_pack_composed needs for n examples. */
size_t orch_pack_composed_workspace(int32_t n);

/* Sec. 5.3, "Rearrangement composition": Pi_M o Pi_E^-1 applied in one pass.  One
 * call moves ONE modality's rows; a batch with several modalities calls it once per
 * modality into the same `packed` buffer.
 *   enc_rows [src_rows, H] 16-bit words: example s's sub_len[s] rows of this modality,
 *            laid out by `src` (the assignment orch_balance produced for sub_len on
 *            D_src instances: instance-major, rows of example s starting at
 *            src->tok_off[i] + cu_i[j]; a segment may be longer than sub_len[s], as in a
 *            padded batch from orch_balance_padded, and its first sub_len[s] rows are used), or, when src is NULL, concatenated in
 *            original example order (a modality that never left its instance)
 *   src      HOST pointer to a struct of device pointers, or NULL
 *   dst      the LLM-phase assignment over the interleaved lengths (D_dst instances)
 *   sub_off[s]  row inside example s's interleaved sequence where this modality's
 *            sub-sequence starts; sub_off[s] + sub_len[s] must not exceed the
 *            sequence's length
 * Result: packed[dst.tok_off[i] - dst.tok_off[inst_begin] + cu_i[j] + sub_off[s] + r, :]
 * = enc_rows[start_src(s) + r, :] for s the j-th sequence of destination instance i,
 * 0 <= r < sub_len[s], inst_begin <= i < inst_end.  Rows of `packed` that belong to
 * other modalities are not touched.  Rows are copied bit for bit.
 * Inconsistent data (a segment outside either buffer, an encoder segment shorter
 * than sub_len, a failed assignment on either side) sets dst.dev_status
 * to ORCH_EDATA and copies nothing. */
int orch_pack_composed(const void *enc_rows, void *packed, const int32_t *sub_len,
                       const int32_t *sub_off, int32_t n, int32_t D_src, const orch_assignment *src,
                       int32_t D_dst, orch_assignment dst, int64_t src_rows, int32_t H,
                       int64_t packed_rows, int32_t inst_begin, int32_t inst_end, void *ws,
                       size_t ws_bytes, void *stream);

/* Bytes of workspace orch_pack_composed_pieces needs for n examples and n_pieces pieces. */
size_t orch_pack_composed_pieces_workspace(int32_t n, int32_t n_pieces);

/* Sec. 6 (subsequence assembly) on top of Sec. 5.3: the composition when one modality
 * contributes SEVERAL sub-sequences to an example's interleaved sequence (several images
 * between pieces of text).  The encoder's output still holds example s's rows of the modality
 * as one run (located through `src` exactly as in orch_pack_composed; its length is the sum of
 * the example's piece lengths); the run is cut into the pieces piece_ptr[s] .. piece_ptr[s+1]-1,
 * in that order:
 *   piece_ptr [n+1]      int32, piece_ptr[0] = 0, non-decreasing, piece_ptr[n] = n_pieces
 *   piece_off [n_pieces] row of the example's interleaved sequence where the piece starts
 *   piece_len [n_pieces] rows of the piece (0 is allowed)
 * The pieces of one example must ascend without overlap and stay inside its sequence.
 * Result: packed[dst.tok_off[i] - dst.tok_off[inst_begin] + cu_i[j] + piece_off[p] + r, :]
 * = enc_rows[start_src(s) + (rows of s's earlier pieces) + r, :], 0 <= r < piece_len[p].
 * One piece per example with piece_off = sub_off, piece_len = sub_len is orch_pack_composed.
 * Inconsistent data sets dst.dev_status = ORCH_EDATA and copies nothing. */
int orch_pack_composed_pieces(const void *enc_rows, void *packed, const int32_t *piece_ptr,
                              const int32_t *piece_off, const int32_t *piece_len, int32_t n,
                              int32_t n_pieces, int32_t D_src, const orch_assignment *src, int32_t D_dst,
                              orch_assignment dst, int64_t src_rows, int32_t H, int64_t packed_rows,
                              int32_t inst_begin, int32_t inst_end, void *ws, size_t ws_bytes, void *stream);

/* Sec. 5.2.2, first loop of the node-wise rearrangement algorithm: the communication-volume
 * matrix of a rearrangement, V[from][to] = tokens that move from the instance they were
 * sampled on to the instance the assignment gives them to.
 *   from[n]   instance each sequence was sampled on, or NULL: contiguous equal blocks,
 *             sequence s on instance floor(s * D_src / n)
 *   dst       an assignment over D_dst instances (only inst and dev_status are used)
 *   V         [D_src * D_dst] u64, row-major, overwritten
 *   node, inter   if inter != NULL and node > 0: inter[D_src] receives, per source instance,
 *             the tokens sent to instances on other nodes (nodes = node consecutive
 *             instances): the quantity the section's All-to-All overhead is proportional to
 * An index outside its range sets dst.dev_status = ORCH_EDATA.  No workspace. */
int orch_comm_volume(const int32_t *lengths, int32_t n, int32_t D_src, const int32_t *from, int32_t D_dst,
                     orch_assignment dst, uint64_t *V, int32_t node, uint64_t *inter, void *stream);

/* Bytes of workspace orch_varlen_attn_fwd needs (4 bytes per sequence and per
 * (256-row query tile, q-head) pair). */
size_t orch_varlen_attn_workspace(int32_t batch, int32_t total_tokens, int32_t Hq);

/* Padding-free attention forward over `batch` sequences stored back to back.
 * For sequence t (rows cu_seqlens[t] .. cu_seqlens[t+1]), q-head h, kv-head
 * g = h / (Hq/Hkv), row i:  out[i,h,:] = softmax_j(scale * q[i,h,:].k[j,g,:]) v[j,g,:]
 * over all rows j of the sequence, or j <= i when causal != 0.
 *   q, out  [total_tokens, Hq, d] bf16      k, v  [total_tokens, Hkv, d] bf16
 *   lse     [Hq, total_tokens] fp32 natural-log-sum-exp, or NULL
 *   cu_seqlens [batch+1] int32, non-decreasing, cu_seqlens[batch] <= total_tokens
 *   max_seqlen  an upper bound on any sequence length (<= total_tokens), or 0 = not known;
 *               a nonzero bound caps the number of workgroups launched, and a sequence
 *               longer than it is a data error
 *   d in {64, 128}; Hq % Hkv == 0; scale <= 0 means 1/sqrt(d)
 *   dev_status  [1] device, may be NULL: receives ORCH_OK, or ORCH_EDATA when cu_seqlens is
 *               not non-decreasing inside [0, total_tokens] or a sequence exceeds a nonzero
 *               max_seqlen; on a data error nothing is written to out and lse
 * bf16 inputs, fp32 accumulation, bf16 output (round to nearest even).
 * Empty sequences write nothing. */
int orch_varlen_attn_fwd(const void *q, const void *k, const void *v, void *out, float *lse,
                         const int32_t *cu_seqlens, int32_t batch, int32_t total_tokens,
                         int32_t max_seqlen, int32_t Hq, int32_t Hkv, int32_t d, float scale,
                         int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* Message for the last non-OK status returned on this thread; never NULL. */
const char *orch_last_error(void);

/* Name of the kernel variant the last orch_varlen_attn_fwd on this thread
 * launched (for profiling logs); never NULL. */
const char *orch_attn_variant(void);

/* Bytes of workspace orch_varlen_attn_bwd needs (it holds delta[Hq, total_tokens] in fp32). */
size_t orch_varlen_attn_bwd_workspace(int32_t batch, int32_t total_tokens, int32_t Hq);

/* Backward of orch_varlen_attn_fwd: the gradients of sum(dout * out) with respect to q, k and v
 * (Sec. 5.3: back-propagation mirrors the forward pass; the operator is Sec. 7's).  With
 * p_ij = exp(scale * q_i.k_j - lse_i), dp_ij = dout_i.v_j, delta_i = dout_i.out_i and
 * ds_ij = p_ij (dp_ij - delta_i), over the visible pairs of every sequence:
 *   dq[i,h,:] = scale * sum_j ds_ij k[j,g,:]
 *   dk[j,g,:] = scale * sum_{h in the group of g} sum_i ds_ij q[i,h,:]
 *   dv[j,g,:] =         sum_{h in the group of g} sum_i p_ij dout[i,h,:]
 *   q, out, dout, dq  [total_tokens, Hq, d] bf16     k, v, dk, dv  [total_tokens, Hkv, d] bf16
 *   lse   [Hq, total_tokens] fp32 as written by the forward pass (required)
 * Same cu_seqlens, max_seqlen, scale, causal, head-dim and dev_status rules as the forward
 * pass (on a data error no gradient is written).  Rows outside every sequence are not
 * written.  No atomics: results are bit-reproducible. */
int orch_varlen_attn_bwd(const void *q, const void *k, const void *v, const void *out, const float *lse,
                         const void *dout, void *dq, void *dk, void *dv, const int32_t *cu_seqlens,
                         int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t Hq, int32_t Hkv,
                         int32_t d, float scale, int32_t causal, int32_t *dev_status, void *ws, size_t ws_bytes,
                         void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ORCH_H */
