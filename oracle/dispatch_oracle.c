/* CPU oracle for the Batch Post-Balancing dispatch step.  TEST INFRASTRUCTURE:
 * only tests, the smoke check and the bench's cpu_baseline leg may call it; it
 * shares no code with the HIP library and is never a fallback for it.
 *
 * What it computes, in the paper's order (OrchMLLM, Sec. 5.1):
 *   - per-sequence cost from the no-padding branch of Eq. 2: a batch's cost
 *     alpha*sum(l) + beta*sum(l^2) is additive over sequences, so sequence s
 *     carries c_s = a*l_s^2 + b*l_s with a = beta, b = alpha (exact, u64);
 *   - Algorithm 1 (Sec. 5.1, batching without paddings) with that cost as the
 *     key: sort descending, then give every sequence in turn to the batch whose
 *     summed key is smallest (longest-processing-time-first greedy).  With
 *     a = 0, b = 1 this is Algorithm 1 literally;
 *   - the packed, padding-free layout each instance then batches along the
 *     sequence dimension (Sec. 7, input preprocessing) and the row movement the
 *     All-to-All Batch Communicator performs (Sec. 5.2.1), on one device;
 *   - the rearrangement composition of Sec. 5.3 (an encoder phase's packed rows
 *     straight into the LLM phase's packed batch), written as the two steps it
 *     composes: reset to original order, then rearrange.
 *
 * Readings where the paper is silent: equal keys keep ascending index order
 * (stable sort); among equally loaded batches the lowest-numbered one is the
 * "top"; the batch created i-th is instance i; sequences stay in push order
 * inside a batch; zero-length sequences are kept as empty segments.
 *
 * Every function takes HOST pointers.  Return value 0 = ok, -1 = bad argument,
 * -5 = bad data (negative length or arithmetic overflow).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Eq. 2, no-padding branch, per sequence. */
int orc_cost(const int32_t *lengths, int32_t n, uint64_t a, uint64_t b, uint64_t *cost)
{
    if (n < 0 || (n > 0 && (!lengths || !cost))) return -1;
    unsigned __int128 total = 0;
    for (int32_t s = 0; s < n; ++s) {
        if (lengths[s] < 0) return -5;
        unsigned __int128 l = (unsigned __int128)(uint32_t)lengths[s];
        unsigned __int128 c = (unsigned __int128)a * l * l + (unsigned __int128)b * l;
        total += c;
        if (total >> 63) return -5;
        cost[s] = (uint64_t)c;
    }
    return 0;
}

/* Algorithm 1, line 1: indices in descending key order; equal keys keep
 * ascending index order.  Bottom-up merge sort, stable. */
int orc_sort_desc(const uint64_t *cost, int32_t n, int32_t *sorted)
{
    if (n < 0 || (n > 0 && (!cost || !sorted))) return -1;
    int32_t *a = sorted, *b = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!b) return -1;
    for (int32_t i = 0; i < n; ++i) a[i] = i;
    for (int64_t w = 1; w < n; w *= 2) {
        for (int64_t lo = 0; lo < n; lo += 2 * w) {
            int64_t mid = lo + w < n ? lo + w : n, hi = lo + 2 * w < n ? lo + 2 * w : n;
            int64_t i = lo, j = mid, k = lo;
            while (i < mid && j < hi) {
                /* take from the right run only when its key is strictly larger */
                if (cost[a[j]] > cost[a[i]]) b[k++] = a[j++];
                else b[k++] = a[i++];
            }
            while (i < mid) b[k++] = a[i++];
            while (j < hi) b[k++] = a[j++];
        }
        int32_t *t = a; a = b; b = t;
    }
    if (a != sorted) { memcpy(sorted, a, sizeof(int32_t) * (size_t)n); b = a; }
    free(b);
    return 0;
}

/* Algorithm 1, lines 2-7.  The priority queue's top() is found by a plain scan:
 * first strictly smaller load wins, so ties go to the lowest instance.
 * rank[s] = how many sequences the batch held before s was pushed. */
int orc_greedy(const uint64_t *cost, const int32_t *sorted, int32_t n, int32_t D,
               int32_t *inst, int32_t *rank, uint64_t *loads, int32_t *counts)
{
    if (n < 0 || D < 1) return -1;
    for (int32_t i = 0; i < D; ++i) { loads[i] = 0; counts[i] = 0; }
    for (int32_t t = 0; t < n; ++t) {
        int32_t s = sorted[t], best = 0;
        for (int32_t i = 1; i < D; ++i)
            if (loads[i] < loads[best]) best = i;
        inst[s] = best;
        rank[s] = counts[best]++;
        loads[best] += cost[s];
    }
    return 0;
}

/* The whole dispatch: cost -> sort -> greedy -> layout.
 *   inst[n]        instance of sequence s
 *   order[n]       sequence ids, instance-major, push order inside an instance
 *   seq_off[D+1]   order[seq_off[i] .. seq_off[i+1]) is instance i
 *   tok_off[D+1]   first packed row of instance i (i64)
 *   cu_seqlens[n+D] instance i's slice starts at seq_off[i]+i, has cnt_i+1
 *                  entries, starts at 0 (rows local to the instance)
 *   loads[D]       summed cost per instance
 */
int orc_balance(const int32_t *lengths, int32_t n, int32_t D, uint64_t a, uint64_t b,
                int32_t *inst, int32_t *order, int32_t *seq_off, int64_t *tok_off,
                int32_t *cu_seqlens, uint64_t *loads)
{
    if (n < 0 || D < 1) return -1;
    size_t nn = (size_t)(n > 0 ? n : 1);
    uint64_t *cost = (uint64_t *)malloc(nn * sizeof(uint64_t));
    int32_t *sorted = (int32_t *)malloc(nn * sizeof(int32_t));
    int32_t *rank = (int32_t *)malloc(nn * sizeof(int32_t));
    int32_t *counts = (int32_t *)malloc((size_t)D * sizeof(int32_t));
    int rc = -1;
    if (!cost || !sorted || !rank || !counts) goto done;
    if ((rc = orc_cost(lengths, n, a, b, cost)) != 0) goto done;
    if ((rc = orc_sort_desc(cost, n, sorted)) != 0) goto done;
    if ((rc = orc_greedy(cost, sorted, n, D, inst, rank, loads, counts)) != 0) goto done;

    seq_off[0] = 0;
    for (int32_t i = 0; i < D; ++i) seq_off[i + 1] = seq_off[i] + counts[i];
    for (int32_t s = 0; s < n; ++s) order[seq_off[inst[s]] + rank[s]] = s;
    tok_off[0] = 0;
    for (int32_t i = 0; i < D; ++i) {
        int32_t *cu = cu_seqlens + seq_off[i] + i;
        int64_t run = 0;
        cu[0] = 0;
        for (int32_t j = 0; j < counts[i]; ++j) {
            run += lengths[order[seq_off[i] + j]];
            if (run > INT32_MAX) { rc = -5; goto done; }
            cu[j + 1] = (int32_t)run;
        }
        tok_off[i + 1] = tok_off[i] + run;
    }
    rc = 0;
done:
    free(cost); free(sorted); free(rank); free(counts);
    return rc;
}

/* Row movement of the rearrangement: sequence s occupies source rows
 * [src_cu[s], src_cu[s]+l_s) (sequences concatenated in original order) and
 * lands at instance-major position tok_off[i] + cu_i[j].  One memcpy per
 * sequence.  Only instances [inst_begin, inst_end) are produced, at rows
 * relative to tok_off[inst_begin].  row_bytes = bytes per token row. */
int orc_pack(const void *tokens, void *packed, const int32_t *lengths, int32_t n, int32_t D,
             int64_t row_bytes, const int32_t *order, const int32_t *seq_off,
             const int64_t *tok_off, const int32_t *cu_seqlens,
             int32_t inst_begin, int32_t inst_end)
{
    if (n < 0 || D < 1 || inst_begin < 0 || inst_end > D || inst_begin > inst_end || row_bytes < 1)
        return -1;
    int64_t *src_cu = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!src_cu) return -1;
    src_cu[0] = 0;
    for (int32_t s = 0; s < n; ++s) src_cu[s + 1] = src_cu[s] + lengths[s];
    const char *src = (const char *)tokens;
    char *dst = (char *)packed;
    for (int32_t i = inst_begin; i < inst_end; ++i) {
        const int32_t *cu = cu_seqlens + seq_off[i] + i;
        for (int32_t j = 0; j < seq_off[i + 1] - seq_off[i]; ++j) {
            int32_t s = order[seq_off[i] + j];
            int64_t drow = tok_off[i] - tok_off[inst_begin] + cu[j];
            memcpy(dst + drow * row_bytes, src + src_cu[s] * row_bytes,
                   (size_t)lengths[s] * (size_t)row_bytes);
        }
    }
    free(src_cu);
    return 0;
}

/* Same movement as an index map: src_row_of_dst[r] = source row that lands in
 * global packed row r (all instances), for checking device output in chunks
 * without holding both buffers on the host. */
int orc_row_map(const int32_t *lengths, int32_t n, int32_t D, const int32_t *order,
                const int32_t *seq_off, const int64_t *tok_off, const int32_t *cu_seqlens,
                int64_t *src_row_of_dst)
{
    if (n < 0 || D < 1) return -1;
    int64_t *src_cu = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!src_cu) return -1;
    src_cu[0] = 0;
    for (int32_t s = 0; s < n; ++s) src_cu[s + 1] = src_cu[s] + lengths[s];
    for (int32_t i = 0; i < D; ++i) {
        const int32_t *cu = cu_seqlens + seq_off[i] + i;
        for (int32_t j = 0; j < seq_off[i + 1] - seq_off[i]; ++j) {
            int32_t s = order[seq_off[i] + j];
            for (int32_t r = 0; r < lengths[s]; ++r)
                src_row_of_dst[tok_off[i] + cu[j] + r] = src_cu[s] + r;
        }
    }
    free(src_cu);
    return 0;
}

/* Rearrangement composition (Sec. 5.3, "MLLM Global Orchestrator").  The rows an
 * encoder produced lie in THAT phase's packed order (its own dispatcher's
 * rearrangement Pi_E, given by e_order / e_seq_off / e_tok_off / e_cu over the
 * per-example sub-lengths).  The result the composition must equal is defined by
 * the two steps the paper composes, taken one after the other here:
 *   1. reset: Pi_E^-1 brings every example's rows back to original example order
 *      (a temporary buffer, examples concatenated in index order);
 *   2. rearrange: Pi_M places example s's rows inside its interleaved sequence on
 *      the destination instance, at row sub_off[s] of that sequence
 *      (m_order / m_seq_off / m_tok_off / m_cu describe the LLM-phase assignment
 *      over the interleaved lengths).
 * e_order == NULL means the rows already are in original order (text: it never
 * left its instance), so step 1 is the identity.
 * Destination rows that belong to other modalities are left untouched.
 * An encoder segment may be longer than sub_len[s] (a padded encoder batch, Sec. 7
 * input preprocessing: audio is batched with paddings); its first sub_len[s] rows
 * are the example's.
 * Returns -5 if a sub-sequence does not fit in its interleaved sequence or in its
 * encoder segment. */
int orc_pack_composed(const void *enc_rows, void *packed, const int32_t *sub_len,
                      const int32_t *sub_off, int32_t n, int64_t row_bytes, int32_t De,
                      const int32_t *e_order, const int32_t *e_seq_off, const int64_t *e_tok_off,
                      const int32_t *e_cu, int32_t Dm, const int32_t *m_order,
                      const int32_t *m_seq_off, const int64_t *m_tok_off, const int32_t *m_cu,
                      int32_t inst_begin, int32_t inst_end)
{
    if (n < 0 || Dm < 1 || inst_begin < 0 || inst_end > Dm || inst_begin > inst_end || row_bytes < 1)
        return -1;
    if (e_order && De < 1) return -1;
    int64_t *sub_cu = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!sub_cu) return -1;
    sub_cu[0] = 0;
    for (int32_t s = 0; s < n; ++s) {
        if (sub_len[s] < 0 || sub_off[s] < 0) { free(sub_cu); return -5; }
        sub_cu[s + 1] = sub_cu[s] + sub_len[s];
    }
    const char *src = (const char *)enc_rows;
    char *tmp = NULL;
    /* step 1: reset to original example order */
    if (e_order) {
        tmp = (char *)malloc((size_t)(sub_cu[n] > 0 ? sub_cu[n] : 1) * (size_t)row_bytes);
        if (!tmp) { free(sub_cu); return -1; }
        for (int32_t i = 0; i < De; ++i) {
            const int32_t *cu = e_cu + e_seq_off[i] + i;
            for (int32_t j = 0; j < e_seq_off[i + 1] - e_seq_off[i]; ++j) {
                int32_t s = e_order[e_seq_off[i] + j];
                if (cu[j + 1] - cu[j] < sub_len[s]) { free(tmp); free(sub_cu); return -5; }
                memcpy(tmp + sub_cu[s] * row_bytes, src + (e_tok_off[i] + cu[j]) * row_bytes,
                       (size_t)sub_len[s] * (size_t)row_bytes);
            }
        }
        src = tmp;
    }
    /* step 2: place inside the interleaved sequences of the destination instances */
    char *dst = (char *)packed;
    int rc = 0;
    for (int32_t i = inst_begin; i < inst_end && rc == 0; ++i) {
        const int32_t *cu = m_cu + m_seq_off[i] + i;
        for (int32_t j = 0; j < m_seq_off[i + 1] - m_seq_off[i]; ++j) {
            int32_t s = m_order[m_seq_off[i] + j];
            if ((int64_t)sub_off[s] + sub_len[s] > (int64_t)cu[j + 1] - cu[j]) { rc = -5; break; }
            int64_t drow = m_tok_off[i] - m_tok_off[inst_begin] + cu[j] + sub_off[s];
            memcpy(dst + drow * row_bytes, src + sub_cu[s] * row_bytes,
                   (size_t)sub_len[s] * (size_t)row_bytes);
        }
    }
    free(tmp);
    free(sub_cu);
    return rc;
}

/* Rearrangement composition with several sub-sequences per example (Sec. 6, subsequence
 * assembly: an example's subsequences of the different modalities are interleaved in a
 * predefined order, and one modality may contribute more than one of them, e.g. several
 * images between pieces of text).  The encoder still hands back example s's rows of this
 * modality as ONE run (its segment of the encoder assignment, or its place in original
 * order); that run is cut into the pieces piece_ptr[s] .. piece_ptr[s+1]-1, taken in that order:
 * piece p has piece_len[p] rows and goes to row piece_off[p] of the example's interleaved
 * sequence.  Same two steps as orc_pack_composed: reset to original example order, then place.
 * Pieces of one example must ascend without overlap (piece_off[p] >= end of the piece before);
 * returns -5 otherwise, or if a piece leaves its sequence, or an encoder segment is too short. */
int orc_pack_composed_pieces(const void *enc_rows, void *packed, const int32_t *piece_ptr,
                             const int32_t *piece_off, const int32_t *piece_len, int32_t n,
                             int64_t row_bytes, int32_t De, const int32_t *e_order,
                             const int32_t *e_seq_off, const int64_t *e_tok_off, const int32_t *e_cu,
                             int32_t Dm, const int32_t *m_order, const int32_t *m_seq_off,
                             const int64_t *m_tok_off, const int32_t *m_cu, int32_t inst_begin,
                             int32_t inst_end)
{
    if (n < 0 || Dm < 1 || inst_begin < 0 || inst_end > Dm || inst_begin > inst_end || row_bytes < 1)
        return -1;
    if (e_order && De < 1) return -1;
    if (piece_ptr[0] != 0) return -5;
    /* rows of this modality per example, and where each example starts in original order */
    int64_t *sub_cu = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n + 1));
    if (!sub_cu) return -1;
    sub_cu[0] = 0;
    for (int32_t s = 0; s < n; ++s) {
        if (piece_ptr[s + 1] < piece_ptr[s]) { free(sub_cu); return -5; }
        int64_t rows = 0;
        for (int32_t p = piece_ptr[s]; p < piece_ptr[s + 1]; ++p) {
            if (piece_len[p] < 0 || piece_off[p] < 0) { free(sub_cu); return -5; }
            rows += piece_len[p];
        }
        sub_cu[s + 1] = sub_cu[s] + rows;
    }
    const char *src = (const char *)enc_rows;
    char *tmp = NULL;
    /* step 1: reset to original example order */
    if (e_order) {
        tmp = (char *)malloc((size_t)(sub_cu[n] > 0 ? sub_cu[n] : 1) * (size_t)row_bytes);
        if (!tmp) { free(sub_cu); return -1; }
        for (int32_t i = 0; i < De; ++i) {
            const int32_t *cu = e_cu + e_seq_off[i] + i;
            for (int32_t j = 0; j < e_seq_off[i + 1] - e_seq_off[i]; ++j) {
                int32_t s = e_order[e_seq_off[i] + j];
                int64_t rows = sub_cu[s + 1] - sub_cu[s];
                if (cu[j + 1] - cu[j] < rows) { free(tmp); free(sub_cu); return -5; }
                memcpy(tmp + sub_cu[s] * row_bytes, src + (e_tok_off[i] + cu[j]) * row_bytes,
                       (size_t)rows * (size_t)row_bytes);
            }
        }
        src = tmp;
    }
    /* step 2: place the pieces inside the interleaved sequences of the destination instances */
    char *dst = (char *)packed;
    int rc = 0;
    for (int32_t i = inst_begin; i < inst_end && rc == 0; ++i) {
        const int32_t *cu = m_cu + m_seq_off[i] + i;
        for (int32_t j = 0; j < m_seq_off[i + 1] - m_seq_off[i] && rc == 0; ++j) {
            int32_t s = m_order[m_seq_off[i] + j];
            int64_t seq_rows = (int64_t)cu[j + 1] - cu[j];
            int64_t drow = m_tok_off[i] - m_tok_off[inst_begin] + cu[j];
            int64_t taken = 0, prev_end = 0;
            for (int32_t p = piece_ptr[s]; p < piece_ptr[s + 1]; ++p) {
                if (piece_off[p] < prev_end || (int64_t)piece_off[p] + piece_len[p] > seq_rows) { rc = -5; break; }
                memcpy(dst + (drow + piece_off[p]) * row_bytes, src + (sub_cu[s] + taken) * row_bytes,
                       (size_t)piece_len[p] * (size_t)row_bytes);
                taken += piece_len[p];
                prev_end = (int64_t)piece_off[p] + piece_len[p];
            }
        }
    }
    free(tmp);
    free(sub_cu);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Algorithm 2 (Sec. 5.1), the balancing for phases that batch with paddings.  A padded
 * batch of k sequences costs k * (its longest sequence) rows (Eq. 1, padding
 * branch); the algorithm sorts ascending, and for an upper bound b on that
 * batch length cuts the sorted list greedily into the fewest batches, then
 * binary-searches the smallest b that needs at most d batches.
 * ------------------------------------------------------------------------- */

/* Algorithm 2, line 1: indices in ascending length order; equal lengths keep
 * ascending index order (stable bottom-up merge sort). */
int orc_sort_asc(const int32_t *lengths, int32_t n, int32_t *sorted)
{
    if (n < 0 || (n > 0 && (!lengths || !sorted))) return -1;
    int32_t *a = sorted, *b = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!b) return -1;
    for (int32_t i = 0; i < n; ++i) a[i] = i;
    for (int64_t w = 1; w < n; w *= 2) {
        for (int64_t lo = 0; lo < n; lo += 2 * w) {
            int64_t mid = lo + w < n ? lo + w : n, hi = lo + 2 * w < n ? lo + 2 * w : n;
            int64_t i = lo, j = mid, k = lo;
            while (i < mid && j < hi) {
                /* take from the right run only when it is strictly shorter */
                if (lengths[a[j]] < lengths[a[i]]) b[k++] = a[j++];
                else b[k++] = a[i++];
            }
            while (i < mid) b[k++] = a[i++];
            while (j < hi) b[k++] = a[j++];
        }
        int32_t *t = a; a = b; b = t;
    }
    if (a != sorted) { memcpy(sorted, a, sizeof(int32_t) * (size_t)n); b = a; }
    free(b);
    return 0;
}

/* The batch-counting helper of Algorithm 2 (Sec. 5.1) for a bound b: walk the ascending list; the current batch
 * is closed (a new, empty one opened) when one more sequence would push its
 * padded length (count + 1) * length above b; the sequence is then put into the
 * last batch whatever its length.  batch_of[t] (may be NULL) receives the batch
 * of sorted position t.  Returns the number of batches, counting the initial
 * one even when it stays empty. */
int64_t orc_least_batches(const int32_t *lengths, const int32_t *sorted, int32_t n, uint64_t bound,
                          int32_t *batch_of)
{
    int64_t batches = 1;  /* the result starts as one empty batch */
    uint64_t in_last = 0;
    for (int32_t t = 0; t < n; ++t) {
        uint64_t len = (uint64_t)(uint32_t)lengths[sorted[t]];
        if ((in_last + 1) * len > bound) {
            ++batches;
            in_last = 0;
        }
        ++in_last;
        if (batch_of) batch_of[t] = (int32_t)(batches - 1);
    }
    return batches;
}

/* The whole of Algorithm 2 plus the layout of the padded batches.
 * Readings where the printed listing is garbled or silent:
 *   - the search starts at left = the shortest length, as printed, and
 *     right = (the LONGEST length) * (floor(n/d) + 1): the printed right bound
 *     takes the first (shortest) element, which need not be feasible, while with
 *     the longest one every batch can hold floor(n/d) + 1 >= ceil(n/d) sequences,
 *     so at most d batches are needed and the search has an answer;
 *   - loop body: mid = floor((left + right) / 2); if the helper at bound mid needs at
 *     most d batches then right = mid, else left = mid + 1;
 *   - the batches returned are the helper's at the final bound (the last mid
 *     tried may have been an infeasible one);
 *   - the k-th batch is instance k; when fewer than d batches result the last
 *     instances stay empty;
 *   - zero-length sequences are ordinary elements (they sort first and occupy a
 *     padded slot each).
 * Outputs (same shapes as orc_balance): inst, order (= the ascending order),
 * seq_off; cu_seqlens: instance i's slice holds j * max_i for j = 0..cnt_i, i.e.
 * every sequence owns max_i rows of the padded batch; tok_off: prefix of the
 * padded batch lengths cnt_i * max_i; loads[i] = Eq. 2's padding branch,
 * a * L_i^2 / cnt_i + b * L_i = cnt_i * (a * max_i^2 + b * max_i); *bound = the
 * smallest feasible b. */
int orc_balance_padded(const int32_t *lengths, int32_t n, int32_t D, uint64_t a, uint64_t b,
                       int32_t *inst, int32_t *order, int32_t *seq_off, int64_t *tok_off,
                       int32_t *cu_seqlens, uint64_t *loads, uint64_t *bound)
{
    if (n < 0 || D < 1) return -1;
    for (int32_t s = 0; s < n; ++s)
        if (lengths[s] < 0) return -5;
    size_t nn = (size_t)(n > 0 ? n : 1);
    int32_t *sorted = (int32_t *)malloc(nn * sizeof(int32_t));
    int32_t *batch_of = (int32_t *)malloc(nn * sizeof(int32_t));
    int rc = -1;
    if (!sorted || !batch_of) goto done;
    if ((rc = orc_sort_asc(lengths, n, sorted)) != 0) goto done;

    uint64_t left = 0, right = 0;
    if (n > 0) {
        left = (uint64_t)lengths[sorted[0]];
        right = (uint64_t)lengths[sorted[n - 1]] * ((uint64_t)(n / D) + 1);
    }
    while (left < right) {
        uint64_t mid = (left + right) / 2;
        if (orc_least_batches(lengths, sorted, n, mid, NULL) <= D) right = mid;
        else left = mid + 1;
    }
    if (orc_least_batches(lengths, sorted, n, left, batch_of) > D) { rc = -5; goto done; }
    if (bound) *bound = left;

    for (int32_t i = 0; i <= D; ++i) seq_off[i] = 0;
    for (int32_t t = 0; t < n; ++t) {
        order[t] = sorted[t];
        inst[sorted[t]] = batch_of[t];
        seq_off[batch_of[t] + 1]++;
    }
    for (int32_t i = 0; i < D; ++i) seq_off[i + 1] += seq_off[i];
    tok_off[0] = 0;
    rc = 0;
    for (int32_t i = 0; i < D; ++i) {
        int32_t cnt = seq_off[i + 1] - seq_off[i];
        uint64_t mx = cnt ? (uint64_t)lengths[order[seq_off[i + 1] - 1]] : 0;
        int32_t *cu = cu_seqlens + seq_off[i] + i;
        if ((uint64_t)cnt * mx > INT32_MAX) { rc = -5; goto done; }
        for (int32_t j = 0; j <= cnt; ++j) cu[j] = (int32_t)((uint64_t)j * mx);
        tok_off[i + 1] = tok_off[i] + (int64_t)((uint64_t)cnt * mx);
        unsigned __int128 c = ((unsigned __int128)a * mx * mx + (unsigned __int128)b * mx) * (unsigned __int128)cnt;
        if (c >> 63) { rc = -5; goto done; }
        loads[i] = (uint64_t)c;
    }
done:
    free(sorted); free(batch_of);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Appendix A, the third balancing algorithm: Algorithm 1 with the priority
 * queue ordered by CMP(a, b): when two batches' length sums differ by less than
 * the tolerance interval v, the one with the smaller sum of squared lengths comes
 * first, otherwise the one with the smaller length sum.  It serves the objective
 * max_i (L_i + lambda * sum_j l_ij^2) when beta << alpha does not hold.
 *
 * CMP is not a strict weak order (a ~ b and b ~ c within v do not give a ~ c), so
 * "the top of a priority queue sorted by CMP" is not defined by the listing.
 * Reading used here, two passes over the d batches:
 *   1. m = the smallest length sum;
 *   2. among the batches whose length sum is less than m + max(v, 1), take the
 *      one with the smallest sum of squares; ties go to the lowest batch index.
 * The chosen batch is never beaten under CMP by any batch inside that window, and
 * every batch outside the window has a length sum at least v above the minimum.
 * v <= 1 makes the window "length sum == m": Algorithm 1 on lengths, with the sum
 * of squares breaking ties; a v above the total length makes it the greedy on the
 * sum of squares alone.
 * Sorting is by length, descending, ties by ascending index (as Algorithm 1).
 * loads[i] = a * sum_sq_i + b * sum_i (Eq. 2, no-padding branch); the layout is
 * that of orc_balance. */
int orc_balance_tolerance(const int32_t *lengths, int32_t n, int32_t D, uint64_t v, uint64_t a,
                          uint64_t b, int32_t *inst, int32_t *order, int32_t *seq_off,
                          int64_t *tok_off, int32_t *cu_seqlens, uint64_t *loads)
{
    if (n < 0 || D < 1) return -1;
    size_t nn = (size_t)(n > 0 ? n : 1);
    uint64_t *key = (uint64_t *)malloc(nn * sizeof(uint64_t));
    int32_t *sorted = (int32_t *)malloc(nn * sizeof(int32_t));
    int32_t *rank = (int32_t *)malloc(nn * sizeof(int32_t));
    int32_t *counts = (int32_t *)calloc((size_t)D, sizeof(int32_t));
    uint64_t *sum = (uint64_t *)calloc((size_t)D, sizeof(uint64_t));
    uint64_t *sq = (uint64_t *)calloc((size_t)D, sizeof(uint64_t));
    int rc = -1;
    if (!key || !sorted || !rank || !counts || !sum || !sq) goto done;
    if ((rc = orc_cost(lengths, n, 0, 1, key)) != 0) goto done;      /* key = length */
    if ((rc = orc_sort_desc(key, n, sorted)) != 0) goto done;
    const uint64_t window = v > 1 ? v : 1;
    for (int32_t t = 0; t < n; ++t) {
        int32_t s = sorted[t];
        uint64_t m = sum[0];
        for (int32_t i = 1; i < D; ++i)
            if (sum[i] < m) m = sum[i];
        int32_t best = -1;
        for (int32_t i = 0; i < D; ++i)
            if (sum[i] - m < window && (best < 0 || sq[i] < sq[best])) best = i;
        uint64_t l = (uint64_t)lengths[s];
        unsigned __int128 nsq = (unsigned __int128)sq[best] + (unsigned __int128)l * l;
        if (nsq >> 63) { rc = -5; goto done; }
        inst[s] = best;
        rank[s] = counts[best]++;
        sum[best] += l;
        sq[best] = (uint64_t)nsq;
    }
    seq_off[0] = 0;
    for (int32_t i = 0; i < D; ++i) seq_off[i + 1] = seq_off[i] + counts[i];
    for (int32_t s = 0; s < n; ++s) order[seq_off[inst[s]] + rank[s]] = s;
    tok_off[0] = 0;
    rc = 0;
    for (int32_t i = 0; i < D; ++i) {
        int32_t *cu = cu_seqlens + seq_off[i] + i;
        int64_t run = 0;
        cu[0] = 0;
        for (int32_t j = 0; j < counts[i]; ++j) {
            run += lengths[order[seq_off[i] + j]];
            if (run > INT32_MAX) { rc = -5; goto done; }
            cu[j + 1] = (int32_t)run;
        }
        tok_off[i + 1] = tok_off[i] + run;
        unsigned __int128 c = (unsigned __int128)a * sq[i] + (unsigned __int128)b * sum[i];
        if (c >> 63) { rc = -5; goto done; }
        loads[i] = (uint64_t)c;
    }
done:
    free(key); free(sorted); free(rank); free(counts); free(sum); free(sq);
    return rc;
}

/* Communication-volume matrix of a rearrangement (Sec. 5.2.2, the node-wise rearrangement
 * algorithm's first loop): for every new batch i and every sequence l in it,
 * cost_matrix[l.from][i] += l.length.  `from` gives the instance a sequence was sampled on;
 * NULL means contiguous equal blocks, sequence s on instance floor(s * D_src / n).
 * Also the quantity the All-to-All overhead is proportional to when nodes hold c
 * consecutive instances (the section's overhead relation): for each source instance,
 * the tokens it sends to instances on OTHER nodes; out_inter may be NULL, c <= 0 skips it.
 * V is row-major [D_src][D_dst]. */
int orc_comm_volume(const int32_t *lengths, int32_t n, int32_t D_src, const int32_t *from,
                    int32_t D_dst, const int32_t *order, const int32_t *seq_off, uint64_t *V,
                    int32_t c, uint64_t *out_inter)
{
    if (n < 0 || D_src < 1 || D_dst < 1) return -1;
    for (int64_t e = 0; e < (int64_t)D_src * D_dst; ++e) V[e] = 0;
    for (int32_t i = 0; i < D_dst; ++i)
        for (int32_t p = seq_off[i]; p < seq_off[i + 1]; ++p) {
            int32_t s = order[p];
            int32_t f = from ? from[s] : (int32_t)(((int64_t)s * D_src) / n);
            if (lengths[s] < 0 || f < 0 || f >= D_src) return -5;
            V[(int64_t)f * D_dst + i] += (uint64_t)lengths[s];
        }
    if (out_inter && c > 0)
        for (int32_t f = 0; f < D_src; ++f) {
            out_inter[f] = 0;
            for (int32_t i = 0; i < D_dst; ++i)
                if (i / c != f / c) out_inter[f] += V[(int64_t)f * D_dst + i];
        }
    return 0;
}
