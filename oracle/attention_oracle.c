/* CPU oracle for variable-length packed attention (forward, and at the end of the file
 * its backward).  TEST
 * INFRASTRUCTURE: only tests, the smoke check and the bench's cpu_baseline leg
 * may call it; it shares no code with the HIP library and is never a fallback.
 *
 * The paper concatenates the sequences of a batch along the token axis without
 * padding and runs a flash-attention operator on them (Sec. 7, input preprocessing;
 * Appendix A); the quantity that operator computes is the Transformer's
 * scaled-dot-product attention whose quadratic term is beta*sum(l^2) in Eq. 2.
 * This file is that definition written out, in fp64, on bf16-rounded inputs:
 *
 *   for each sequence t (rows cu[t] .. cu[t+1]), q-head h, kv-head
 *   g = h / (Hq/Hkv), row i:
 *       s_j = scale * sum_x q[i,h,x] * k[j,g,x]   over visible j
 *             (all rows of the sequence; j <= i when causal)
 *       p_j = exp(s_j - max s) / sum_j exp(s_j - max s)
 *       out[i,h,:] = sum_j p_j * v[j,g,:]
 *       lse[h,i]   = max s + log(sum_j exp(s_j - max s))
 *
 * Layout: q [T,Hq,d], k,v [T,Hkv,d], token-major, bf16 bit patterns (uint16).
 * Outputs are fp64 (not rounded).  No blocking, no online softmax.
 * Return value 0 = ok, -1 = bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* One output row: sequence rows [r0, r1), query at absolute row i, head h. */
static void attn_row(const uint16_t *q, const uint16_t *k, const uint16_t *v, int64_t r0, int64_t r1,
                     int64_t i, int32_t h, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                     int causal, double *s, double *out_row, double *lse)
{
    int32_t g = h / (Hq / Hkv);
    int64_t jend = causal ? i + 1 : r1;
    const uint16_t *qi = q + ((size_t)i * Hq + h) * d;
    double m = -INFINITY;
    for (int64_t j = r0; j < jend; ++j) {
        const uint16_t *kj = k + ((size_t)j * Hkv + g) * d;
        double acc = 0.0;
        for (int32_t x = 0; x < d; ++x) acc += bf16_to_double(qi[x]) * bf16_to_double(kj[x]);
        s[j - r0] = acc * scale;
        if (s[j - r0] > m) m = s[j - r0];
    }
    double z = 0.0;
    for (int64_t j = r0; j < jend; ++j) { s[j - r0] = exp(s[j - r0] - m); z += s[j - r0]; }
    for (int32_t x = 0; x < d; ++x) out_row[x] = 0.0;
    for (int64_t j = r0; j < jend; ++j) {
        const uint16_t *vj = v + ((size_t)j * Hkv + g) * d;
        double p = s[j - r0] / z;
        for (int32_t x = 0; x < d; ++x) out_row[x] += p * bf16_to_double(vj[x]);
    }
    if (lse) *lse = m + log(z);
}

/* Full forward.  out: fp64 [T,Hq,d]; lse: fp64 [Hq,T] or NULL, where T =
 * total_tokens >= cu[batch] is the row count of the buffers.
 * nthreads <= 0 means one thread.  Returns the thread count used via *used. */
int orc_attn_fwd(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *out, double *lse,
                 const int32_t *cu, int32_t batch, int64_t total_tokens, int32_t Hq, int32_t Hkv,
                 int32_t d, double scale, int causal, int nthreads, int *used)
{
    if (batch < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || !cu) return -1;
    for (int32_t t = 0; t < batch; ++t) if (cu[t + 1] < cu[t]) return -1;
    if (scale <= 0) scale = 1.0 / sqrt((double)d);
    int64_t T = total_tokens;
    if (batch > 0 && cu[batch] > T) return -1;
    int32_t maxlen = 0;
    for (int32_t t = 0; t < batch; ++t) if (cu[t + 1] - cu[t] > maxlen) maxlen = cu[t + 1] - cu[t];
    if (nthreads < 1) nthreads = 1;
    int nused = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
    {
#ifdef _OPENMP
#pragma omp single
        nused = omp_get_num_threads();
#endif
        double *s = (double *)malloc(sizeof(double) * (size_t)(maxlen > 0 ? maxlen : 1));
#ifdef _OPENMP
#pragma omp for collapse(2) schedule(dynamic, 1)
#endif
        for (int32_t t = 0; t < batch; ++t)
            for (int32_t h = 0; h < Hq; ++h)
                for (int64_t i = cu[t]; i < cu[t + 1]; ++i)
                    attn_row(q, k, v, cu[t], cu[t + 1], i, h, Hq, Hkv, d, scale, causal, s,
                             out + ((size_t)i * Hq + h) * d, lse ? lse + (size_t)h * T + i : NULL);
        free(s);
    }
    if (used) *used = nused;
    return 0;
}

/* Sampled rows: for each m, output row (abs_row[m], head[m]) of sequence seq[m].
 * out: fp64 [M, d]; lse: fp64 [M] or NULL. */
int orc_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *cu,
                  int32_t batch, int32_t Hq, int32_t Hkv, int32_t d, double scale, int causal,
                  const int32_t *seq, const int32_t *head, const int32_t *abs_row, int32_t M,
                  double *out, double *lse, int nthreads)
{
    if (batch < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || M < 0) return -1;
    if (scale <= 0) scale = 1.0 / sqrt((double)d);
    int32_t maxlen = 0;
    for (int32_t m = 0; m < M; ++m) {
        int32_t t = seq[m];
        if (t < 0 || t >= batch || head[m] < 0 || head[m] >= Hq) return -1;
        if (abs_row[m] < cu[t] || abs_row[m] >= cu[t + 1]) return -1;
        if (cu[t + 1] - cu[t] > maxlen) maxlen = cu[t + 1] - cu[t];
    }
    if (nthreads < 1) nthreads = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(maxlen > 0 ? maxlen : 1));
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int32_t m = 0; m < M; ++m) {
            int32_t t = seq[m];
            attn_row(q, k, v, cu[t], cu[t + 1], abs_row[m], head[m], Hq, Hkv, d, scale, causal, s,
                     out + (size_t)m * d, lse ? lse + m : NULL);
        }
        free(s);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Backward of the attention defined above, for one (sequence, kv-head) unit: the
 * gradient of  sum_{i,h,x} dout[i,h,x] * out[i,h,x]  with respect to q, k and v,
 * written out from the definition in fp64 (the back-propagation that mirrors the
 * forward pass, Sec. 5.3):
 *   p_ij   as in the forward pass
 *   dp_ij  = sum_x dout[i,h,x] * v[j,g,x]
 *   delta_i = sum_j p_ij * dp_ij
 *   ds_ij  = p_ij * (dp_ij - delta_i)
 *   dq[i,h,:]  = scale * sum_j ds_ij * k[j,g,:]
 *   dk[j,g,:]  = scale * sum_{h in group of g} sum_i ds_ij * q[i,h,:]
 *   dv[j,g,:]  =         sum_{h in group of g} sum_i p_ij  * dout[i,h,:]
 * Rows [r0, r1) are the sequence; outputs are local to the unit:
 *   dq_out [r1-r0, group, d], dk_out and dv_out [r1-r0, d], all fp64, overwritten.
 * Threads split the query rows; each keeps its own dk/dv partial sums, added in thread order.
 * ------------------------------------------------------------------------- */
int orc_attn_bwd_unit(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *dout,
                      int64_t r0, int64_t r1, int32_t g, int32_t Hq, int32_t Hkv, int32_t d,
                      double scale, int causal, double *dq_out, double *dk_out, double *dv_out,
                      int nthreads)
{
    if (r1 < r0 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1 || g < 0 || g >= Hkv) return -1;
    if (scale <= 0) scale = 1.0 / sqrt((double)d);
    const int32_t group = Hq / Hkv;
    const int64_t L = r1 - r0;
    if (nthreads < 1) nthreads = 1;
    for (int64_t e = 0; e < L * d; ++e) { dk_out[e] = 0.0; dv_out[e] = 0.0; }
    double *part = (double *)calloc((size_t)nthreads * 2 * (size_t)(L > 0 ? L : 1) * (size_t)d, sizeof(double));
    if (!part) return -1;
    int nused = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(nthreads)
#endif
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#pragma omp single
        nused = omp_get_num_threads();
#endif
        double *pk = part + (size_t)tid * 2 * (size_t)L * d, *pv = pk + (size_t)L * d;
        double *p = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        double *dp = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
#ifdef _OPENMP
#pragma omp for collapse(2) schedule(dynamic, 4)
#endif
        for (int32_t hh = 0; hh < group; ++hh)
            for (int64_t i = r0; i < r1; ++i) {
                const int32_t h = g * group + hh;
                const int64_t jend = causal ? i + 1 : r1;
                const uint16_t *qi = q + ((size_t)i * Hq + h) * d;
                const uint16_t *doi = dout + ((size_t)i * Hq + h) * d;
                double m = -INFINITY;
                for (int64_t j = r0; j < jend; ++j) {
                    const uint16_t *kj = k + ((size_t)j * Hkv + g) * d;
                    const uint16_t *vj = v + ((size_t)j * Hkv + g) * d;
                    double s = 0.0, t = 0.0;
                    for (int32_t x = 0; x < d; ++x) {
                        s += bf16_to_double(qi[x]) * bf16_to_double(kj[x]);
                        t += bf16_to_double(doi[x]) * bf16_to_double(vj[x]);
                    }
                    p[j - r0] = s * scale;
                    dp[j - r0] = t;
                    if (p[j - r0] > m) m = p[j - r0];
                }
                double z = 0.0;
                for (int64_t j = r0; j < jend; ++j) { p[j - r0] = exp(p[j - r0] - m); z += p[j - r0]; }
                double delta = 0.0;
                for (int64_t j = r0; j < jend; ++j) { p[j - r0] /= z; delta += p[j - r0] * dp[j - r0]; }
                double *dqi = dq_out + ((size_t)(i - r0) * group + hh) * d;
                for (int32_t x = 0; x < d; ++x) dqi[x] = 0.0;
                for (int64_t j = r0; j < jend; ++j) {
                    const uint16_t *kj = k + ((size_t)j * Hkv + g) * d;
                    const double pij = p[j - r0], ds = pij * (dp[j - r0] - delta) * scale;
                    double *dkj = pk + (size_t)(j - r0) * d, *dvj = pv + (size_t)(j - r0) * d;
                    for (int32_t x = 0; x < d; ++x) {
                        dqi[x] += ds * bf16_to_double(kj[x]);
                        dkj[x] += ds * bf16_to_double(qi[x]);
                        dvj[x] += pij * bf16_to_double(doi[x]);
                    }
                }
            }
        free(p);
        free(dp);
    }
    for (int t = 0; t < nused; ++t) {
        const double *pk = part + (size_t)t * 2 * (size_t)L * d, *pv = pk + (size_t)L * d;
        for (int64_t e = 0; e < L * d; ++e) { dk_out[e] += pk[e]; dv_out[e] += pv[e]; }
    }
    free(part);
    return 0;
}
