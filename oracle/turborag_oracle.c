/*
 * TurboRAG online-prefill hot path: plain CPU reference ("oracle"), fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the HIP library computes.  It shares no code, header, table or helper
 * with the GPU path and must never be linked or called by it.  Only the test
 * suite, the smoke check and the bench's cpu_baseline leg may use it.
 *
 * Every function follows the paper's definition directly (arXiv 2410.07590):
 *   - RoPE rotation .................. Eq. 3 (Sec. 3.1), theta_m = base^(-2m/d)
 *   - scaled scores, mask, softmax ... Eq. 2, Eq. 4 and the text after Eq. 4
 *   - independent attention mask ..... Sec. 3.2 (no cross-attention between chunks)
 *   - composite / reordered ids ...... Sec. 3.2
 *   - KV-cache formation / prefill ... Sec. 3.4, steps 2, 5 and 6
 * There is no blocking, fusion or reordering: one loop nest per definition.
 * Storage-typed inputs (fp32 or bf16 bit patterns) are widened exactly to
 * double on load; all arithmetic is double; OpenMP only splits independent
 * (query row, head) pairs across cores.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (closed forms, invariants, library routines on special cases, brute force).
 * The paper prints no worked numeric attention example, so no printed value
 * pins the attention numbers; they are pinned by those independent routes.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_ROPE_INTERLEAVED = 0, ORC_ROPE_HALF = 1 };
enum { ORC_POS_COMPOSITE = 0, ORC_POS_REORDERED = 1 };

/* ---- storage <-> double -------------------------------------------------- */

/* Exact widening of element i of a storage-typed array. */
static double load_elem(const void* p, int64_t i, int dtype)
{
    if (dtype == ORC_F32) return (double)((const float*)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t*)p)[i] << 16; /* bf16 = top half of an fp32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Round a double to the nearest bfloat16 (ties to even), by the definition of
 * rounding: scale so that one unit in the last place becomes 1, round to the
 * nearest integer (ties to even), scale back.  bf16 has 8 significant bits and
 * fp32's exponent range (min normal exponent -126, subnormal ulp 2^-133). */
static uint16_t round_to_bf16(double x)
{
    float f;
    if (isnan(x)) {
        f = NAN;
    } else if (isinf(x) || x == 0.0) {
        f = (float)x;
    } else {
        int e;
        frexp(x, &e);              /* |x| = m * 2^e, 0.5 <= m < 1  ->  2^(e-1) <= |x| < 2^e */
        int ulp_exp = (e - 1) - 7; /* 8 significant bits */
        if (ulp_exp < -133) ulp_exp = -133;
        double q = nearbyint(ldexp(x, -ulp_exp)); /* default rounding mode: ties to even */
        double r = ldexp(q, ulp_exp);
        if (fabs(r) >= ldexp(1.0, 128)) r = copysign(INFINITY, x); /* above the largest finite bf16 */
        f = (float)r;              /* exact: r is representable */
    }
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return (uint16_t)(bits >> 16);
}

/* out[i] = round_to_storage(x[i]); out is float* (ORC_F32) or uint16_t* (ORC_BF16). */
void orc_round(const double* x, int64_t n, int dtype, void* out)
{
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == ORC_F32) ((float*)out)[i] = (float)x[i];
        else ((uint16_t*)out)[i] = round_to_bf16(x[i]);
    }
}

/* out[i] = (double)storage[i] */
void orc_widen(const void* x, int64_t n, int dtype, double* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = load_elem(x, i, dtype);
}

/* ---- RoPE (Eq. 3) ---------------------------------------------------------- */

/* theta[m] = base^(-2m/d), m = 0 .. d/2-1 (text after Eq. 3; base is 10000 there). */
void orc_theta(double base, int d, double* theta)
{
    for (int m = 0; m < d / 2; ++m) theta[m] = pow(base, -2.0 * (double)m / (double)d);
}

/* Rotate one head vector x[0..d) by position p into y (Eq. 3).  Pair m is
 * (x[2m], x[2m+1]) in the interleaved layout the equation prints, or
 * (x[m], x[m+d/2]) in the half-split layout; both turn the pair by p*theta_m:
 *   y_a = x_a cos - x_b sin ,  y_b = x_b cos + x_a sin. */
static void rope_vec(const double* x, double* y, int d, double p, const double* theta, int layout)
{
    for (int m = 0; m < d / 2; ++m) {
        int a = (layout == ORC_ROPE_INTERLEAVED) ? 2 * m : m;
        int b = (layout == ORC_ROPE_INTERLEAVED) ? 2 * m + 1 : m + d / 2;
        double ang = p * theta[m];
        double c = cos(ang), s = sin(ang);
        double xa = x[a], xb = x[b];
        y[a] = xa * c - xb * s;
        y[b] = xb * c + xa * s;
    }
}

/* x: storage-typed [n_rows, n_heads, d]; pos[n_rows] (may be negative);
 * out: double [n_rows, n_heads, d] = R(pos[row]) x. */
void orc_rope(const void* x, int dtype, int64_t n_rows, int n_heads, int d,
              const int64_t* pos, double base, int layout, double* out)
{
    double* theta = (double*)malloc(sizeof(double) * (size_t)(d / 2));
    double* tmp = (double*)malloc(sizeof(double) * (size_t)d);
    orc_theta(base, d, theta);
    for (int64_t r = 0; r < n_rows; ++r)
        for (int h = 0; h < n_heads; ++h) {
            int64_t o = (r * n_heads + h) * (int64_t)d;
            for (int e = 0; e < d; ++e) tmp[e] = load_elem(x, o + e, dtype);
            rope_vec(tmp, out + o, d, (double)pos[r], theta, layout);
        }
    free(tmp);
    free(theta);
}

/* Same, for an input already in double (used to chain rotations in tests). */
void orc_rope_f64(const double* x, int64_t n_rows, int n_heads, int d,
                  const int64_t* pos, double base, int layout, double* out)
{
    double* theta = (double*)malloc(sizeof(double) * (size_t)(d / 2));
    double* tmp = (double*)malloc(sizeof(double) * (size_t)d);
    orc_theta(base, d, theta);
    for (int64_t r = 0; r < n_rows; ++r)
        for (int h = 0; h < n_heads; ++h) {
            int64_t o = (r * n_heads + h) * (int64_t)d;
            memcpy(tmp, x + o, sizeof(double) * (size_t)d);
            rope_vec(tmp, out + o, d, (double)pos[r], theta, layout);
        }
    free(tmp);
    free(theta);
}

/* ---- gather plan and position ids (Sec. 3.2; Sec. 3.4 step 5) --------------- */

/* row_start[n_store+1]: chunk c of the store owns rows [row_start[c], row_start[c+1]).
 * For the k retrieved ids, in order:
 *   offsets[i] = sum of the lengths of the chunks before i, offsets[k] = n_doc;
 *   delta[i]   = rotation still owed to chunk i's stored keys, which already sit
 *                at chunk-local positions: 0 (composite) or offsets[i] (reordered);
 *   pos[offsets[i] + t] = t (composite) or offsets[i] + t (reordered).
 * pos may be NULL.  Returns 0, or -1 when an id is outside [0, n_store). */
int orc_plan(const int64_t* row_start, int n_store, const int32_t* chunk_ids, int k,
             int pos_mode, int64_t* offsets, int64_t* delta, int32_t* pos)
{
    int64_t off = 0;
    for (int i = 0; i < k; ++i) {
        int32_t c = chunk_ids[i];
        if (c < 0 || c >= n_store) return -1;
        int64_t len = row_start[c + 1] - row_start[c];
        offsets[i] = off;
        delta[i] = (pos_mode == ORC_POS_REORDERED) ? off : 0;
        if (pos)
            for (int64_t t = 0; t < len; ++t)
                pos[off + t] = (int32_t)((pos_mode == ORC_POS_REORDERED) ? off + t : t);
        off += len;
    }
    offsets[k] = off;
    return 0;
}

/* ---- contextual KV-cache formation (Sec. 3.4 step 5) ------------------------ */

/* k_store, v_store: storage-typed [store_rows, n_kv, d]; keys stored already
 * rotated at chunk-local positions.  out_k, out_v: double [n_doc, n_kv, d]:
 *   out_v[offsets[i]+t] = V_store[c_i][t]
 *   out_k[offsets[i]+t] = R(delta[i]) K'_store[c_i][t]      (delta 0: plain copy)
 * Rotating a key that sits at position t by delta puts it at position t+delta,
 * which is what "Eq. 3 with the new position IDs" yields (Sec. 3.2). */
void orc_assemble(const void* k_store, const void* v_store, int dtype,
                  const int64_t* row_start, const int32_t* chunk_ids, int k,
                  const int64_t* offsets, const int64_t* delta,
                  int n_kv, int d, double base, int layout,
                  double* out_k, double* out_v)
{
    double* theta = (double*)malloc(sizeof(double) * (size_t)(d / 2));
    double* tmp = (double*)malloc(sizeof(double) * (size_t)d);
    orc_theta(base, d, theta);
    for (int i = 0; i < k; ++i) {
        int64_t src0 = row_start[chunk_ids[i]];
        int64_t len = row_start[chunk_ids[i] + 1] - src0;
        for (int64_t t = 0; t < len; ++t)
            for (int h = 0; h < n_kv; ++h) {
                int64_t so = ((src0 + t) * n_kv + h) * (int64_t)d;
                int64_t dn = ((offsets[i] + t) * n_kv + h) * (int64_t)d;
                for (int e = 0; e < d; ++e) {
                    out_v[dn + e] = load_elem(v_store, so + e, dtype);
                    tmp[e] = load_elem(k_store, so + e, dtype);
                }
                if (delta[i] == 0) memcpy(out_k + dn, tmp, sizeof(double) * (size_t)d);
                else rope_vec(tmp, out_k + dn, d, (double)delta[i], theta, layout);
            }
    }
    free(tmp);
    free(theta);
}

/* ---- masked softmax attention (Eq. 2, Eq. 4, Sec. 3.2) ---------------------- */

/* One output row: query vector qv (already rotated), keys/values of KV head kvh
 * in k, v [*, n_kv, d]; the visible keys are rows lo..hi inclusive.  Masked keys
 * get zero weight (score -inf before the softmax).  scratch holds hi-lo+1 doubles. */
static void attend_row(const double* qv, const double* k, const double* v, int n_kv, int kvh, int d,
                       int64_t lo, int64_t hi, double* scratch, double* o)
{
    double scale = 1.0 / sqrt((double)d);
    double smax = -INFINITY;
    for (int64_t j = lo; j <= hi; ++j) {
        const double* kv = k + (j * n_kv + kvh) * (int64_t)d;
        double s = 0.0;
        for (int e = 0; e < d; ++e) s += qv[e] * kv[e];
        s *= scale;
        scratch[j - lo] = s;
        if (s > smax) smax = s;
    }
    double denom = 0.0;
    for (int64_t j = lo; j <= hi; ++j) {
        scratch[j - lo] = exp(scratch[j - lo] - smax);
        denom += scratch[j - lo];
    }
    for (int e = 0; e < d; ++e) o[e] = 0.0;
    for (int64_t j = lo; j <= hi; ++j) {
        const double* vv = v + (j * n_kv + kvh) * (int64_t)d;
        double w = scratch[j - lo] / denom;
        for (int e = 0; e < d; ++e) o[e] += w * vv[e];
    }
}

/* Query prefill over an assembled cache (Sec. 3.4 step 6).
 *   q_rot [n_q, n_qh, d] rotated queries; k, v [kv_len, n_kv, d]; the last n_q
 *   cache rows are the query tokens themselves.  Query token i sees every
 *   document row and query rows up to itself: j <= kv_len - n_q + i.
 *   Query head h reads KV head h / (n_qh / n_kv).
 * Only the tokens listed in rows[0..n_rows) are computed:
 *   out [n_rows, n_qh, d]. */
void orc_attn_prefix(const double* q_rot, const double* k, const double* v,
                     int n_q, int64_t kv_len, int n_qh, int n_kv, int d,
                     const int32_t* rows, int n_rows, double* out)
{
    int g = n_qh / n_kv;
    int64_t n_doc = kv_len - n_q;
    int64_t work = (int64_t)n_rows * n_qh;
#pragma omp parallel
    {
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(kv_len > 0 ? kv_len : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < work; ++w) {
            int r = (int)(w / n_qh), h = (int)(w % n_qh);
            int i = rows[r];
            attend_row(q_rot + ((int64_t)i * n_qh + h) * d, k, v, n_kv, h / g, d,
                       0, n_doc + i, scratch, out + ((int64_t)r * n_qh + h) * d);
        }
        free(scratch);
    }
}

/* Offline chunk prefill (Sec. 3.4 step 2) under independent attention (Sec. 3.2):
 * tokens of all chunks packed [T, heads, d]; chunk c owns rows [cu[c], cu[c+1]).
 * Token t of chunk c sees rows cu[c] .. t of its own chunk only.
 * q_rot, k_rot are already rotated at chunk-local positions t - cu[c].
 * rows[] lists the packed token indices to compute: out [n_rows, n_qh, d]. */
void orc_attn_blockdiag(const double* q_rot, const double* k_rot, const double* v,
                        const int32_t* cu, int n_chunks, int n_qh, int n_kv, int d,
                        const int32_t* rows, int n_rows, double* out)
{
    int g = n_qh / n_kv;
    int64_t work = (int64_t)n_rows * n_qh;
    int64_t max_len = 1;
    for (int c = 0; c < n_chunks; ++c)
        if (cu[c + 1] - cu[c] > max_len) max_len = cu[c + 1] - cu[c];
#pragma omp parallel
    {
        double* scratch = (double*)malloc(sizeof(double) * (size_t)max_len);
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < work; ++w) {
            int r = (int)(w / n_qh), h = (int)(w % n_qh);
            int t = rows[r];
            int c = 0;
            while (!(cu[c] <= t && t < cu[c + 1])) ++c; /* the chunk that owns token t */
            attend_row(q_rot + ((int64_t)t * n_qh + h) * d, k_rot, v, n_kv, h / g, d,
                       cu[c], t, scratch, out + ((int64_t)r * n_qh + h) * d);
        }
        free(scratch);
    }
}

/* ---- one pass over a packed sequence with a per-token visible range (Sec. 3.3: fine-tuning uses the masks and
 * position ids of inference; Sec. 3.2 independent attention for the documents, full attention for the query).
 * Token t sees rows lo[t] .. t.  q_rot, k_rot are already rotated at the tokens' position ids.
 * rows[] lists the packed token indices to compute: out [n_rows, n_qh, d]. */
void orc_attn_rows(const double* q_rot, const double* k_rot, const double* v, const int32_t* lo, int64_t total,
                   int n_qh, int n_kv, int d, const int32_t* rows, int n_rows, double* out)
{
    int g = n_qh / n_kv;
    int64_t work = (int64_t)n_rows * n_qh;
#pragma omp parallel
    {
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t w = 0; w < work; ++w) {
            int r = (int)(w / n_qh), h = (int)(w % n_qh);
            int t = rows[r];
            attend_row(q_rot + ((int64_t)t * n_qh + h) * d, k_rot, v, n_kv, h / g, d,
                       lo[t], t, scratch, out + ((int64_t)r * n_qh + h) * d);
        }
        free(scratch);
    }
}

/* Number of OpenMP threads the attention loops will use. */
int orc_num_threads(void)
{
    return omp_get_max_threads();
}
