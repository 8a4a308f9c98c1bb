/* The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.
 *
 * Built by tests/test_sanitizers.py together with oracle/turborag_oracle.c (gcc -fsanitize=address,undefined).
 * Every exported routine runs on small ragged inputs held in exactly sized heap blocks, so that a read or write
 * one element outside any of them stops the run.  A few results with closed forms are checked as well (a rotation
 * keeps the norm; attention over constant values returns that constant), so that the calls cannot be optimised
 * into nothing.  Exit status 0 and "oracle sanitizer run ok" on stdout mean nothing fired. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

enum { F32 = 0, BF16 = 1 };

void orc_round(const double* x, int64_t n, int dtype, void* out);
void orc_widen(const void* x, int64_t n, int dtype, double* out);
void orc_theta(double base, int d, double* theta);
void orc_rope(const void* x, int dtype, int64_t n_rows, int n_heads, int d, const int64_t* pos, double base, int layout, double* out);
void orc_rope_f64(const double* x, int64_t n_rows, int n_heads, int d, const int64_t* pos, double base, int layout, double* out);
int orc_plan(const int64_t* row_start, int n_store, const int32_t* chunk_ids, int k, int pos_mode, int64_t* offsets, int64_t* delta, int32_t* pos);
void orc_assemble(const void* k_store, const void* v_store, int dtype, const int64_t* row_start, const int32_t* chunk_ids, int k,
                  const int64_t* offsets, const int64_t* delta, int n_kv, int d, double base, int layout, double* out_k, double* out_v);
void orc_attn_prefix(const double* q_rot, const double* k, const double* v, int n_q, int64_t kv_len, int n_qh, int n_kv, int d,
                     const int32_t* rows, int n_rows, double* out);
void orc_attn_blockdiag(const double* q_rot, const double* k_rot, const double* v, const int32_t* cu, int n_chunks, int n_qh, int n_kv, int d,
                        const int32_t* rows, int n_rows, double* out);
void orc_attn_rows(const double* q_rot, const double* k_rot, const double* v, const int32_t* lo, int64_t total, int n_qh, int n_kv, int d,
                   const int32_t* rows, int n_rows, double* out);
int orc_num_threads(void);

static uint64_t rng_state = 88172645463325252ull;
static double draw(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 4.0 - 2.0;
}
static int draw_int(int lo, int hi) { return lo + (int)((draw() + 2.0) / 4.0 * (hi - lo + 1)) % (hi - lo + 1); }

static void* exact(size_t n, size_t elem)
{
    void* p = malloc((n * elem) != 0 ? n * elem : 1);
    if (!p) { fprintf(stderr, "oracle_san: out of memory\n"); exit(2); }
    return p;
}
static double* doubles(size_t n, int constant, double value)
{
    double* p = (double*)exact(n, sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = constant ? value : draw();
    return p;
}
#define CHECK(cond, msg) do { if (!(cond)) { fprintf(stderr, "oracle_san: %s:%d: %s\n", __FILE__, __LINE__, msg); exit(1); } } while (0)

static void one_case(int dtype, int n_qh, int n_kv, int d, int layout, double base)
{
    const size_t esz = dtype == BF16 ? 2 : 4;
    /* a ragged store, one empty chunk included */
    const int n_store = draw_int(2, 7);
    int64_t* row_start = (int64_t*)exact((size_t)n_store + 1, sizeof(int64_t));
    row_start[0] = 0;
    for (int c = 0; c < n_store; ++c) row_start[c + 1] = row_start[c] + (c == 1 ? 0 : draw_int(1, 37));
    const int64_t store_rows = row_start[n_store];
    const size_t store_elems = (size_t)store_rows * n_kv * d;
    double* wide = doubles(store_elems, 0, 0);
    void* ks = exact(store_elems, esz);
    void* vs = exact(store_elems, esz);
    orc_round(wide, (int64_t)store_elems, dtype, ks);
    orc_round(wide, (int64_t)store_elems, dtype, vs);
    double* back = (double*)exact(store_elems, sizeof(double));
    orc_widen(ks, (int64_t)store_elems, dtype, back);
    for (size_t i = 0; i < store_elems; ++i) CHECK(fabs(back[i] - wide[i]) <= 0.00782 * fabs(wide[i]) + 1e-30, "rounding moved a value by more than half a bf16 step");

    /* plan: an out-of-range id is refused, a valid list fills offsets, delta and pos exactly */
    const int k = draw_int(1, 6);
    int32_t* ids = (int32_t*)exact((size_t)k, sizeof(int32_t));
    int64_t n_doc = 0;
    for (int i = 0; i < k; ++i) { ids[i] = draw_int(0, n_store - 1); n_doc += row_start[ids[i] + 1] - row_start[ids[i]]; }
    int64_t* offsets = (int64_t*)exact((size_t)k + 1, sizeof(int64_t));
    int64_t* delta = (int64_t*)exact((size_t)k, sizeof(int64_t));
    int32_t* pos = (int32_t*)exact((size_t)n_doc, sizeof(int32_t));
    for (int mode = 0; mode < 2; ++mode) {
        CHECK(orc_plan(row_start, n_store, ids, k, mode, offsets, delta, pos) == 0, "plan refused valid ids");
        CHECK(offsets[k] == n_doc, "plan: total length");
        CHECK(orc_plan(row_start, n_store, ids, k, mode, offsets, delta, NULL) == 0, "plan without position ids");
    }
    {
        int32_t bad = n_store;
        int64_t o2[2], d2[1];
        CHECK(orc_plan(row_start, n_store, &bad, 1, 0, o2, d2, NULL) == -1, "plan accepted an id past the store");
        bad = -1;
        CHECK(orc_plan(row_start, n_store, &bad, 1, 0, o2, d2, NULL) == -1, "plan accepted a negative id");
    }

    /* assemble under reordered positions: keys keep their norm, values are copied */
    const size_t doc_elems = (size_t)n_doc * n_kv * d;
    double* ak = (double*)exact(doc_elems, sizeof(double));
    double* av = (double*)exact(doc_elems, sizeof(double));
    orc_assemble(ks, vs, dtype, row_start, ids, k, offsets, delta, n_kv, d, base, layout, ak, av);
    for (int i = 0; i < k; ++i) {
        const int64_t len = row_start[ids[i] + 1] - row_start[ids[i]];
        for (int64_t t = 0; t < len; ++t) {
            double n0 = 0, n1 = 0;
            for (int e = 0; e < n_kv * d; ++e) {
                const double x = back[(row_start[ids[i]] + t) * n_kv * d + e], y = ak[(offsets[i] + t) * n_kv * d + e];
                n0 += x * x;
                n1 += y * y;
                CHECK(av[(offsets[i] + t) * n_kv * d + e] == x, "assemble changed a value row");
            }
            CHECK(fabs(n0 - n1) <= 1e-9 * (n0 + 1), "assemble changed the norm of a key row");
        }
    }

    /* rope on storage-typed and on double rows, negative positions included */
    const int n_q = draw_int(1, 9);
    const size_t q_elems = (size_t)n_q * n_qh * d;
    double* qw = doubles(q_elems, 0, 0);
    void* qs = exact(q_elems, esz);
    orc_round(qw, (int64_t)q_elems, dtype, qs);
    int64_t* qpos = (int64_t*)exact((size_t)n_q, sizeof(int64_t));
    for (int i = 0; i < n_q; ++i) qpos[i] = n_doc + i - (i == 0 ? 3 * n_doc + 5 : 0);
    double* q_rot = (double*)exact(q_elems, sizeof(double));
    double* q_rot2 = (double*)exact(q_elems, sizeof(double));
    orc_rope(qs, dtype, n_q, n_qh, d, qpos, base, layout, q_rot);
    orc_rope_f64(q_rot, n_q, n_qh, d, qpos, base, layout, q_rot2);
    double* theta = (double*)exact((size_t)d / 2, sizeof(double));
    orc_theta(base, d, theta);
    CHECK(theta[0] == 1.0 && theta[d / 2 - 1] < 1.0, "theta");

    /* query prefill over [documents | query tokens] with constant values: every output equals the constant */
    const int64_t kv_len = n_doc + n_q;
    const size_t kv_elems = (size_t)kv_len * n_kv * d;
    double* ck = doubles(kv_elems, 0, 0);
    double* cv = doubles(kv_elems, 1, 0.625);
    int32_t* rows = (int32_t*)exact((size_t)n_q, sizeof(int32_t));
    for (int i = 0; i < n_q; ++i) rows[i] = n_q - 1 - i;
    double* out = (double*)exact(q_elems, sizeof(double));
    orc_attn_prefix(q_rot, ck, cv, n_q, kv_len, n_qh, n_kv, d, rows, n_q, out);
    for (size_t i = 0; i < q_elems; ++i) CHECK(fabs(out[i] - 0.625) < 1e-12, "prefix attention over constant values");
    orc_attn_prefix(q_rot, ck, cv, n_q, kv_len, n_qh, n_kv, d, rows, 1, out); /* a single listed row */

    /* block-diagonal and per-row-range attention over packed ragged chunks, first and last token of each chunk */
    const int n_chunks = draw_int(1, 5);
    int32_t* cu = (int32_t*)exact((size_t)n_chunks + 1, sizeof(int32_t));
    cu[0] = 0;
    for (int c = 0; c < n_chunks; ++c) cu[c + 1] = cu[c] + draw_int(1, 23);
    const int T = cu[n_chunks];
    double* pq = doubles((size_t)T * n_qh * d, 0, 0);
    double* pk = doubles((size_t)T * n_kv * d, 0, 0);
    double* pv = doubles((size_t)T * n_kv * d, 1, -1.5);
    int32_t* lo = (int32_t*)exact((size_t)T, sizeof(int32_t));
    int32_t* prow = (int32_t*)exact((size_t)2 * n_chunks, sizeof(int32_t));
    for (int c = 0; c < n_chunks; ++c) {
        for (int t = cu[c]; t < cu[c + 1]; ++t) lo[t] = cu[c];
        prow[2 * c] = cu[c];
        prow[2 * c + 1] = cu[c + 1] - 1;
    }
    double* pout = (double*)exact((size_t)2 * n_chunks * n_qh * d, sizeof(double));
    orc_attn_blockdiag(pq, pk, pv, cu, n_chunks, n_qh, n_kv, d, prow, 2 * n_chunks, pout);
    for (size_t i = 0; i < (size_t)2 * n_chunks * n_qh * d; ++i) CHECK(fabs(pout[i] + 1.5) < 1e-12, "block-diagonal attention over constant values");
    orc_attn_rows(pq, pk, pv, lo, T, n_qh, n_kv, d, prow, 2 * n_chunks, pout);
    for (size_t i = 0; i < (size_t)2 * n_chunks * n_qh * d; ++i) CHECK(fabs(pout[i] + 1.5) < 1e-12, "row-range attention over constant values");

    free(pout); free(prow); free(lo); free(pv); free(pk); free(pq); free(cu);
    free(out); free(rows); free(cv); free(ck); free(theta); free(q_rot2); free(q_rot); free(qpos); free(qs); free(qw);
    free(av); free(ak); free(pos); free(delta); free(offsets); free(ids); free(back); free(vs); free(ks); free(wide); free(row_start);
}

int main(void)
{
    static const int heads[][2] = {{4, 4}, {28, 4}, {8, 1}, {6, 2}};
    int cases = 0;
    for (int rep = 0; rep < 6; ++rep)
        for (int hi = 0; hi < 4; ++hi)
            for (int dt = 0; dt < 2; ++dt) {
                one_case(dt, heads[hi][0], heads[hi][1], (rep + hi) % 2 ? 128 : 64, (rep + dt) % 2, rep % 2 ? 1e6 : 1e4);
                ++cases;
            }
    printf("oracle sanitizer run ok: %d cases, %d threads\n", cases, orc_num_threads());
    return 0;
}
