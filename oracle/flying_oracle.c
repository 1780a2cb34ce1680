/*
 * flying_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU implementation (fp64 arithmetic, plain
 * loops) of what the GPU hot path computes:
 *
 *   - the KV Cache Adaptor's layout views (paper Sec. 4.2.2, Eq. 2 and Eq. 3;
 *     Alg. 1 step 4 / Eq. 4: B_req = B_base * N_eng, H_req = H_base / N_eng),
 *   - paged single-query (decode) attention through such a view
 *     (Sec. 2.1 "Attention Layer": softmax attention over the cached K/V;
 *     Sec. 4.1.1: a TP rank owns a disjoint, contiguous subset of heads),
 *   - paged multi-token causal attention through a view (a prefill chunk or
 *     the recompute of Soft Preempt, Sec. 5.2.2; chunked prefill, Sec. 3),
 *   - scatter / gather of logical K/V rows to / from pool blocks (the stand-in
 *     for the paper's "KV cache kernel", Sec. 4.2.3),
 *   - the byte-exact block repack between two views (this build's replacement
 *     for the KV recompute of Soft Preempt, Sec. 5.2.2 / Fig. 6(b)).
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call into this file.  It shares no code with the HIP path: every address
 * is re-derived here from the formulas.
 *
 * Physical layout assumed (the reading of Eq. 2-4 used by this build): the pool
 * is n_blocks blocks of 2 * plane_elems bf16 elements, plane_elems =
 * B_base * H_kv * d.  A block read under a view with capacity Bv tokens and Hrow
 * heads per token row is the array [2 (K,V)][Bv][Hrow][d].  Bv * Hrow is the same
 * for every view, which is Eq. 2's "M_block constant".
 *
 * Every function in this file is pinned by tests that do not use the file
 * itself as the expected value (paper's printed Fig. 4 capacities, brute-force
 * bijection of the address map, numpy textbook attention on logical tensors,
 * closed forms for one token / equal keys, round-trip identities).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

enum { ORACLE_LAYOUT_DP = 0, ORACLE_LAYOUT_TP = 1 };

/* A resolved view: all the integers that Eq. 2-4 and the head partition fix. */
typedef struct {
    int32_t Hq, Hkv, d, B0; /* geometry: query heads, KV heads, head dim, B_base */
    int32_t layout, p, r;   /* block arrangement, TP degree, rank in the group   */
    int32_t Bv;             /* tokens per block under this view (Eq. 3)          */
    int32_t Hrow;           /* KV heads stored in one token row of a block       */
    int32_t Hl;             /* KV heads this view exposes (Eq. 4: H_base / N)    */
    int32_t Hql;            /* query heads this view exposes                     */
    int32_t h0;             /* first global KV head exposed: r * Hl              */
    int32_t row0;           /* where head h0 sits inside a token row             */
    int64_t plane_elems;    /* B0 * Hkv * d                                      */
} oracle_view;

/*
 * Eq. 3 / Eq. 4 and Sec. 4.1.1.  Layout DP with p == 1: the replica view.
 * Layout TP: a block holds p*B0 tokens of Hkv/p heads; rank r owns KV heads
 * [r*Hkv/p, (r+1)*Hkv/p) and query heads [r*Hq/p, (r+1)*Hq/p).
 * Layout DP with p > 1: rank r's head slice read in place from DP-arranged
 * blocks (capacity and row width stay those of DP; only the exposed heads
 * shrink).
 */
int oracle_view_resolve(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                        int32_t layout, int32_t p, int32_t r, oracle_view* v)
{
    if (!v) return ORACLE_EINVAL;
    if (Hq <= 0 || Hkv <= 0 || d <= 0 || B0 <= 0) return ORACLE_EINVAL;
    if (Hq % Hkv != 0) return ORACLE_EINVAL;
    if (layout != ORACLE_LAYOUT_DP && layout != ORACLE_LAYOUT_TP) return ORACLE_EINVAL;
    if (p < 1 || r < 0 || r >= p) return ORACLE_EINVAL;
    if (Hkv % p != 0 || Hq % p != 0) return ORACLE_EINVAL;
    v->Hq = Hq; v->Hkv = Hkv; v->d = d; v->B0 = B0;
    v->layout = layout; v->p = p; v->r = r;
    v->Hl = Hkv / p;
    v->Hql = Hq / p;
    v->h0 = r * v->Hl;
    v->plane_elems = (int64_t)B0 * Hkv * d;
    if (layout == ORACLE_LAYOUT_TP) {
        v->Bv = p * B0;
        v->Hrow = Hkv / p;
        v->row0 = 0;
    } else {
        v->Bv = B0;
        v->Hrow = Hkv;
        v->row0 = v->h0;
    }
    return ORACLE_OK;
}

/* Flat export of a resolved view for the Python side (10 integers). */
int oracle_view_query(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                      int32_t layout, int32_t p, int32_t r, int64_t* out10)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    out10[0] = v.Bv; out10[1] = v.Hrow; out10[2] = v.Hl; out10[3] = v.Hql;
    out10[4] = v.h0; out10[5] = v.row0; out10[6] = v.plane_elems;
    out10[7] = 2 * v.plane_elems * 2;          /* block bytes: K and V planes, bf16 */
    out10[8] = (int64_t)v.Hrow * v.d;          /* token stride in elements          */
    out10[9] = (int64_t)v.Hq / v.Hkv;          /* GQA group size G                  */
    return ORACLE_OK;
}

/*
 * Element index of (block, plane, slot, local head hl, element e) in the pool.
 * plane 0 = K, 1 = V; slot in [0,Bv); hl in [0,Hl); e in [0,d).
 */
static int64_t elem_index(const oracle_view* v, int64_t blk, int plane, int slot,
                          int hl, int e)
{
    return blk * (2 * v->plane_elems) + (int64_t)plane * v->plane_elems +
           (int64_t)slot * ((int64_t)v->Hrow * v->d) + (int64_t)(v->row0 + hl) * v->d + e;
}

int64_t oracle_elem_index(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                          int32_t layout, int32_t p, int32_t r,
                          int64_t blk, int32_t plane, int32_t slot, int32_t hl, int32_t e)
{
    oracle_view v;
    if (oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v)) return -1;
    if (plane < 0 || plane > 1 || slot < 0 || slot >= v.Bv || hl < 0 || hl >= v.Hl ||
        e < 0 || e >= d || blk < 0)
        return -1;
    return elem_index(&v, blk, plane, slot, hl, e);
}

/* bf16 bit pattern -> double, exact. */
static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Token t of a sequence: which block (through the table) and which slot. */
static int64_t token_block(const oracle_view* v, const int32_t* table_row, int64_t t)
{
    return (int64_t)table_row[t / v->Bv];
}
static int token_slot(const oracle_view* v, int64_t t) { return (int)(t % v->Bv); }

/*
 * One output row: sequence with n cached tokens, local query head whose KV
 * head is hl.  Two passes, fp64: scores, max, then weights and weighted sum.
 * If stats != NULL the row is left un-normalised and stats = {max, sum of
 * weights} (used to pin the split-merge identity); else out = sum / weights.
 * t_begin/t_end restrict the tokens taken (whole context: 0, n).
 */
static void decode_row(const oracle_view* v, const uint16_t* q_row, const uint16_t* pool,
                       const int32_t* table_row, int64_t t_begin, int64_t t_end, int hl,
                       double scale, double* out, double* stats)
{
    const int d = v->d;
    for (int e = 0; e < d; ++e) out[e] = 0.0;
    if (stats) { stats[0] = -INFINITY; stats[1] = 0.0; }
    if (t_end <= t_begin) return;
    const int64_t n = t_end - t_begin;
    double* score = (double*)malloc((size_t)n * sizeof(double));
    double m = -INFINITY;
    for (int64_t t = t_begin; t < t_end; ++t) {
        const int64_t k0 = elem_index(v, token_block(v, table_row, t), 0, token_slot(v, t), hl, 0);
        double s = 0.0;
        for (int e = 0; e < d; ++e) s += bf16_to_f64(q_row[e]) * bf16_to_f64(pool[k0 + e]);
        s *= scale;
        score[t - t_begin] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int64_t t = t_begin; t < t_end; ++t) {
        const double w = exp(score[t - t_begin] - m);
        const int64_t v0 = elem_index(v, token_block(v, table_row, t), 1, token_slot(v, t), hl, 0);
        denom += w;
        for (int e = 0; e < d; ++e) out[e] += w * bf16_to_f64(pool[v0 + e]);
    }
    free(score);
    if (stats) { stats[0] = m; stats[1] = denom; return; }
    for (int e = 0; e < d; ++e) out[e] /= denom;
}

static double resolve_scale(double scale, int d) { return scale > 0.0 ? scale : 1.0 / sqrt((double)d); }

/*
 * Paged decode attention through a view, for a list of (sequence, local query
 * head) pairs.  q: [batch][Hql][d] bf16 bits.  table: [batch][table_stride]
 * int32.  out: [n_pairs][d] fp64.  Local query head i reads local KV head
 * i / G (G = Hq / Hkv, unchanged by the partition).
 */
int oracle_paged_decode_pairs(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                              int32_t layout, int32_t p, int32_t r,
                              const uint16_t* q, const uint16_t* pool,
                              const int32_t* table, int64_t table_stride,
                              const int32_t* ctx_lens, const int32_t* pair_seq,
                              const int32_t* pair_head, int64_t n_pairs, double scale,
                              double* out)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    const int G = Hq / Hkv;
    const double sc = resolve_scale(scale, d);
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n_pairs; ++k) {
        const int s = pair_seq[k], i = pair_head[k];
        if (i < 0 || i >= v.Hql || ctx_lens[s] < 0) { bad = 1; continue; }
        decode_row(&v, q + ((int64_t)s * v.Hql + i) * d, pool, table + (int64_t)s * table_stride,
                   0, ctx_lens[s], i / G, sc, out + k * d, NULL);
    }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/* All rows of a batch: out [batch][Hql][d] fp64. */
int oracle_paged_decode(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                        int32_t layout, int32_t p, int32_t r,
                        const uint16_t* q, const uint16_t* pool,
                        const int32_t* table, int64_t table_stride,
                        const int32_t* ctx_lens, int32_t batch, double scale, double* out)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    const int64_t n_pairs = (int64_t)batch * v.Hql;
    int32_t* ps = (int32_t*)malloc((size_t)(n_pairs ? n_pairs : 1) * sizeof(int32_t));
    int32_t* ph = (int32_t*)malloc((size_t)(n_pairs ? n_pairs : 1) * sizeof(int32_t));
    for (int64_t k = 0; k < n_pairs; ++k) { ps[k] = (int32_t)(k / v.Hql); ph[k] = (int32_t)(k % v.Hql); }
    rc = oracle_paged_decode_pairs(Hq, Hkv, d, B0, layout, p, r, q, pool, table, table_stride,
                                   ctx_lens, ps, ph, n_pairs, scale, out);
    free(ps); free(ph);
    return rc;
}

/*
 * Multi-token (chunked prefill / recompute) causal attention through a view
 * (Sec. 2.1: a prefill step attends over the prompt with a causal mask; Sec.
 * 5.2.2: Soft Preempt recomputes the KV of taken-over requests, which is such a
 * step; Sec. 3: chunked prefill is preserved).  Sequence s has ctx_lens[s]
 * tokens in the cache, the last q_len[s] = q_off[s+1] - q_off[s] of which are
 * the new ones: query j of the sequence sits at position
 * pos = ctx_lens[s] - q_len[s] + j and attends to tokens 0..pos.
 * q: [total_q][Hql][d] bf16 bits, sequence s owning rows [q_off[s], q_off[s+1]).
 * Rows are selected by (row index into q, local head); out: [n_rows][d] fp64.
 * Each row is, by definition, single-query attention over the first pos + 1
 * tokens: computed as exactly that.
 */
int oracle_paged_prefill_rows(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                              int32_t layout, int32_t p, int32_t r,
                              const uint16_t* q, const uint16_t* pool,
                              const int32_t* table, int64_t table_stride,
                              const int32_t* ctx_lens, const int64_t* q_off, int32_t batch,
                              const int64_t* row_q, const int32_t* row_head, int64_t n_rows,
                              double scale, double* out)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    const int G = Hq / Hkv;
    const double sc = resolve_scale(scale, d);
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n_rows; ++k) {
        const int64_t row = row_q[k];
        const int i = row_head[k];
        int s = -1;
        for (int c = 0; c < batch; ++c)
            if (row >= q_off[c] && row < q_off[c + 1]) s = c;
        if (s < 0 || i < 0 || i >= v.Hql) { bad = 1; continue; }
        const int64_t q_len = q_off[s + 1] - q_off[s];
        const int64_t pos = (int64_t)ctx_lens[s] - q_len + (row - q_off[s]);
        if (pos < 0) { bad = 1; continue; }
        decode_row(&v, q + (row * v.Hql + i) * d, pool, table + (int64_t)s * table_stride,
                   0, pos + 1, i / G, sc, out + k * d, NULL);
    }
    return bad ? ORACLE_EINVAL : ORACLE_OK;
}

/*
 * Un-normalised partial over tokens [t_begin, t_end) of one (sequence, head):
 * acc[d] = sum_t exp(s_t - m) V_t, stats = {m, sum_t exp(s_t - m)}.
 */
int oracle_paged_decode_partial(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                                int32_t layout, int32_t p, int32_t r,
                                const uint16_t* q, const uint16_t* pool,
                                const int32_t* table, int64_t table_stride,
                                int32_t seq, int32_t head, int64_t t_begin, int64_t t_end,
                                double scale, double* acc, double* stats)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    if (head < 0 || head >= v.Hql) return ORACLE_EINVAL;
    decode_row(&v, q + ((int64_t)seq * v.Hql + head) * d, pool, table + (int64_t)seq * table_stride,
               t_begin, t_end, head / (Hq / Hkv), resolve_scale(scale, d), acc, stats);
    return ORACLE_OK;
}

/*
 * Dense decode attention with no pool, no table and no view: K and V are the
 * logical tensors [total_tokens][Hkv][d] (sequence s owns tokens
 * [seq_off[s], seq_off[s+1])), q is [batch][Hq][d] with ALL query heads.
 * Output [batch][Hq][d] fp64.  Written differently from decode_row on purpose
 * (normalised weight vector first, then the weighted sum per element) so that
 * the two check each other.
 */
int oracle_dense_decode(int32_t Hq, int32_t Hkv, int32_t d, const uint16_t* q,
                        const uint16_t* K, const uint16_t* V, const int64_t* seq_off,
                        int32_t batch, double scale, double* out)
{
    if (Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return ORACLE_EINVAL;
    const int G = Hq / Hkv;
    const double sc = resolve_scale(scale, d);
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < batch; ++s) {
        for (int h = 0; h < Hq; ++h) {
            const int64_t t0 = seq_off[s], n = seq_off[s + 1] - seq_off[s];
            double* o = out + ((int64_t)s * Hq + h) * d;
            for (int e = 0; e < d; ++e) o[e] = 0.0;
            if (n <= 0) continue;
            const int g = h / G;
            const uint16_t* qr = q + ((int64_t)s * Hq + h) * d;
            double* w = (double*)malloc((size_t)n * sizeof(double));
            double m = -INFINITY;
            for (int64_t t = 0; t < n; ++t) {
                const uint16_t* kr = K + ((t0 + t) * Hkv + g) * d;
                double dot = 0.0;
                for (int e = 0; e < d; ++e) dot += bf16_to_f64(kr[e]) * bf16_to_f64(qr[e]);
                w[t] = dot * sc;
                if (w[t] > m) m = w[t];
            }
            double z = 0.0;
            for (int64_t t = 0; t < n; ++t) { w[t] = exp(w[t] - m); z += w[t]; }
            for (int64_t t = 0; t < n; ++t) w[t] /= z;
            for (int e = 0; e < d; ++e) {
                double a = 0.0;
                for (int64_t t = 0; t < n; ++t) a += w[t] * bf16_to_f64(V[((t0 + t) * Hkv + g) * d + e]);
                o[e] = a;
            }
            free(w);
        }
    }
    return ORACLE_OK;
}

/*
 * Scatter (dir = 0): write logical rows K,V[seq_off[s] + t][g][:] for t <
 * n_tokens[s] and every global head g the view exposes into the pool, through
 * the table.  Gather (dir = 1): the reverse copy, pool -> logical (only the
 * exposed heads are written).  16-bit copies, nothing is converted.
 */
static int scatter_gather(int dir, int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                          int32_t layout, int32_t p, int32_t r, uint16_t* pool,
                          const int32_t* table, int64_t table_stride, const int32_t* n_tokens,
                          int32_t n_seqs, const int64_t* seq_off, uint16_t* K, uint16_t* V)
{
    oracle_view v;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, layout, p, r, &v);
    if (rc) return rc;
    for (int s = 0; s < n_seqs; ++s) {
        const int32_t* row = table + (int64_t)s * table_stride;
        for (int64_t t = 0; t < n_tokens[s]; ++t) {
            const int64_t blk = token_block(&v, row, t);
            const int slot = token_slot(&v, t);
            for (int hl = 0; hl < v.Hl; ++hl) {
                const int g = v.h0 + hl;
                const int64_t lk = ((seq_off[s] + t) * Hkv + g) * d;
                const int64_t pk = elem_index(&v, blk, 0, slot, hl, 0);
                const int64_t pv = elem_index(&v, blk, 1, slot, hl, 0);
                for (int e = 0; e < d; ++e) {
                    if (dir == 0) { pool[pk + e] = K[lk + e]; pool[pv + e] = V[lk + e]; }
                    else          { K[lk + e] = pool[pk + e]; V[lk + e] = pool[pv + e]; }
                }
            }
        }
    }
    return ORACLE_OK;
}

int oracle_scatter(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0, int32_t layout, int32_t p,
                   int32_t r, uint16_t* pool, const int32_t* table, int64_t table_stride,
                   const int32_t* n_tokens, int32_t n_seqs, const int64_t* seq_off,
                   const uint16_t* K, const uint16_t* V)
{
    return scatter_gather(0, Hq, Hkv, d, B0, layout, p, r, pool, table, table_stride, n_tokens,
                          n_seqs, seq_off, (uint16_t*)K, (uint16_t*)V);
}

int oracle_gather(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0, int32_t layout, int32_t p,
                  int32_t r, const uint16_t* pool, const int32_t* table, int64_t table_stride,
                  const int32_t* n_tokens, int32_t n_seqs, const int64_t* seq_off, uint16_t* K,
                  uint16_t* V)
{
    return scatter_gather(1, Hq, Hkv, d, B0, layout, p, r, (uint16_t*)pool, table, table_stride,
                          n_tokens, n_seqs, seq_off, K, V);
}

/*
 * Repack: for every sequence s, token t < n_tokens[s], plane, and every global
 * KV head exposed by BOTH views, copy the d-element row from its address under
 * the source view (through src_table) to its address under the destination
 * view (through dst_table).  All other bytes of the pool keep their value.
 * Source and destination block sets must be disjoint (not checked here).
 */
int oracle_repack(int32_t Hq, int32_t Hkv, int32_t d, int32_t B0,
                  int32_t src_layout, int32_t src_p, int32_t src_r,
                  int32_t dst_layout, int32_t dst_p, int32_t dst_r, uint16_t* pool,
                  const int32_t* src_table, int64_t src_stride, const int32_t* dst_table,
                  int64_t dst_stride, const int32_t* n_tokens, int32_t n_seqs)
{
    oracle_view sv, dv;
    int rc = oracle_view_resolve(Hq, Hkv, d, B0, src_layout, src_p, src_r, &sv);
    if (rc) return rc;
    rc = oracle_view_resolve(Hq, Hkv, d, B0, dst_layout, dst_p, dst_r, &dv);
    if (rc) return rc;
    const int g_lo = sv.h0 > dv.h0 ? sv.h0 : dv.h0;
    const int g_hi = (sv.h0 + sv.Hl) < (dv.h0 + dv.Hl) ? (sv.h0 + sv.Hl) : (dv.h0 + dv.Hl);
    for (int s = 0; s < n_seqs; ++s) {
        const int32_t* srow = src_table + (int64_t)s * src_stride;
        const int32_t* drow = dst_table + (int64_t)s * dst_stride;
        for (int64_t t = 0; t < n_tokens[s]; ++t) {
            for (int g = g_lo; g < g_hi; ++g) {
                for (int plane = 0; plane < 2; ++plane) {
                    const int64_t a = elem_index(&sv, token_block(&sv, srow, t), plane,
                                                 token_slot(&sv, t), g - sv.h0, 0);
                    const int64_t b = elem_index(&dv, token_block(&dv, drow, t), plane,
                                                 token_slot(&dv, t), g - dv.h0, 0);
                    for (int e = 0; e < d; ++e) pool[b + e] = pool[a + e];
                }
            }
        }
    }
    return ORACLE_OK;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
