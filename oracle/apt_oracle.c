/*
 * CPU oracle for hybrid-cache decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision evaluation of what the decode attention step
 * computes for one batch whose requests keep their context either in a paged KV
 * cache or in a hidden cache (the attention layer's input hidden vectors, from
 * which K and V are projected again).  It is written from the paper's
 * definitions and shares no code, header, table or helper with the GPU library;
 * only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What is evaluated, per request r and head h with n = ctx_lens[r] attended
 * token positions j = 0..n-1 (Section 2.1, Eq. 1-3; Section 2.2 "KV Cache
 * Technique"; Section 3.1 "Opportunity I"; Section 4.3 for the block pool):
 *
 *   KV kind:      k_j, v_j  read from the request's K blocks and V blocks
 *   hidden kind:  x_j read from the request's hidden blocks,
 *                 k_j = x_j W_K[:, head h] + b_K[head h]      (Eq. 1, plus bias)
 *                 v_j = x_j W_V[:, head h] + b_V[head h]
 *   s_j   = scale * <q_{r,h}, k_j>                            (Eq. 2 exponent)
 *   a_j   = exp(s_j) / sum_m exp(s_m)                         (Eq. 2)
 *   out   = sum_j a_j v_j                                     (Eq. 3 without W_o;
 *           the printed v_i is read as v_j, as the sentence before Eq. 3 says)
 *
 * Readings of the paper taken here: the output projection W_o is not applied;
 * scale is passed in (1/sqrt(head_dim) in the multi-head reading of Eq. 2's
 * sqrt(d)); W is stored [d_in][d_out] so that k = x W + b (the transpose of the
 * paper's column-vector W x); ctx_lens counts every attended position including
 * the current token, whose vectors are already in the cache.
 *
 * Inputs are the already rounded fp32 / fp16 / bf16 values, converted exactly to
 * double; nothing is rounded inside; results are double.
 *
 * Storage layout read here (this is the documented input format of the step):
 *   pool blocks of bs*d elements; hidden block [slot][d]; K or V block
 *   [head][slot][head_dim]; block_tables int32 [B][2][max_blocks], row 0 = K or
 *   hidden blocks, row 1 = V blocks; token j lives in block j / bs, slot j % bs
 *   (a block holds consecutive token positions; blocks of a request may lie
 *   anywhere in the pool, Section 4.3).
 *
 * Pins (tests/test_oracle_*.py): hidden kind == KV kind on materialised x W + b;
 * softmax weights sum to one; brute force on tiny inputs; closed forms (n = 1,
 * q = 0, equal tokens, W = I); the absorbed-weight identity; split invariance of
 * the merge; page-permutation invariance; the Section 4.3 worked block mapping.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };
enum { ORACLE_KV = 0, ORACLE_HIDDEN = 1 };

typedef struct {
    int32_t d_model, n_heads, head_dim, block_size, dtype, max_blocks;
    double scale;
} oracle_shape;

static double half_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double elem(const void* base, int64_t idx, int dtype) {
    switch (dtype) {
    case ORACLE_F32: return (double)((const float*)base)[idx];
    case ORACLE_F16: return half_bits_to_double(((const uint16_t*)base)[idx]);
    default:         return bf16_bits_to_double(((const uint16_t*)base)[idx]);
    }
}

int apt_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Physical location of token j of request r in block-table row `row`:
 * block id and slot inside the block.  (Section 4.3: cache map.) */
void apt_oracle_locate(const int32_t* block_tables, int max_blocks, int bs, int r, int row, int j,
                       int32_t* block, int32_t* slot) {
    *block = block_tables[((int64_t)r * 2 + row) * max_blocks + j / bs];
    *slot = j % bs;
}

/* Fill k[(j-t0)*hd + c], v[...] for tokens j in [t0,t1) of (request r, head h). */
static void gather_kv(const oracle_shape* s, const void* k_pages, const void* v_pages, const void* hidden_pages,
                      const void* W_K, const void* b_K, const void* W_V, const void* b_V,
                      const int32_t* block_tables, int kind, int r, int h, int t0, int t1,
                      double* k, double* v) {
    const int d = s->d_model, hd = s->head_dim, bs = s->block_size, dt = s->dtype;
    const int64_t blk_elems = (int64_t)bs * d;
    if (kind == ORACLE_KV) {
        for (int j = t0; j < t1; ++j) {
            int32_t bk, bv, slot;
            apt_oracle_locate(block_tables, s->max_blocks, bs, r, 0, j, &bk, &slot);
            apt_oracle_locate(block_tables, s->max_blocks, bs, r, 1, j, &bv, &slot);
            /* K/V block layout [head][slot][head_dim] */
            int64_t off = ((int64_t)h * bs + slot) * hd;
            for (int c = 0; c < hd; ++c) {
                k[(int64_t)(j - t0) * hd + c] = elem(k_pages, bk * blk_elems + off + c, dt);
                v[(int64_t)(j - t0) * hd + c] = elem(v_pages, bv * blk_elems + off + c, dt);
            }
        }
        return;
    }
    /* hidden kind: project x_j again (Eq. 1 with bias), W is [d_in][d_out] */
    double* wk = (double*)malloc(sizeof(double) * (size_t)d * hd);
    double* wv = (double*)malloc(sizeof(double) * (size_t)d * hd);
    double* x = (double*)malloc(sizeof(double) * (size_t)d);
    for (int i = 0; i < d; ++i)
        for (int c = 0; c < hd; ++c) {
            wk[(int64_t)i * hd + c] = elem(W_K, (int64_t)i * d + (int64_t)h * hd + c, dt);
            wv[(int64_t)i * hd + c] = elem(W_V, (int64_t)i * d + (int64_t)h * hd + c, dt);
        }
    for (int j = t0; j < t1; ++j) {
        int32_t bx, slot;
        apt_oracle_locate(block_tables, s->max_blocks, bs, r, 0, j, &bx, &slot);
        /* hidden block layout [slot][d] */
        for (int i = 0; i < d; ++i) x[i] = elem(hidden_pages, bx * blk_elems + (int64_t)slot * d + i, dt);
        double* kj = k + (int64_t)(j - t0) * hd;
        double* vj = v + (int64_t)(j - t0) * hd;
        for (int c = 0; c < hd; ++c) {
            kj[c] = elem(b_K, (int64_t)h * hd + c, dt);
            vj[c] = elem(b_V, (int64_t)h * hd + c, dt);
        }
        for (int i = 0; i < d; ++i) {
            const double xi = x[i];
            const double* wki = wk + (int64_t)i * hd;
            const double* wvi = wv + (int64_t)i * hd;
            for (int c = 0; c < hd; ++c) {
                kj[c] += xi * wki[c];
                vj[c] += xi * wvi[c];
            }
        }
    }
    free(wk);
    free(wv);
    free(x);
}

/*
 * One-piece attention (Eq. 1-3) for n_sel (request, head) pairs.
 *   sel_r, sel_h : the pairs (NULL, NULL => all B*H pairs in [r][h] order, n_sel = B*H)
 *   out          : double [n_sel][head_dim]
 *   weights      : optional double [sum of ctx_lens over the selected pairs], the
 *                  softmax weights a_j of each pair back to back (NULL to skip)
 * Returns 0, or -1 on a bad argument (ctx_len < 1, unknown kind).
 */
int apt_oracle_attn(const oracle_shape* s, int B, const void* q,
                    const void* k_pages, const void* v_pages, const void* hidden_pages,
                    const void* W_K, const void* b_K, const void* W_V, const void* b_V,
                    const int32_t* block_tables, const int32_t* ctx_lens, const uint8_t* cache_kind,
                    const int32_t* sel_r, const int32_t* sel_h, int n_sel,
                    double* out, double* weights) {
    const int H = s->n_heads, hd = s->head_dim;
    if (!sel_r) n_sel = B * H;
    int64_t* woff = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_sel + 1));
    woff[0] = 0;
    for (int p = 0; p < n_sel; ++p) {
        int r = sel_r ? sel_r[p] : p / H;
        if (r < 0 || r >= B || ctx_lens[r] < 1 || cache_kind[r] > 1) { free(woff); return -1; }
        woff[p + 1] = woff[p] + ctx_lens[r];
    }
    #pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < n_sel; ++p) {
        const int r = sel_r ? sel_r[p] : p / H;
        const int h = sel_h ? sel_h[p] : p % H;
        const int n = ctx_lens[r];
        double* k = (double*)malloc(sizeof(double) * (size_t)n * hd);
        double* v = (double*)malloc(sizeof(double) * (size_t)n * hd);
        double* sc = (double*)malloc(sizeof(double) * (size_t)n);
        gather_kv(s, k_pages, v_pages, hidden_pages, W_K, b_K, W_V, b_V, block_tables,
                  cache_kind[r], r, h, 0, n, k, v);
        double mx = -INFINITY;
        for (int j = 0; j < n; ++j) {
            double dot = 0.0;
            for (int c = 0; c < hd; ++c)
                dot += elem(q, ((int64_t)r * H + h) * hd + c, s->dtype) * k[(int64_t)j * hd + c];
            sc[j] = s->scale * dot;
            if (sc[j] > mx) mx = sc[j];
        }
        /* subtracting the maximum multiplies numerator and denominator of Eq. 2
         * by the same factor */
        double den = 0.0;
        for (int j = 0; j < n; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
        double* o = out + (int64_t)p * hd;
        for (int c = 0; c < hd; ++c) o[c] = 0.0;
        for (int j = 0; j < n; ++j) {
            const double a = sc[j] / den;
            if (weights) weights[woff[p] + j] = a;
            for (int c = 0; c < hd; ++c) o[c] += a * v[(int64_t)j * hd + c];
        }
        free(k); free(v); free(sc);
    }
    free(woff);
    return 0;
}

/*
 * Partial result of one token range [t0,t1) of (request r, head h): the running
 * maximum m = max_j s_j, l = sum_j exp(s_j - m), acc[c] = sum_j exp(s_j - m) v_j[c].
 * Splitting the sums of Eq. 2-3 over ranges and factoring exp(m) out of each is an
 * exact re-association; apt_oracle_merge undoes it.
 */
int apt_oracle_partial(const oracle_shape* s, const void* q,
                       const void* k_pages, const void* v_pages, const void* hidden_pages,
                       const void* W_K, const void* b_K, const void* W_V, const void* b_V,
                       const int32_t* block_tables, int kind, int r, int h, int t0, int t1,
                       double* m_out, double* l_out, double* acc /* [head_dim] */) {
    const int H = s->n_heads, hd = s->head_dim, n = t1 - t0;
    if (n < 1 || kind > 1 || kind < 0) return -1;
    double* k = (double*)malloc(sizeof(double) * (size_t)n * hd);
    double* v = (double*)malloc(sizeof(double) * (size_t)n * hd);
    double* sc = (double*)malloc(sizeof(double) * (size_t)n);
    gather_kv(s, k_pages, v_pages, hidden_pages, W_K, b_K, W_V, b_V, block_tables, kind, r, h, t0, t1, k, v);
    double mx = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double dot = 0.0;
        for (int c = 0; c < hd; ++c)
            dot += elem(q, ((int64_t)r * H + h) * hd + c, s->dtype) * k[(int64_t)j * hd + c];
        sc[j] = s->scale * dot;
        if (sc[j] > mx) mx = sc[j];
    }
    double l = 0.0;
    for (int c = 0; c < hd; ++c) acc[c] = 0.0;
    for (int j = 0; j < n; ++j) {
        const double e = exp(sc[j] - mx);
        l += e;
        for (int c = 0; c < hd; ++c) acc[c] += e * v[(int64_t)j * hd + c];
    }
    *m_out = mx;
    *l_out = l;
    free(k); free(v); free(sc);
    return 0;
}

/*
 * Merge of n_splits partials of one (request, head):
 *   m* = max_s m_s,  l* = sum_s l_s exp(m_s - m*),  out = sum_s acc_s exp(m_s - m*) / l*.
 */
int apt_oracle_merge(int n_splits, int hd, const double* m, const double* l, const double* acc /* [n_splits][hd] */,
                     double* out /* [hd] */) {
    if (n_splits < 1) return -1;
    double ms = -INFINITY;
    for (int s = 0; s < n_splits; ++s) if (m[s] > ms) ms = m[s];
    double ls = 0.0;
    for (int c = 0; c < hd; ++c) out[c] = 0.0;
    for (int s = 0; s < n_splits; ++s) {
        const double w = exp(m[s] - ms);
        ls += l[s] * w;
        for (int c = 0; c < hd; ++c) out[c] += acc[(int64_t)s * hd + c] * w;
    }
    for (int c = 0; c < hd; ++c) out[c] /= ls;
    return 0;
}

/*
 * Cache append (Section 5.1: the cache engine writes the vectors of the token just
 * processed into the request's blocks; Section 4.3 for where they go).  For request r
 * with n = ctx_lens[r] tokens after the append, position n-1 receives
 *   hidden kind: x_new[r][0..d)             -> hidden block [slot][d]
 *   KV kind:     k_new[r][h][c], v_new[...] -> K block, V block [head][slot][head_dim]
 * Bytes are copied unchanged (element size from the dtype).  Returns 0, -1 on a bad argument.
 */
int apt_oracle_append(const oracle_shape* s, int B, const void* x_new, const void* k_new, const void* v_new,
                      void* k_pages, void* v_pages, void* hidden_pages,
                      const int32_t* block_tables, const int32_t* ctx_lens, const uint8_t* cache_kind) {
    const int d = s->d_model, H = s->n_heads, hd = s->head_dim, bs = s->block_size;
    const int eb = s->dtype == ORACLE_F32 ? 4 : 2;
    const int64_t blk_elems = (int64_t)bs * d;
    for (int r = 0; r < B; ++r) {
        if (ctx_lens[r] < 1 || cache_kind[r] > 1) return -1;
        const int j = ctx_lens[r] - 1;
        int32_t b0, b1, slot;
        apt_oracle_locate(block_tables, s->max_blocks, bs, r, 0, j, &b0, &slot);
        if (cache_kind[r] == ORACLE_HIDDEN) {
            for (int i = 0; i < d; ++i)
                memcpy((char*)hidden_pages + (b0 * blk_elems + (int64_t)slot * d + i) * eb,
                       (const char*)x_new + ((int64_t)r * d + i) * eb, eb);
        } else {
            apt_oracle_locate(block_tables, s->max_blocks, bs, r, 1, j, &b1, &slot);
            for (int h = 0; h < H; ++h)
                for (int c = 0; c < hd; ++c) {
                    const int64_t off = ((int64_t)h * bs + slot) * hd + c;
                    const int64_t src = ((int64_t)r * H + h) * hd + c;
                    memcpy((char*)k_pages + (b0 * blk_elems + off) * eb, (const char*)k_new + src * eb, eb);
                    memcpy((char*)v_pages + (b1 * blk_elems + off) * eb, (const char*)v_new + src * eb, eb);
                }
        }
    }
    return 0;
}

/*
 * Cache write of a run of new tokens per request (the prefill's cache write; Section 2.2,
 * Section 4.3 for the placement).  Request r has n_r = new_offsets[r+1] - new_offsets[r] new
 * tokens whose vectors are rows new_offsets[r].. of x_new / k_new / v_new; they go to positions
 * ctx_lens[r] - n_r .. ctx_lens[r] - 1, one position at a time by the same rule as
 * apt_oracle_append.  Returns 0, -1 on a bad argument.
 */
int apt_oracle_write(const oracle_shape* s, int B, const int32_t* new_offsets, const void* x_new, const void* k_new,
                     const void* v_new, void* k_pages, void* v_pages, void* hidden_pages,
                     const int32_t* block_tables, const int32_t* ctx_lens, const uint8_t* cache_kind) {
    const int d = s->d_model, H = s->n_heads, hd = s->head_dim, bs = s->block_size;
    const int eb = s->dtype == ORACLE_F32 ? 4 : 2;
    const int64_t blk_elems = (int64_t)bs * d;
    for (int r = 0; r < B; ++r) {
        const int n_new = new_offsets[r + 1] - new_offsets[r];
        if (n_new < 0 || n_new > ctx_lens[r] || cache_kind[r] > 1) return -1;
        for (int t = 0; t < n_new; ++t) {
            const int j = ctx_lens[r] - n_new + t;
            const int64_t row = new_offsets[r] + t;
            int32_t b0, b1, slot;
            apt_oracle_locate(block_tables, s->max_blocks, bs, r, 0, j, &b0, &slot);
            if (cache_kind[r] == ORACLE_HIDDEN) {
                for (int i = 0; i < d; ++i)
                    memcpy((char*)hidden_pages + (b0 * blk_elems + (int64_t)slot * d + i) * eb,
                           (const char*)x_new + (row * d + i) * eb, eb);
            } else {
                apt_oracle_locate(block_tables, s->max_blocks, bs, r, 1, j, &b1, &slot);
                for (int h = 0; h < H; ++h)
                    for (int c = 0; c < hd; ++c) {
                        const int64_t off = ((int64_t)h * bs + slot) * hd + c;
                        const int64_t src = (row * H + h) * hd + c;
                        memcpy((char*)k_pages + (b0 * blk_elems + off) * eb, (const char*)k_new + src * eb, eb);
                        memcpy((char*)v_pages + (b1 * blk_elems + off) * eb, (const char*)v_new + src * eb, eb);
                    }
            }
        }
    }
    return 0;
}
