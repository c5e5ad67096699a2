/*
 * difa_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, dense fp64 CPU statement of what the head-wise joint-attention
 * operator of DiTFastAttnV2 computes (Sec. 3.1 "Head-wise Arrow Attention",
 * Sec. 3.2 "Head-wise Caching", Sec. 3.3 "Fused Kernel for Multi-Strategy
 * Attention", and the last three statements of Alg. 1).  It exists so that the
 * GPU library can be checked against something that shares no code with it.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What is computed, per batch entry b and head h (layout [B,H,N,D], D contiguous):
 *   - mode CACHE (Sec. 3.2; Alg. 1 "O[idx] = O_cache[idx]"): the head's rows of
 *     `cache` are copied, bit for bit, to the raw output.
 *   - mode FULL: softmax(scale * q k^T) v over all N keys.
 *   - mode ARROW (Sec. 3.1): the same, restricted to the allowed pairs.  Tokens
 *     [0, n_text) are text, [n_text, N) are image tokens in flattened order.  The
 *     three quadrants that involve text are kept whole; the image-image quadrant
 *     keeps a band around the diagonal:
 *         allowed(i, j) = i < n_text  or  j < n_text  or  |i - j| <= w_h .
 *     Pairs that are not allowed get weight exactly 0 and the softmax is taken
 *     over the allowed set only.
 * There is no tiling, no running maximum and no skipping beyond "a pair that is
 * not allowed contributes nothing": each row is score -> max -> exp -> sum ->
 * weighted mean, in that order, in double precision.
 *
 * Block-granular band (Sec. 3.3 and Fig. 4: the paper's kernel turns a block that mixes kept
 * and discarded pairs into a dense block): with block sizes (bm, bn) given, an ARROW head
 * attends to pair (i, j) iff the block of bm query rows and bn keys that holds it contains at
 * least one pair of the exact pattern above.  The block table is filled from that sentence as
 * it stands: every pair of the exact pattern marks its block.
 *
 * Readings of points the paper leaves open (text tokens first; w is a half-width,
 * inclusive; 1-D band on the flattened image index; scale given by the caller)
 * are listed with their reasons in the repository's design notes.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o libdifa_oracle.so difa_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_FULL = 0, ORACLE_ARROW = 1, ORACLE_CACHE = 2 };
enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
static double widen(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[idx];
}

static size_t elem_size(int dtype) { return dtype == ORACLE_BF16 ? 2 : 4; }

/* Sec. 3.1: which (query i, key j) pairs a head in a given mode attends to.  The text tokens sit in
 * front of the image tokens (image_first == 0: text is [0, n_text)) or behind them (image_first != 0:
 * text is [n_img, n_img + n_text)); the paper only says the two are concatenated. */
int difa_oracle_allowed_order(int mode, int i, int j, int n_text, int n_img, int w, int image_first)
{
    const int t0 = image_first ? n_img : 0;     /* first text token */
    if (mode == ORACLE_FULL) return 1;
    if (i >= t0 && i < t0 + n_text) return 1;   /* language-to-anything            */
    if (j >= t0 && j < t0 + n_text) return 1;   /* visual-to-language              */
    return abs(i - j) <= w;                     /* visual-to-visual: local band    */
}

int difa_oracle_allowed(int mode, int i, int j, int n_text, int w)
{
    return difa_oracle_allowed_order(mode, i, j, n_text, 0, w, 0);
}

/* Sec. 3.3 / Fig. 4: blocks[(i / bm) * n_kb + j / bn] = 1 iff the block holds a pair the exact
 * arrow pattern keeps.  Returns NULL when memory runs out. */
static unsigned char *block_table(int N, int n_text, int n_img, int image_first, int w, int bm, int bn, int *n_kb_out)
{
    const int n_qb = (N + bm - 1) / bm, n_kb = (N + bn - 1) / bn;
    unsigned char *t = (unsigned char *)calloc((size_t)n_qb * n_kb, 1);
    if (!t) return NULL;
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j)
            if (difa_oracle_allowed_order(ORACLE_ARROW, i, j, n_text, n_img, w, image_first)) t[(size_t)(i / bm) * n_kb + j / bn] = 1;
    *n_kb_out = n_kb;
    return t;
}

int difa_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * q, k, v, cache : [B,H,N,D] host arrays of `dtype` (cache may be NULL iff no head is CACHE)
 * head_plan[H], window[H] : per-head mode and half-width (window read for ARROW heads only)
 * rows[n_rows]   : query rows to evaluate, or rows == NULL for all N rows (then R = N)
 * out            : [B,H,R,D] fp64 results (for CACHE heads: the cached values widened)
 * out_raw        : optional [B,H,R,D] of `dtype`; written for CACHE heads only (raw copy)
 * probs          : optional [B,H,R,N] fp64 softmax weights (zero where not allowed;
 *                  untouched for CACHE heads)
 * block_m, block_n : 0, 0 for the exact band; otherwise the block sizes of the block-granular band
 * returns 0, -1 on an invalid argument, -2 when host memory runs out.
 */
int difa_oracle_joint_attention_order(const void *q, const void *k, const void *v, const void *cache,
                                      int dtype, int B, int H, int D,
                                      const int32_t *head_plan, const int32_t *window,
                                      int n_text, int n_img, int image_first, double scale,
                                      const int32_t *rows, int n_rows, int block_m, int block_n,
                                      double *out, void *out_raw, double *probs)
{
    const int N = n_text + n_img;
    if (!q || !k || !v || !out || !head_plan || B <= 0 || H <= 0 || D <= 0 || N <= 0) return -1;
    if (n_text < 0 || n_img < 0) return -1;
    if (block_m < 0 || block_n < 0 || (block_m == 0) != (block_n == 0)) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32) return -1;
    const int R = rows ? n_rows : N;
    for (int h = 0; h < H; ++h) {
        if (head_plan[h] < 0 || head_plan[h] > 2) return -1;
        if (head_plan[h] == ORACLE_CACHE && !cache) return -1;
        if (head_plan[h] == ORACLE_ARROW && (!window || window[h] < 0)) return -1;
    }
    for (int r = 0; r < R; ++r) {
        int i = rows ? rows[r] : r;
        if (i < 0 || i >= N) return -1;
    }
    const size_t es = elem_size(dtype);

    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const size_t head_off = ((size_t)b * H + h) * (size_t)N * D;   /* into q,k,v,cache */
            const size_t out_off = ((size_t)b * H + h) * (size_t)R * D;
            const int mode = head_plan[h];

            if (mode == ORACLE_CACHE) {
                /* Sec. 3.3 / Alg. 1: the skipped head is filled from the cached output. */
                for (int r = 0; r < R; ++r) {
                    const int i = rows ? rows[r] : r;
                    for (int d = 0; d < D; ++d)
                        out[out_off + (size_t)r * D + d] =
                            widen(cache, dtype, head_off + (size_t)i * D + d);
                    if (out_raw)
                        memcpy((char *)out_raw + (out_off + (size_t)r * D) * es,
                               (const char *)cache + (head_off + (size_t)i * D) * es, (size_t)D * es);
                }
                continue;
            }
            const int w = (mode == ORACLE_ARROW) ? window[h] : 0;
            /* block-granular band: which (query block, key block) pairs this head keeps */
            unsigned char *blocks = NULL;
            int n_kb = 0;
            if (mode == ORACLE_ARROW && block_m > 0) {
                blocks = block_table(N, n_text, n_img, image_first, w, block_m, block_n, &n_kb);
                if (!blocks) return -2;
            }
#define KEPT(i, j) (blocks ? blocks[(size_t)((i) / block_m) * n_kb + (j) / block_n] \
                           : difa_oracle_allowed_order(mode, (i), (j), n_text, n_img, w, image_first))

            /* this head's keys and values, widened once (exact) */
            double *kd = (double *)malloc((size_t)N * D * sizeof(double));
            double *vd = (double *)malloc((size_t)N * D * sizeof(double));
            if (!kd || !vd) { free(kd); free(vd); free(blocks); return -2; }
            for (size_t e = 0; e < (size_t)N * D; ++e) {
                kd[e] = widen(k, dtype, head_off + e);
                vd[e] = widen(v, dtype, head_off + e);
            }

#pragma omp parallel
            {
                double *p = (double *)malloc((size_t)N * sizeof(double));
                double *qi = (double *)malloc((size_t)D * sizeof(double));
                double *acc = (double *)malloc((size_t)D * sizeof(double));
#pragma omp for schedule(dynamic, 4)
                for (int r = 0; r < R; ++r) {
                    const int i = rows ? rows[r] : r;
                    for (int d = 0; d < D; ++d) qi[d] = widen(q, dtype, head_off + (size_t)i * D + d);

                    /* scores of the allowed keys and their maximum */
                    double m = -INFINITY;
                    for (int j = 0; j < N; ++j) {
                        if (!KEPT(i, j)) continue;
                        double s = 0.0;
                        for (int d = 0; d < D; ++d)
                            s += qi[d] * kd[(size_t)j * D + d];
                        s *= scale;
                        p[j] = s;
                        if (s > m) m = s;
                    }
                    /* weights: exp(s - m) on allowed pairs, exactly 0 elsewhere */
                    double l = 0.0;
                    for (int j = 0; j < N; ++j) {
                        if (KEPT(i, j)) {
                            p[j] = exp(p[j] - m);
                            l += p[j];
                        } else {
                            p[j] = 0.0;
                        }
                    }
                    /* weighted mean of the value rows */
                    for (int d = 0; d < D; ++d) acc[d] = 0.0;
                    for (int j = 0; j < N; ++j) {
                        if (p[j] == 0.0) continue;
                        for (int d = 0; d < D; ++d)
                            acc[d] += p[j] * vd[(size_t)j * D + d];
                    }
                    for (int d = 0; d < D; ++d) out[out_off + (size_t)r * D + d] = acc[d] / l;
                    if (probs)
                        for (int j = 0; j < N; ++j)
                            probs[(((size_t)b * H + h) * R + r) * (size_t)N + j] = p[j] / l;
                }
                free(p);
                free(qi);
                free(acc);
            }
            free(kd);
            free(vd);
            free(blocks);
#undef KEPT
        }
    }
    return 0;
}

/* Text tokens first. */
int difa_oracle_joint_attention_blocks(const void *q, const void *k, const void *v, const void *cache,
                                       int dtype, int B, int H, int D,
                                       const int32_t *head_plan, const int32_t *window,
                                       int n_text, int n_img, double scale,
                                       const int32_t *rows, int n_rows, int block_m, int block_n,
                                       double *out, void *out_raw, double *probs)
{
    return difa_oracle_joint_attention_order(q, k, v, cache, dtype, B, H, D, head_plan, window, n_text, n_img, 0,
                                             scale, rows, n_rows, block_m, block_n, out, out_raw, probs);
}

/* The exact band (Sec. 3.1). */
int difa_oracle_joint_attention(const void *q, const void *k, const void *v, const void *cache,
                                int dtype, int B, int H, int D,
                                const int32_t *head_plan, const int32_t *window,
                                int n_text, int n_img, double scale,
                                const int32_t *rows, int n_rows,
                                double *out, void *out_raw, double *probs)
{
    return difa_oracle_joint_attention_blocks(q, k, v, cache, dtype, B, H, D, head_plan, window, n_text, n_img,
                                              scale, rows, n_rows, 0, 0, out, out_raw, probs);
}
