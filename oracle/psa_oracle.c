/*
 * psa_oracle.c -- plain, slow, fp64 CPU oracle for the decode-step hot path of
 * Progressive Sparse Attention (PSA).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library, and the HIP library never calls it.
 *
 * What it computes, and the passage of the paper each part follows:
 *   oracle_dense_attention      S = QK^T/sqrt(d), P = softmax(S), O = PV         (Sec. 2.1, the
 *                               unnumbered attention equation), two passes, fp64.
 *   oracle_block_metadata       per-block, per-channel min and max of the keys: the "bounding
 *                               cuboid" flavour of block metadata                (Sec. 2.2,
 *                               "KV Cache Selection").
 *   oracle_block_scores         criticality score CS = q . B_meta                (Algorithm 1, line 5),
 *                               read as the largest value q.k/sqrt(d) can take inside the cuboid,
 *                               then reduced with max over the query heads that share a KV head.
 *   oracle_block_order          rank blocks by CS, most critical first            (Algorithm 1, line 6),
 *                               ties to the smaller logical block index.
 *   oracle_psa_decode           the progressive loop                              (Algorithm 1, lines
 *                               2-4 and 7-19; Sec. 3.2 prose on the microbatch size m and on the
 *                               batched form where every query stops on its own).
 *   oracle_attend_prefix        softmax attention restricted to the first n ranked blocks, by the
 *                               definition (used to check the merge of Algorithm 1, line 11, and as
 *                               the fixed top-k control of Sec. 1 / Sec. 2.2), with the log of its
 *                               denominator.
 * The Python side (psa_oracle.py) adds, in numpy: topk_attention (ranking + oracle_attend_prefix) and
 * append_kv (the cache after one more token per request, Sec. 3.1).
 *
 * Readings of points the paper leaves open are listed where they are used; they are the same list
 * the repository's design document carries.
 *
 * Parity pins (tests, CPU only): dense against a numpy/scipy softmax; metadata and the bounding
 * property of the score by brute force; order invariants; threshold 1 equals dense; the selected
 * set is a prefix; attained estimate > threshold or all blocks; true mass >= estimate under the
 * ideal order; the n(m) identity that follows from P_acc being non-decreasing; a hand-computed
 * three-block case stored under tests/golden.
 * Parity unpinned (no passage or closed form fixes them; they are this build's readings): the max
 * reduce over a GQA group, the treatment of a partly filled last block, the order of -0 and +0 in
 * the metadata, and the cuboid-centre scorer as a reading of the "cuboid-mean" metadata the paper
 * names without defining (its arithmetic is pinned; that it is what the paper means is not).
 *
 * Storage formats: K, V, Q and metadata are IEEE binary16 ("f16", dtype 0) or bfloat16 (dtype 1),
 * passed as raw uint16_t and decoded exactly to double here.
 *
 * Layouts (all row-major):
 *   k_pool, v_pool  [num_pages][num_kv_heads][page_size][head_dim]
 *   meta            [num_pages][num_kv_heads][2][head_dim]      (0 = min, 1 = max)
 *   q               [batch][num_q_heads][head_dim]
 *   block_table     [batch][max_blocks]   logical block -> physical page
 *   ctx_lens        [batch]               tokens of each request
 *   order           [batch][num_kv_heads][max_blocks]  ranked logical blocks, -1 beyond N_r
 */

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t batch, num_q_heads, num_kv_heads, head_dim, page_size, num_pages, max_blocks;
    int32_t dtype; /* 0 = f16, 1 = bf16 */
} oracle_shape;

/* ---------- exact decoders --------------------------------------------------------------- */

static double decode_f16(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24); /* subnormal: frac * 2^-10 * 2^-14 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

static double decode_bf16(uint16_t h) {
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double decode(uint16_t h, int dtype) { return dtype ? decode_bf16(h) : decode_f16(h); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int blocks_of(int ctx, int page_size) { return (ctx + page_size - 1) / page_size; }

static int valid_tokens(int ctx, int page_size, int b) {
    int left = ctx - b * page_size;
    return left < page_size ? left : page_size;
}

/* ---------- block metadata (Sec. 2.2): per-channel min / max over the block's valid keys ---- */
/*
 * page_fill[p] = number of valid tokens in page p (NULL: every page is full).  A page with no
 * valid token gets min = max = +0.  The result is one of the inputs, so it is exact in the
 * storage type and written back as the same 16 bits.  Reading of an open point: where -0 and +0
 * meet, min prefers -0 and max prefers +0 (a total order), so that the result has defined bits.
 */
static int before(uint16_t a, uint16_t b, int dtype) { /* a strictly below b in that total order */
    double x = decode(a, dtype), y = decode(b, dtype);
    if (x < y) return 1;
    if (x > y) return 0;
    return (a >> 15) > (b >> 15); /* equal values: the negative zero is the smaller one */
}

void oracle_block_metadata(const oracle_shape *sh, const uint16_t *k_pool, const int32_t *page_fill,
                           uint16_t *meta) {
    const int H = sh->num_kv_heads, T = sh->page_size, D = sh->head_dim;
#pragma omp parallel for schedule(static)
    for (int p = 0; p < sh->num_pages; ++p) {
        int fill = page_fill ? page_fill[p] : T;
        if (fill > T) fill = T;
        for (int h = 0; h < H; ++h) {
            const uint16_t *kb = k_pool + ((size_t)p * H + h) * T * D;
            uint16_t *mn = meta + ((size_t)p * H + h) * 2 * D;
            uint16_t *mx = mn + D;
            for (int c = 0; c < D; ++c) {
                if (fill <= 0) { mn[c] = 0; mx[c] = 0; continue; }
                uint16_t lo = kb[c], hi = kb[c];
                for (int t = 1; t < fill; ++t) {
                    uint16_t x = kb[(size_t)t * D + c];
                    if (before(x, lo, sh->dtype)) lo = x;
                    if (before(hi, x, sh->dtype)) hi = x;
                }
                mn[c] = lo;
                mx[c] = hi;
            }
        }
    }
}

/* ---------- mean-key metadata (Sec. 2.2 "KV Cache Selection": metadata vectors that represent a block's
 * keys; the per-channel mean is the smallest of the constructions in use, half the bytes of the cuboid) ---- */
/*
 * Rounds a binary64 value to the 16-bit storage type, once, to nearest with ties to even: the exponent comes from
 * frexp, the scaling is by powers of two (exact), the rounding is nearbyint's in the default rounding mode.  The
 * values this is used on are means of storage-type numbers, so neither overflow nor NaN occurs; infinities and NaN
 * are passed on as the type's own.
 */
static uint16_t encode(double x, int dtype) {
    const int mant_bits = dtype ? 7 : 10, bias = dtype ? 127 : 15, exp_max = dtype ? 255 : 31;
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    if (isnan(x)) return (uint16_t)(sign | ((unsigned)exp_max << mant_bits) | 1u);
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | ((unsigned)exp_max << mant_bits));
    int e;
    (void)frexp(a, &e);                      /* a = f * 2^e, f in [0.5, 1): the leading bit has weight 2^(e-1) */
    int lead = e - 1;
    int emin = 1 - bias;                     /* exponent of the smallest normal number */
    if (lead < emin) {                       /* subnormal range: a fixed grid of 2^(emin - mant_bits) */
        double steps = nearbyint(ldexp(a, mant_bits - emin));
        return (uint16_t)(sign | (unsigned)steps);       /* (reaching 2^mant_bits is the smallest normal: same bits) */
    }
    double frac = nearbyint(ldexp(a, mant_bits - lead));  /* in [2^mant_bits, 2^(mant_bits+1)] */
    if (frac >= ldexp(1.0, mant_bits + 1)) { frac = ldexp(1.0, mant_bits); lead += 1; }
    if (lead + bias >= exp_max) return (uint16_t)(sign | ((unsigned)exp_max << mant_bits));
    return (uint16_t)(sign | ((unsigned)(lead + bias) << mant_bits) | ((unsigned)frac - (1u << mant_bits)));
}

/*
 * means[p][h][c] = the mean over the page's valid tokens of k[t][c], summed token by token in binary64 (exact for
 * any keys whose magnitudes in one channel span less than 2^38, which covers every generated input), divided by
 * the count and rounded once to the storage type.  A page with no valid token gets +0, and so does a channel
 * whose mean is zero (the sum starts from +0).
 */
void oracle_block_means(const oracle_shape *sh, const uint16_t *k_pool, const int32_t *page_fill,
                        uint16_t *means) {
    const int H = sh->num_kv_heads, T = sh->page_size, D = sh->head_dim;
#pragma omp parallel for schedule(static)
    for (int p = 0; p < sh->num_pages; ++p) {
        int fill = page_fill ? page_fill[p] : T;
        if (fill > T) fill = T;
        for (int h = 0; h < H; ++h) {
            const uint16_t *kb = k_pool + ((size_t)p * H + h) * T * D;
            uint16_t *out = means + ((size_t)p * H + h) * D;
            for (int c = 0; c < D; ++c) {
                if (fill <= 0) { out[c] = 0; continue; }
                double sum = 0.0;
                for (int t = 0; t < fill; ++t) sum += decode(kb[(size_t)t * D + c], sh->dtype);
                out[c] = encode(sum / (double)fill, sh->dtype);
            }
        }
    }
}

/* ---------- criticality scores (Algorithm 1, line 5) -------------------------------------- */
/*
 * scorer 0 (the default reading of q . B_meta for cuboid metadata):
 *   UB[g][b] = (1/sqrt d) * sum_c max(q[g][c]*kmin[b][c], q[g][c]*kmax[b][c]): no key inside the
 *   cuboid [kmin, kmax] can give a larger scaled logit.
 * scorer 1 (a reading of the "cuboid-mean" metadata that Sec. 3.1 names as the default without
 *   defining it): the scaled logit of the cuboid's centre, q . (kmin + kmax)/2 / sqrt d, which is
 *   also the mean of the largest and the smallest logit the cuboid allows.  Parity unpinned.
 * scorer 2 (mean-key metadata, `meta` is then the [page][KV head][channel] array of oracle_block_means): the
 *   scaled logit of the block's mean key, q . mean / sqrt d -- the mean of the block's token logits, up to the
 *   rounding of the stored mean.  Parity unpinned (a construction the paper names among others, Sec. 2.2).
 * CS[b] = max over the heads g of the group (reading: one ranking per KV head must serve all its
 * query heads; for scorer 0 max keeps the bound valid for each of them).
 * ub: [batch][num_q_heads][max_blocks] per-head scores, cs: [batch][num_kv_heads][max_blocks];
 * entries at b >= N_r are left untouched.
 */
void oracle_block_scores(const oracle_shape *sh, const uint16_t *q, const uint16_t *meta,
                         const int32_t *block_table, const int32_t *ctx_lens, int32_t scorer,
                         double *ub, double *cs) {
    const int Hq = sh->num_q_heads, H = sh->num_kv_heads, D = sh->head_dim, G = Hq / H;
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    for (int r = 0; r < sh->batch; ++r) {
        int N = blocks_of(ctx_lens[r], sh->page_size);
        for (int h = 0; h < H; ++h) {
            for (int b = 0; b < N; ++b) {
                int page = block_table[(size_t)r * sh->max_blocks + b];
                const uint16_t *mn = meta + ((size_t)page * H + h) * (scorer == 2 ? 1 : 2) * D;
                const uint16_t *mx = scorer == 2 ? mn : mn + D;        /* (one vector per block with scorer 2) */
                double best = -INFINITY;
                for (int g = 0; g < G; ++g) {
                    const uint16_t *qg = q + ((size_t)r * Hq + h * G + g) * D;
                    double acc = 0.0;
                    for (int c = 0; c < D; ++c) {
                        double qc = decode(qg[c], sh->dtype);
                        double a = qc * decode(mn[c], sh->dtype);
                        double z = qc * decode(mx[c], sh->dtype);
                        acc += scorer == 2 ? a : (scorer == 1 ? 0.5 * (a + z) : (a > z ? a : z));
                    }
                    acc *= inv_sqrt_d;
                    if (ub) ub[((size_t)r * Hq + h * G + g) * sh->max_blocks + b] = acc;
                    if (acc > best) best = acc;
                }
                cs[((size_t)r * H + h) * sh->max_blocks + b] = best;
            }
        }
    }
}

/* ---------- ranking (Algorithm 1, line 6) --------------------------------------------------- */
/* Insertion into a sorted list, most critical first; a block goes behind every block whose score
 * is greater or equal, which sends ties to the smaller logical index.  O(N^2) moves at worst but
 * there is nothing to get wrong.  keys are whatever the caller ranks by (CS, or a test's own). */
void oracle_block_order(const oracle_shape *sh, const double *keys, const int32_t *ctx_lens,
                        int32_t *order) {
    const int H = sh->num_kv_heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int r = 0; r < sh->batch; ++r) {
        for (int h = 0; h < H; ++h) {
            int N = blocks_of(ctx_lens[r], sh->page_size);
            const double *k = keys + ((size_t)r * H + h) * sh->max_blocks;
            int32_t *o = order + ((size_t)r * H + h) * sh->max_blocks;
            for (int b = 0; b < N; ++b) {
                /* binary search for the first position whose score is strictly below k[b] */
                int lo = 0, hi = b;
                while (lo < hi) {
                    int mid = (lo + hi) / 2;
                    if (k[o[mid]] >= k[b]) lo = mid + 1; else hi = mid;
                }
                memmove(o + lo + 1, o + lo, (size_t)(b - lo) * sizeof(int32_t));
                o[lo] = b;
            }
            for (int b = N; b < sh->max_blocks; ++b) o[b] = -1;
        }
    }
}

/* ---------- scaled logits of one block for one query head ---------------------------------- */
static void block_logits(const oracle_shape *sh, const uint16_t *qg, const uint16_t *kb, int valid,
                         double *s) {
    const int D = sh->head_dim;
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    for (int t = 0; t < valid; ++t) {
        double acc = 0.0;
        for (int c = 0; c < D; ++c)
            acc += decode(qg[c], sh->dtype) * decode(kb[(size_t)t * D + c], sh->dtype);
        s[t] = acc * inv_sqrt_d;
    }
}

/* ---------- dense attention (Sec. 2.1) ------------------------------------------------------- */
/* out: [batch][num_q_heads][head_dim]; lse (may be NULL): [batch][num_q_heads] = log sum_t e^{s_t}.
 * A request with no token gives out = 0 and lse = -inf. */
void oracle_dense_attention(const oracle_shape *sh, const uint16_t *q, const uint16_t *k_pool,
                            const uint16_t *v_pool, const int32_t *block_table,
                            const int32_t *ctx_lens, double *out, double *lse) {
    const int Hq = sh->num_q_heads, H = sh->num_kv_heads, D = sh->head_dim, T = sh->page_size;
    const int G = Hq / H;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int r = 0; r < sh->batch; ++r) {
        for (int hq = 0; hq < Hq; ++hq) {
            const int h = hq / G;
            const int ctx = ctx_lens[r], N = blocks_of(ctx, T);
            const uint16_t *qg = q + ((size_t)r * Hq + hq) * D;
            double *o = out + ((size_t)r * Hq + hq) * D;
            for (int c = 0; c < D; ++c) o[c] = 0.0;
            if (N == 0) { if (lse) lse[(size_t)r * Hq + hq] = -INFINITY; continue; }
            double *s = (double *)malloc((size_t)N * T * sizeof(double));
            /* pass 1: all logits and their maximum */
            double smax = -INFINITY;
            for (int b = 0; b < N; ++b) {
                int page = block_table[(size_t)r * sh->max_blocks + b];
                int valid = valid_tokens(ctx, T, b);
                block_logits(sh, qg, k_pool + ((size_t)page * H + h) * T * D, valid, s + (size_t)b * T);
                for (int t = 0; t < valid; ++t)
                    if (s[(size_t)b * T + t] > smax) smax = s[(size_t)b * T + t];
            }
            /* pass 2: P = softmax(S), O = P V */
            double denom = 0.0;
            for (int b = 0; b < N; ++b) {
                int valid = valid_tokens(ctx, T, b);
                for (int t = 0; t < valid; ++t) denom += exp(s[(size_t)b * T + t] - smax);
            }
            for (int b = 0; b < N; ++b) {
                int page = block_table[(size_t)r * sh->max_blocks + b];
                int valid = valid_tokens(ctx, T, b);
                const uint16_t *vb = v_pool + ((size_t)page * H + h) * T * D;
                for (int t = 0; t < valid; ++t) {
                    double p = exp(s[(size_t)b * T + t] - smax) / denom;
                    for (int c = 0; c < D; ++c) o[c] += p * decode(vb[(size_t)t * D + c], sh->dtype);
                }
            }
            if (lse) lse[(size_t)r * Hq + hq] = smax + log(denom);
            free(s);
        }
    }
}

/* ---------- attention over a ranked prefix, by the definition ------------------------------ */
/* For query head (r, hq): softmax attention over the tokens of blocks order[0 .. n_take-1].
 * n_take: [batch][num_q_heads].  n_take = 0 gives out = 0. */
void oracle_attend_prefix(const oracle_shape *sh, const uint16_t *q, const uint16_t *k_pool,
                          const uint16_t *v_pool, const int32_t *block_table,
                          const int32_t *ctx_lens, const int32_t *order, const int32_t *n_take,
                          double *out, double *lse /* [batch][Hq] log of the softmax denominator, or NULL */) {
    const int Hq = sh->num_q_heads, H = sh->num_kv_heads, D = sh->head_dim, T = sh->page_size;
    const int G = Hq / H;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int r = 0; r < sh->batch; ++r) {
        for (int hq = 0; hq < Hq; ++hq) {
            const int h = hq / G, ctx = ctx_lens[r];
            const int n = n_take[(size_t)r * Hq + hq];
            const uint16_t *qg = q + ((size_t)r * Hq + hq) * D;
            const int32_t *ord = order + ((size_t)r * H + h) * sh->max_blocks;
            double *o = out + ((size_t)r * Hq + hq) * D;
            for (int c = 0; c < D; ++c) o[c] = 0.0;
            if (lse) lse[(size_t)r * Hq + hq] = -INFINITY;
            if (n <= 0) continue;
            double *s = (double *)malloc((size_t)n * T * sizeof(double));
            double smax = -INFINITY, denom = 0.0;
            for (int i = 0; i < n; ++i) {
                int b = ord[i], page = block_table[(size_t)r * sh->max_blocks + b];
                int valid = valid_tokens(ctx, T, b);
                block_logits(sh, qg, k_pool + ((size_t)page * H + h) * T * D, valid, s + (size_t)i * T);
                for (int t = 0; t < valid; ++t)
                    if (s[(size_t)i * T + t] > smax) smax = s[(size_t)i * T + t];
            }
            for (int i = 0; i < n; ++i) {
                int valid = valid_tokens(ctx, T, ord[i]);
                for (int t = 0; t < valid; ++t) denom += exp(s[(size_t)i * T + t] - smax);
            }
            if (lse) lse[(size_t)r * Hq + hq] = smax + log(denom);
            for (int i = 0; i < n; ++i) {
                int b = ord[i], page = block_table[(size_t)r * sh->max_blocks + b];
                int valid = valid_tokens(ctx, T, b);
                const uint16_t *vb = v_pool + ((size_t)page * H + h) * T * D;
                for (int t = 0; t < valid; ++t) {
                    double p = exp(s[(size_t)i * T + t] - smax) / denom;
                    for (int c = 0; c < D; ++c) o[c] += p * decode(vb[(size_t)t * D + c], sh->dtype);
                }
            }
            free(s);
        }
    }
}

/* ---------- the progressive loop (Algorithm 1, lines 7-19; Sec. 3.2) ------------------------------ */
/*
 * Every query head is walked on its own over the ranking of its KV head (Sec. 3.2, batched form: a
 * query drops out as soon as it has passed the threshold).  The head keeps four things while it
 * consumes blocks in ranked order: the attention output over the blocks consumed so far, the sum of
 * their weights, the smallest weight any single consumed block had, and the count of blocks not yet
 * consumed.  A block's "weight" AS is the sum over its valid tokens of exp(scaled logit); its own
 * output O is softmax attention inside the block.  Consuming a block merges O into the running output
 * in proportion to the two weights, adds AS to the running sum, and lowers the minimum if AS is
 * smaller.  The share of the total attention already covered is then estimated by pretending that
 * every block still unread weighs as much as the lightest one seen:
 *     P_acc = AS_acc / (AS_acc + AS_min * N_left),
 * and the head stops at the first tested position where P_acc exceeds eps.
 *
 * Only ratios of weights enter any result, so every exponent is taken relative to one per-head
 * constant s_ref (the head's largest logit): exp() stays inside double range, no ratio changes.
 *
 * Readings of open points:
 *   - microbatch m (Sec. 3.2): the test is made only after every m-th block and after the last
 *     block; the minimum stays a per-block quantity and N_left counts blocks.
 *   - the comparison is strict, as Algorithm 1 prints it; so eps = 1 never stops early.
 *   - the comparison is taken in binary32: (float)P_acc > (float)eps.  The threshold crosses the C
 *     ABI as a float, so eps is a binary32 number to begin with; P_acc is rounded to the same type so
 *     that "exceeds" means the same thing on both sides of a parity test when P_acc and eps agree to
 *     more digits than binary32 holds (only there can the rounding decide).
 *   - a partly filled last block takes part like any other, with its valid tokens only.
 *
 * Outputs: out [batch][num_q_heads][head_dim]; n_selected, mass_est [batch][num_q_heads];
 * blocks_read [batch][num_kv_heads] = max over the group of n_selected.
 * Optional curves (may be NULL), each [batch][num_q_heads][max_blocks], entry n-1 for n consumed
 * blocks, computed over ALL blocks regardless of the stop: p_acc_curve = P_acc(n);
 * true_mass_curve = AS_acc(n) / AS_acc(N);  as_curve = log of the n-th consumed block's AS + s_ref.
 */
void oracle_psa_decode(const oracle_shape *sh, const uint16_t *q, const uint16_t *k_pool,
                       const uint16_t *v_pool, const int32_t *block_table, const int32_t *ctx_lens,
                       const int32_t *order, double eps, int32_t m, double *out,
                       int32_t *n_selected, double *mass_est, int32_t *blocks_read,
                       double *p_acc_curve, double *true_mass_curve, double *as_curve) {
    const int Hq = sh->num_q_heads, H = sh->num_kv_heads, D = sh->head_dim, T = sh->page_size;
    const int G = Hq / H;
    if (m < 1) m = 1;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int r = 0; r < sh->batch; ++r) {
        for (int hq = 0; hq < Hq; ++hq) {
            const int h = hq / G, ctx = ctx_lens[r], N = blocks_of(ctx, T);
            const size_t qi = (size_t)r * Hq + hq;
            const uint16_t *qg = q + qi * D;
            const int32_t *ord = order + ((size_t)r * H + h) * sh->max_blocks;
            double *o_out = out + qi * D;
            for (int c = 0; c < D; ++c) o_out[c] = 0.0;
            n_selected[qi] = 0;
            mass_est[qi] = 0.0;
            if (N == 0) continue;

            /* logits of every block, and the reference exponent */
            double *s = (double *)malloc((size_t)N * T * sizeof(double));
            double s_ref = -INFINITY;
            for (int b = 0; b < N; ++b) {
                int page = block_table[(size_t)r * sh->max_blocks + b];
                int valid = valid_tokens(ctx, T, b);
                block_logits(sh, qg, k_pool + ((size_t)page * H + h) * T * D, valid, s + (size_t)b * T);
                for (int t = 0; t < valid; ++t)
                    if (s[(size_t)b * T + t] > s_ref) s_ref = s[(size_t)b * T + t];
            }

            double *O_acc = (double *)calloc((size_t)D, sizeof(double));
            double *O = (double *)malloc((size_t)D * sizeof(double));
            double AS_acc = 0.0, AS_min = INFINITY;
            int N_left = N, stopped = 0;
            for (int n = 1; n <= N; ++n) {
                const int b = ord[n - 1];
                const int page = block_table[(size_t)r * sh->max_blocks + b];
                const int valid = valid_tokens(ctx, T, b);
                const uint16_t *vb = v_pool + ((size_t)page * H + h) * T * D;
                /* the block's own attention: weight AS and output O */
                double AS = 0.0;
                for (int t = 0; t < valid; ++t) AS += exp(s[(size_t)b * T + t] - s_ref);
                for (int c = 0; c < D; ++c) O[c] = 0.0;
                if (AS > 0.0)
                    for (int t = 0; t < valid; ++t) {
                        double p = exp(s[(size_t)b * T + t] - s_ref) / AS;
                        for (int c = 0; c < D; ++c) O[c] += p * decode(vb[(size_t)t * D + c], sh->dtype);
                    }
                /* merge (only while this head has not stopped: its output is frozen after) */
                if (!stopped && AS_acc + AS > 0.0)
                    for (int c = 0; c < D; ++c) O_acc[c] = (AS_acc * O_acc[c] + AS * O[c]) / (AS_acc + AS);
                AS_acc += AS;
                /* lightest block so far, blocks left, estimated share */
                if (AS < AS_min) AS_min = AS;
                N_left -= 1;
                double AS_total = AS_acc + AS_min * (double)N_left;
                double P_acc = AS_total > 0.0 ? AS_acc / AS_total : 0.0;
                if (p_acc_curve) p_acc_curve[qi * sh->max_blocks + (n - 1)] = P_acc;
                if (true_mass_curve) true_mass_curve[qi * sh->max_blocks + (n - 1)] = AS_acc; /* scaled below */
                if (as_curve) as_curve[qi * sh->max_blocks + (n - 1)] = log(AS) + s_ref;
                /* the stop test, once per microbatch of m blocks and at the end */
                if (!stopped && (n % m == 0 || n == N)) {
                    if ((float)P_acc > (float)eps || n == N) {
                        stopped = 1;
                        n_selected[qi] = n;
                        mass_est[qi] = P_acc;
                        for (int c = 0; c < D; ++c) o_out[c] = O_acc[c];
                        if (!p_acc_curve && !true_mass_curve && !as_curve) break;
                    }
                }
            }
            if (true_mass_curve)
                for (int n = 1; n <= N; ++n) true_mass_curve[qi * sh->max_blocks + (n - 1)] /= AS_acc;
            free(s); free(O); free(O_acc);
        }
    }
    if (blocks_read)
        for (int r = 0; r < sh->batch; ++r)
            for (int h = 0; h < H; ++h) {
                int mx = 0;
                for (int g = 0; g < G; ++g) {
                    int v = n_selected[(size_t)r * Hq + h * G + g];
                    if (v > mx) mx = v;
                }
                blocks_read[(size_t)r * H + h] = mx;
            }
}
