/*
 * CO3 gradient codec -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded reference for the per-iteration uplink path of
 * the CO3 protocol (Algorithm 1 of the paper: error correction, fp conversion,
 * Huffman compression on the user side; decompression and averaging on the
 * parameter-server side).  Nothing in the product may call into this file: it
 * exists so that tests, the smoke check and the benchmark's CPU leg have an
 * independent statement of what every step computes.  It shares no code, table
 * or constant with the HIP library.
 *
 * Everything here is scalar and in the order the method states it.  Floating
 * point that the method performs in fp32 is performed in fp32 with one IEEE
 * operation per stated operation (build with -ffp-contract=off, no fast-math);
 * the quantiser itself is evaluated in double, where every intermediate is
 * exact, following the nearest-representative rule of Sec. III (i).
 *
 * Readings of the paper that the text leaves open (integer exponent anchor in
 * place of the real-valued bias, ties-to-even, gradual underflow, one zero,
 * Huffman tie-breaks, bit order) are listed in the repository's design notes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define CO3O_OK 0
#define CO3O_EINVAL (-1)
#define CO3O_ECAP (-2)
#define CO3O_ENOCODE (-3)
#define CO3O_EBADSTREAM (-4)

/* ---------------------------------------------------------------------- */
/* Sec. III (i): the representative set of the sign/exponent/mantissa      */
/* format, with the exponent bias realised as an integer anchor A: the top */
/* exponent field maps to binade 2^A.                                      */
/* ---------------------------------------------------------------------- */

/* magnitude of the level with exponent field f and mantissa field m */
double co3o_level(int f, int m, int A, int E, int M)
{
    int F = (1 << E) - 1;
    int e_min = A - F + 1;
    double frac = (double)m / (double)(1 << M);
    if (f == 0)
        return ldexp(frac, e_min);          /* gradual underflow, includes 0 */
    return ldexp(1.0 + frac, e_min + f - 1);
}

/* round to nearest integer, ties to the even integer; t >= 0 */
static double round_half_even(double t)
{
    double lo = floor(t);
    double d = t - lo; /* exact: t has at most 24 significant bits here */
    if (d > 0.5)
        return lo + 1.0;
    if (d < 0.5)
        return lo;
    return (fmod(lo, 2.0) == 0.0) ? lo : lo + 1.0;
}

/* Nearest representative of the magnitude a >= 0: returns fields (f, m). */
static void quantize_magnitude(double a, int A, int E, int M, int *f_out, int *m_out)
{
    int F = (1 << E) - 1;
    int e_min = A - F + 1;
    double two_M = (double)(1 << M);
    if (a == 0.0) {
        *f_out = 0;
        *m_out = 0;
        return;
    }
    if (isinf(a)) { /* beyond every level: the largest one is the closest */
        *f_out = F;
        *m_out = (1 << M) - 1;
        return;
    }
    int ex2;
    (void)frexp(a, &ex2);   /* a = frac * 2^ex2, frac in [0.5, 1) */
    int ex = ex2 - 1;       /* floor(log2 a) */
    int e = ex > e_min ? ex : e_min; /* clamped exponent */
    double t = ldexp(a, -(e - M));   /* a in units of the local quantum; exact */
    double r = round_half_even(t);
    if (ex >= e_min) { /* normal range of the format */
        if (r == 2.0 * two_M) {
            e += 1;
            r = two_M;
        }
        int f = e - e_min + 1;
        int m = (int)(r - two_M);
        if (f > F) { /* above the top binade: saturate to the largest level */
            f = F;
            m = (1 << M) - 1;
        }
        *f_out = f;
        *m_out = m;
    } else { /* below the smallest normal level */
        if (r == two_M) {
            *f_out = 1;
            *m_out = 0;
        } else {
            *f_out = 0;
            *m_out = (int)r;
        }
    }
}

/* Q_fp as a real-valued map, any (E, M) and any integer anchor (no clamp):
 * used to pin the quantiser against library float formats. */
double co3o_quantize_value(double x, int A, int E, int M)
{
    int f, m;
    quantize_magnitude(fabs(x), A, E, M, &f, &m);
    double v = co3o_level(f, m, A, E, M);
    return (signbit(x) && v != 0.0) ? -v : v;
}

/* array form of co3o_quantize_value (x given as fp32) */
void co3o_quantize_values(const float *x, int64_t n, int A, int E, int M, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = co3o_quantize_value((double)x[i], A, E, M);
}

/* symbol byte = sign | exponent field | mantissa field; the negative zero
 * pattern is never produced */
int co3o_quantize_symbol(float x, int A, int E, int M)
{
    int f, m;
    quantize_magnitude(fabs((double)x), A, E, M, &f, &m);
    int s = (signbit(x) && !(f == 0 && m == 0)) ? 1 : 0;
    return (s << (E + M)) | (f << M) | m;
}

/* value of a symbol byte under anchor A (always exactly an fp32 number for
 * the anchors co3o_anchor produces) */
float co3o_symbol_value(int sym, int A, int E, int M)
{
    int s = (sym >> (E + M)) & 1;
    int f = (sym >> M) & ((1 << E) - 1);
    int m = sym & ((1 << M) - 1);
    double v = co3o_level(f, m, A, E, M);
    return (float)(s ? -v : v);
}

/* ---------------------------------------------------------------------- */
/* Exponent anchor per segment (one segment = one tensor / layer): the     */
/* binade of the largest gradient magnitude, A = floor(log2 max|g|),       */
/* clamped so that every level is an fp32 number.                          */
/* ---------------------------------------------------------------------- */
int co3o_anchor(const float *g, int64_t n, const int64_t *seg_off, int nseg, int E, int32_t *anchor)
{
    int F = (1 << E) - 1;
    if (nseg < 0 || E < 1)
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        if (seg_off[s] < 0 || seg_off[s + 1] < seg_off[s] || seg_off[s + 1] > n)
            return CO3O_EINVAL;
        float amax = 0.0f;
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            float a = fabsf(g[i]);
            if (a > amax)
                amax = a;
        }
        int A;
        if (amax == 0.0f) {
            A = F - 126;
        } else if (isinf(amax)) {
            A = 127;
        } else {
            int ex2;
            (void)frexpf(amax, &ex2);
            A = ex2 - 1;
        }
        if (A < F - 126)
            A = F - 126;
        if (A > 127)
            A = 127;
        anchor[s] = A;
    }
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* Algorithm 1, user side: x = g + gamma*m_{t-1};  ghat = Q_fp(x);         */
/* m_t = x - ghat.  err holds m_{t-1} on entry and m_t on return.          */
/* ---------------------------------------------------------------------- */
int co3o_convert_ef(const float *g, float *err, uint8_t *sym, int64_t n, const int64_t *seg_off, int nseg,
                    const int32_t *anchor, float gamma, int E, int M)
{
    if (E < 1 || M < 0 || 1 + E + M > 8 || nseg < 0 || (nseg > 0 && seg_off[nseg] > n))
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        int A = anchor[s];
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            volatile float decayed = gamma * err[i]; /* one rounding */
            volatile float x = g[i] + decayed;       /* one rounding */
            int q = co3o_quantize_symbol(x, A, E, M);
            float v = co3o_symbol_value(q, A, E, M);
            volatile float e_new = x - v;            /* one rounding */
            sym[i] = (uint8_t)q;
            err[i] = e_new;
        }
    }
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* Empirical symbol counts (stand-in for the model pmf of Sec. III (ii)).  */
/* ---------------------------------------------------------------------- */
int co3o_histogram(const uint8_t *sym, int64_t n, int K, uint32_t *counts)
{
    for (int k = 0; k < K; ++k)
        counts[k] = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (sym[i] >= K)
            return CO3O_EINVAL;
        counts[sym[i]] += 1;
    }
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* Sec. III (ii): Huffman code lengths.  Textbook two-queue construction:  */
/* leaves sorted by (weight, symbol) ascending wait in queue 1; merged     */
/* nodes join queue 2 in creation order; each step removes the two lowest  */
/* fronts, a leaf winning a tie against a merged node.                     */
/* ---------------------------------------------------------------------- */
int co3o_huffman_lengths(const uint32_t *weights, int K, uint8_t *len)
{
    if (K < 1 || K > 256)
        return CO3O_EINVAL;
    int leaf_sym[256];
    int nact = 0;
    for (int k = 0; k < K; ++k) {
        len[k] = 0;
        if (weights[k] > 0)
            leaf_sym[nact++] = k;
    }
    if (nact == 0)
        return CO3O_OK;
    if (nact == 1) {
        len[leaf_sym[0]] = 1;
        return CO3O_OK;
    }
    /* insertion sort of the leaves by (weight asc, symbol asc) */
    for (int i = 1; i < nact; ++i) {
        int s = leaf_sym[i];
        int j = i - 1;
        while (j >= 0 && (weights[leaf_sym[j]] > weights[s] ||
                          (weights[leaf_sym[j]] == weights[s] && leaf_sym[j] > s))) {
            leaf_sym[j + 1] = leaf_sym[j];
            --j;
        }
        leaf_sym[j + 1] = s;
    }
    /* nodes 0..nact-1 are the sorted leaves, nact..2*nact-2 merged nodes */
    uint64_t w[512];
    int parent[512];
    for (int i = 0; i < nact; ++i)
        w[i] = weights[leaf_sym[i]];
    int q1 = 0;          /* front of the leaf queue */
    int q2 = nact;       /* front of the merged-node queue */
    int next = nact;     /* next merged node to create */
    for (int step = 0; step < nact - 1; ++step) {
        int pick[2];
        for (int c = 0; c < 2; ++c) {
            int have_leaf = q1 < nact;
            int have_node = q2 < next;
            if (have_leaf && (!have_node || w[q1] <= w[q2]))
                pick[c] = q1++;
            else
                pick[c] = q2++;
        }
        w[next] = w[pick[0]] + w[pick[1]];
        parent[pick[0]] = next;
        parent[pick[1]] = next;
        ++next;
    }
    int root = next - 1;
    for (int i = 0; i < nact; ++i) {
        int depth = 0;
        for (int v = i; v != root; v = parent[v])
            ++depth;
        len[leaf_sym[i]] = (uint8_t)depth;
    }
    return CO3O_OK;
}

/* Canonical codewords: symbols ordered by (length, symbol); the first gets
 * the all-zero word, each next one is (previous + 1) shifted left by the
 * growth in length. */
int co3o_canonical_codes(const uint8_t *len, int K, uint64_t *code)
{
    int have_prev = 0;
    uint64_t prev_code = 0;
    int prev_len = 0;
    for (int k = 0; k < K; ++k)
        code[k] = 0;
    for (int l = 1; l <= 64; ++l) {
        for (int k = 0; k < K; ++k) {
            if (len[k] != l)
                continue;
            if (!have_prev) {
                code[k] = 0;
                have_prev = 1;
            } else {
                code[k] = (prev_code + 1) << (l - prev_len);
            }
            prev_code = code[k];
            prev_len = l;
        }
    }
    for (int k = 0; k < K; ++k)
        if (len[k] > 64)
            return CO3O_EINVAL;
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* h_Hf: concatenate the codewords of sym[0..n) most-significant bit       */
/* first.  Stream bit p lives in bit 63-(p mod 64) of words[p / 64]; the   */
/* last word is zero padded.  chunk_bitoff[c] is the stream position of    */
/* symbol c*chunk_syms, chunk_bitoff[nchunks] the total length.            */
/* ---------------------------------------------------------------------- */
int co3o_encode(const uint8_t *sym, int64_t n, const uint8_t *len, const uint64_t *code, int K, int64_t chunk_syms,
                uint64_t *words, int64_t cap_words, uint64_t *chunk_bitoff, uint64_t *total_bits)
{
    if (chunk_syms < 1 || n < 0)
        return CO3O_EINVAL;
    uint64_t total = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (sym[i] >= K || len[sym[i]] == 0)
            return CO3O_ENOCODE;
        total += len[sym[i]];
    }
    if ((total + 63) / 64 > (uint64_t)cap_words)
        return CO3O_ECAP;
    for (uint64_t wdx = 0; wdx < (total + 63) / 64; ++wdx)
        words[wdx] = 0;
    uint64_t p = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (i % chunk_syms == 0)
            chunk_bitoff[i / chunk_syms] = p;
        int l = len[sym[i]];
        uint64_t c = code[sym[i]];
        for (int b = l - 1; b >= 0; --b) {
            if ((c >> b) & 1)
                words[p / 64] |= (uint64_t)1 << (63 - (p % 64));
            ++p;
        }
    }
    int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    chunk_bitoff[nchunks] = p;
    *total_bits = p;
    return CO3O_OK;
}

/* Inverse of h_Hf: walk the code tree one stream bit at a time. */
int co3o_decode(const uint64_t *words, uint64_t total_bits, const uint8_t *len, const uint64_t *code, int K,
                int64_t n, uint8_t *sym_out)
{
    /* binary trie over the codewords; node 0 is the root */
    int cap = 2;
    for (int k = 0; k < K; ++k)
        cap += len[k];
    int(*child)[2] = malloc(sizeof(int[2]) * (size_t)cap);
    int *leaf = malloc(sizeof(int) * (size_t)cap);
    if (!child || !leaf) {
        free(child);
        free(leaf);
        return CO3O_EINVAL;
    }
    int nnodes = 1;
    child[0][0] = child[0][1] = -1;
    leaf[0] = -1;
    for (int k = 0; k < K; ++k) {
        if (len[k] == 0)
            continue;
        int v = 0;
        for (int b = len[k] - 1; b >= 0; --b) {
            int bit = (int)((code[k] >> b) & 1);
            if (child[v][bit] < 0) {
                child[nnodes][0] = child[nnodes][1] = -1;
                leaf[nnodes] = -1;
                child[v][bit] = nnodes++;
            }
            v = child[v][bit];
        }
        leaf[v] = k;
    }
    int rc = CO3O_OK;
    uint64_t p = 0;
    for (int64_t i = 0; i < n && rc == CO3O_OK; ++i) {
        int v = 0;
        while (leaf[v] < 0) {
            if (p >= total_bits) {
                rc = CO3O_EBADSTREAM;
                break;
            }
            int bit = (int)((words[p / 64] >> (63 - (p % 64))) & 1);
            ++p;
            v = child[v][bit];
            if (v < 0) {
                rc = CO3O_EBADSTREAM;
                break;
            }
        }
        if (rc == CO3O_OK)
            sym_out[i] = (uint8_t)leaf[v];
    }
    if (rc == CO3O_OK && p != total_bits)
        rc = CO3O_EBADSTREAM;
    free(child);
    free(leaf);
    return rc;
}

/* ---------------------------------------------------------------------- */
/* Parameter server: average of the reconstructed user gradients,          */
/* (1/U) * sum_u ghat^(u), users added in index order in fp32, then one    */
/* fp32 division.  sym is [U][stride]; anchor is [U][nseg].                */
/* ---------------------------------------------------------------------- */
int co3o_aggregate(const uint8_t *sym, int64_t n, int U, int64_t stride, const int64_t *seg_off, int nseg,
                   const int32_t *anchor, int E, int M, float *avg)
{
    if (U < 1)
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            volatile float acc = 0.0f;
            for (int u = 0; u < U; ++u) {
                float v = co3o_symbol_value(sym[(int64_t)u * stride + i], anchor[(int64_t)u * nseg + s], E, M);
                acc = acc + v;
            }
            volatile float mean = acc / (float)U;
            avg[i] = mean;
        }
    }
    (void)n;
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* Sec. IV-B, "fp exponent bias": the bias of Sec. III (i) as a function   */
/* of the GenNorm parameters of the tensor.  The bias is read as a real    */
/* multiplier c applied to the corrected gradient before it is rounded     */
/* onto a fixed grid (the printed approximation scales as 1/sigma, which   */
/* only a multiplier does), and "sigma" as the GenNorm scale parameter     */
/* alpha: under that reading the printed polynomial is the L2-optimal      */
/* multiplier of a 4-bit grid to about one per cent (pinned by a test).    */
/* ---------------------------------------------------------------------- */

/* first absolute and second moment sums of x = g + gamma*m per tensor */
int co3o_moments(const float *g, const float *err, int64_t n, const int64_t *seg_off, int nseg, float gamma,
                 double *sums /* [nseg][2] */)
{
    if (nseg < 0 || (nseg > 0 && seg_off[nseg] > n))
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        double s1 = 0.0, s2 = 0.0;
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            volatile float decayed = gamma * err[i];
            volatile float x = g[i] + decayed;
            double xd = (double)x;
            s1 += fabs(xd);
            s2 += xd * xd;
        }
        sums[2 * s] = s1;
        sums[2 * s + 1] = s2;
    }
    return CO3O_OK;
}

/* (E|X|)^2 / E[X^2] of GenNorm(beta): Gamma(2/b)^2 / (Gamma(1/b) Gamma(3/b)); rises from 0 to 3/4 */
double co3o_gennorm_ratio(double beta)
{
    return exp(2.0 * lgamma(2.0 / beta) - lgamma(1.0 / beta) - lgamma(3.0 / beta));
}

#define CO3O_FIT_BETA_LO 0.05
#define CO3O_FIT_BETA_HI 50.0

/* Moment matching: the beta whose ratio equals s1^2 / (n s2), found by bisection, and the scale
 * alpha that reproduces the second moment.  A tensor of zeros gives beta = 1, alpha = 0. */
int co3o_gennorm_fit(double s1, double s2, int64_t n, double *beta, double *alpha)
{
    if (n <= 0 || !(s2 > 0.0)) {
        *beta = 1.0;
        *alpha = 0.0;
        return CO3O_OK;
    }
    double rho = s1 * s1 / ((double)n * s2);
    double lo = CO3O_FIT_BETA_LO, hi = CO3O_FIT_BETA_HI;
    if (rho <= co3o_gennorm_ratio(lo)) {
        hi = lo;
    } else if (rho >= co3o_gennorm_ratio(hi)) {
        lo = hi;
    } else {
        for (int it = 0; it < 200; ++it) {
            double mid = 0.5 * (lo + hi);
            if (co3o_gennorm_ratio(mid) < rho)
                lo = mid;
            else
                hi = mid;
        }
    }
    double b = 0.5 * (lo + hi);
    *beta = b;
    *alpha = sqrt(s2 / (double)n * exp(lgamma(1.0 / b) - lgamma(3.0 / b)));
    return CO3O_OK;
}

/* the printed fourth-degree fit, beta clamped to the range over which the paper plots it */
double co3o_bias_poly(double beta)
{
    double b = beta < 0.4 ? 0.4 : (beta > 1.6 ? 1.6 : beta);
    return 0.46 - 2.85 * b + 5.37 * b * b - 2.85 * b * b * b + 0.52 * b * b * b * b;
}

/* multiplier c = poly(beta) / alpha as an fp32 number kept inside [2^-96, 2^96]; 1 for a zero tensor */
float co3o_bias_scale(double beta, double alpha)
{
    if (!(alpha > 0.0))
        return 1.0f;
    double c = co3o_bias_poly(beta) / alpha;
    const double lim = ldexp(1.0, 96);
    if (!(c < lim))
        c = lim;
    if (!(c > 1.0 / lim))
        c = 1.0 / lim;
    return (float)c;
}

/* Algorithm 1 with the multiplier: x = g + gamma*m; y = c*x; ghat = Q_A(y) / c; m' = x - ghat.
 * One fp32 rounding per stated operation.  scale is [nseg], anchor the fixed grid's anchor. */
int co3o_convert_ef_scaled(const float *g, float *err, uint8_t *sym, int64_t n, const int64_t *seg_off, int nseg,
                           const int32_t *anchor, const float *scale, float gamma, int E, int M)
{
    if (E < 1 || M < 0 || 1 + E + M > 8 || nseg < 0 || (nseg > 0 && seg_off[nseg] > n))
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        int A = anchor[s];
        float c = scale[s];
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            volatile float decayed = gamma * err[i];
            volatile float x = g[i] + decayed;
            volatile float y = c * x;
            int q = co3o_quantize_symbol(y, A, E, M);
            volatile float ghat = co3o_symbol_value(q, A, E, M) / c;
            volatile float e_new = x - ghat;
            sym[i] = (uint8_t)q;
            err[i] = e_new;
        }
    }
    return CO3O_OK;
}

/* parameter server with multipliers: each user's level is divided by that user's c before the sum */
int co3o_aggregate_scaled(const uint8_t *sym, int64_t n, int U, int64_t stride, const int64_t *seg_off, int nseg,
                          const int32_t *anchor, const float *scale, int E, int M, float *avg)
{
    if (U < 1)
        return CO3O_EINVAL;
    for (int s = 0; s < nseg; ++s) {
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            volatile float acc = 0.0f;
            for (int u = 0; u < U; ++u) {
                float v = co3o_symbol_value(sym[(int64_t)u * stride + i], anchor[(int64_t)u * nseg + s], E, M);
                volatile float ghat = v / scale[(int64_t)u * nseg + s];
                acc = acc + ghat;
            }
            volatile float mean = acc / (float)U;
            avg[i] = mean;
        }
    }
    (void)n;
    return CO3O_OK;
}

/* ---------------------------------------------------------------------- */
/* Sec. III (ii) assigns the codes per layer: every layer (tensor) has a   */
/* code of its own, and all users share the code of a layer.  A user's     */
/* stream is still one concatenation of codewords over all its elements;   */
/* the codeword of element i comes from the code of the tensor that holds  */
/* i.  len and code are [nseg][K].                                         */
/* ---------------------------------------------------------------------- */

/* symbol counts per tensor: counts is [nseg][K] */
int co3o_histogram_layers(const uint8_t *sym, int64_t n, const int64_t *seg_off, int nseg, int K, uint32_t *counts)
{
    if (nseg < 0 || (nseg > 0 && seg_off[nseg] > n))
        return CO3O_EINVAL;
    for (int64_t j = 0; j < (int64_t)nseg * K; ++j)
        counts[j] = 0;
    for (int s = 0; s < nseg; ++s)
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            if (sym[i] >= K) /* not a symbol of the format: rejected, as in co3o_histogram */
                return CO3O_EINVAL;
            counts[(int64_t)s * K + sym[i]] += 1;
        }
    return CO3O_OK;
}

int co3o_encode_layers(const uint8_t *sym, int64_t n, const int64_t *seg_off, int nseg, const uint8_t *len,
                       const uint64_t *code, int K, int64_t chunk_syms, uint64_t *words, int64_t cap_words,
                       uint64_t *chunk_bitoff, uint64_t *total_bits)
{
    if (chunk_syms < 1 || n < 0 || nseg < 1 || seg_off[0] != 0 || seg_off[nseg] != n)
        return CO3O_EINVAL;
    uint64_t total = 0;
    for (int s = 0; s < nseg; ++s)
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            if (sym[i] >= K || len[(int64_t)s * K + sym[i]] == 0)
                return CO3O_ENOCODE;
            total += len[(int64_t)s * K + sym[i]];
        }
    if ((total + 63) / 64 > (uint64_t)cap_words)
        return CO3O_ECAP;
    for (uint64_t wdx = 0; wdx < (total + 63) / 64; ++wdx)
        words[wdx] = 0;
    uint64_t p = 0;
    for (int s = 0; s < nseg; ++s)
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            if (i % chunk_syms == 0)
                chunk_bitoff[i / chunk_syms] = p;
            int l = len[(int64_t)s * K + sym[i]];
            uint64_t c = code[(int64_t)s * K + sym[i]];
            for (int b = l - 1; b >= 0; --b) {
                if ((c >> b) & 1)
                    words[p / 64] |= (uint64_t)1 << (63 - (p % 64));
                ++p;
            }
        }
    int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    chunk_bitoff[nchunks] = p;
    *total_bits = p;
    return CO3O_OK;
}

/* inverse: for each element, extend the read prefix one stream bit at a time until it equals a
 * codeword of the element's tensor (codes are prefix-free, so the first match is the symbol) */
int co3o_decode_layers(const uint64_t *words, uint64_t total_bits, const int64_t *seg_off, int nseg,
                       const uint8_t *len, const uint64_t *code, int K, int64_t n, uint8_t *sym_out)
{
    if (nseg < 1 || seg_off[0] != 0 || seg_off[nseg] != n)
        return CO3O_EINVAL;
    uint64_t p = 0;
    for (int s = 0; s < nseg; ++s) {
        const uint8_t *ls = len + (int64_t)s * K;
        const uint64_t *cs = code + (int64_t)s * K;
        for (int64_t i = seg_off[s]; i < seg_off[s + 1]; ++i) {
            uint64_t prefix = 0;
            int found = -1;
            for (int l = 1; l <= 64 && found < 0; ++l) {
                if (p >= total_bits)
                    return CO3O_EBADSTREAM;
                prefix = (prefix << 1) | ((words[p / 64] >> (63 - (p % 64))) & 1);
                ++p;
                for (int k = 0; k < K; ++k)
                    if (ls[k] == l && cs[k] == prefix) {
                        found = k;
                        break;
                    }
            }
            if (found < 0)
                return CO3O_EBADSTREAM;
            sym_out[i] = (uint8_t)found;
        }
    }
    return p == total_bits ? CO3O_OK : CO3O_EBADSTREAM;
}
