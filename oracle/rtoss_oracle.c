/*
 * rtoss_oracle.c -- plain fp64 CPU statement of what the R-TOSS hot path computes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is compared
 * against.  It shares no code, table or header with the GPU library and must never be
 * linked into, or called from, the product path.
 *
 * Everything here is the definition written out with no blocking, fusion or reordering:
 *   - pattern dictionary: all k-subsets of the 9 taps of a 3x3 kernel (Section IV.B, Eq. 1)
 *     that pass an adjacency filter (Section IV.B, first narrowing criterion);
 *   - pattern selection: for every group of 9 weights, the dictionary entry whose
 *     retained L2 norm is largest (Section IV.C prose around Algorithm 2);
 *   - masking: W (.) M, and the left-over tail of a flattened 1x1 tensor set to zero
 *     (Section II.B "Semi-structured pruning"; Section IV.D, Algorithm 3);
 *   - convolution: ordinary 2-D cross-correlation with zero padding over the masked
 *     weights (Section II.B cost model: only non-zero weights contribute).
 *
 * Tap numbering: tap t of a group is row t/3, column t%3 of the 3x3 kernel, which is also
 * offset t inside the 9 contiguous weights of the group.  Bit t of a mask <-> tap t.
 *
 * Parity pins (tests/test_oracle_*.py): dictionary counts against Eq. 1 and an independent
 * graph search; selection against exhaustive search and, for the unfiltered dictionary,
 * against plain magnitude sorting; convolution against torch.nn.functional.conv2d in
 * float64, unit impulses, and a float64 matmul for 1x1.
 * Parity unpinned: the paper's second narrowing criterion ("most used" patterns under
 * random kernels, the final 21 patterns) is not computed here at all.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

enum { ORACLE_RULE_ALL = 0, ORACLE_RULE_ANYPAIR4 = 1, ORACLE_RULE_CONNECTED4 = 2, ORACLE_RULE_CONNECTED8 = 3 };

static int tap_row(int t) { return t / 3; }
static int tap_col(int t) { return t % 3; }
static int iabs(int v) { return v < 0 ? -v : v; }

/* 4-neighbour: share an edge.  8-neighbour: share an edge or a corner. */
static int taps_adjacent(int a, int b, int eight)
{
    int dr = iabs(tap_row(a) - tap_row(b));
    int dc = iabs(tap_col(a) - tap_col(b));
    if (a == b) return 0;
    if (eight) return dr <= 1 && dc <= 1;
    return dr + dc == 1;
}

static int popcount9(unsigned m)
{
    int c = 0;
    for (int t = 0; t < 9; ++t) c += (m >> t) & 1u;
    return c;
}

/* Is the set of live taps one connected component under the chosen neighbourhood? */
static int mask_connected(unsigned m, int eight)
{
    unsigned seen = 0, frontier = 0;
    for (int t = 0; t < 9; ++t)
        if ((m >> t) & 1u) { frontier = 1u << t; break; }
    if (!frontier) return 0;
    while (frontier) {
        seen |= frontier;
        unsigned next = 0;
        for (int a = 0; a < 9; ++a) {
            if (!((frontier >> a) & 1u)) continue;
            for (int b = 0; b < 9; ++b)
                if (((m >> b) & 1u) && !((seen >> b) & 1u) && taps_adjacent(a, b, eight))
                    next |= 1u << b;
        }
        frontier = next;
    }
    return seen == m;
}

/* Does the mask hold at least one pair of 4-adjacent live taps?  (A single tap passes.) */
static int mask_has_adjacent_pair(unsigned m)
{
    if (popcount9(m) == 1) return 1;
    for (int a = 0; a < 9; ++a)
        for (int b = a + 1; b < 9; ++b)
            if (((m >> a) & 1u) && ((m >> b) & 1u) && taps_adjacent(a, b, 0)) return 1;
    return 0;
}

static int mask_passes(unsigned m, int rule)
{
    switch (rule) {
    case ORACLE_RULE_ALL:        return 1;
    case ORACLE_RULE_ANYPAIR4:   return mask_has_adjacent_pair(m);
    case ORACLE_RULE_CONNECTED4: return mask_connected(m, 0);
    case ORACLE_RULE_CONNECTED8: return mask_connected(m, 1);
    default:                     return 0;
    }
}

/*
 * Section IV.B, Eq. 1 + first criterion.  Enumerates the k-subsets of {0..8} as ascending
 * tuples in lexicographic order, keeps those that pass `rule`, and writes their bit masks
 * to masks[0..cap).  Returns the number kept (which may exceed cap; only cap are written),
 * or -1 for a bad k / rule.
 */
int rtoss_oracle_pattern_dict(int k, int rule, uint16_t *masks, int cap)
{
    if (k < 1 || k > 9 || rule < 0 || rule > 3) return -1;
    int tup[9];
    for (int i = 0; i < k; ++i) tup[i] = i;
    int count = 0;
    for (;;) {
        unsigned m = 0;
        for (int i = 0; i < k; ++i) m |= 1u << tup[i];
        if (mask_passes(m, rule)) {
            if (masks && count < cap) masks[count] = (uint16_t)m;
            ++count;
        }
        /* next ascending tuple in lexicographic order */
        int i = k - 1;
        while (i >= 0 && tup[i] == 9 - k + i) --i;
        if (i < 0) break;
        ++tup[i];
        for (int j = i + 1; j < k; ++j) tup[j] = tup[j - 1] + 1;
    }
    return count;
}

/*
 * Section IV.C (Algorithm 2, scoring loop and best-fit choice), applied to the flat view
 * used by Section IV.D (Algorithm 3): weights w[0..n_elems) are cut into G = n_elems/9
 * groups of 9 contiguous values.  For each group and each pattern p the score is the sum,
 * over the live taps of mask p in ascending tap order, of w_t * w_t, accumulated in fp64
 * starting from 0.  The winner is found by a strict `>` scan from p = 0 that starts below
 * every real score, so equal scores resolve to the lowest pattern index, a NaN score
 * never wins, and a group whose scores are all NaN gets index 0.  (The square root of the
 * norm is monotone and is left out.)
 */
void rtoss_oracle_select(const double *w, int64_t n_elems, const uint16_t *masks, int P, uint8_t *idx)
{
    int64_t G = n_elems / 9;
    for (int64_t g = 0; g < G; ++g) {
        const double *wg = w + 9 * g;
        int best = 0;
        double best_score = -1.0; /* every real score is >= 0, so pattern 0 wins first */
        for (int p = 0; p < P; ++p) {
            double s = 0.0;
            for (int t = 0; t < 9; ++t)
                if ((masks[p] >> t) & 1u) s = s + wg[t] * wg[t];
            if (s > best_score) { best = p; best_score = s; }
        }
        idx[g] = (uint8_t)best;
    }
}

/*
 * W' = W (.) mask[idx] per group (Section II.B; Algorithm 2 mask write), and the
 * n_elems % 9 left-over weights at the end of the flat list become zero (Section IV.D,
 * Algorithm 3 else-branch).
 */
void rtoss_oracle_mask(const double *w, int64_t n_elems, const uint16_t *masks, const uint8_t *idx, double *w_out)
{
    int64_t G = n_elems / 9;
    for (int64_t g = 0; g < G; ++g)
        for (int t = 0; t < 9; ++t)
            w_out[9 * g + t] = ((masks[idx[g]] >> t) & 1u) ? w[9 * g + t] : 0.0;
    for (int64_t i = 9 * G; i < n_elems; ++i) w_out[i] = 0.0;
}

static int64_t out_extent(int in, int ks, int stride, int pad) { return (in + 2 * pad - ks) / stride + 1; }

/* One output element of the cross-correlation, all taps, ascending (ci, kh, kw). */
static double conv_point(const double *x, const double *w, int Ci, int H, int W, int ks, int stride, int pad,
                         int n, int co, int oh, int ow)
{
    double acc = 0.0;
    for (int ci = 0; ci < Ci; ++ci)
        for (int kh = 0; kh < ks; ++kh)
            for (int kw = 0; kw < ks; ++kw) {
                int ih = oh * stride - pad + kh;
                int iw = ow * stride - pad + kw;
                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                double xv = x[(((int64_t)n * Ci + ci) * H + ih) * W + iw];
                double wv = w[(((int64_t)co * Ci + ci) * ks + kh) * ks + kw];
                acc = acc + wv * xv;
            }
    return acc;
}

/*
 * Direct convolution, PyTorch conv2d semantics (cross-correlation, zero padding, no bias,
 * groups 1, dilation 1).  x is [N][Ci][H][W], w is [Co][Ci][ks][ks] (already masked),
 * y is [N][Co][Ho][Wo], all fp64 row-major.  relu != 0 applies max(.,0) afterwards.
 * The loop over (n, co) is shared among threads; each output is still one serial sum.
 */
void rtoss_oracle_conv2d(const double *x, const double *w, double *y, int N, int Ci, int H, int W, int Co, int ks,
                         int stride, int pad, int relu)
{
    int Ho = (int)out_extent(H, ks, stride, pad), Wo = (int)out_extent(W, ks, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Co; ++co)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double v = conv_point(x, w, Ci, H, W, ks, stride, pad, n, co, oh, ow);
                    if (relu && v < 0.0) v = 0.0;
                    y[(((int64_t)n * Co + co) * Ho + oh) * Wo + ow] = v;
                }
}

/* The same sum for a list of output coordinates pts[4*i..] = (n, co, oh, ow). */
void rtoss_oracle_conv2d_points(const double *x, const double *w, const int32_t *pts, int64_t npts, double *out,
                                int Ci, int H, int W, int ks, int stride, int pad, int relu)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; ++i) {
        double v = conv_point(x, w, Ci, H, W, ks, stride, pad, pts[4 * i], pts[4 * i + 1], pts[4 * i + 2], pts[4 * i + 3]);
        if (relu && v < 0.0) v = 0.0;
        out[i] = v;
    }
}

/*
 * Variant that visits only the live taps of each 3x3 kernel (what "skipping the zeros"
 * means in Section II.B).  w is the UNMASKED [Co][Ci][3][3] tensor; masks/idx pick the
 * live taps of kernel (co, ci).  Taps are visited in ascending order, so the result is
 * the same fp64 sum as the masked-dense loop minus its exact zero terms.
 */
void rtoss_oracle_conv2d_live3x3(const double *x, const double *w, const uint16_t *masks, const uint8_t *idx, double *y,
                                 int N, int Ci, int H, int W, int Co, int stride, int relu)
{
    const int ks = 3, pad = 1;
    int Ho = (int)out_extent(H, ks, stride, pad), Wo = (int)out_extent(W, ks, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Co; ++co)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int ci = 0; ci < Ci; ++ci) {
                        unsigned m = masks[idx[(int64_t)co * Ci + ci]];
                        for (int t = 0; t < 9; ++t) {
                            if (!((m >> t) & 1u)) continue;
                            int ih = oh * stride - pad + t / 3, iw = ow * stride - pad + t % 3;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc = acc + w[((int64_t)co * Ci + ci) * 9 + t] *
                                            x[(((int64_t)n * Ci + ci) * H + ih) * W + iw];
                        }
                    }
                    if (relu && acc < 0.0) acc = 0.0;
                    y[(((int64_t)n * Co + co) * Ho + oh) * Wo + ow] = acc;
                }
}

int rtoss_oracle_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
