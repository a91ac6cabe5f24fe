/*
 * CPU oracle for the distance-based and the angle-based pruning of a k-NN graph in the
 * Collect-Filter-Store procedure (paper section 5.1, the algorithm "CFS procedure of
 * pruning"; the NSG, Vamana, NSSG and DPG rows of the table of pruning strategies and their
 * description in section 3.2).
 *
 * THIS IS TEST INFRASTRUCTURE: a plain, slow, single-threaded definition written out,
 * used only by the test-suite.  It shares no code with the HIP library.
 *
 * For every node p:
 *   Collect  hops = 1: the candidates are p's neighbours in the k-NN graph;
 *            hops = 2: those and the neighbours of each of them.
 *            p itself, ids without a row and repeats are no candidates.  The candidates
 *            are ordered by (dis(p, c), id) and the first cand_size of them go on.
 *   Filter   the serial rule of section 3.2: the candidates are taken closest first; p' is
 *            inserted into R iff for every p* already in R
 *                dis(p, p') < alpha * dis(p*, p')            (alpha = 1: NSG; alpha > 1: Vamana)
 *            until R holds d_out nodes.  dis is the Euclidean distance; this library stores
 *            its square, so the test is  sq(p, p') < alpha^2 * sq(p*, p').
 *            Angle rule (NSSG): p' is inserted iff for every p* already in R the angle between
 *            p -> p* and p -> p' exceeds gamma.  With a = sq(p, p*), b = sq(p, p'), c = sq(p*, p')
 *            the cosine of that angle is (a + b - c) / (2 sqrt(a b)), so the test is
 *                t < 0  or  t^2 < 4 cos^2(gamma) (a b),   t = a + b - c      (0 < gamma <= 90 degrees).
 *            Dispersion rule (DPG; section 5.1 reaches it with the angle metric and a threshold of 0): R is
 *            to make the sum of the pairwise angles at p large, by greedy insertion.  The nearest candidate
 *            is inserted first; then, until R holds d_out nodes or no candidate is left, the candidate
 *            whose angles to the nodes in R add up to the most is inserted (equal sums: the nearer one).
 *            The angle is acos(t / (2 sqrt(a b))) (0 when a b = 0: a node at p's position has no
 *            direction), with the arc cosine taken from the eight-term polynomial of Abramowitz and
 *            Stegun 4.4.46, acos(x) = sqrt(1 - x) (a0 + a1 x + ... + a7 x^7) on [0, 1] (|error| <= 2e-8)
 *            and acos(-x) = pi - acos(x), so that both sides can take every step in the same arithmetic.
 *   Store    R in insertion order, padded with -1.
 *
 * Precision: squared distances are summed in double from the float inputs and then rounded
 * to float; the comparisons above are taken in float, every operation rounded to float in the
 * order written: alpha^2 * sq;  t = (a + b) - c, t * t, c4 * (a * b) with c4 = 4 cos^2(gamma)
 * formed in double and rounded once (a cosine below 1e-12 counts as 0: gamma = 90 degrees).
 * The dispersion rule takes a b, sqrt, the quotient, 1 - |x|, sqrt, the polynomial (Horner, one fused
 * multiply-add per coefficient), the product and pi - r in float, each rounded once, and adds a
 * candidate's angles in the order of insertion.
 * This is the precision the GPU decides in.  On integer-valued data below 2^24 every one of
 * these values is exact.
 *
 * Pinning (tests/test_oracle_filter.py): closed forms on a line and on a circle, the strict
 * inequality on an isosceles triangle, alpha -> infinity reduces to "the d_out nearest
 * candidates", duplicates, 2-hop collection against a set union in Python, invariants.
 * The angle rule (tests/test_oracle_filter_angle.py): line, circle, a right angle with gamma = 90,
 * angles measured with arccos, equality with the distance rule on a sphere.  The dispersion rule
 * (tests/test_oracle_filter_dpg.py): the arc cosine against the library's, a hand-made example,
 * a greedy in double precision written in the test, twins, prefix and scaling invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

static const float *g_X;
static int g_d;

static double sq64(int64_t a, int64_t b)
{
    const float *x = g_X + a * g_d, *y = g_X + b * g_d;
    double s = 0.0;
    for (int j = 0; j < g_d; ++j) { double t = (double)x[j] - (double)y[j]; s += t * t; }
    return s;
}

static double norm64(int64_t a)
{
    const float *x = g_X + a * g_d;
    double s = 0.0;
    for (int j = 0; j < g_d; ++j) s += (double)x[j] * (double)x[j];
    return s;
}

/* angle at p between p -> r and p -> c from the squared lengths a = |p r|^2, b = |p c|^2, c = |r c|^2 */
float oangle_at(float a, float b, float c)
{
    const float ab = a * b;
    if (!(ab > 0.0f)) return 0.0f;
    const float den = 2.0f * sqrtf(ab);
    const float t = (a + b) - c;
    float x = t / den;
    if (x > 1.0f) x = 1.0f;
    if (x < -1.0f) x = -1.0f;
    const float ax = fabsf(x);
    float pol = -0.0012624911f;
    pol = fmaf(pol, ax, 0.0066700901f);
    pol = fmaf(pol, ax, -0.0170881256f);
    pol = fmaf(pol, ax, 0.0308918810f);
    pol = fmaf(pol, ax, -0.0501743046f);
    pol = fmaf(pol, ax, 0.0889789874f);
    pol = fmaf(pol, ax, -0.2145988016f);
    pol = fmaf(pol, ax, 1.5707963050f);
    const float r = sqrtf(1.0f - ax) * pol;
    return x < 0.0f ? 3.14159265358979323846f - r : r;
}

void oangle_at_many(const float *a, const float *b, const float *c, float *out, int64_t count)
{
    for (int64_t i = 0; i < count; ++i) out[i] = oangle_at(a[i], b[i], c[i]);
}

typedef struct { float dist; int32_t id; } cand_t;

static int cand_less(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->dist != b->dist) return a->dist < b->dist ? -1 : 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

/* Prunes the rows of nodes 0 .. n_do-1 (n_do <= n; the rest of the graph is only read).
 * out_ids: n_do x d_out; out_deg: n_do (may be NULL); out_margin: n_do (may be NULL): the
 * smallest distance of any decision taken for the row from flipping, |lhs - rhs| divided by
 * the sum of the squared norms of the nodes involved (0 when equal keys were ordered by id).
 * A row whose margin is far above float rounding has one possible result in any arithmetic.
 * Returns 0, or -1 on bad arguments. */
/* rule 0: distance rule, thres = alpha >= 1.  rule 1: angle rule, thres = gamma in degrees, 0 < gamma <= 90.
 * rule 2: dispersion rule, thres unused; the margin of its rows is the smallest lead, in radians, of an inserted
 * candidate's sum over the runner-up's (and the ordering gaps as for the other rules). */
int ofilter(const float *X, int64_t n, int d, const int32_t *ids, int k, int64_t n_do,
            int hops, int cand_size, int rule, float thres, int d_out,
            int32_t *out_ids, int32_t *out_deg, double *out_margin)
{
    if (!X || !ids || !out_ids || n < 1 || d < 1 || k < 1 || n_do < 0 || n_do > n) return -1;
    if ((hops != 1 && hops != 2) || cand_size < 1 || d_out < 1) return -1;
    if (rule < 0 || rule > 2) return -1;
    if (rule == 0 && !(thres >= 1.0f)) return -1;
    if (rule == 1 && !(thres > 0.0f && thres <= 90.0f)) return -1;
    g_X = X; g_d = d;
    const float a2 = thres * thres;
    double cg = cos((double)thres * 3.14159265358979323846 / 180.0);
    if (fabs(cg) < 1e-12) cg = 0.0;
    const float c4 = (float)(4.0 * cg * cg);
    int64_t cap = (int64_t)k + (hops == 2 ? (int64_t)k * k : 0);
    cand_t *cand = (cand_t *)malloc((size_t)cap * sizeof(cand_t));
    int64_t *stamp = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    int32_t *R = (int32_t *)malloc((size_t)d_out * sizeof(int32_t));
    float *score = (float *)malloc((size_t)(cand_size > 0 ? cand_size : 1) * sizeof(float));
    char *in = (char *)malloc((size_t)(cand_size > 0 ? cand_size : 1));
    for (int64_t i = 0; i < n; ++i) stamp[i] = -1;
    for (int64_t p = 0; p < n_do; ++p) {
        /* Collect */
        int64_t m = 0;
        const int32_t *Np = ids + p * k;
        for (int i = 0; i < k; ++i) {
            int32_t u = Np[i];
            if (u < 0 || u >= n || u == p || stamp[u] == p) continue;
            stamp[u] = p; cand[m++].id = u;
        }
        if (hops == 2) {
            int64_t m1 = m;
            for (int64_t i = 0; i < m1; ++i) {
                const int32_t *Nu = ids + (int64_t)cand[i].id * k;
                for (int j = 0; j < k; ++j) {
                    int32_t w = Nu[j];
                    if (w < 0 || w >= n || w == p || stamp[w] == p) continue;
                    stamp[w] = p; cand[m++].id = w;
                }
            }
        }
        for (int64_t i = 0; i < m; ++i) cand[i].dist = (float)sq64(p, cand[i].id);
        qsort(cand, (size_t)m, sizeof(cand_t), cand_less);
        double margin = INFINITY;
        double np_ = norm64(p);
        int64_t mc = m < cand_size ? m : cand_size;
        if (out_margin) {
            int64_t last = mc < m ? mc : mc - 1;       /* includes the cut between kept and dropped candidates */
            for (int64_t i = 0; i < last; ++i) {
                double sc = np_ + norm64(cand[i].id) + norm64(cand[i + 1].id);
                double g = fabs((double)cand[i + 1].dist - (double)cand[i].dist) / (sc > 0 ? sc : 1.0);
                if (g < margin) margin = g;
            }
        }
        /* Filter */
        int deg = 0;
        if (rule == 2) {
            for (int64_t i = 0; i < mc; ++i) { score[i] = 0.0f; in[i] = 0; }
            int64_t last = -1;
            while (deg < d_out && deg < mc) {
                int64_t best = -1, second = -1;
                for (int64_t i = 0; i < mc; ++i) {
                    if (in[i]) continue;
                    if (last >= 0) score[i] += oangle_at(cand[last].dist, cand[i].dist, (float)sq64(cand[last].id, cand[i].id));
                    if (best < 0 || score[i] > score[best]) { second = best; best = i; }
                    else if (second < 0 || score[i] > score[second]) second = i;
                }
                if (second >= 0 && last >= 0) {
                    double g = (double)score[best] - (double)score[second];
                    if (g < margin) margin = g;
                }
                in[best] = 1;
                R[deg++] = cand[best].id;
                last = best;
            }
        }
        for (int64_t i = 0; rule != 2 && i < mc && deg < d_out; ++i) {
            int32_t c = cand[i].id;
            float lhs = cand[i].dist;
            int keep = 1;
            double m_keep = INFINITY, m_drop = 0.0;
            for (int r = 0; r < deg; ++r) {
                float drc = (float)sq64(R[r], c);
                double sc = np_ + norm64(c) + norm64(R[r]);
                int pass;
                double g;
                if (rule == 0) {
                    float rhs = a2 * drc;
                    pass = lhs < rhs;
                    g = fabs((double)lhs - (double)rhs) / (sc > 0 ? sc : 1.0);
                } else {
                    float a = (float)sq64(p, R[r]);
                    float t = (a + lhs) - drc;
                    float tt = t * t;
                    float ab = a * lhs;
                    float rhs = c4 * ab;
                    pass = t < 0.0f || tt < rhs;
                    /* distance from flipping: of t from 0, or of t^2 from the threshold, in squared-length units */
                    double g1 = fabs((double)t), g2 = fabs((double)tt - (double)rhs) / (fabs((double)t) + sqrt((double)rhs) + 1e-300);
                    g = (t < 0.0f ? g1 : (g1 < g2 ? g1 : g2)) / (sc > 0 ? sc : 1.0);
                }
                if (pass) { if (g < m_keep) m_keep = g; }
                else { keep = 0; if (g > m_drop) m_drop = g; }
            }
            double mcand = keep ? m_keep : m_drop;      /* dropped: safe if one occluder is safe */
            if (mcand < margin) margin = mcand;
            if (keep) R[deg++] = c;
        }
        /* Store */
        for (int t = 0; t < d_out; ++t) out_ids[p * d_out + t] = t < deg ? R[t] : -1;
        if (out_deg) out_deg[p] = deg;
        if (out_margin) out_margin[p] = margin;
    }
    free(cand); free(stamp); free(R); free(score); free(in);
    return 0;
}

int ofilter_dist(const float *X, int64_t n, int d, const int32_t *ids, int k, int64_t n_do,
                 int hops, int cand_size, float alpha, int d_out,
                 int32_t *out_ids, int32_t *out_deg, double *out_margin)
{
    return ofilter(X, n, d, ids, k, n_do, hops, cand_size, 0, alpha, d_out, out_ids, out_deg, out_margin);
}
