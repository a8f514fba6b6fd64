/*
 * CPU oracle for farthest point sampling, minimum-distance-prediction sampling
 * (MDPS) and ball query -- FastPoint, arXiv 2507.23480.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * statement of what the GPU library must compute.  Nothing in the product path
 * may include, link or call it; it shares no code, header, table or helper
 * with the HIP sources.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg load it.
 *
 * Arithmetic conventions (fixed so that index results can be compared
 * bit-for-bit):
 *   - "distance" in Algorithm 1 / Algorithm 2 is the SQUARED Euclidean
 *     distance in IEEE binary32, evaluated as ((dx*dx) + (dy*dy)) + (dz*dz)
 *     with every operation rounded separately (build with -ffp-contract=off,
 *     never -ffast-math).  Squaring keeps every comparison and argmax of the
 *     paper's algorithms, which only ever compare distances.
 *   - argmax and "find any available point" take the LOWEST index among
 *     equals / candidates (the paper leaves both open: the arg-max of
 *     Alg. 1, findAnyOne of Alg. 2).
 *   - the curve estimator works in binary64 and rounds each threshold once
 *     to binary32.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * against brute-force restatements, closed-form cases and hand-worked examples
 * (tests/golden/).  The one thing no test can pin to the paper is the CHOICE of
 * estimator constants (exponent, bias, fit window): the paper fits them on data
 * sets that are not available ("parity unpinned" for those constants only; the
 * arithmetic that uses them is pinned by closed forms).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_MAX_SEG 16

/* squared distance, the one rounding order used everywhere */
static float ref_dist2(const float *a, const float *b)
{
    float dx = a[0] - b[0];
    float dy = a[1] - b[1];
    float dz = a[2] - b[2];
    float t = dx * dx;
    t = t + dy * dy;
    t = t + dz * dz;
    return t;
}

/* Alg. 1, distance-update loop: fold one sample into the running min-distance array */
static void ref_fold(const float *xyz, int32_t N, int32_t s, float *dists)
{
    const float *c = xyz + 3 * (size_t)s;
    for (int32_t j = 0; j < N; ++j) {
        float d = ref_dist2(c, xyz + 3 * (size_t)j);
        if (dists[j] > d)
            dists[j] = d;
    }
}

/* Alg. 1, arg-max step: index of the maximum, lowest index among equal maxima */
static int32_t ref_argmax(const float *dists, int32_t N)
{
    int32_t best = 0;
    for (int32_t j = 1; j < N; ++j)
        if (dists[j] > dists[best])
            best = j;
    return best;
}

/*
 * Exact farthest point sampling -- Algorithm 1 (Section 3.3).
 *   xyz      [N][3] points
 *   start    seed index (first step of Alg. 1; the paper draws it at random)
 *   out_idx  [n]  sampled indices, out_idx[0] = start
 *   out_mdc  [n]  or NULL: out_mdc[i] = max(min_dists) at the moment sample i
 *            was picked (the "minimum distance curve", Section 4 and the prefix
 *            loop of Alg. 2), squared; out_mdc[0] = +inf.
 * Returns 0, or -1 on bad arguments.
 */
int ref_fps_exact(const float *xyz, int32_t N, int32_t n, int32_t start,
                  int32_t *out_idx, float *out_mdc)
{
    if (!xyz || !out_idx || N < 1 || n < 1 || n > N || start < 0 || start >= N)
        return -1;
    float *dists = (float *)malloc(sizeof(float) * (size_t)N);
    if (!dists)
        return -1;
    for (int32_t j = 0; j < N; ++j)
        dists[j] = INFINITY;
    out_idx[0] = start;
    if (out_mdc)
        out_mdc[0] = INFINITY;
    for (int32_t i = 1; i < n; ++i) {
        ref_fold(xyz, N, out_idx[i - 1], dists);
        int32_t best = ref_argmax(dists, N);
        out_idx[i] = best;
        if (out_mdc)
            out_mdc[i] = dists[best];
    }
    free(dists);
    return 0;
}

/* ------------------------------------------------------------------ MDPS -- */

typedef struct {
    float p;              /* prefix ratio of exact FPS iterations (Sec. 4.1: 0.1)    */
    int32_t nseg;         /* number of curve segments (Sec. 5.3 default 6), 1..16    */
    double exponent;      /* e of the power-law curve C(x) = a / x^e (App. A.3),
                             in SQUARED-distance space, x = sample index            */
    float bias;           /* multiplies the predicted DISTANCE (so bias^2 on d^2)    */
    int32_t fit_window;   /* W: number of trailing prefix points that determine a    */
    int32_t m_min;        /* lower limit of prefix iterations                        */
    int32_t use_override; /* nonzero: take thresholds from thr_override (tests)      */
    float thr_override[REF_MAX_SEG];
    float level_scale[REF_MAX_SEG]; /* offline per-segment correction of the predicted
                                       SQUARED value (1 = pure power function)       */
    const float *mlp;     /* NULL: power-function estimator.  Else the weights of the
                             MLP estimator of App. A.3 (REF_MLP_WEIGHTS floats, layout
                             at ref_mlp_curve)                                       */
    int32_t scan_order;   /* which available point the threshold phase takes (Sec. 4.1
                             step 3 says "randomly selected among the available points"):
                             0 the lowest index; 1 the first in the scattered order of
                             ref_scan_stride                                         */
} ref_mdps_params;

typedef struct {
    int32_t m;                          /* prefix iterations actually run             */
    int32_t et_index;                   /* first sample index filled by the remainder
                                           FPS (early termination), n if none         */
    int32_t level_start[REF_MAX_SEG];   /* sample index at which level l+1 became
                                           current, -1 if it never did                */
    int32_t level_exhausted[REF_MAX_SEG]; /* 1 if level l+1 ran out of available points */
    float thr2[REF_MAX_SEG];            /* squared thresholds R_l^2 used              */
} ref_mdps_info;

/* number of prefix iterations: floor(p*n), at least m_min; the caller treats
 * m >= n-1 as "everything is exact FPS" */
int32_t ref_mdps_prefix_len(const ref_mdps_params *prm, int32_t n)
{
    int32_t m = (int32_t)floor((double)prm->p * (double)n);
    if (m < prm->m_min)
        m = prm->m_min;
    return m;
}

/*
 * x^e for an integer x >= 1, binary64.  The estimator needs a power function
 * whose result does not depend on the math library at hand (the thresholds
 * derived from it decide integer picks), so it is spelled out with + - * /
 * only, each of which IEEE 754 rounds the same way everywhere:
 *   x = f * 2^k with f in [sqrt(1/2), sqrt(2));  ln f = 2 atanh((f-1)/(f+1))
 *   by its series (13 terms, |s| < 0.172);  y = e * (k ln2 + ln f);
 *   y = q ln2 + r with q = round(y / ln2);  exp r by its Taylor series
 *   (20 terms, |r| < 0.35);  result = exp(r) * 2^q.
 * Relative error stays below 2e-14 (ln 2 is itself rounded); tests pin it against libm pow.
 */
double ref_pow_int_base(int64_t x, double e)
{
    const double LN2 = 0.6931471805599453;
    int k = 0;
    while (((int64_t)1 << (k + 1)) <= x)
        ++k;
    double f = (double)x / (double)((int64_t)1 << k);   /* exact, in [1,2) */
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k = k + 1;
    }
    double s = (f - 1.0) / (f + 1.0);
    double s2 = s * s;
    double sum = 0.0;
    for (int t = 12; t >= 0; --t)
        sum = sum * s2 + 1.0 / (double)(2 * t + 1);
    double lnx = ((double)k * LN2) + ((2.0 * s) * sum);
    double y = e * lnx;
    double q = floor(y / LN2 + 0.5);
    double r = y - q * LN2;
    double acc = 1.0;
    for (int t = 20; t >= 1; --t)
        acc = 1.0 + acc * (r / (double)t);
    return ldexp(acc, (int)q);                           /* exact scaling */
}

/* ln v for a normal positive binary64 v, with + - * / only, in a fixed order:
 * v = f * 2^k with f in [sqrt(1/2), sqrt(2)), ln f = 2 atanh((f-1)/(f+1)) by 13 terms of
 * its series.  The same steps as inside ref_pow_int_base. */
double ref_ln_fixed(double v)
{
    const double LN2 = 0.6931471805599453;
    int k = 0;
    double f = frexp(v, &k);          /* exact: v = f * 2^k, f in [0.5, 1) */
    f = f * 2.0;
    k = k - 1;                        /* f in [1, 2) */
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k = k + 1;
    }
    double s = (f - 1.0) / (f + 1.0);
    double s2 = s * s;
    double sum = 0.0;
    for (int t = 12; t >= 0; --t)
        sum = sum * s2 + 1.0 / (double)(2 * t + 1);
    return ((double)k * LN2) + ((2.0 * s) * sum);
}

/* exp y, fixed order: y = q ln2 + r, q = round(y / ln2), exp r by 20 terms of its Taylor
 * series, times 2^q.  y is first brought into [-700, 700] (NaN counts as -700), so that
 * the scaling by 2^q is exact and defined for whatever a network puts out. */
double ref_exp_fixed(double y)
{
    const double LN2 = 0.6931471805599453;
    if (!(y >= -700.0))
        y = -700.0;
    if (y > 700.0)
        y = 700.0;
    double q = floor(y / LN2 + 0.5);
    double r = y - q * LN2;
    double acc = 1.0;
    for (int t = 20; t >= 1; --t)
        acc = 1.0 + acc * (r / (double)t);
    return ldexp(acc, (int)q);
}

/*
 * MLP curve estimator (Appendix A.3): a three-layer perceptron 32-128-128-64 that takes
 * the first segment of the minimum distance curve "represented by 32 values" and returns
 * the rest of the curve "represented by 64 values".  The paper fixes neither the
 * representation, the activation nor the precision; this build takes
 *   input k (0..31)   ln( mdc[i_k] / mdc[m] ),  i_k = max(1, floor(m (k+1) / 32))
 *   output j (0..63)  ln( C(x_j) / mdc[m] ) at x_j = m + (n-1-m) (j+1) / 64
 *   hidden layers with ReLU, the output layer linear, every layer with a bias
 *   arithmetic in binary64, a neuron's sum starting from its bias and adding the
 *   products in ascending input order, each product and sum rounded on its own
 * (logarithms of ratios make the estimator independent of the cloud's scale and density).
 * Weights, binary32, input-major so that consecutive outputs are adjacent:
 *   W1[32][128] b1[128] W2[128][128] b2[128] W3[128][64] b3[64]   (REF_MLP_WEIGHTS floats)
 *   out[64] receives the output layer
 */
#define REF_MLP_WEIGHTS (32 * 128 + 128 + 128 * 128 + 128 + 128 * 64 + 64)
int ref_mlp_curve(const float *mdc, int32_t m, const float *w, double *out)
{
    if (!mdc || !w || !out || m < 1)
        return -1;
    double in[32], h1[128], h2[128];
    for (int k = 0; k < 32; ++k) {
        int64_t i = ((int64_t)m * (k + 1)) / 32;
        if (i < 1)
            i = 1;
        /* a curve never rises, so the ratio is >= 1; anything else (mdc[m] = 0: all
         * remaining points coincide with samples) reads as 0 */
        double ratio = (double)mdc[i] / (double)mdc[m];
        in[k] = (ratio >= 1.0 && ratio <= 1e300) ? ref_ln_fixed(ratio) : 0.0;
    }
    const float *W1 = w, *b1 = W1 + 32 * 128, *W2 = b1 + 128, *b2 = W2 + 128 * 128;
    const float *W3 = b2 + 128, *b3 = W3 + 128 * 64;
    for (int o = 0; o < 128; ++o) {
        double acc = (double)b1[o];
        for (int k = 0; k < 32; ++k)
            acc = acc + (double)W1[k * 128 + o] * in[k];
        h1[o] = acc > 0.0 ? acc : 0.0;
    }
    for (int o = 0; o < 128; ++o) {
        double acc = (double)b2[o];
        for (int k = 0; k < 128; ++k)
            acc = acc + (double)W2[k * 128 + o] * h1[k];
        h2[o] = acc > 0.0 ? acc : 0.0;
    }
    for (int o = 0; o < 64; ++o) {
        double acc = (double)b3[o];
        for (int k = 0; k < 128; ++k)
            acc = acc + (double)W3[k * 64 + o] * h2[k];
        out[o] = acc;
    }
    return 0;
}

/* The estimated curve at sample position b (m < b <= n-1), squared: linear interpolation
 * of the MLP's outputs (log of the ratio to mdc[m]; the ratio is 1 at position m). */
static double ref_mlp_value(const double *out, const float *mdc, int32_t n, int32_t m, int64_t b)
{
    double u = ((double)(b - m) * 64.0) / (double)(n - 1 - m);      /* in (0, 64] */
    int j0 = (int)floor(u);
    if (j0 > 64)
        j0 = 64;
    double frac = u - (double)j0;
    double v0 = j0 == 0 ? 0.0 : out[j0 - 1];
    double v1 = j0 >= 64 ? out[63] : out[j0];
    double y = v0 + frac * (v1 - v0);
    return (double)mdc[m] * ref_exp_fixed(y);
}

/*
 * Curve estimator and segment thresholds (Section 4.1 step 1, Eq. 1, with the
 * power-function estimator of Appendix A.3; the threshold set-up of Alg. 2,
 * Section 4.1 step 2).
 *   mdc[0..m]  measured curve of the prefix (mdc[0] unused)
 *   C(x) = a / x^e ; a = mean over the last W prefix points of mdc[i] * i^e
 *   R_l^2 = curve value at the END of segment l, index b_l = floor(n*l/nseg)
 *           clamped to [1, n-1]: the measured value if b_l <= m, else the
 *           prediction times bias^2 times level_scale[l] (an offline-fitted
 *           shape correction per segment, 1 for the pure power function).  R_l
 *           serves as the lower bound of the spacing inside segment l
 *           (Section 4.1 step 3), hence the end.
 *   thresholds are kept >= FLT_MIN and non-increasing.
 */
int ref_mdps_thresholds(const float *mdc, int32_t n, int32_t m,
                        const ref_mdps_params *prm, float *thr2)
{
    if (!mdc || !prm || !thr2 || prm->nseg < 1 || prm->nseg > REF_MAX_SEG || m < 1 || m >= n)
        return -1;
    if (prm->use_override) {
        for (int32_t l = 0; l < prm->nseg; ++l)
            thr2[l] = prm->thr_override[l];
        return 0;
    }
    int32_t W = prm->fit_window < m ? prm->fit_window : m;
    if (W < 1)
        return -1;
    double e = prm->exponent;
    double a = 0.0;
    for (int32_t i = m - W + 1; i <= m; ++i)
        a += (double)mdc[i] * ref_pow_int_base(i, e);
    a = a / (double)W;
    double bias2 = (double)prm->bias * (double)prm->bias;
    double mlp_out[64];
    if (prm->mlp && ref_mlp_curve(mdc, m, prm->mlp, mlp_out) != 0)
        return -1;
    for (int32_t l = 1; l <= prm->nseg; ++l) {
        int64_t b = ((int64_t)n * l) / prm->nseg;
        if (b < 1)
            b = 1;
        if (b > n - 1)
            b = n - 1;
        float r;
        if (b <= m)
            r = mdc[b];
        else if (prm->mlp)
            r = (float)((bias2 * (double)prm->level_scale[l - 1]) * ref_mlp_value(mlp_out, mdc, n, m, b));
        else
            r = (float)(((bias2 * (double)prm->level_scale[l - 1]) * a) / ref_pow_int_base(b, e));
        if (!(r >= FLT_MIN))
            r = FLT_MIN;
        if (l >= 2 && r > thr2[l - 2])
            r = thr2[l - 2];
        thr2[l - 1] = r;
    }
    return 0;
}

static void ref_info_init(ref_mdps_info *info, int32_t n)
{
    memset(info, 0, sizeof(*info));
    info->et_index = n;
    for (int l = 0; l < REF_MAX_SEG; ++l)
        info->level_start[l] = -1;
}

/* quota rule of Alg. 2 (the level floor of a sample position): the segment that sample index i belongs to */
static int32_t ref_quota_level(int32_t i, int32_t n, int32_t nseg)
{
    return 1 + (int32_t)(((int64_t)i * nseg) / n);
}

/*
 * Scattered scan order of the threshold phase.  The paper takes a random available point
 * (Section 4.1 step 3); a fixed pseudo-random order keeps that spirit and stays reproducible:
 * the points are visited in the order j_t = (t * A) mod N, t = 0, 1, ..., N-1, a walk with the
 * golden-ratio stride, A = the smallest integer >= max(1, floor(0.6180339887498949 * N)) that has
 * no common divisor with N (so that the walk visits every point once).  In a cloud whose
 * neighbours in space are neighbours in the index (scans), consecutive points of the walk lie far
 * apart.  ref_scan_stride returns A.
 */
static int64_t ref_gcd(int64_t a, int64_t b)
{
    while (b != 0) {
        int64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}

int64_t ref_scan_stride(int32_t N)
{
    if (N < 1)
        return 0;
    int64_t A = (int64_t)floor(0.6180339887498949 * (double)N);
    if (A < 1)
        A = 1;
    while (ref_gcd(A, (int64_t)N) != 1)
        ++A;
    return A;
}

/* The first available point (dists[j] >= r2) in the chosen scan order, -1 if there is none. */
static int32_t ref_first_available(const float *dists, int32_t N, float r2, int32_t scan_order)
{
    if (scan_order == 0) {
        for (int32_t j = 0; j < N; ++j)
            if (dists[j] >= r2)
                return j;
        return -1;
    }
    const int64_t A = ref_scan_stride(N);
    int64_t j = 0;
    for (int32_t t = 0; t < N; ++t) {
        if (dists[j] >= r2)
            return (int32_t)j;
        j += A;
        if (j >= N)
            j -= N;
    }
    return -1;
}

/*
 * MDPS -- Algorithm 2 (Appendix A.1), running-min-distance form.
 *
 * Availability of point j at level l is kept implicitly: the bitmap bit of
 * Alg. 2 is 0 exactly when some already chosen sample lies closer than R_l,
 * i.e. when dists[j] < R_l^2 where dists is the same running min-distance
 * array exact FPS keeps.  ref_mdps_literal() below builds the exclusion lists
 * and bitmaps explicitly and must return the same indices.
 *
 * Steps:
 *  S1  exact FPS for i = 1..m recording mdc (the prefix loop of Alg. 2); the prefix
 *      samples stay in the output and sampling continues at i = m+1.
 *  S2  thresholds from the estimated curve (the estimator call and the threshold set-up of Alg. 2).
 *  S3  threshold sampling (the main loop of Alg. 2): level = max(level, quota level of i);
 *      pick the first available point of the current level in the scan order (the lowest
 *      index, or the first of the scattered walk); if none, move to the next level without
 *      consuming a sample slot.
 *  S4  early termination (the closing part of Alg. 2): once the last level is exhausted the
 *      remaining samples come from exact FPS on the (already current) dists.
 */
int ref_mdps_sample(const float *xyz, int32_t N, int32_t n, int32_t start,
                    const ref_mdps_params *prm, int32_t *out_idx, ref_mdps_info *info_out)
{
    if (!xyz || !out_idx || !prm || N < 1 || n < 1 || n > N || start < 0 || start >= N ||
        prm->nseg < 1 || prm->nseg > REF_MAX_SEG || prm->scan_order < 0 || prm->scan_order > 1)
        return -1;
    ref_mdps_info info;
    ref_info_init(&info, n);
    int32_t m = ref_mdps_prefix_len(prm, n);
    if (m >= n - 1) {               /* nothing left to predict: all exact FPS */
        info.m = n - 1;
        info.et_index = n;
        if (info_out)
            *info_out = info;
        return ref_fps_exact(xyz, N, n, start, out_idx, NULL);
    }
    info.m = m;
    float *dists = (float *)malloc(sizeof(float) * (size_t)N);
    float *mdc = (float *)malloc(sizeof(float) * (size_t)(m + 1));
    if (!dists || !mdc) {
        free(dists);
        free(mdc);
        return -1;
    }
    /* S1 */
    for (int32_t j = 0; j < N; ++j)
        dists[j] = INFINITY;
    out_idx[0] = start;
    mdc[0] = INFINITY;
    for (int32_t i = 1; i <= m; ++i) {
        ref_fold(xyz, N, out_idx[i - 1], dists);
        int32_t best = ref_argmax(dists, N);
        out_idx[i] = best;
        mdc[i] = dists[best];
    }
    /* S2 */
    if (ref_mdps_thresholds(mdc, n, m, prm, info.thr2) != 0) {
        free(dists);
        free(mdc);
        return -1;
    }
    /* S3 */
    int32_t seg = 0;
    int32_t i = m + 1;
    int32_t applied = m - 1;        /* last sample index folded into dists */
    while (i < n) {
        int32_t q = ref_quota_level(i, n, prm->nseg);
        if (q > seg) {
            seg = q;
            if (seg <= prm->nseg && info.level_start[seg - 1] < 0)
                info.level_start[seg - 1] = i;
        }
        if (seg > prm->nseg)
            break;
        while (applied < i - 1) {
            ++applied;
            ref_fold(xyz, N, out_idx[applied], dists);
        }
        float r2 = info.thr2[seg - 1];
        int32_t pick = ref_first_available(dists, N, r2, prm->scan_order);
        if (pick < 0) {             /* level exhausted */
            info.level_exhausted[seg - 1] = 1;
            ++seg;
            if (seg <= prm->nseg && info.level_start[seg - 1] < 0)
                info.level_start[seg - 1] = i;
            continue;
        }
        out_idx[i] = pick;
        ++i;
    }
    /* S4 */
    if (i < n) {
        info.et_index = i;
        while (applied < i - 1) {
            ++applied;
            ref_fold(xyz, N, out_idx[applied], dists);
        }
        /* remainder FPS in the order of the closing loop of Alg. 2 (the first fold
         * repeats sample i-1, which is already in dists: a no-op) */
        for (; i < n; ++i) {
            ref_fold(xyz, N, out_idx[i - 1], dists);
            out_idx[i] = ref_argmax(dists, N);
        }
    }
    if (info_out)
        *info_out = info;
    free(dists);
    free(mdc);
    return 0;
}

/* growable index list */
typedef struct {
    int32_t *v;
    int32_t len, cap;
} ref_list;

static int ref_list_push(ref_list *l, int32_t x)
{
    if (l->len == l->cap) {
        int32_t nc = l->cap ? 2 * l->cap : 8;
        int32_t *nv = (int32_t *)realloc(l->v, sizeof(int32_t) * (size_t)nc);
        if (!nv)
            return -1;
        l->v = nv;
        l->cap = nc;
    }
    l->v[l->len++] = x;
    return 0;
}

/*
 * MDPS with the data structures of Algorithm 2 kept explicitly, as a check that the
 * running-distance form of ref_mdps_sample is the same method: an exclusion list per
 * (level, point), an availability bitmap per level, and nothing else deciding a pick.
 * O(N^2) time and memory: tiny clouds only.  The helpers below are the operations on the
 * two structures; ref_mdps_literal strings them together.
 */

/* All exclusion lists of a cloud: list (l, a) receives every b with dist2(a, b) < thr2[l],
 * in ascending b; one distance per pair serves all levels. */
static int lit_build_lists(const float *xyz, int32_t N, const float *thr2, int32_t nseg, ref_list *excl)
{
    for (int32_t a = 0; a < N; ++a)
        for (int32_t b = 0; b < N; ++b) {
            float d = ref_dist2(xyz + 3 * (size_t)a, xyz + 3 * (size_t)b);
            for (int32_t l = 0; l < nseg; ++l)
                if (d < thr2[l] && ref_list_push(&excl[(size_t)l * N + a], b) != 0)
                    return -1;
        }
    return 0;
}

/* A sample makes the members of its lists unavailable on levels first_level .. nseg-1. */
static void lit_exclude(uint8_t *bitmap, const ref_list *excl, int32_t N, int32_t nseg, int32_t first_level,
                        int32_t sample)
{
    for (int32_t l = first_level; l < nseg; ++l) {
        const ref_list *li = &excl[(size_t)l * N + sample];
        for (int32_t t = 0; t < li->len; ++t)
            bitmap[(size_t)l * N + li->v[t]] = 0;
    }
}

/* "Any available point" of a level is taken to be the first set bit in the scan order (the lowest
 * index, or the first of the scattered walk of ref_scan_stride); -1 if the level has none. */
static int32_t lit_first_available(const uint8_t *bitmap, int32_t N, int32_t level, int32_t scan_order)
{
    const int64_t A = scan_order == 0 ? 1 : ref_scan_stride(N);
    int64_t j = 0;
    for (int32_t t = 0; t < N; ++t) {
        if (bitmap[(size_t)level * N + j])
            return (int32_t)j;
        j += A;
        if (j >= N)
            j -= N;
    }
    return -1;
}

/* Early termination: the distance of every point to its nearest sample, taken from the
 * sampled members of its widest (level-1) list on top of what dists already holds. */
static void lit_distances_from_lists(const float *xyz, int32_t N, const ref_list *excl,
                                     const uint8_t *is_sampled, float *dists)
{
    for (int32_t a = 0; a < N; ++a) {
        const ref_list *li = &excl[a];               /* level 1 is stored first */
        for (int32_t t = 0; t < li->len; ++t)
            if (is_sampled[li->v[t]]) {
                float d = ref_dist2(xyz + 3 * (size_t)a, xyz + 3 * (size_t)li->v[t]);
                if (dists[a] > d)
                    dists[a] = d;
            }
    }
}

int ref_mdps_literal(const float *xyz, int32_t N, int32_t n, int32_t start,
                     const ref_mdps_params *prm, int32_t *out_idx, ref_mdps_info *info_out)
{
    if (!xyz || !out_idx || !prm || N < 1 || n < 1 || n > N || start < 0 || start >= N ||
        prm->nseg < 1 || prm->nseg > REF_MAX_SEG || prm->scan_order < 0 || prm->scan_order > 1)
        return -1;
    ref_mdps_info info;
    ref_info_init(&info, n);
    int32_t m = ref_mdps_prefix_len(prm, n);
    if (m >= n - 1) {
        info.m = n - 1;
        if (info_out)
            *info_out = info;
        return ref_fps_exact(xyz, N, n, start, out_idx, NULL);
    }
    info.m = m;
    const int32_t nseg = prm->nseg;
    float *dists = (float *)malloc(sizeof(float) * (size_t)N);
    float *mdc = (float *)malloc(sizeof(float) * (size_t)(m + 1));
    ref_list *excl = (ref_list *)calloc((size_t)nseg * (size_t)N, sizeof(ref_list));
    uint8_t *bitmap = (uint8_t *)malloc((size_t)nseg * (size_t)N);
    uint8_t *is_sampled = (uint8_t *)calloc((size_t)N, 1);
    int rc = -1;
    if (!dists || !mdc || !excl || !bitmap || !is_sampled)
        goto done;

    /* the exact iterations that open the method, with the curve they measure */
    for (int32_t j = 0; j < N; ++j)
        dists[j] = INFINITY;
    out_idx[0] = start;
    mdc[0] = INFINITY;
    for (int32_t i = 1; i <= m; ++i) {
        ref_fold(xyz, N, out_idx[i - 1], dists);
        int32_t best = ref_argmax(dists, N);
        out_idx[i] = best;
        mdc[i] = dists[best];
    }
    if (ref_mdps_thresholds(mdc, n, m, prm, info.thr2) != 0)
        goto done;
    if (lit_build_lists(xyz, N, info.thr2, nseg, excl) != 0)
        goto done;
    /* every point starts available on every level; the samples kept from the opening
     * iterations (0..m-1; sample m is excluded by the loop below) then exclude theirs */
    memset(bitmap, 1, (size_t)nseg * (size_t)N);
    for (int32_t s = 0; s < m; ++s)
        lit_exclude(bitmap, excl, N, nseg, 0, out_idx[s]);

    int32_t seg = 0;
    int32_t i = m + 1;
    while (i < n) {
        int32_t q = ref_quota_level(i, n, nseg);
        if (q > seg) {
            seg = q;
            if (seg <= nseg && info.level_start[seg - 1] < 0)
                info.level_start[seg - 1] = i;
        }
        if (seg > nseg)
            break;
        lit_exclude(bitmap, excl, N, nseg, seg - 1, out_idx[i - 1]);
        int32_t pick = lit_first_available(bitmap, N, seg - 1, prm->scan_order);
        if (pick < 0) {
            info.level_exhausted[seg - 1] = 1;
            ++seg;
            if (seg <= nseg && info.level_start[seg - 1] < 0)
                info.level_start[seg - 1] = i;
            continue;
        }
        out_idx[i] = pick;
        ++i;
    }
    if (i < n) {
        /* the last level ran out before n samples: the rest is exact FPS, on distances that
         * so far only know the samples 0..m-1 */
        info.et_index = i;
        for (int32_t s = 0; s < i; ++s)
            is_sampled[out_idx[s]] = 1;
        lit_distances_from_lists(xyz, N, excl, is_sampled, dists);
        for (; i < n; ++i) {
            ref_fold(xyz, N, out_idx[i - 1], dists);
            out_idx[i] = ref_argmax(dists, N);
        }
    }
    if (info_out)
        *info_out = info;
    rc = 0;
done:
    if (excl)
        for (size_t t = 0; t < (size_t)nseg * (size_t)N; ++t)
            free(excl[t].v);
    free(excl);
    free(bitmap);
    free(is_sampled);
    free(dists);
    free(mdc);
    return rc;
}

/* ------------------------------------------------------------ ball query -- */
/*
 * Ball query (Section 3.1 step 2): for each centre (a point of the same
 * cloud, given by index) the neighbours closer than `radius`.  The paper
 * fixes neither k, the order nor the padding; this build takes the first k
 * hits in ascending index order, strict "<" on squared binary32 distances
 * (the comparison Alg. 2 builds its lists with), and pads unused slots with the first
 * hit.  out_cnt[q] = min(hits, k) >= 1 because a centre always hits itself.
 *   out_idx [M][k], out_cnt [M] or NULL
 */
int ref_ball_query(const float *xyz, int32_t N, const int32_t *center_idx, int32_t M,
                   float radius, int32_t k, int32_t *out_idx, int32_t *out_cnt)
{
    if (!xyz || !center_idx || !out_idx || N < 1 || M < 0 || k < 1 || !(radius > 0.0f) ||
        !isfinite(radius))
        return -1;
    float r2 = radius * radius;
    for (int32_t q = 0; q < M; ++q) {
        int32_t c = center_idx[q];
        if (c < 0 || c >= N)
            return -1;
        int32_t cnt = 0;
        int32_t *row = out_idx + (size_t)q * k;
        for (int32_t j = 0; j < N && cnt < k; ++j)
            if (ref_dist2(xyz + 3 * (size_t)c, xyz + 3 * (size_t)j) < r2)
                row[cnt++] = j;
        for (int32_t t = cnt; t < k; ++t)
            row[t] = cnt > 0 ? row[0] : -1;
        if (out_cnt)
            out_cnt[q] = cnt;
    }
    return 0;
}

/* gather of sampled coordinates (input of the next stage of a hierarchy) */
int ref_gather_xyz(const float *xyz, int32_t N, const int32_t *idx, int32_t M, float *out_xyz)
{
    if (!xyz || !idx || !out_xyz)
        return -1;
    for (int32_t q = 0; q < M; ++q) {
        if (idx[q] < 0 || idx[q] >= N)
            return -1;
        memcpy(out_xyz + 3 * (size_t)q, xyz + 3 * (size_t)idx[q], 3 * sizeof(float));
    }
    return 0;
}

/* ------------------------------------------------------- exclusion lists -- */
/*
 * Exclusion lists -- the list-building loops of Algorithm 2 (Section 4.1 step 2), plus the extra
 * list at the ball-query radius of Section 4.2, as a data structure of its own:
 * for every level l and every point i the points j with dist2(P_i, P_j) < thr2[l],
 * in the order the paper's loop over j appends them (ascending j; i itself is a
 * member whenever thr2[l] > 0).  One distance per pair serves all levels.
 *   thr2    [L] squared radii, any order (the MDPS thresholds are non-increasing,
 *           the ball-query radius may lie anywhere among them)
 *   offsets [L*N + 1] row r = l*N + i occupies entries[offsets[r] .. offsets[r+1])
 *   entries NULL: only the offsets are produced (a caller sizes the array from
 *           offsets[L*N]); else it receives the members, `capacity` of them at most
 * Returns 0, -1 on bad arguments, -2 if `capacity` is too small.
 */
int ref_excl_lists(const float *xyz, int32_t N, const float *thr2, int32_t L,
                   int64_t *offsets, int32_t *entries, int64_t capacity)
{
    if (!xyz || !thr2 || !offsets || N < 1 || L < 1)
        return -1;
    const size_t rows = (size_t)L * (size_t)N;
    for (size_t r = 0; r <= rows; ++r)
        offsets[r] = 0;
    /* sizes first: offsets[r + 1] = members of row r */
    for (int32_t i = 0; i < N; ++i)
        for (int32_t j = 0; j < N; ++j) {
            float d = ref_dist2(xyz + 3 * (size_t)i, xyz + 3 * (size_t)j);
            for (int32_t l = 0; l < L; ++l)
                if (d < thr2[l])
                    ++offsets[(size_t)l * N + i + 1];
        }
    for (size_t r = 0; r < rows; ++r)
        offsets[r + 1] += offsets[r];
    if (!entries)
        return 0;
    if (offsets[rows] > capacity)
        return -2;
    for (int32_t i = 0; i < N; ++i) {
        for (int32_t j = 0; j < N; ++j) {
            float d = ref_dist2(xyz + 3 * (size_t)i, xyz + 3 * (size_t)j);
            for (int32_t l = 0; l < L; ++l)
                if (d < thr2[l]) {
                    /* append: the cursor of row r is kept in place of its start and put back below */
                    size_t r = (size_t)l * N + i;
                    entries[offsets[r]++] = j;
                }
        }
    }
    /* every row's cursor now sits at its end = the next row's start: shift back */
    for (size_t r = rows; r > 0; --r)
        offsets[r] = offsets[r - 1];
    offsets[0] = 0;
    return 0;
}

/*
 * Ball query by lookup in an exclusion list (Section 4.2: the neighbours of a
 * centre are its list at the query radius): the first k members of row
 * level*N + centre in list order, unused slots repeating the first member,
 * out_cnt = min(members, k).  An empty row gives -1 in every slot and count 0.
 */
int ref_ball_query_lists(const int64_t *offsets, const int32_t *entries, int32_t N, int32_t level,
                         const int32_t *center_idx, int32_t M, int32_t k, int32_t *out_idx,
                         int32_t *out_cnt)
{
    if (!offsets || !entries || !center_idx || !out_idx || N < 1 || level < 0 || M < 0 || k < 1)
        return -1;
    for (int32_t q = 0; q < M; ++q) {
        int32_t c = center_idx[q];
        if (c < 0 || c >= N)
            return -1;
        size_t r = (size_t)level * N + c;
        int64_t len = offsets[r + 1] - offsets[r];
        int32_t cnt = len < k ? (int32_t)len : k;
        for (int32_t t = 0; t < k; ++t)
            out_idx[(size_t)q * k + t] = cnt == 0 ? -1 : entries[offsets[r] + (t < cnt ? t : 0)];
        if (out_cnt)
            out_cnt[q] = cnt;
    }
    return 0;
}

/* ------------------------------------------------------ k nearest samples -- */
/*
 * k-NN of the up-sampling (feature propagation) step, Section 3.1: for every
 * point of the cloud its k nearest SAMPLED points.  Section 4.2 ("Redundancy-Free
 * k-NN") reaches the same result from a reduced search space, so the oracle is
 * the plain definition: all n squared binary32 distances of point j, then k
 * times the smallest one not taken yet.  The paper does not order equal
 * distances; here the sample with the lower position q comes first.
 *   sample_idx [n] indices into the cloud (the sampler's output), 1 <= k <= n
 *   point_idx  NULL: all N points, M = N.  Else [M] indices of the points wanted (lets a test
 *              check a sample of a large cloud)
 *   out_pos [M][k] positions q (into sample_idx), nearest first
 *   out_d2  [M][k] the squared distances, ascending
 */
int ref_knn(const float *xyz, int32_t N, const int32_t *sample_idx, int32_t n, int32_t k,
            const int32_t *point_idx, int32_t M, int32_t *out_pos, float *out_d2)
{
    if (!xyz || !sample_idx || !out_pos || !out_d2 || N < 1 || n < 1 || k < 1 || k > n)
        return -1;
    if (!point_idx)
        M = N;
    for (int32_t r = 0; point_idx && r < M; ++r)
        if (point_idx[r] < 0 || point_idx[r] >= N)
            return -1;
    for (int32_t q = 0; q < n; ++q)
        if (sample_idx[q] < 0 || sample_idx[q] >= N)
            return -1;
    float *d = (float *)malloc((size_t)n * sizeof(float));
    unsigned char *taken = (unsigned char *)malloc((size_t)n);
    if (!d || !taken) {
        free(d);
        free(taken);
        return -2;
    }
    for (int32_t r = 0; r < M; ++r) {
        int32_t j = point_idx ? point_idx[r] : r;
        for (int32_t q = 0; q < n; ++q) {
            d[q] = ref_dist2(xyz + 3 * (size_t)j, xyz + 3 * (size_t)sample_idx[q]);
            taken[q] = 0;
        }
        for (int32_t t = 0; t < k; ++t) {
            int32_t best = -1;
            for (int32_t q = 0; q < n; ++q)
                if (!taken[q] && (best < 0 || d[q] < d[best]))
                    best = q;
            taken[best] = 1;
            out_pos[(size_t)r * k + t] = best;
            out_d2[(size_t)r * k + t] = d[best];
        }
    }
    free(d);
    free(taken);
    return 0;
}

/* --------------------------------------------------------- quality metrics -- */
/* binary64 Euclidean distance from the binary32 inputs */
static double ref_dist_f64(const float *a, const float *b)
{
    double dx = (double)a[0] - (double)b[0];
    double dy = (double)a[1] - (double)b[1];
    double dz = (double)a[2] - (double)b[2];
    return sqrt(dx * dx + dy * dy + dz * dz);
}

/* coverage radius: max over points of the distance to the nearest sample */
double ref_coverage_radius(const float *xyz, int32_t N, const int32_t *idx, int32_t n)
{
    double worst = 0.0;
    for (int32_t j = 0; j < N; ++j) {
        double best = INFINITY;
        for (int32_t s = 0; s < n; ++s) {
            double d = ref_dist_f64(xyz + 3 * (size_t)j, xyz + 3 * (size_t)idx[s]);
            if (d < best)
                best = d;
        }
        if (best > worst)
            worst = best;
    }
    return worst;
}

/* the paper's sampling-quality metric (Section 5.2, Table 1): mean over samples
 * of the distance to the nearest other sample */
double ref_mean_spacing(const float *xyz, const int32_t *idx, int32_t n)
{
    if (n < 2)
        return 0.0;
    double sum = 0.0;
    for (int32_t s = 0; s < n; ++s) {
        double best = INFINITY;
        for (int32_t t = 0; t < n; ++t) {
            if (t == s)
                continue;
            double d = ref_dist_f64(xyz + 3 * (size_t)idx[s], xyz + 3 * (size_t)idx[t]);
            if (d < best)
                best = d;
        }
        sum += best;
    }
    return sum / (double)n;
}
