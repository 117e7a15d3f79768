/*
 * tern_oracle.c -- plain scalar CPU oracle for the ternary 3D convolution of TernaryNet.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU library can be checked
 * element by element against something a reader can verify against the paper by eye.  Only the
 * test-suite, the smoke check and the benchmark's cpu_baseline leg may call it; the GPU library
 * never does, and the two share no code.
 *
 * What it computes (paper, section 2, "Ternary convolutions and complexity analysis"): the paper
 * replaces the inner product of a ternary input patch I and a ternary filter W, both in
 * {-1,0,+1}^c with c = kernel volume x input channels, by boolean operations and two bit counts
 * (Eq. 9).  That bitwise form *is* the ordinary inner product, so the oracle is the ordinary inner
 * product written out: a direct cross-correlation on unpacked int8 values with int32 accumulation,
 * no bit tricks, no blocking, no reordering.  Everything here is integer (or a float comparison),
 * so results are exact and independent of summation order.
 *
 * Readings of the paper taken here (each is also listed in the design document):
 *   - cross-correlation, no kernel flip (the paper's implementation is a deep-learning framework
 *     whose conv layers correlate);
 *   - out-of-volume taps contribute 0 (zero padding = the ternary value 0, which Eq. 9's mask
 *     excludes like any other zero);
 *   - the hard activation tern(x) of Eq. 6 (+1 if x > 0.5, 0 if |x| <= 0.5, -1 else) with the
 *     per-channel scale alpha (below Eq. 4) and batch-norm (section 2, last paragraph) folded
 *     into two integer cut points per channel: code = +1 if acc > hi, -1 if acc < lo, else 0,
 *     strict comparisons, inclusive zero band, lo <= hi + 1 (lo = hi + 1: empty zero band);
 *   - the 2-bit storage of Fig. 3 as two bit-planes packed along channels: bit j of word q of a
 *     voxel's mask plane is 1 iff channel 32q+j is nonzero; the same bit of the sign plane is 1
 *     iff that channel is -1 (and 0 when the value is 0).  The figure's caption draws the first
 *     bit set for +1 and the second bit as a zero flag; this is the complement convention and
 *     does not change any result.
 *
 * Pins: tests/test_oracle_pins.py (brute force, closed forms, library cross-checks, invariants).
 * Nothing in this file is "parity unpinned".
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o liboracle.so tern_oracle.c   (see oracle/build.py)
 * Threads are used only to split the outer (n, c_out, z) loops; each output is still one scalar
 * sum.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EARG -1   /* null pointer, non-positive extent, lo > hi */
#define ORACLE_EVALUE -2 /* value outside {-1,0,+1} or an invalid 2-bit code point */

typedef struct {
    int n, c_in, d, h, w;         /* input  [n][c_in][d][h][w]                  */
    int c_out, kd, kh, kw;        /* filter [c_out][c_in][kd][kh][kw]           */
    int sd, sh, sw;               /* stride                                     */
    int pd, ph, pw;               /* zero padding on both sides                 */
    int dd, dh, dw;               /* dilation                                   */
} oracle_geom;

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* Output extent of one axis: floor((x + 2p - dil*(k-1) - 1)/s) + 1, or 0 if the dilated kernel
 * does not fit. */
static int out_extent(int x, int k, int s, int p, int dil)
{
    int span = x + 2 * p - dil * (k - 1) - 1;
    if (span < 0) return 0;
    return span / s + 1;
}

int oracle_out_dims(const oracle_geom* g, int* od, int* oh, int* ow)
{
    if (!g || !od || !oh || !ow) return ORACLE_EARG;
    if (g->n <= 0 || g->c_in <= 0 || g->d <= 0 || g->h <= 0 || g->w <= 0) return ORACLE_EARG;
    if (g->c_out <= 0 || g->kd <= 0 || g->kh <= 0 || g->kw <= 0) return ORACLE_EARG;
    if (g->sd <= 0 || g->sh <= 0 || g->sw <= 0) return ORACLE_EARG;
    if (g->dd <= 0 || g->dh <= 0 || g->dw <= 0) return ORACLE_EARG;
    if (g->pd < 0 || g->ph < 0 || g->pw < 0) return ORACLE_EARG;
    *od = out_extent(g->d, g->kd, g->sd, g->pd, g->dd);
    *oh = out_extent(g->h, g->kh, g->sh, g->ph, g->dh);
    *ow = out_extent(g->w, g->kw, g->sw, g->pw, g->dw);
    if (*od <= 0 || *oh <= 0 || *ow <= 0) return ORACLE_EARG;
    return ORACLE_OK;
}

/* The inner product of the paper's section 2 for one output element: sum over input channels and
 * kernel taps of weight x activation, activations outside the volume counting as 0. */
static int32_t conv_at(const oracle_geom* g, const int8_t* act, const int8_t* wgt,
                       int n, int co, int z, int y, int x)
{
    int32_t acc = 0;
    for (int ci = 0; ci < g->c_in; ++ci)
        for (int a = 0; a < g->kd; ++a)
            for (int b = 0; b < g->kh; ++b)
                for (int c = 0; c < g->kw; ++c) {
                    int iz = z * g->sd - g->pd + a * g->dd;
                    int iy = y * g->sh - g->ph + b * g->dh;
                    int ix = x * g->sw - g->pw + c * g->dw;
                    if (iz < 0 || iz >= g->d || iy < 0 || iy >= g->h || ix < 0 || ix >= g->w)
                        continue;
                    size_t ai = ((((size_t)n * g->c_in + ci) * g->d + iz) * g->h + iy) * g->w + ix;
                    size_t wi = ((((size_t)co * g->c_in + ci) * g->kd + a) * g->kh + b) * g->kw + c;
                    acc += (int32_t)wgt[wi] * (int32_t)act[ai];
                }
    return acc;
}

/* acc[n][c_out][od][oh][ow] = ternary cross-correlation of act with wgt. */
int oracle_conv3d(const oracle_geom* g, const int8_t* act, const int8_t* wgt, int32_t* acc)
{
    int od, oh, ow;
    if (!act || !wgt || !acc) return ORACLE_EARG;
    int rc = oracle_out_dims(g, &od, &oh, &ow);
    if (rc) return rc;
#pragma omp parallel for collapse(3) schedule(static)
    for (int n = 0; n < g->n; ++n)
        for (int co = 0; co < g->c_out; ++co)
            for (int z = 0; z < od; ++z)
                for (int y = 0; y < oh; ++y)
                    for (int x = 0; x < ow; ++x) {
                        size_t oi = ((((size_t)n * g->c_out + co) * od + z) * oh + y) * ow + x;
                        acc[oi] = conv_at(g, act, wgt, n, co, z, y, x);
                    }
    return ORACLE_OK;
}

/* The same sum at a list of output coordinates pts[i] = (n, co, z, y, x); used to spot-check
 * volumes too large to compute whole. */
int oracle_conv3d_points(const oracle_geom* g, const int8_t* act, const int8_t* wgt,
                         const int32_t* pts, int64_t n_pts, int32_t* acc)
{
    int od, oh, ow;
    if (!act || !wgt || !acc || !pts || n_pts < 0) return ORACLE_EARG;
    int rc = oracle_out_dims(g, &od, &oh, &ow);
    if (rc) return rc;
    for (int64_t i = 0; i < n_pts; ++i) {
        const int32_t* p = pts + 5 * i;
        if (p[0] < 0 || p[0] >= g->n || p[1] < 0 || p[1] >= g->c_out || p[2] < 0 || p[2] >= od ||
            p[3] < 0 || p[3] >= oh || p[4] < 0 || p[4] >= ow)
            return ORACLE_EARG;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_pts; ++i) {
        const int32_t* p = pts + 5 * i;
        acc[i] = conv_at(g, act, wgt, p[0], p[1], p[2], p[3], p[4]);
    }
    return ORACLE_OK;
}

/* Eq. 6 with scale and batch-norm folded into integer cut points:
 * code = +1 if v > hi[c]; -1 if v < lo[c]; else 0.   v is [n][c][d][h][w], spatial = d*h*w. */
int oracle_threshold_i32(const int32_t* v, int n, int c, int64_t spatial,
                         const int32_t* lo, const int32_t* hi, int8_t* code)
{
    if (!v || !lo || !hi || !code || n <= 0 || c <= 0 || spatial <= 0) return ORACLE_EARG;
    /* lo = hi + 1 is allowed: when the scale folded into the cut points exceeds 1, the zero band
     * |y| <= 0.5 of Eq. 6 may contain no integer, and the -1 and +1 ranges are then adjacent.
     * Beyond that the two ranges would overlap, which Eq. 6 cannot produce. */
    for (int ch = 0; ch < c; ++ch)
        if ((int64_t)lo[ch] > (int64_t)hi[ch] + 1) return ORACLE_EARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int ch = 0; ch < c; ++ch)
            for (int64_t i = 0; i < spatial; ++i) {
                size_t k = ((size_t)b * c + ch) * spatial + i;
                code[k] = (int8_t)(v[k] > hi[ch] ? 1 : (v[k] < lo[ch] ? -1 : 0));
            }
    return ORACLE_OK;
}

/* Eq. 6 on raw float intensities (first layer): same rule with float cut points (the paper's own
 * are -0.5 and +0.5).  A NaN compares false both ways and becomes 0. */
int oracle_threshold_f32(const float* v, int n, int c, int64_t spatial,
                         const float* lo, const float* hi, int8_t* code)
{
    if (!v || !lo || !hi || !code || n <= 0 || c <= 0 || spatial <= 0) return ORACLE_EARG;
    for (int ch = 0; ch < c; ++ch)
        if (!(lo[ch] <= hi[ch])) return ORACLE_EARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < n; ++b)
        for (int ch = 0; ch < c; ++ch)
            for (int64_t i = 0; i < spatial; ++i) {
                size_t k = ((size_t)b * c + ch) * spatial + i;
                code[k] = (int8_t)(v[k] > hi[ch] ? 1 : (v[k] < lo[ch] ? -1 : 0));
            }
    return ORACLE_OK;
}

/* 2-bit storage (Fig. 3): x is [n][c][spatial] int8 in {-1,0,+1}; packed is
 * [n][spatial][2][ceil(c/32)] uint32, plane 0 = nonzero mask, plane 1 = sign (1 = negative).
 * Bits of channels >= c are 0.  Any other input value is an error. */
int oracle_pack(const int8_t* x, int n, int c, int64_t spatial, uint32_t* packed)
{
    if (!x || !packed || n <= 0 || c <= 0 || spatial <= 0) return ORACLE_EARG;
    int words = (c + 31) / 32;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : bad)
    for (int b = 0; b < n; ++b)
        for (int64_t i = 0; i < spatial; ++i) {
            uint32_t* vox = packed + ((size_t)b * spatial + i) * 2 * words;
            for (int q = 0; q < 2 * words; ++q) vox[q] = 0;
            for (int ch = 0; ch < c; ++ch) {
                int8_t t = x[((size_t)b * c + ch) * spatial + i];
                if (t != 0 && t != 1 && t != -1) { bad = 1; continue; }
                if (t != 0) vox[ch / 32] |= (uint32_t)1 << (ch % 32);
                if (t < 0) vox[words + ch / 32] |= (uint32_t)1 << (ch % 32);
            }
        }
    return bad ? ORACLE_EVALUE : ORACLE_OK;
}

/* Inverse of oracle_pack.  A set sign bit under a clear mask bit (the unused fourth code point of
 * Fig. 3) or a set bit for a channel >= c is an error. */
int oracle_unpack(const uint32_t* packed, int n, int c, int64_t spatial, int8_t* x)
{
    if (!x || !packed || n <= 0 || c <= 0 || spatial <= 0) return ORACLE_EARG;
    int words = (c + 31) / 32;
    int bad = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : bad)
    for (int b = 0; b < n; ++b)
        for (int64_t i = 0; i < spatial; ++i) {
            const uint32_t* vox = packed + ((size_t)b * spatial + i) * 2 * words;
            for (int bit = 0; bit < 32 * words; ++bit) {
                int m = (vox[bit / 32] >> (bit % 32)) & 1;
                int s = (vox[words + bit / 32] >> (bit % 32)) & 1;
                if (bit >= c) { if (m || s) bad = 1; continue; }
                if (s && !m) bad = 1;
                x[((size_t)b * c + bit) * spatial + i] = (int8_t)(m ? (s ? -1 : 1) : 0);
            }
        }
    return bad ? ORACLE_EVALUE : ORACLE_OK;
}
