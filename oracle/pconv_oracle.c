/*
 * CPU oracle for PCONV sparse 3x3 convolution.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definitions that the HIP library is checked
 * against.  Nothing in the product path may call into this file; it shares no
 * code with the GPU implementation.
 *
 * What it computes (paper, "Theory of Sparse Convolution Patterns"):
 *   - pattern pruning: every 3x3 kernel is multiplied element-wise by a binary
 *     mask P (the kernel's Sparse Convolution Pattern);
 *   - connectivity pruning: whole kernels, i.e. (filter f, channel c) pairs, are
 *     removed;
 *   - the layer output is the ordinary DNN convolution, Eq. (1) of "The
 *     Convolution Operator" (un-flipped form g(x,y) = sum f(x+k, y+l) h(k,l)),
 *     over the masked weights.
 * Because the method only skips structural zeros, the oracle is that definition
 * written out: masked weights, then seven plain loops, accumulated in fp64.
 *
 * The reference packer implements the canonical filter-kernel-reorder layout
 * ("Filter kernel reorder" paragraph of the compiler section): filters ordered
 * so that similar filters are adjacent, kernels inside a filter grouped by
 * pattern.  The paper leaves the similarity metric open; the ordering keys used
 * here are stated next to the code.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * (brute force in exact rational arithmetic, impulse-response closed form,
 * reduction to a library dense convolution, linearity / zeroed-kernel
 * invariants, pack/unpack round trip).  The paper prints no numeric activation
 * values, so no absolute paper output is pinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_NCHW = 0, ORC_NHWC = 1 };

/* ---- bf16 rounding (round to nearest, ties to even) ---------------------- */

static uint32_t bits_of(float v) { uint32_t u; memcpy(&u, &v, 4); return u; }
static float float_of(uint32_t u) { float v; memcpy(&v, &u, 4); return v; }

uint16_t orc_bf16_bits(float v)
{
    uint32_t u = bits_of(v);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0)
        return (uint16_t)((u >> 16) | 0x0040u);          /* NaN stays NaN */
    uint32_t keep = u >> 16;                             /* truncated result   */
    uint32_t rest = u & 0xFFFFu;                         /* discarded 16 bits  */
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))
        keep += 1;                                       /* may carry into exponent: correct */
    return (uint16_t)keep;
}

float orc_bf16_value(float v) { return float_of((uint32_t)orc_bf16_bits(v) << 16); }

/* ---- masked weights: W~ = W (.) P (.) conn ------------------------------- */

/* wt[f][c][r][s] (double).  pattern ids on removed kernels are don't-care. */
void orc_masked_weights(const float *w, const uint8_t *pattern_id, const uint8_t *conn,
                        const uint16_t *table, int c_out, int c_in, int wdtype, double *wt)
{
    for (int f = 0; f < c_out; ++f)
        for (int c = 0; c < c_in; ++c) {
            size_t k = (size_t)f * c_in + c;
            unsigned mask = conn[k] ? table[pattern_id[k]] : 0u;
            for (int t = 0; t < 9; ++t) {
                float v = w[k * 9 + t];
                if (wdtype == ORC_BF16) v = orc_bf16_value(v);
                wt[k * 9 + t] = ((mask >> t) & 1u) ? (double)v : 0.0;
            }
        }
}

static size_t act_index(int layout, int n, int c, int y, int x, int C, int H, int W)
{
    if (layout == ORC_NCHW) return (((size_t)n * C + c) * H + y) * W + x;
    return (((size_t)n * H + y) * W + x) * C + c;
}

/* ---- Eq. (1) on chosen output points: the literal seven loops ------------ */

/* pts[i] = (n, f, y, x).  y_out[i] = act(b[f] + sum_c sum_r sum_s W~ * Xpad),
 * s_out[i] = |b[f]| + sum |W~ * Xpad|  (the per-output tolerance scale).      */
void orc_conv2d_points(const float *x, int layout, int n_img, int c_in, int h, int w,
                       const double *wt, int c_out, const float *bias,
                       int stride, int pad, int relu,
                       const int32_t *pts, int64_t npts, double *y_out, double *s_out)
{
    (void)n_img; (void)c_out;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; ++i) {
        int n = pts[4 * i], f = pts[4 * i + 1], oy = pts[4 * i + 2], ox = pts[4 * i + 3];
        double acc = bias ? (double)bias[f] : 0.0;
        double sab = fabs(acc);
        for (int c = 0; c < c_in; ++c)
            for (int r = 0; r < 3; ++r)
                for (int s = 0; s < 3; ++s) {
                    int iy = oy * stride + r - pad, ix = ox * stride + s - pad;
                    if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;   /* zero padding */
                    double p = wt[((size_t)f * c_in + c) * 9 + 3 * r + s] *
                               (double)x[act_index(layout, n, c, iy, ix, c_in, h, w)];
                    acc += p;
                    sab += fabs(p);
                }
        y_out[i] = (relu && acc < 0.0) ? 0.0 : acc;
        s_out[i] = sab;
    }
}

/* ---- Eq. (1) on the whole output ----------------------------------------- */

/* Same sums in the same (c, r, s) order as orc_conv2d_points, with the output
 * plane of one (n, f) as the innermost data so that the host compiler can
 * vectorise.  y_out / s_out use the same layout as x, with c_out channels.    */
void orc_conv2d(const float *x, int layout, int n_img, int c_in, int h, int w,
                const double *wt, int c_out, const float *bias,
                int stride, int pad, int relu, double *y_out, double *s_out)
{
    const int ho = (h + 2 * pad - 3) / stride + 1, wo = (w + 2 * pad - 3) / stride + 1;
    #pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < n_img; ++n)
        for (int f = 0; f < c_out; ++f) {
            double *acc = (double *)malloc(sizeof(double) * (size_t)ho * wo);
            double *sab = (double *)malloc(sizeof(double) * (size_t)ho * wo);
            double *row = (double *)malloc(sizeof(double) * (size_t)w);
            double b = bias ? (double)bias[f] : 0.0;
            for (int i = 0; i < ho * wo; ++i) { acc[i] = b; sab[i] = fabs(b); }
            for (int c = 0; c < c_in; ++c)
                for (int r = 0; r < 3; ++r)
                    for (int s = 0; s < 3; ++s) {
                        double wv = wt[((size_t)f * c_in + c) * 9 + 3 * r + s];
                        for (int oy = 0; oy < ho; ++oy) {
                            int iy = oy * stride + r - pad;
                            if (iy < 0 || iy >= h) continue;
                            for (int ix = 0; ix < w; ++ix)
                                row[ix] = (double)x[act_index(layout, n, c, iy, ix, c_in, h, w)];
                            for (int ox = 0; ox < wo; ++ox) {
                                int ix = ox * stride + s - pad;
                                if (ix < 0 || ix >= w) continue;
                                double p = wv * row[ix];
                                acc[oy * wo + ox] += p;
                                sab[oy * wo + ox] += fabs(p);
                            }
                        }
                    }
            for (int oy = 0; oy < ho; ++oy)
                for (int ox = 0; ox < wo; ++ox) {
                    double v = acc[oy * wo + ox];
                    size_t o = act_index(layout, n, f, oy, ox, c_out, ho, wo);
                    y_out[o] = (relu && v < 0.0) ? 0.0 : v;
                    s_out[o] = sab[oy * wo + ox];
                }
            free(acc); free(sab); free(row);
        }
}

/* ---- 2x2 / stride-2 max-pool (between VGG blocks) ------------------------ */

void orc_maxpool2x2(const float *x, int layout, int n_img, int c, int h, int w, float *y)
{
    const int ho = h / 2, wo = w / 2;
    for (int n = 0; n < n_img; ++n)
        for (int ch = 0; ch < c; ++ch)
            for (int oy = 0; oy < ho; ++oy)
                for (int ox = 0; ox < wo; ++ox) {
                    float m = x[act_index(layout, n, ch, 2 * oy, 2 * ox, c, h, w)];
                    for (int dy = 0; dy < 2; ++dy)
                        for (int dx = 0; dx < 2; ++dx) {
                            float v = x[act_index(layout, n, ch, 2 * oy + dy, 2 * ox + dx, c, h, w)];
                            if (v > m) m = v;
                        }
                    y[act_index(layout, n, ch, oy, ox, c, ho, wo)] = m;
                }
}

/* ---- reference packer: canonical filter-kernel-reorder layout ------------ */
/*
 * Logical layout (a deterministic function of the inputs):
 *   kcnt[f]      kept kernels of filter f;  hist[f][p] how many use pattern p
 *   perm[]       filters sorted by (kcnt desc, hist[f][0] desc, ..., hist[f][P-1] desc,
 *                f asc): filters with similar kernels end up adjacent
 *   row_ptr[i]   first kernel of the filter at position i of perm; row_ptr[F] = K
 *   pat_cnt[i][p] = hist[perm[i]][p]
 *   inside a filter kernels are ordered by (pattern id asc, input channel asc)
 *   cin[k]       input channel of kernel k
 *   vals         for each kernel, in order, the weights under the mask's set bits in
 *                ascending bit order (3r+s); fp32 bit copies, or bf16 RNE bit patterns
 * Removed kernels and masked-out taps are not stored.
 */
typedef struct { int f; int kcnt; const int *hist; int np; } orc_key;

static int key_cmp(const void *pa, const void *pb)
{
    const orc_key *a = (const orc_key *)pa, *b = (const orc_key *)pb;
    if (a->kcnt != b->kcnt) return a->kcnt > b->kcnt ? -1 : 1;
    for (int p = 0; p < a->np; ++p)
        if (a->hist[p] != b->hist[p]) return a->hist[p] > b->hist[p] ? -1 : 1;
    return a->f < b->f ? -1 : (a->f > b->f ? 1 : 0);
}

/* number of kept kernels (K) and stored weights (nnz) */
void orc_pack_sizes(const uint8_t *pattern_id, const uint8_t *conn, const uint16_t *table,
                    int c_out, int c_in, int64_t *k_out, int64_t *nnz_out)
{
    int64_t k = 0, nnz = 0;
    for (size_t i = 0; i < (size_t)c_out * c_in; ++i)
        if (conn[i]) { k += 1; nnz += __builtin_popcount(table[pattern_id[i]]); }
    *k_out = k; *nnz_out = nnz;
}

/* vals: float[nnz] when wdtype == ORC_F32, uint16_t[nnz] when ORC_BF16 */
void orc_pack(const float *w, const uint8_t *pattern_id, const uint8_t *conn,
              const uint16_t *table, int np, int c_out, int c_in, int wdtype,
              uint16_t *perm, uint32_t *row_ptr, uint16_t *pat_cnt, uint16_t *cin, void *vals)
{
    int *hist = (int *)calloc((size_t)c_out * np, sizeof(int));
    orc_key *keys = (orc_key *)malloc(sizeof(orc_key) * (size_t)c_out);
    for (int f = 0; f < c_out; ++f) {
        int cnt = 0;
        for (int c = 0; c < c_in; ++c)
            if (conn[(size_t)f * c_in + c]) { cnt++; hist[(size_t)f * np + pattern_id[(size_t)f * c_in + c]]++; }
        keys[f].f = f; keys[f].kcnt = cnt; keys[f].hist = hist + (size_t)f * np; keys[f].np = np;
    }
    qsort(keys, (size_t)c_out, sizeof(orc_key), key_cmp);
    uint32_t k = 0; size_t v = 0;
    for (int i = 0; i < c_out; ++i) {
        int f = keys[i].f;
        perm[i] = (uint16_t)f;
        row_ptr[i] = k;
        for (int p = 0; p < np; ++p) {
            pat_cnt[(size_t)i * np + p] = (uint16_t)keys[i].hist[p];
            for (int c = 0; c < c_in; ++c) {
                size_t e = (size_t)f * c_in + c;
                if (!conn[e] || pattern_id[e] != p) continue;
                cin[k++] = (uint16_t)c;
                for (int t = 0; t < 9; ++t)
                    if ((table[p] >> t) & 1u) {
                        float val = w[e * 9 + t];
                        if (wdtype == ORC_BF16) ((uint16_t *)vals)[v++] = orc_bf16_bits(val);
                        else                    ((float *)vals)[v++] = val;   /* bit copy */
                    }
            }
        }
    }
    row_ptr[c_out] = k;
    free(keys); free(hist);
}

/* inverse: dense masked weights (fp32; bf16 values widened exactly), zeros elsewhere */
void orc_unpack(const uint16_t *perm, const uint32_t *row_ptr, const uint16_t *pat_cnt,
                const uint16_t *cin, const void *vals, const uint16_t *table, int np,
                int c_out, int c_in, int wdtype, float *w_out)
{
    memset(w_out, 0, sizeof(float) * (size_t)c_out * c_in * 9);
    size_t v = 0;
    for (int i = 0; i < c_out; ++i) {
        int f = perm[i];
        uint32_t k = row_ptr[i];
        for (int p = 0; p < np; ++p)
            for (int j = 0; j < pat_cnt[(size_t)i * np + p]; ++j, ++k) {
                size_t e = (size_t)f * c_in + cin[k];
                for (int t = 0; t < 9; ++t)
                    if ((table[p] >> t) & 1u) {
                        if (wdtype == ORC_BF16)
                            w_out[e * 9 + t] = float_of((uint32_t)((const uint16_t *)vals)[v++] << 16);
                        else
                            w_out[e * 9 + t] = ((const float *)vals)[v++];
                    }
            }
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    #pragma omp parallel
    {
        #pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
