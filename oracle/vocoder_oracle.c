/*
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU oracle for the vocoder side of incremental synthesis (Sec. 2.1.4:
 * a HiFi-GAN-based generator G of transposed convolutions and multi-receptive
 * field fusion blocks; Eq. 3: the current mel chunk is preceded by frames from
 * the tail of the previous one, and the overlapping audio is fused with
 * equal-power fade coefficients; Eq. 4: the previous chunk's mel and audio are
 * replaced by the current ones; Sec. 3.1: 128 initial channels, upsampling
 * factors 8, 8, 2, 2).  Scalar loops, double accumulation.  Shares no code with
 * the HIP library.
 *
 * Readings (the paper fixes only the two figures above):
 *   - G = conv_pre (kernel 7, n_mel -> C0), then per stage i: leaky ReLU,
 *     transposed convolution (stride u_i, kernel 2 u_i, padding u_i / 2,
 *     C -> C / 2), then the mean of three residual blocks with kernels 3, 7, 11;
 *     finally leaky ReLU, conv_post (kernel 7, C -> 1), tanh.  Output length is
 *     exactly prod(u_i) = 256 samples per frame.
 *   - residual block with kernel k: for d in (1, 3, 5):
 *         x = x + conv_{k,1}(lrelu(conv_{k,d}(lrelu(x))))
 *     every convolution zero padded to keep the length ("same").
 *   - leaky ReLU slope 0.1 everywhere; weight normalisation folded into the
 *     weights; cross-correlation orientation x[t + (j - (k-1)/2) d].
 *   - transposed convolution by its definition: input sample t spreads to
 *     outputs t * stride + j - padding, j = 0 .. kernel - 1.
 *   - equal-power cross-fade over N overlapping samples:
 *         alpha_i = sin(pi/2 * (i + 1/2) / N),  beta_i = cos(pi/2 * (i + 1/2) / N)
 *     (fade-in for the current chunk's head, fade-out for the previous chunk's
 *     tail; alpha^2 + beta^2 = 1).  The sampling of the fade at the mid-points
 *     (i + 1/2) / N is a reading: the paper names the fade only.
 *
 * Pins (tests/test_vocoder_oracle.py): torch.nn.functional.conv1d /
 * conv_transpose1d (library routines) on random shapes with dilation, impulse
 * responses worked by hand, the generator recomposed from those library
 * routines, output length and shift behaviour, alpha^2 + beta^2 = 1 and the
 * fade's end values.  No printed value exists in the paper for this block:
 * beyond those pins it is "parity unpinned".
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define ORC_PI 3.14159265358979323846

/* y[t][co] = b[co] + sum_ci sum_j w[co][ci][j] x[t + (j - (k-1)/2) dil][ci], x = 0 outside [0, T) */
void orc_conv1d(int T, int c_in, int c_out, int k, int dil, const float *w, const float *b,
                const double *x, double *y)
{
    int half = (k - 1) / 2;
    for (int t = 0; t < T; ++t)
        for (int co = 0; co < c_out; ++co) {
            double s = (double)b[co];
            for (int ci = 0; ci < c_in; ++ci)
                for (int j = 0; j < k; ++j) {
                    int tt = t + (j - half) * dil;
                    if (tt < 0 || tt >= T) continue;
                    s += (double)w[((size_t)co * c_in + ci) * k + j] * x[(size_t)tt * c_in + ci];
                }
            y[(size_t)t * c_out + co] = s;
        }
}

/* Transposed convolution, w is [c_in][c_out][k]: x[t][ci] adds w[ci][co][j] x[t][ci] to
 * y[t * stride + j - pad][co]; y has T * stride rows (requires k - 2 pad = stride). */
void orc_conv_transpose1d(int T, int c_in, int c_out, int k, int stride, int pad, const float *w,
                          const float *b, const double *x, double *y)
{
    int To = T * stride;
    for (int o = 0; o < To; ++o)
        for (int co = 0; co < c_out; ++co) y[(size_t)o * c_out + co] = (double)b[co];
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int o = t * stride + j - pad;
            if (o < 0 || o >= To) continue;
            for (int ci = 0; ci < c_in; ++ci) {
                double xv = x[(size_t)t * c_in + ci];
                for (int co = 0; co < c_out; ++co)
                    y[(size_t)o * c_out + co] += (double)w[((size_t)ci * c_out + co) * k + j] * xv;
            }
        }
}

void orc_leaky_relu(size_t n, double slope, const double *x, double *y)
{
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > 0.0 ? x[i] : slope * x[i];
}

/* One residual block with kernel k: w[2 i], b[2 i] is the dilated convolution of pair i
 * (dilation dils[i]), w[2 i + 1], b[2 i + 1] the undilated one.  In place on x [T][c]. */
void orc_resblock(int T, int c, int k, int n_pairs, const int *dils, const float *const *w,
                  const float *const *b, double slope, double *x)
{
    size_t n = (size_t)T * c;
    double *a = (double *)malloc(sizeof(double) * (n ? n : 1));
    double *t = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (int i = 0; i < n_pairs; ++i) {
        orc_leaky_relu(n, slope, x, a);
        orc_conv1d(T, c, c, k, dils[i], w[2 * i], b[2 * i], a, t);
        orc_leaky_relu(n, slope, t, a);
        orc_conv1d(T, c, c, k, 1, w[2 * i + 1], b[2 * i + 1], a, t);
        for (size_t q = 0; q < n; ++q) x[q] += t[q];
    }
    free(a); free(t);
}

typedef struct {
    int n_mel, c0, n_stages, n_blocks, n_pairs, k_pre, k_post;
    const int *rates;      /* [n_stages] */
    const int *block_k;    /* [n_blocks] */
    const int *dils;       /* [n_pairs]  */
    double slope;
    const float *pre_w, *pre_b, *post_w, *post_b;
    const float *const *up_w, *const *up_b;      /* [n_stages] */
    const float *const *res_w, *const *res_b;    /* [n_stages][n_blocks][2 n_pairs], flattened */
} orc_generator_t;

/* audio [T * prod(rates)] = G(mel [T][n_mel]) */
void orc_generator(const orc_generator_t *g, int T, const double *mel, double *audio)
{
    int c = g->c0, len = T;
    double *x = (double *)malloc(sizeof(double) * (size_t)(T ? T : 1) * c);
    orc_conv1d(T, g->n_mel, c, g->k_pre, 1, g->pre_w, g->pre_b, mel, x);
    for (int s = 0; s < g->n_stages; ++s) {
        int u = g->rates[s], co = c / 2, lo = len * u;
        size_t n_in = (size_t)len * c, n_out = (size_t)lo * co;
        double *a = (double *)malloc(sizeof(double) * (n_in ? n_in : 1));
        double *y = (double *)malloc(sizeof(double) * (n_out ? n_out : 1));
        double *acc = (double *)calloc(n_out ? n_out : 1, sizeof(double));
        double *r = (double *)malloc(sizeof(double) * (n_out ? n_out : 1));
        orc_leaky_relu(n_in, g->slope, x, a);
        orc_conv_transpose1d(len, c, co, 2 * u, u, u / 2, g->up_w[s], g->up_b[s], a, y);
        for (int bk = 0; bk < g->n_blocks; ++bk) {
            size_t base = ((size_t)s * g->n_blocks + bk) * 2 * g->n_pairs;
            memcpy(r, y, sizeof(double) * n_out);
            orc_resblock(lo, co, g->block_k[bk], g->n_pairs, g->dils, g->res_w + base, g->res_b + base, g->slope, r);
            for (size_t q = 0; q < n_out; ++q) acc[q] += r[q];
        }
        for (size_t q = 0; q < n_out; ++q) acc[q] /= (double)g->n_blocks;
        free(x); free(a); free(y); free(r);
        x = acc; c = co; len = lo;
    }
    {
        size_t n = (size_t)len * c;
        double *a = (double *)malloc(sizeof(double) * (n ? n : 1));
        orc_leaky_relu(n, g->slope, x, a);
        orc_conv1d(len, c, 1, g->k_post, 1, g->post_w, g->post_b, a, audio);
        for (int t = 0; t < len; ++t) audio[t] = tanh(audio[t]);
        free(a);
    }
    free(x);
}

/* Equal-power fade coefficients over n samples. */
void orc_fade(int n, double *alpha, double *beta)
{
    for (int i = 0; i < n; ++i) {
        double u = ((double)i + 0.5) / (double)n;
        alpha[i] = sin(0.5 * ORC_PI * u);
        beta[i] = cos(0.5 * ORC_PI * u);
    }
}

/* Eq. 3, second line: fused[i] = alpha_i head_cur[i] + beta_i tail_pre[i] */
void orc_crossfade(int n, const double *head_cur, const double *tail_pre, double *fused)
{
    double *al = (double *)malloc(sizeof(double) * (n ? n : 1));
    double *be = (double *)malloc(sizeof(double) * (n ? n : 1));
    orc_fade(n, al, be);
    for (int i = 0; i < n; ++i) fused[i] = al[i] * head_cur[i] + be[i] * tail_pre[i];
    free(al); free(be);
}
