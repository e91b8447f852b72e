/*
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU oracle for the incremental Tacotron-2-style decoder step of
 * "Efficient Incremental Text-to-Speech on GPUs" (Sec. 2.1.3, Eq. 2), applied
 * to one request at a time.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no code with the
 * HIP library and is deliberately slow and literal: scalar loops, double
 * accumulation, no blocking, no fusion, no BLAS.
 *
 * Pool semantics (Sec. 2.2.2): pooling and dynamic batching are a scheduling
 * device; Eq. 2 never mixes two requests, so the reference result of a pooled
 * run is each request decoded alone.  orc_pool_decode() does exactly that
 * (optionally one OpenMP thread per request; the arithmetic per request is
 * unchanged).
 *
 * Parity pins: every block below is pinned by tests against closed forms,
 * invariants and CPU library routines (LSTMCell, conv1d, softmax).  The full
 * multi-step trajectory has no printed value in the paper to compare with:
 * beyond a second, independently written composition of library routines it
 * is "parity unpinned".
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - LSTM gate rows are ordered i, f, g, o; one merged bias per LSTM.
 *   - The location convolution is a cross-correlation with zero "same"
 *     padding over channels (W_last, W_acc) (or W_acc alone if the model has
 *     one input channel); prenet, query, memory, location and v layers carry
 *     no bias; the mel and stop projections do.
 *   - All carried state starts at zero (Sec. 2.1.3 lists the state set).
 *   - Positions at or beyond the request's encoder length do not exist: they
 *     get no energy, no weight and contribute nothing to the convolution.
 *   - W_acc is updated after the attention and decoder LSTM of the same step
 *     (order of Eq. 2), so attention at step t sees the sum of weights of
 *     steps < t.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int n_mel, prenet_dim, enc_dim, att_rnn_dim, dec_rnn_dim, att_dim;
    int loc_filters, loc_kernel, loc_in_channels;
} orc_dims;

/* fp32 row-major [out, in]; the same arrays the HIP library is created from */
typedef struct {
    const float *prenet1, *prenet2;
    const float *att_w_ih, *att_w_hh, *att_b;
    const float *q_w, *mem_w, *loc_conv, *loc_w, *v;
    const float *dec_w_ih, *dec_w_hh, *dec_b;
    const float *mel_w, *mel_b, *stop_w, *stop_b;
} orc_weights;

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* fp32 -> nearest bfloat16, ties to even, returned as double */
static double bf16_rne(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t lsb = (u >> 16) & 1u;
    u = (u + 0x7FFFu + lsb) & 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Eq. 2, line 1, "Pre(M_last)": two bias-free linear layers, each followed
 * by ReLU; dropout off. */
void orc_prenet(const orc_dims *d, const float *W1, const float *W2,
                const double *m, double *p)
{
    double *hid = (double *)malloc(sizeof(double) * d->prenet_dim);
    for (int o = 0; o < d->prenet_dim; ++o) {
        double s = 0.0;
        for (int i = 0; i < d->n_mel; ++i) s += (double)W1[o * d->n_mel + i] * m[i];
        hid[o] = s > 0.0 ? s : 0.0;
    }
    for (int o = 0; o < d->prenet_dim; ++o) {
        double s = 0.0;
        for (int i = 0; i < d->prenet_dim; ++i) s += (double)W2[o * d->prenet_dim + i] * hid[i];
        p[o] = s > 0.0 ? s : 0.0;
    }
    free(hid);
}

/* One LSTM cell step (Eq. 2, lines 1 and 3): gates = W_ih x + W_hh h + b,
 * row blocks i, f, g, o; c <- sig(f) c + sig(i) tanh(g); h <- sig(o) tanh(c). */
void orc_lstm_cell(int in_dim, int hid, const float *W_ih, const float *W_hh,
                   const float *b, const double *x, double *h, double *c)
{
    double *g = (double *)malloc(sizeof(double) * 4 * hid);
    for (int r = 0; r < 4 * hid; ++r) {
        double s = (double)b[r];
        for (int k = 0; k < in_dim; ++k) s += (double)W_ih[(size_t)r * in_dim + k] * x[k];
        for (int k = 0; k < hid; ++k) s += (double)W_hh[(size_t)r * hid + k] * h[k];
        g[r] = s;
    }
    for (int u = 0; u < hid; ++u) {
        double gi = sigmoid(g[u]);
        double gf = sigmoid(g[hid + u]);
        double gg = tanh(g[2 * hid + u]);
        double go = sigmoid(g[3 * hid + u]);
        c[u] = gf * c[u] + gi * gg;
        h[u] = go * tanh(c[u]);
    }
    free(g);
}

/* Processed memory PM = F W_mem^T, computed once when a request joins the
 * pool.  With round_bf16 the stored value is narrowed to bfloat16 (the
 * bf16-memory mode of the library stores it that way). */
void orc_memory_projection(const orc_dims *d, const float *mem_w, const float *F,
                           int L, int round_bf16, double *PM)
{
    for (int j = 0; j < L; ++j)
        for (int a = 0; a < d->att_dim; ++a) {
            double s = 0.0;
            for (int k = 0; k < d->enc_dim; ++k)
                s += (double)mem_w[a * d->enc_dim + k] * (double)F[(size_t)j * d->enc_dim + k];
            PM[(size_t)j * d->att_dim + a] = round_bf16 ? bf16_rne(s) : s;
        }
}

/* Location features: loc[j][f] = sum_c sum_k K[f][c][k] u[c][j + k - pad],
 * pad = (ksz-1)/2, terms outside [0, L) are zero. */
void orc_location_features(int L, int n_filt, int n_ch, int ksz, const float *K,
                           const double *u /* [n_ch][L] */, double *loc /* [L][n_filt] */)
{
    int pad = (ksz - 1) / 2;
    for (int j = 0; j < L; ++j)
        for (int f = 0; f < n_filt; ++f) {
            double s = 0.0;
            for (int c = 0; c < n_ch; ++c)
                for (int k = 0; k < ksz; ++k) {
                    int jj = j + k - pad;
                    if (jj < 0 || jj >= L) continue;
                    s += (double)K[(f * n_ch + c) * ksz + k] * u[(size_t)c * L + jj];
                }
            loc[(size_t)j * n_filt + f] = s;
        }
}

/* Location-sensitive attention (Eq. 2, line 2):
 *   q = W_q h_att;  pl_j = W_loc loc_j;  e_j = v . tanh(q + pl_j + PM_j);
 *   w = softmax over the request's own L positions;  ctx = sum_j w_j F_j.
 * Outputs e[L], w[L], ctx[enc_dim]. */
void orc_lsa(const orc_dims *d, const orc_weights *W, int L, const float *F,
             const double *PM, const double *h_att, const double *w_last,
             const double *w_acc, double *e, double *w, double *ctx)
{
    int A = d->att_dim, NF = d->loc_filters, C = d->loc_in_channels;
    double *q = (double *)malloc(sizeof(double) * A);
    double *u = (double *)malloc(sizeof(double) * (size_t)C * L);
    double *loc = (double *)malloc(sizeof(double) * (size_t)L * NF);

    for (int a = 0; a < A; ++a) {
        double s = 0.0;
        for (int k = 0; k < d->att_rnn_dim; ++k) s += (double)W->q_w[a * d->att_rnn_dim + k] * h_att[k];
        q[a] = s;
    }
    if (C == 2) {
        memcpy(u, w_last, sizeof(double) * L);
        memcpy(u + L, w_acc, sizeof(double) * L);
    } else {
        memcpy(u, w_acc, sizeof(double) * L);
    }
    orc_location_features(L, NF, C, d->loc_kernel, W->loc_conv, u, loc);

    for (int j = 0; j < L; ++j) {
        double ej = 0.0;
        for (int a = 0; a < A; ++a) {
            double pl = 0.0;
            for (int f = 0; f < NF; ++f) pl += (double)W->loc_w[a * NF + f] * loc[(size_t)j * NF + f];
            ej += (double)W->v[a] * tanh(q[a] + pl + PM[(size_t)j * A + a]);
        }
        e[j] = ej;
    }
    double mx = e[0];
    for (int j = 1; j < L; ++j) if (e[j] > mx) mx = e[j];
    double den = 0.0;
    for (int j = 0; j < L; ++j) { w[j] = exp(e[j] - mx); den += w[j]; }
    for (int j = 0; j < L; ++j) w[j] /= den;

    for (int k = 0; k < d->enc_dim; ++k) {
        double s = 0.0;
        for (int j = 0; j < L; ++j) s += w[j] * (double)F[(size_t)j * d->enc_dim + k];
        ctx[k] = s;
    }
    free(q); free(u); free(loc);
}

/* Eq. 2, line 5, "Linear(H_dec, A)": mel and stop projections of [h_dec; ctx]. */
void orc_projection(const orc_dims *d, const orc_weights *W, const double *h_dec,
                    const double *ctx, double *mel, double *stop)
{
    int H = d->dec_rnn_dim, E = d->enc_dim, IN = H + E;
    for (int o = 0; o < d->n_mel; ++o) {
        double s = (double)W->mel_b[o];
        for (int k = 0; k < H; ++k) s += (double)W->mel_w[(size_t)o * IN + k] * h_dec[k];
        for (int k = 0; k < E; ++k) s += (double)W->mel_w[(size_t)o * IN + H + k] * ctx[k];
        mel[o] = s;
    }
    double s = (double)W->stop_b[0];
    for (int k = 0; k < H; ++k) s += (double)W->stop_w[k] * h_dec[k];
    for (int k = 0; k < E; ++k) s += (double)W->stop_w[H + k] * ctx[k];
    *stop = s;
}

/* ---- one request: the pool item of Sec. 2.2.2 restricted to module D ---- */

typedef struct orc_request {
    orc_dims d;
    orc_weights W;
    const float *F;     /* [L, enc_dim], borrowed */
    int L, n_steps, t, finished;
    double stop_threshold;           /* outside [0,1] = disabled */
    double *PM;                      /* [L, att_dim] */
    double *m, *a, *w_last, *w_acc;  /* M_last, A, W_last, W_acc */
    double *h_att, *c_att, *h_dec, *c_dec;
} orc_request;

static double *zeros(size_t n) { return (double *)calloc(n ? n : 1, sizeof(double)); }

orc_request *orc_request_new(const orc_dims *d, const orc_weights *W, const float *F,
                             int L, int n_steps, int pm_round_bf16, double stop_threshold)
{
    if (L < 1 || n_steps < 0) return NULL;
    orc_request *r = (orc_request *)calloc(1, sizeof(orc_request));
    r->d = *d; r->W = *W; r->F = F; r->L = L; r->n_steps = n_steps;
    r->stop_threshold = stop_threshold;
    r->finished = (n_steps == 0);
    r->PM = zeros((size_t)L * d->att_dim);
    orc_memory_projection(d, W->mem_w, F, L, pm_round_bf16, r->PM);
    r->m = zeros(d->n_mel); r->a = zeros(d->enc_dim);
    r->w_last = zeros(L); r->w_acc = zeros(L);
    r->h_att = zeros(d->att_rnn_dim); r->c_att = zeros(d->att_rnn_dim);
    r->h_dec = zeros(d->dec_rnn_dim); r->c_dec = zeros(d->dec_rnn_dim);
    return r;
}

void orc_request_free(orc_request *r)
{
    if (!r) return;
    free(r->PM); free(r->m); free(r->a); free(r->w_last); free(r->w_acc);
    free(r->h_att); free(r->c_att); free(r->h_dec); free(r->c_dec);
    free(r);
}

/* One frame (Eq. 2, top to bottom).  Returns 1 if a frame was produced,
 * 0 if the request had already finished. */
int orc_request_step(orc_request *r, double *mel_out, double *stop_out)
{
    if (r->finished) return 0;
    const orc_dims *d = &r->d;
    int att_in = d->prenet_dim + d->enc_dim, dec_in = d->att_rnn_dim + d->enc_dim;
    double *x = (double *)malloc(sizeof(double) * (att_in > dec_in ? att_in : dec_in));
    double *e = (double *)malloc(sizeof(double) * r->L);
    double *w = (double *)malloc(sizeof(double) * r->L);
    double stop;

    /* H_att, C_att = LSTM_att([Pre(M_last), A], H_att, C_att) */
    orc_prenet(d, r->W.prenet1, r->W.prenet2, r->m, x);
    memcpy(x + d->prenet_dim, r->a, sizeof(double) * d->enc_dim);
    orc_lstm_cell(att_in, d->att_rnn_dim, r->W.att_w_ih, r->W.att_w_hh, r->W.att_b, x, r->h_att, r->c_att);

    /* A, W_last = LSA(H_att, F_enc, W_acc) */
    orc_lsa(d, &r->W, r->L, r->F, r->PM, r->h_att, r->w_last, r->w_acc, e, w, r->a);

    /* H_dec, C_dec = LSTM_dec([H_att, A], H_dec, C_dec) */
    memcpy(x, r->h_att, sizeof(double) * d->att_rnn_dim);
    memcpy(x + d->att_rnn_dim, r->a, sizeof(double) * d->enc_dim);
    orc_lstm_cell(dec_in, d->dec_rnn_dim, r->W.dec_w_ih, r->W.dec_w_hh, r->W.dec_b, x, r->h_dec, r->c_dec);

    /* W_acc = W_acc + W_last */
    for (int j = 0; j < r->L; ++j) { r->w_last[j] = w[j]; r->w_acc[j] += w[j]; }

    /* M_last = Linear(H_dec, A) */
    orc_projection(d, &r->W, r->h_dec, r->a, r->m, &stop);

    if (mel_out) memcpy(mel_out, r->m, sizeof(double) * d->n_mel);
    if (stop_out) *stop_out = stop;
    r->t += 1;
    /* the stop token exceeding the threshold flags the end (Sec. 2.2.1);
     * the frame that trips it is kept */
    if (r->t >= r->n_steps) r->finished = 1;
    if (r->stop_threshold >= 0.0 && r->stop_threshold <= 1.0 && sigmoid(stop) > r->stop_threshold)
        r->finished = 1;
    free(x); free(e); free(w);
    return 1;
}

/* state access for tests: which = 0 m, 1 a, 2 w_last, 3 w_acc, 4 h_att,
 * 5 c_att, 6 h_dec, 7 c_dec, 8 PM.  Returns the element count. */
static double *state_ptr(orc_request *r, int which, int *n)
{
    const orc_dims *d = &r->d;
    switch (which) {
    case 0: *n = d->n_mel; return r->m;
    case 1: *n = d->enc_dim; return r->a;
    case 2: *n = r->L; return r->w_last;
    case 3: *n = r->L; return r->w_acc;
    case 4: *n = d->att_rnn_dim; return r->h_att;
    case 5: *n = d->att_rnn_dim; return r->c_att;
    case 6: *n = d->dec_rnn_dim; return r->h_dec;
    case 7: *n = d->dec_rnn_dim; return r->c_dec;
    case 8: *n = r->L * d->att_dim; return r->PM;
    default: *n = 0; return NULL;
    }
}

int orc_request_get(orc_request *r, int which, double *out)
{
    int n; double *p = state_ptr(r, which, &n);
    if (p && out) memcpy(out, p, sizeof(double) * n);
    return n;
}

int orc_request_set(orc_request *r, int which, const double *in)
{
    int n; double *p = state_ptr(r, which, &n);
    if (p && in) memcpy(p, in, sizeof(double) * n);
    return n;
}

int orc_request_frames(const orc_request *r) { return r->t; }
int orc_request_finished(const orc_request *r) { return r->finished; }

/* Decode every request alone for min(n_steps[i], window) frames.
 * mel_out is [n_req][window][n_mel], stop_out [n_req][window]; rows past a
 * request's last frame are left untouched.  frames_out[i] = frames written.
 * n_threads > 1 runs requests on separate OpenMP threads. */
int orc_pool_decode(const orc_dims *d, const orc_weights *W, int n_req,
                    const float *const *F, const int *L, const int *n_steps,
                    int window, int pm_round_bf16, double stop_threshold,
                    int n_threads, double *mel_out, double *stop_out, int *frames_out)
{
    int used = 1;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
    #pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
#endif
    for (int i = 0; i < n_req; ++i) {
        int n = n_steps[i] < window ? n_steps[i] : window;
        orc_request *r = orc_request_new(d, W, F[i], L[i], n, pm_round_bf16, stop_threshold);
        int t = 0;
        while (r && !r->finished) {
            orc_request_step(r, mel_out + ((size_t)i * window + t) * d->n_mel,
                             stop_out ? stop_out + (size_t)i * window + t : NULL);
            ++t;
        }
        if (frames_out) frames_out[i] = t;
        orc_request_free(r);
    }
#ifdef _OPENMP
    used = n_threads < n_req ? n_threads : n_req;
#endif
    return used;
}
