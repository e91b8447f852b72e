/*
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU oracle for the acoustic encoder (Sec. 2.1.2, Eq. 1): the token
 * embedding and the three prosodic-structure embeddings are summed and passed
 * through the "CBRL" network -- three convolutions with batch normalisation
 * and ReLU, then a bidirectional LSTM -- to give F_enc.  It runs once per
 * request (Sec. 2.2.1).  Scalar loops, double accumulation.  Shares no code
 * with the HIP library; the LSTM cell is the one of tts_oracle.c.
 *
 * Readings (the paper says "based on the Tacotron 2 encoder" and no more):
 *   - embeddings of width 512; E_all[j] = E_token[tok_j] + E_pw[pw_j] +
 *     E_pph[pph_j] + E_iph[iph_j];
 *   - three 1-D convolutions over the token axis, kernel 5, zero "same"
 *     padding, 512 -> 512, cross-correlation orientation x[j + k - 2]; batch
 *     normalisation at inference is a per-channel affine map, taken as folded
 *     into the weights and one bias per channel; ReLU after each; dropout off;
 *   - one bidirectional LSTM layer, 256 units per direction, gate rows
 *     i, f, g, o, one merged bias per direction, zero initial state; the
 *     backward direction starts at the last token of the request's own length
 *     (no padding exists); F_enc[j] = [h_fwd[j], h_bwd[j]].
 *
 * Pins (tests/test_encoder_oracle.py): torch.nn.LSTM (bidirectional) and
 * torch.nn.functional.conv1d as library routines, the embedding sum by
 * indexing, zero-weight closed forms, the reversal symmetry of the two
 * directions.  No printed value exists in the paper for this block: beyond
 * those pins it is "parity unpinned".
 */
#include <stdlib.h>
#include <string.h>

void orc_lstm_cell(int in_dim, int hid, const float *W_ih, const float *W_hh,
                   const float *b, const double *x, double *h, double *c);

/* E[j][:] = sum over tables t of table_t[ids_t[j]][:] */
void orc_encoder_embed(int L, int dim, int n_tables, const float *const *tables,
                       const int *const *ids, double *E)
{
    for (int j = 0; j < L; ++j)
        for (int d = 0; d < dim; ++d) {
            double s = 0.0;
            for (int t = 0; t < n_tables; ++t) s += (double)tables[t][(size_t)ids[t][j] * dim + d];
            E[(size_t)j * dim + d] = s;
        }
}

/* y[j][co] = relu(b[co] + sum_ci sum_k w[co][ci][k] x[j + k - (ksz-1)/2][ci]), x = 0 outside [0, L) */
void orc_encoder_conv_relu(int L, int c_in, int c_out, int ksz, const float *w, const float *b,
                           const double *x, double *y)
{
    int half = (ksz - 1) / 2;
    for (int j = 0; j < L; ++j)
        for (int co = 0; co < c_out; ++co) {
            double s = (double)b[co];
            for (int ci = 0; ci < c_in; ++ci)
                for (int k = 0; k < ksz; ++k) {
                    int jj = j + k - half;
                    if (jj < 0 || jj >= L) continue;
                    s += (double)w[((size_t)co * c_in + ci) * ksz + k] * x[(size_t)jj * c_in + ci];
                }
            y[(size_t)j * c_out + co] = s > 0.0 ? s : 0.0;
        }
}

/* out[j] = [h_fwd[j], h_bwd[j]]: the forward direction reads x[0], x[1], ...; the backward one
 * x[L-1], x[L-2], ...; both from a zero state. */
void orc_bilstm(int L, int in_dim, int hid,
                const float *W_ih_f, const float *W_hh_f, const float *b_f,
                const float *W_ih_b, const float *W_hh_b, const float *b_b,
                const double *x, double *out)
{
    double *h = (double *)calloc((size_t)hid, sizeof(double));
    double *c = (double *)calloc((size_t)hid, sizeof(double));
    for (int j = 0; j < L; ++j) {
        orc_lstm_cell(in_dim, hid, W_ih_f, W_hh_f, b_f, x + (size_t)j * in_dim, h, c);
        memcpy(out + (size_t)j * 2 * hid, h, sizeof(double) * hid);
    }
    memset(h, 0, sizeof(double) * hid);
    memset(c, 0, sizeof(double) * hid);
    for (int j = L - 1; j >= 0; --j) {
        orc_lstm_cell(in_dim, hid, W_ih_b, W_hh_b, b_b, x + (size_t)j * in_dim, h, c);
        memcpy(out + (size_t)j * 2 * hid + hid, h, sizeof(double) * hid);
    }
    free(h); free(c);
}

/* Eq. 1: F_enc [L][2 hid] from the four id sequences. */
void orc_encoder(int L, int dim, int hid, int n_tables, const float *const *tables, const int *const *ids,
                 int n_conv, int ksz, const float *const *conv_w, const float *const *conv_b,
                 const float *W_ih_f, const float *W_hh_f, const float *b_f,
                 const float *W_ih_b, const float *W_hh_b, const float *b_b, double *F_enc)
{
    size_t n = (size_t)(L ? L : 1) * dim;
    double *a = (double *)malloc(sizeof(double) * n);
    double *t = (double *)malloc(sizeof(double) * n);
    orc_encoder_embed(L, dim, n_tables, tables, ids, a);
    for (int l = 0; l < n_conv; ++l) {
        orc_encoder_conv_relu(L, dim, dim, ksz, conv_w[l], conv_b[l], a, t);
        double *s = a; a = t; t = s;
    }
    orc_bilstm(L, dim, hid, W_ih_f, W_hh_f, b_f, W_ih_b, W_hh_b, b_b, a, F_enc);
    free(a); free(t);
}
