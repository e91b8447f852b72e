/*
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain CPU oracle for the PostNet of the acoustic decoder (Sec. 2.1.3 names
 * it; Sec. 3.1 says the decoder has the parameters of the original Tacotron 2)
 * and for its chunk-wise use in incremental synthesis (Sec. 2.2.1: the decoder
 * produces one chunk of mel frames at a time).  Scalar loops, double
 * accumulation.  Shares no code with the HIP library.
 *
 * Readings (the paper gives no detail of the PostNet):
 *   - five 1-D convolutions over time, kernel 5, zero "same" padding (2 on
 *     each side), channels n_mel -> C -> C -> C -> n_mel; tanh after every
 *     layer but the last; cross-correlation orientation x[t + k - 2];
 *   - batch normalisation at inference is a per-channel affine map: it is
 *     taken as folded into the convolution weights and one bias per output
 *     channel; dropout is off;
 *   - the result is added to the input: out = mel + stack(mel).
 *   - Chunk-wise: chunk [s, e) of a request is post-processed when its frames
 *     exist, as part of "the utterance so far": the whole stack applied to
 *     frames [0, e) (zero padding at both ends, at every layer), restricted
 *     to [s, e).  The last chunk therefore equals the non-incremental result;
 *     an earlier chunk differs from it only in its last 2 * n_layers frames,
 *     which see zeros where later frames will be.
 *
 * Pins (tests/test_postnet_oracle.py): torch.nn.functional.conv1d chains,
 * centre-tap identity kernels (closed form tanh chain), shifted delta
 * kernels (orientation, padding), receptive field (which input frames a
 * chunk depends on), last chunk = whole utterance.  No printed value exists
 * in the paper for this block: beyond those pins it is "parity unpinned".
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define ORC_PN_TAPS 5

/* One layer: y[t][co] = b[co] + sum_ci sum_k w[co][ci][k] x[t + k - 2][ci], x = 0 outside [0, T). */
void orc_conv5(int T, int c_in, int c_out, const float *w, const float *b,
               const double *x, int apply_tanh, double *y)
{
    for (int t = 0; t < T; ++t)
        for (int co = 0; co < c_out; ++co) {
            double s = (double)b[co];
            for (int ci = 0; ci < c_in; ++ci)
                for (int k = 0; k < ORC_PN_TAPS; ++k) {
                    int tt = t + k - ORC_PN_TAPS / 2;
                    if (tt < 0 || tt >= T) continue;
                    s += (double)w[((size_t)co * c_in + ci) * ORC_PN_TAPS + k] * x[(size_t)tt * c_in + ci];
                }
            y[(size_t)t * c_out + co] = apply_tanh ? tanh(s) : s;
        }
}

/* The whole stack on a sequence of T frames: out = mel + conv_n(tanh(... tanh(conv_1(mel)))).
 * w[l] is [c_out_l][c_in_l][5], b[l] is [c_out_l]; hidden width `channels`. */
void orc_postnet(int n_layers, int n_mel, int channels, const float *const *w, const float *const *b,
                 int T, const double *mel, double *out)
{
    size_t wide = (size_t)T * (channels > n_mel ? channels : n_mel);
    double *cur = (double *)malloc(sizeof(double) * (wide ? wide : 1));
    double *nxt = (double *)malloc(sizeof(double) * (wide ? wide : 1));
    memcpy(cur, mel, sizeof(double) * (size_t)T * n_mel);
    for (int l = 0; l < n_layers; ++l) {
        int c_in = l == 0 ? n_mel : channels;
        int c_out = l == n_layers - 1 ? n_mel : channels;
        orc_conv5(T, c_in, c_out, w[l], b[l], cur, l != n_layers - 1, nxt);
        double *t = cur; cur = nxt; nxt = t;
    }
    for (size_t i = 0; i < (size_t)T * n_mel; ++i) out[i] = mel[i] + cur[i];
    free(cur); free(nxt);
}

/* Chunk [s, e) of an utterance whose first e frames are `mel` ([e][n_mel]): the stack applied to
 * the utterance so far, restricted to the chunk.  out is [e - s][n_mel]. */
void orc_postnet_chunk(int n_layers, int n_mel, int channels, const float *const *w, const float *const *b,
                       int s, int e, const double *mel, double *out)
{
    double *all = (double *)malloc(sizeof(double) * (size_t)(e ? e : 1) * n_mel);
    orc_postnet(n_layers, n_mel, channels, w, b, e, mel, all);
    memcpy(out, all + (size_t)s * n_mel, sizeof(double) * (size_t)(e - s) * n_mel);
    free(all);
}
