/*
 * tts_encoder.h -- C ABI of the acoustic encoder (paper Sec. 2.1.2, Eq. 1:
 * E_all = E_token + E_pw + E_pph + E_iph, F_enc = CBRL(E_all), where CBRL is
 * three convolutions with batch normalisation and ReLU followed by a
 * bidirectional LSTM; Sec. 2.2.1: the encoder is not incremental and runs
 * once per request; Sec. 2.2.2: it runs on the dynamic batch of the requests
 * that joined in this iteration, and its output F_enc is part of the pool
 * item).
 *
 * The paper says "based on the Tacotron 2 encoder" and no more.  This library
 * takes it as: four embedding tables of width 512; three 1-D convolutions over
 * the token axis, kernel 5, zero "same" padding inside each request, 512 -> 512,
 * batch normalisation folded into the weights and one bias per channel, ReLU;
 * one bidirectional LSTM layer with 256 units per direction (gate rows
 * i, f, g, o, one merged bias per direction, zero initial state), the backward
 * direction starting at the request's own last token;
 * F_enc[j] = [h_forward[j], h_backward[j]].
 *
 * The output is fp32 [tokens][512] in device memory, ready to be handed to
 * tts_pool_add_request as a device pointer.  All kernels are queued on the
 * stream given at creation; device memory comes from the caller's arena;
 * nothing is allocated on the device (creation allocates one pinned host
 * buffer, through which the ids travel).  Conventions as in tts_pool.h: 0 on
 * success, negative tts_status otherwise, text in tts_last_error(); one owner
 * thread per object.
 */
#ifndef TTS_ENCODER_H
#define TTS_ENCODER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tts_encoder tts_encoder;

#define TTS_ENCODER_TABLES 4       /* phoneme tokens, prosodic word, phonological phrase, intonational phrase */
#define TTS_ENCODER_CONVS 3
#define TTS_ENCODER_MAX_BATCH 256  /* requests in one call */

typedef struct {
    int dim;                          /* 512: embedding width = convolution channels (the kernels are built for 512 / 256) */
    int hid;                          /* 256: LSTM units per direction; F_enc has 2 * hid channels */
    int vocab[TTS_ENCODER_TABLES];    /* rows of each embedding table */
    int max_tokens;                   /* most tokens one call may carry, summed over its requests */
    int max_len;                      /* longest single request, 1 .. 32767 */
    int weight_dtype;                 /* TTS_DTYPE_F32 / TTS_DTYPE_BF16 of tts_pool.h (0 / 1): matrices and the activations
                                         that feed them; embedding sum, accumulation, biases, cell state and F_enc are fp32 */
} tts_encoder_config;

/* HOST pointers, fp32, copied at creation.  Direction 0 = forward, 1 = backward.
 *   tables[t] [vocab[t]][dim]; conv_w[l] [dim][dim][5], conv_b[l] [dim];
 *   w_ih[d] [4 hid][dim], w_hh[d] [4 hid][hid], b[d] [4 hid] (gate row blocks i, f, g, o)              */
typedef struct {
    const float *tables[TTS_ENCODER_TABLES];
    const float *conv_w[TTS_ENCODER_CONVS], *conv_b[TTS_ENCODER_CONVS];
    const float *w_ih[2], *w_hh[2], *b[2];
} tts_encoder_weights;

/* Bytes of device memory tts_encoder_create needs for this configuration (0 if the configuration is invalid). */
size_t tts_encoder_workspace_bytes(const tts_encoder_config *cfg);

/*
 * Create an encoder.  `dev_arena` is DEVICE memory of at least tts_encoder_workspace_bytes(cfg) bytes, 256-byte
 * aligned, owned by the caller and kept alive until tts_encoder_destroy.  `hip_stream` is a hipStream_t.
 */
int tts_encoder_create(const tts_encoder_config *cfg, const tts_encoder_weights *weights, void *dev_arena,
                       size_t arena_bytes, void *hip_stream, tts_encoder **out);

/*
 * Encode one dynamic batch of n requests.
 *   ids     HOST int [TTS_ENCODER_TABLES][total]: for each table the ids of all requests back to back
 *           (total = sum of lens); every id must lie in [0, vocab[t]).
 *   lens    HOST [n]: tokens of request i, 1 .. max_len.
 *   d_out   DEVICE fp32 [total][2 * hid]: F_enc of the requests back to back.
 * Asynchronous on the stream (ids and lens are consumed before the call returns).
 * Errors: TTS_E_INVAL for null pointers, n outside 1 .. TTS_ENCODER_MAX_BATCH, bad lengths, more than
 * max_tokens tokens, or an id outside its table.
 */
int tts_encoder_run(tts_encoder *enc, const int *ids, const int *lens, int n, float *d_out);

/* Device time of the last tts_encoder_run in milliseconds (HIP events on the stream); waits for the stream. */
int tts_encoder_elapsed_ms(tts_encoder *enc, float *out_ms);

void tts_encoder_destroy(tts_encoder *enc);

#ifdef __cplusplus
}
#endif
#endif
