/*
 * tts_postnet.h -- C ABI of the chunk-wise PostNet of the acoustic decoder
 * (paper Sec. 2.1.3: "a PostNet for improving the Mel reconstruction";
 * Sec. 2.2.1: the decoder is incremental and produces one chunk of mel frames
 * at a time; Sec. 2.2.2: every module runs on the dynamic batch of pool items
 * that need it in this iteration).
 *
 * The paper fixes nothing about the PostNet beyond "the parameters of the
 * original Tacotron 2" (Sec. 3.1).  This library takes it as: n_layers
 * (5) one-dimensional convolutions over time, kernel 5, zero "same" padding,
 * channels n_mel -> C -> ... -> C -> n_mel, tanh after every layer but the last,
 * batch normalisation folded into the weights and one bias per output channel,
 * result added to the input mel.  Chunk-wise it is applied to "the utterance so
 * far": chunk [s, e) of a request is the whole stack on frames [0, e), zero
 * padded at both ends, restricted to [s, e).  Frames older than 2 * n_layers
 * before the chunk cannot influence it, so the caller hands over WINDOWS:
 * the chunk's frames preceded by up to 2 * n_layers frames of context.
 *
 * One call = one dynamic batch: n windows of different lengths, packed back to
 * back.  All kernels are queued on the stream given at creation; device memory
 * comes from the caller's arena; nothing is allocated on the device.
 *
 * Conventions as in tts_pool.h: 0 on success, negative tts_status otherwise,
 * text in tts_last_error(); one owner thread per object.
 */
#ifndef TTS_POSTNET_H
#define TTS_POSTNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tts_postnet tts_postnet;

#define TTS_POSTNET_LAYERS 5
#define TTS_POSTNET_TAPS 5
#define TTS_POSTNET_CONTEXT (2 * TTS_POSTNET_LAYERS) /* frames in front of a chunk that can influence it */

typedef struct {
    int n_mel;         /* 80 */
    int channels;      /* 512: width of the hidden layers (the kernels are built for 80 / 512) */
    int max_columns;   /* most frames (context included) one call may carry, summed over its windows */
    int weight_dtype;  /* TTS_DTYPE_F32 / TTS_DTYPE_BF16 of tts_pool.h (0 / 1): weights and the activations between layers;
                          accumulation, bias, tanh and the residual sum are fp32 */
} tts_postnet_config;

/* HOST pointers, fp32; conv_w[l] is [c_out][c_in][5] (c_in = n_mel for l = 0, channels otherwise; c_out = n_mel
 * for the last layer, channels otherwise), conv_b[l] is [c_out].  Copied at creation. */
typedef struct {
    const float *conv_w[TTS_POSTNET_LAYERS];
    const float *conv_b[TTS_POSTNET_LAYERS];
} tts_postnet_weights;

/* Bytes of device memory tts_postnet_create needs for this configuration (0 if the configuration is invalid). */
size_t tts_postnet_workspace_bytes(const tts_postnet_config *cfg);

/*
 * Create a PostNet.  `dev_arena` is DEVICE memory of at least
 * tts_postnet_workspace_bytes(cfg) bytes, 256-byte aligned, owned by the caller
 * and kept alive until tts_postnet_destroy.  `hip_stream` is a hipStream_t.
 */
int tts_postnet_create(const tts_postnet_config *cfg, const tts_postnet_weights *weights, void *dev_arena,
                       size_t arena_bytes, void *hip_stream, tts_postnet **out);

/*
 * Post-process one dynamic batch.
 *   d_mel     DEVICE, fp32 [sum_i win_len[i]][n_mel]: the windows back to back.  Window i holds frames
 *             [e_i - win_len[i], e_i) of its request, e_i = the request's frames so far.
 *   win_len   HOST [n]: frames in window i (context + chunk), >= 1.
 *   keep_from HOST [n]: index inside window i of the chunk's first frame, i.e. the number of context frames
 *             in front (0 <= keep_from[i] < win_len[i]).  A window that does not start at the request's
 *             frame 0 must carry TTS_POSTNET_CONTEXT context frames for its chunk to be exact: frames in
 *             front of a window are taken as zero, which is right only at the start of an utterance.
 *   d_out     DEVICE, fp32 [sum_i (win_len[i] - keep_from[i])][n_mel]: the post-processed chunks back to back.
 * Asynchronous on the stream (win_len / keep_from are consumed before the call returns).
 * Errors: TTS_E_INVAL for null pointers, n < 1, bad lengths, or more than max_columns frames.
 */
int tts_postnet_run(tts_postnet *pn, const float *d_mel, const int *win_len, const int *keep_from, int n,
                    float *d_out);

/*
 * The same call for callers that cannot allocate or be handed a workspace where they run: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, results (bit for bit) and errors are
 * those of tts_postnet_run, but the scratch of the call -- the activations between the layers and the per-column
 * tables -- lives in a static array inside the library instead of the arena: TTS_POSTNET_STATIC_BYTES bytes per GPU
 * that runs it, held until the process ends.  The call allocates nothing (no hipMalloc, no hipFree, no allocating
 * library routine) and records no events (tts_postnet_elapsed_ms does not see it).  A batch may carry at most
 * TTS_POSTNET_STATIC_MAX_COLUMNS frames (context included) whatever max_columns says: more is TTS_E_INVAL.  Every
 * call on a GPU, from any tts_postnet object, uses that GPU's one array: calls that overlap on one GPU (two streams,
 * two threads) race; calls queued on one stream do not.  The device the object was created on must be current.
 */
#define TTS_POSTNET_STATIC_MAX_COLUMNS 4096
#define TTS_POSTNET_STATIC_BYTES (2u * TTS_POSTNET_STATIC_MAX_COLUMNS * 512u * 4u + 2u * TTS_POSTNET_STATIC_MAX_COLUMNS * 4u)
int tts_postnet_run_static(tts_postnet *pn, const float *d_mel, const int *win_len, const int *keep_from, int n,
                           float *d_out);

/* Device time of the last tts_postnet_run in milliseconds (HIP events on the stream); waits for the stream. */
int tts_postnet_elapsed_ms(tts_postnet *pn, float *out_ms);

void tts_postnet_destroy(tts_postnet *pn);

#ifdef __cplusplus
}
#endif
#endif
