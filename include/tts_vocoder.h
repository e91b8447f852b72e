/*
 * tts_vocoder.h -- C ABI of the vocoder side of incremental synthesis
 * (paper Sec. 2.1.4: a HiFi-GAN-based generator G of transposed convolutions
 * and multi-receptive-field fusion blocks turns one mel chunk at a time into
 * one waveform chunk; Eq. 3: G runs on [tail(M_pre), M_cur] and the head of
 * S_cur is fused with the tail of S_pre by equal-power fade coefficients;
 * Sec. 2.2.2 / Eq. 4: M_pre, S_pre are per-request state, replaced by M_cur,
 * S_cur after every chunk, and the module runs on the dynamic batch of the
 * requests that have a chunk ready; Sec. 3.1: 128 initial channels,
 * upsampling factors 8, 8, 2, 2, i.e. 256 samples per frame).
 *
 * The paper fixes only those two figures of G.  This library takes the rest
 * as: conv_pre (kernel 7, n_mel -> 128); per stage leaky ReLU, transposed
 * convolution (stride u, kernel 2u, padding u/2, channels halved), then the
 * mean of three residual blocks with kernels 3, 7, 11, each
 * x += conv_{k,1}(lrelu(conv_{k,d}(lrelu(x)))) for d = 1, 3, 5; finally
 * leaky ReLU, conv_post (kernel 7, -> 1 channel), tanh.  Leaky slope 0.1,
 * zero "same" padding everywhere, weight normalisation folded.  The weights
 * are random stand-ins: the module is built for its arithmetic and its
 * throughput, not for its sound.
 *
 * What one response carries (the paper does not say): the region where two
 * chunks overlap is sent once, fused, with the chunk that completes it.  So a
 * chunk that is not the request's last holds back its final overlap * 256
 * samples, and the responses of a request tile its waveform:
 *   first chunk of n frames      256 (n - overlap) samples
 *   middle chunk                 256 n             (fused head + body)
 *   last chunk                   256 (overlap + n) (everything)
 *   a request of a single chunk  256 n
 * Fade coefficients over the N = 256 * overlap samples of the fused region:
 *   alpha_i = sin(pi/2 (i + 1/2) / N) on the current chunk's head,
 *   beta_i  = cos(pi/2 (i + 1/2) / N) on the previous chunk's tail.
 *
 * All kernels are queued on the stream given at creation; device memory comes
 * from the caller's arena; nothing is allocated on the device.  Conventions as
 * in tts_pool.h: 0 on success, negative tts_status otherwise, text in
 * tts_last_error(); one owner thread per object.
 */
#ifndef TTS_VOCODER_H
#define TTS_VOCODER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tts_vocoder tts_vocoder;

#define TTS_VOCODER_STAGES 4
#define TTS_VOCODER_BLOCKS 3       /* residual blocks per stage: kernels 3, 7, 11 */
#define TTS_VOCODER_PAIRS 3        /* convolution pairs per block: dilations 1, 3, 5 */
#define TTS_VOCODER_HOP 256        /* samples per frame: 8 * 8 * 2 * 2 */
#define TTS_VOCODER_MAX_BATCH 256  /* chunks in one call */
#define TTS_VOCODER_MAX_OVERLAP 16

#define TTS_VOCODER_FIRST 1        /* flags: the request's first chunk (state is reset) */
#define TTS_VOCODER_LAST 2         /* flags: the request's last chunk (nothing is held back; the slot becomes free) */

typedef struct {
    int n_mel;          /* 80 */
    int c0;             /* 128: channels after conv_pre (the kernels are built for 80 / 128 / rates 8, 8, 2, 2) */
    int overlap;        /* frames of the previous chunk in front of the current one, 0 .. TTS_VOCODER_MAX_OVERLAP */
    int max_chunk;      /* most frames in one chunk (>= max(overlap, 1)) */
    int max_requests;   /* state slots: requests that can be between their first and last chunk at one time */
    int max_batch;      /* most chunks in one call, 1 .. TTS_VOCODER_MAX_BATCH */
    int weight_dtype;   /* TTS_DTYPE_F32 / TTS_DTYPE_BF16 of tts_pool.h (0 / 1): weights and the convolutions' inputs;
                           accumulation, bias, residual sums, activations in memory, tanh and the fade are fp32 */
} tts_vocoder_config;

/* HOST pointers, fp32, copied at creation.  With c = channels of stage s (64, 32, 16, 8) and u = its factor:
 *   pre_w [c0][n_mel][7], pre_b [c0]
 *   up_w[s] [2c][c][2u] (input channel first, as for a transposed convolution), up_b[s] [c]
 *   res_w[s][b][2p], res_w[s][b][2p+1]: the dilated and the plain convolution of pair p of block b,
 *                                       [c][c][k_b] with k_b = 3, 7, 11; res_b likewise [c]
 *   post_w [1][8][7], post_b [1]                                                                        */
typedef struct {
    const float *pre_w, *pre_b;
    const float *up_w[TTS_VOCODER_STAGES], *up_b[TTS_VOCODER_STAGES];
    const float *res_w[TTS_VOCODER_STAGES][TTS_VOCODER_BLOCKS][2 * TTS_VOCODER_PAIRS];
    const float *res_b[TTS_VOCODER_STAGES][TTS_VOCODER_BLOCKS][2 * TTS_VOCODER_PAIRS];
    const float *post_w, *post_b;
} tts_vocoder_weights;

/* Bytes of device memory tts_vocoder_create needs for this configuration (0 if the configuration is invalid). */
size_t tts_vocoder_workspace_bytes(const tts_vocoder_config *cfg);

/*
 * Create a vocoder.  `dev_arena` is DEVICE memory of at least tts_vocoder_workspace_bytes(cfg) bytes, 256-byte
 * aligned, owned by the caller and kept alive until tts_vocoder_destroy.  `hip_stream` is a hipStream_t.
 */
int tts_vocoder_create(const tts_vocoder_config *cfg, const tts_vocoder_weights *weights, void *dev_arena,
                       size_t arena_bytes, void *hip_stream, tts_vocoder **out);

/*
 * One dynamic batch: chunk i is the next n_frames[i] mel frames of the request that owns state slot
 * state_slot[i].
 *   d_mel        DEVICE, fp32 [sum_i n_frames[i]][n_mel]: the chunks back to back (M_cur of every item).
 *   n_frames     HOST [n]: 1 .. max_chunk; at least `overlap` unless the chunk is the request's last.
 *   state_slot   HOST [n]: 0 .. max_requests - 1, each at most once per call.  The slot holds tail(M_pre) and
 *                tail(S_pre) of its request between calls (Eq. 4 is applied by this call).
 *   flags        HOST [n]: TTS_VOCODER_FIRST and / or TTS_VOCODER_LAST.  A chunk without FIRST needs a slot whose
 *                previous chunk went through this object and was not LAST.
 *   d_audio      DEVICE, fp32: the responses back to back; response i has out_samples[i] samples (see the table
 *                at the top; at most 256 * (overlap + n_frames[i])).  The caller provides room for the sum.
 *   out_samples  HOST [n], written before the call returns.
 * Asynchronous on the stream (the host arrays are consumed before the call returns).
 * Errors: TTS_E_INVAL for null pointers, n outside 1 .. max_batch, bad lengths, slots or flags; the state is
 * unchanged then.
 */
int tts_vocoder_run(tts_vocoder *v, const float *d_mel, const int *n_frames, const int *state_slot, const int *flags,
                    int n, float *d_audio, int *out_samples);

/* Device time of the last tts_vocoder_run in milliseconds (HIP events on the stream); waits for the stream. */
int tts_vocoder_elapsed_ms(tts_vocoder *v, float *out_ms);

void tts_vocoder_destroy(tts_vocoder *v);

#ifdef __cplusplus
}
#endif
#endif
