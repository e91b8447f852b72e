/*
 * tts_pool — pooled, dynamically batched autoregressive decoder step for
 * incremental TTS on one AMD MI355X (gfx950).
 *
 * What it computes: the per-frame recurrence of the Tacotron-2-style acoustic
 * decoder (paper Sec. 2.1.3, Eq. 2)
 *
 *     H_att, C_att = LSTM_att([Pre(M_last), A], H_att, C_att)
 *     A, W_last    = LSA(H_att, F_enc, W_acc)        (W_last also feeds the location conv)
 *     H_dec, C_dec = LSTM_dec([H_att, A], H_dec, C_dec)
 *     W_acc        = W_acc + W_last
 *     M_last       = Linear(H_dec, A)   (+ stop logit)
 *
 * for every request of an "instant request pool" (Sec. 2.2.2): requests join
 * at any time, are advanced together from the next step on (module-wise
 * dynamic batching restricted to the decoder module D), emit mel frames in
 * chunks (Sec. 2.2.1) and leave at completion.  Each request has its own
 * encoder length and frame count; positions beyond a request's length do not
 * exist (no padding work, zero attention weight).
 *
 * All entry points are plain C.  Return value: TTS_OK (0) or a negative
 * tts_status; the text of the last error of the calling thread is available
 * from tts_last_error().  Nothing aborts or throws across this boundary.
 *
 * Threading: one owner thread per pool.  All device work is queued on the
 * HIP stream given at create time; calls that hand data back to the host
 * (drain, get_state, sync) wait for that stream.
 */
#ifndef TTS_POOL_H
#define TTS_POOL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TTS_OK = 0,
    TTS_E_INVAL = -1,     /* bad argument (null pointer, L < 1, L > max_enc_len, n_steps out of range, ...) */
    TTS_E_FULL = -2,      /* pool already holds max_pool requests */
    TTS_E_NOTFOUND = -3,  /* unknown or already retired request id */
    TTS_E_HIP = -4,       /* a HIP call failed; tts_last_error() carries its text */
    TTS_E_ARENA = -5,     /* device arena too small or misaligned */
    TTS_E_UNSUPPORTED = -6, /* dimensions outside what the kernels are built for, or a device with fewer than 256 CUs */
    TTS_E_LOST = -7       /* tts_pool_sync: requests were ended early by the device since the last call (see there) */
} tts_status;

enum { TTS_DTYPE_F32 = 0, TTS_DTYPE_BF16 = 1 };

/* Which carried state of Eq. 2 / Sec. 2.1.3 get_state / set_state address. */
enum {
    TTS_STATE_M_LAST = 0,  /* [n_mel]        */
    TTS_STATE_A = 1,       /* [enc_dim]      */
    TTS_STATE_W_LAST = 2,  /* [L]            */
    TTS_STATE_W_ACC = 3,   /* [L]            */
    TTS_STATE_H_ATT = 4,   /* [att_rnn_dim]  */
    TTS_STATE_C_ATT = 5,   /* [att_rnn_dim]  */
    TTS_STATE_H_DEC = 6,   /* [dec_rnn_dim]  */
    TTS_STATE_C_DEC = 7    /* [dec_rnn_dim]  */
};

typedef struct tts_pool tts_pool; /* opaque */

/* Model and pool geometry.  All ints are 32-bit. */
typedef struct {
    /* decoder dimensions ("same model parameters as the original" Tacotron 2, Sec. 3.1).
     * The kernels are specialised for 80, 256, 512, 1024, 1024, 128, 32, 31, {1,2};
     * anything else is rejected with TTS_E_UNSUPPORTED. */
    int n_mel, prenet_dim, enc_dim, att_rnn_dim, dec_rnn_dim, att_dim;
    int loc_filters, loc_kernel, loc_in_channels;
    int max_pool;      /* 1..256: most requests in the pool at once */
    int max_enc_len;   /* 1..1024: longest encoder output accepted */
    int max_steps;     /* >= 1: most frames one request may produce (size of its mel ring) */
    int chunk_frames;  /* >= 1: frames handed out per drain ("configurable size of the chunk", Sec. 2.2.1) */
    int weight_dtype;  /* TTS_DTYPE_F32: fp32 weights and activations.
                          TTS_DTYPE_BF16: the weight matrices are bfloat16 VALUES (given values are rounded to
                          bfloat16, ties to even, at upload); accumulation and cell / softmax arithmetic are fp32.
                          On the device the matrices are held as IEEE half, which holds every bfloat16 value of
                          magnitude >= 2^-14 exactly (smaller ones within 2^-25), and the activations multiplied
                          with them are rounded to IEEE half: same bytes and MFMA rate as bfloat16 operands,
                          8 x less operand rounding.  max_steps <= 65504 in this mode. */
    int memory_dtype;  /* storage of F_enc and of the processed memory F_enc W_mem^T.
                          TTS_DTYPE_BF16 requires weight_dtype == TTS_DTYPE_BF16. */
    int use_graph;     /* non-zero: each step is one hipGraph launch */
    float stop_threshold; /* a request ends when sigmoid(stop logit) > threshold (Sec. 2.2.1);
                             outside [0,1] = disabled, requests end at their n_steps */
} tts_config;

/* HOST pointers to fp32, row-major [out, in] tensors; all are copied (and
 * re-laid out) during tts_pool_create and may be freed afterwards.
 * LSTM rows are ordered i, f, g, o; att_b / dec_b are the merged biases. */
typedef struct {
    const float *prenet1, *prenet2;               /* [256,80], [256,256], no bias, ReLU after each      */
    const float *att_w_ih, *att_w_hh, *att_b;     /* [4096,768] on [Pre(M_last);A], [4096,1024], [4096] */
    const float *q_w, *mem_w, *loc_conv, *loc_w, *v; /* [128,1024], [128,512], [32,C,31], [128,32], [128] */
    const float *dec_w_ih, *dec_w_hh, *dec_b;     /* [4096,1536] on [H_att;A], [4096,1024], [4096]      */
    const float *mel_w, *mel_b, *stop_w, *stop_b; /* [80,1536] on [H_dec;A], [80], [1,1536], [1]        */
} tts_weights;

/* Bytes of device memory a pool of this geometry needs (0 if the config is invalid). */
size_t tts_pool_workspace_bytes(const tts_config *cfg);

/*
 * Create a pool.  `dev_arena` is DEVICE memory of at least
 * tts_pool_workspace_bytes(cfg) bytes, 256-byte aligned, owned by the caller
 * and kept alive until tts_pool_destroy; the library allocates no device
 * memory itself (it allocates two small pieces of pinned host memory: a status
 * word and a staging buffer of one chunk).  `hip_stream` is a hipStream_t (NULL = the default stream) on
 * which every kernel and copy of this pool is queued; it stays owned by the
 * caller.  Weights are uploaded and re-laid out here (synchronous).
 */
int tts_pool_create(const tts_config *cfg, const tts_weights *weights,
                    void *dev_arena, size_t arena_bytes, void *hip_stream, tts_pool **out);

/*
 * Add a request to the pool ("once a new request arrives, it is immediately
 * added to the pool", Sec. 2.2.2).  `enc_out` is the encoder output
 * F_enc [L, enc_dim], fp32 row-major, HOST or DEVICE memory (detected).  It is
 * copied: a host buffer may be freed on return; a device buffer must stay
 * valid until the work queued on the pool's stream by this call has run.
 * The processed memory F_enc W_mem^T is computed once here and the request's
 * state is zeroed.  `n_steps` (1..max_steps) is the hard cap on frames.  The
 * request is advanced from the next tts_pool_step on.  *out_id receives a
 * pool-unique id (never reused).
 */
int tts_pool_add_request(tts_pool *pool, const float *enc_out, int L, int n_steps, int64_t *out_id);

/*
 * Add `n` requests at once: an iteration of the pool takes every request that is waiting (Sec. 2.2.2).  Same
 * result, bit for bit, as `n` calls of tts_pool_add_request in this order (enc_out[i], L[i], n_steps[i] -> out_ids[i],
 * each buffer HOST or DEVICE memory), but requests whose encoder outputs are in device memory are set up by one
 * launch per 64 of them.  Arguments and room are checked first: on TTS_E_INVAL or TTS_E_FULL nothing was added.
 */
int tts_pool_add_requests(tts_pool *pool, int n, const float *const *enc_out, const int *L, const int *n_steps,
                          int64_t *out_ids);

/*
 * One decoder step: every unfinished request in the pool produces one more
 * mel frame (Eq. 2).  Asynchronous on the pool's stream.  *out_n_active (may
 * be NULL) receives the number of requests advanced; 0 on an empty pool, which
 * is a no-op.  A request that reaches its n_steps, or trips the stop
 * threshold, stops advancing but keeps its slot until retired.
 */
int tts_pool_step(tts_pool *pool, int *out_n_active);

/* `n` consecutive steps (no joins in between); *out_frames (may be NULL)
 * receives the total number of frames produced.  Same frames and state, bit
 * for bit, as n calls of tts_pool_step; the steps of one call are queued more
 * tightly (one graph launch for up to a chunk of steps; in pools of at most 64
 * slots with two-byte weights and memory a step that follows another step of
 * the same call is two kernel launches instead of three). */
int tts_pool_step_n(tts_pool *pool, int n, int64_t *out_frames);

/*
 * Hand out the next chunk of mel frames of request `id` into HOST memory
 * `dst` [chunk_frames, n_mel] fp32.  If fewer than chunk_frames undrained
 * frames exist and the request is unfinished, *out_frames = 0 and TTS_OK.  The
 * last chunk of a finished request may be short.  *out_finished = 1 once the
 * request is finished AND everything has been drained.  Waits for the stream.
 * A request the device ended early (tts_pool_sync, tts_pool_lost) hands out the frames it has like any finished one.
 */
int tts_pool_drain_chunk(tts_pool *pool, int64_t id, float *dst, int *out_frames, int *out_finished);

/*
 * The same hand-out for a consumer on the device (the chunk-level modules that follow the decoder step,
 * Sec. 2.2.2: each module builds its batch from the pool items that are ready): copy the next chunk of
 * request `id`, preceded by up to `context` earlier frames of the same request, into DEVICE memory `d_dst`
 * (room for (context + chunk_frames) * n_mel floats).  *out_context = frames in front of the chunk that were
 * copied (fewer than `context` only at the start of the utterance), *out_frames = frames of the chunk (0 if
 * none is ready: nothing is copied), *out_finished as in tts_pool_drain_chunk.  The copy is queued on the
 * pool's stream; the chunk counts as handed out.
 */
int tts_pool_chunk_window(tts_pool *pool, int64_t id, int context, float *d_dst, int *out_context, int *out_frames,
                          int *out_finished);

/* Stop logits of frames [first, first+count) of request `id` into HOST `dst`; waits for the stream. */
int tts_pool_get_stop_logits(tts_pool *pool, int64_t id, int first, int count, float *dst);

/* Remove a request ("if a request completes, its item is removed from the pool
 * immediately", Sec. 2.2.2); also allowed for an unfinished request.  Frees its slot. */
int tts_pool_retire(tts_pool *pool, int64_t id);

/* Copy one carried state of request `id` to HOST `dst` (fp32, `cap` elements of
 * room); *out_n receives the element count.  Waits for the stream. */
int tts_pool_get_state(tts_pool *pool, int64_t id, int which, float *dst, int cap, int *out_n);

/* Overwrite one carried state of request `id` from HOST `src` (`n` fp32
 * elements, must equal the state's size).  Takes effect at the next step. */
int tts_pool_set_state(tts_pool *pool, int64_t id, int which, const float *src, int n);

/* Frames produced so far by request `id` (waits for the stream only if the stop threshold is enabled). */
int tts_pool_frames(tts_pool *pool, int64_t id, int *out_frames, int *out_finished);

/* Requests currently holding a slot / requests the next step would advance. */
int tts_pool_size(const tts_pool *pool);
int tts_pool_n_active(const tts_pool *pool);

/* Slots the next step's kernels must cover (one past the highest running request's slot), and how many times a
 * running request has been moved to a lower slot since creation.  The pool of Sec. 2.2.2 shrinks as requests leave;
 * when the running requests would fit fewer 16-slot tiles than the kernels cover, and enough lower slots are free,
 * the pool moves them down on the device before the next step.  Nothing a caller sees depends on the slot: ids,
 * frames and states stay with the request, bit for bit.  Spans of 16 and fewer are left alone. */
int tts_pool_span(const tts_pool *pool);
long long tts_pool_moves(const tts_pool *pool);

/* Wait until everything queued on the pool's stream has run.
 * Workgroups of one launch hand each other words (the projection's partial sums, the attention energies of a
 * request) and wait for them a bounded number of polls.  Should such a wait ever run out (the GPU so oversubscribed by
 * other work that a partner is not scheduled for a quarter of a second), the kernels still finish and only the
 * requests whose words were missing are affected: the device stores nothing more for them from that step on (the
 * frames they have are valid and can be drained; they count as finished and hold their slots until retired), every
 * other request in the pool goes on undisturbed.  The first tts_pool_sync after such an incident returns TTS_E_LOST
 * with the ids in tts_last_error(); tts_pool_lost tells for one request.  Nothing else is needed to go on using the
 * pool.  (A consumer on the device, tts_pool_chunk_window, can only know of steps that have already run: wait with
 * this call before trusting chunks handed over from steps still in flight.) */
int tts_pool_sync(tts_pool *pool);

/* *out_lost = 1 if request `id` was ended early by the device because a step could not be completed for it. */
int tts_pool_lost(tts_pool *pool, int64_t id, int *out_lost);

/* The bound of those waits, in polls (default 2^18).  Waits for the stream.  0 makes every such wait give up at
 * once: the kernels run through as always, and the path above can be exercised without anything hanging. */
int tts_pool_set_wait_polls(tts_pool *pool, int polls);

/* Device time of the kernels of the most recent tts_pool_step / step_n call,
 * measured with HIP events on the pool's stream.  Timing is off by default;
 * enable != 0 turns it on.  elapsed_ms waits for the stream. */
int tts_pool_timing(tts_pool *pool, int enable);
int tts_pool_elapsed_ms(tts_pool *pool, float *out_ms);

/* Profiling aid: run `n` steps WITHOUT the graph, queued back to back with a
 * HIP event between consecutive kernels, and return the average device time of
 * each kernel of the step in microseconds in out_us (room for `cap` values;
 * *out_n_kernels receives how many there are: attention LSTM, attention,
 * decoder LSTM, projection + prenet; pools with two-byte weights have no
 * decoder-LSTM kernel - it is part of the last kernel's launch (above 64
 * slots: from 17 slots spanned) - and report 0 for it).  The n steps are launched as one call of n steps launches them:
 * in those pools the last kernel of every step but the call's last also forms
 * the next step's attention LSTM, so only the first step has an
 * attention-LSTM kernel (that one launch is the figure reported) and the
 * projection's figure is the average over the steps whose launch carried that
 * extra part.  The device cost of an event itself is
 * measured with adjacent events and subtracted; if cap > *out_n_kernels it is
 * stored after the kernel times, and if cap > *out_n_kernels + 1 the time of
 * the last kernel without the extra part (the call's last step; 0 where no
 * step differs) after that.  The intervals still contain the launch gap,
 * so they are upper bounds of the kernels' own durations.  The steps are real:
 * requests advance.  Waits for the stream. */
int tts_pool_kernel_times(tts_pool *pool, int n, float *out_us, int cap, int *out_n_kernels);

void tts_pool_destroy(tts_pool *pool);

const char *tts_last_error(void);

/*
 * Host-only model of the pool's bookkeeping (slots, ids, membership, frame
 * counters, chunk cursor): exactly the class the pool uses, without any
 * device work.  For schedulers and CPU tests of the pooling semantics of
 * Sec. 2.2.2 / 2.2.3 (e.g. the membership trace of the timeline figure).
 */
typedef struct tts_book tts_book;
tts_book *tts_book_create(int max_pool, int max_enc_len, int max_steps, int chunk_frames);
int tts_book_add(tts_book *b, int L, int n_steps, int64_t *out_id);
/* advances every active request; ids of the requests advanced go to out_ids (room for max_pool) */
int tts_book_step(tts_book *b, int64_t *out_ids, int *out_n_active);
/* frames the next drain would hand out (0 if the chunk is not ready) */
int tts_book_drain(tts_book *b, int64_t id, int *out_first, int *out_frames, int *out_finished);
int tts_book_retire(tts_book *b, int64_t id);
/* slot of request `id` (-1: no such request) */
int tts_book_slot(const tts_book *b, int64_t id);
/* Packs the running requests into fewer 16-slot tiles (below one tile: a smaller power of two), not below `min_span`, if the free slots allow it
 * (the pool does this before a step, with min_span 16).  Returns the number of moves carried out and writes the first
 * `cap` of them as out_from[i] -> out_to[i]; 0 if there is nothing to gain or finished requests block the low slots. */
int tts_book_compact(tts_book *b, int min_span, int *out_from, int *out_to, int cap);
void tts_book_destroy(tts_book *b);

#ifdef __cplusplus
}
#endif
#endif /* TTS_POOL_H */
