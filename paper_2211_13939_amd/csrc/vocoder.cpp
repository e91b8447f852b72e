// Host side of the tts_vocoder C ABI: argument checks, arena carve-up, weight re-layout (every convolution,
// the transposed ones included, becomes the A operand of one GEMM), the per-call batch table and the state
// slots' bookkeeping.  All arithmetic on audio and mel data is in vocoder.hip.
#include "../../include/tts_vocoder.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <vector>

#include "hostutil.h"
#include "vocoder_kernels.h"

using namespace tts;

namespace {

int check(const tts_vocoder_config* c)
{
    if (!c) return fail(TTS_E_INVAL, "config is null");
    if (c->n_mel != VOC_N_MEL || c->c0 != VOC_C0)
        return fail(TTS_E_UNSUPPORTED, "kernels are built for %d mel bins and %d initial channels", VOC_N_MEL, VOC_C0);
    if (c->overlap < 0 || c->overlap > VOC_MAX_OVERLAP) return fail(TTS_E_INVAL, "overlap must be in 0..%d", VOC_MAX_OVERLAP);
    if (c->max_chunk < 1 || c->max_chunk < c->overlap || c->max_chunk > 4096)
        return fail(TTS_E_INVAL, "max_chunk must be in max(overlap, 1)..4096");
    if (c->max_requests < 1 || c->max_requests > 65535) return fail(TTS_E_INVAL, "max_requests must be in 1..65535");
    if (c->max_batch < 1 || c->max_batch > VOC_MAX_BATCH) return fail(TTS_E_INVAL, "max_batch must be in 1..%d", VOC_MAX_BATCH);
    if (c->weight_dtype != TTS_DTYPE_F32 && c->weight_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "weight_dtype must be 0 (fp32) or 1 (bf16)");
    return TTS_OK;
}

// one convolution as the GEMM's A operand: rows x (taps * c_in), padded to whole 16-row tiles and whole fragments
struct ConvShape {
    int rows, rows_pad, c_in, taps, k_pad;
};
ConvShape shape_of(int rows, int c_in, int taps, bool bf)
{
    const int kb = bf ? 32 : 16;
    return {rows, (rows + 15) / 16 * 16, c_in, taps, (taps * c_in + kb - 1) / kb * kb};
}
size_t bytes_of(const ConvShape& s, bool bf) { return (size_t)s.rows_pad * s.k_pad * (bf ? 2 : 4); }

ConvShape pre_shape(bool bf) { return shape_of(VOC_C0, VOC_N_MEL, VOC_K_PRE, bf); }
ConvShape up_shape(int s, bool bf) { return shape_of(voc_rate(s) * voc_channels(s), 2 * voc_channels(s), 3, bf); }
ConvShape res_shape(int s, int b, bool bf) { return shape_of(voc_channels(s), voc_channels(s), voc_block_k(b), bf); }
ConvShape post_shape(bool bf) { return shape_of(1, voc_channels(VOC_STAGES - 1), VOC_K_POST, bf); }

struct VocLayout {
    size_t pre_w, pre_b, up_w[VOC_STAGES], up_b[VOC_STAGES];
    size_t res_w[VOC_STAGES][VOC_BLOCKS][2 * VOC_PAIRS], res_b[VOC_STAGES][VOC_BLOCKS][2 * VOC_PAIRS];
    size_t post_w, post_b, alpha, beta, m_tail, s_tail, len, x_mel, x0, y, r[VOC_BLOCKS], audio, total;
    size_t state_begin;   // everything from here on is cleared at creation
};

VocLayout layout_of(const tts_vocoder_config& c)
{
    const bool bf = c.weight_dtype == TTS_DTYPE_BF16;
    const size_t window = (size_t)c.overlap + c.max_chunk;
    const size_t frames = window * c.max_batch;
    const size_t n_ov = (size_t)(c.overlap > 0 ? c.overlap : 1);
    Carver a;
    VocLayout l;
    l.pre_w = a.take(bytes_of(pre_shape(bf), bf));
    l.pre_b = a.take(VOC_C0 * 4);
    for (int s = 0; s < VOC_STAGES; ++s) {
        l.up_w[s] = a.take(bytes_of(up_shape(s, bf), bf));
        l.up_b[s] = a.take(voc_channels(s) * 4);
        for (int b = 0; b < VOC_BLOCKS; ++b)
            for (int i = 0; i < 2 * VOC_PAIRS; ++i) {
                l.res_w[s][b][i] = a.take(bytes_of(res_shape(s, b, bf), bf));
                l.res_b[s][b][i] = a.take(voc_channels(s) * 4);
            }
    }
    l.post_w = a.take(bytes_of(post_shape(bf), bf));
    l.post_b = a.take(16);
    l.alpha = a.take(n_ov * VOC_HOP * 4);
    l.beta = a.take(n_ov * VOC_HOP * 4);
    l.state_begin = a.off;
    l.m_tail = a.take((size_t)c.max_requests * n_ov * VOC_N_MEL * 4);
    l.s_tail = a.take((size_t)c.max_requests * n_ov * VOC_HOP * 4);
    l.len = a.take(VOC_MAX_BATCH * 4);
    l.x_mel = a.take(frames * VOC_N_MEL * 4);
    l.x0 = a.take(frames * VOC_C0 * 4);
    // positions x channels per frame: 8 * 64, 64 * 32, 128 * 16, 256 * 8 -- at most 2048
    const size_t act = frames * 2048 * 4;
    l.y = a.take(act);
    for (int b = 0; b < VOC_BLOCKS; ++b) l.r[b] = a.take(act);
    l.audio = a.take(frames * VOC_HOP * 4);
    l.total = a.off;
    return l;
}

}  // namespace

struct tts_vocoder {
    tts_vocoder_config cfg;
    VocoderPtrs d;
    hipStream_t stream = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    bool ev_valid = false;
    std::vector<uint8_t> open;      // per state slot: a chunk went through and was not the last
};

extern "C" size_t tts_vocoder_workspace_bytes(const tts_vocoder_config* cfg)
{
    if (check(cfg) != TTS_OK) return 0;
    return layout_of(*cfg).total;
}

extern "C" int tts_vocoder_create(const tts_vocoder_config* cfg, const tts_vocoder_weights* w, void* dev_arena,
                                  size_t arena_bytes, void* hip_stream, tts_vocoder** out)
{
    if (!out) return fail(TTS_E_INVAL, "out is null");
    *out = nullptr;
    int rc = check(cfg);
    if (rc) return rc;
    if (!w || !dev_arena) return fail(TTS_E_INVAL, "null argument");
    bool all = w->pre_w && w->pre_b && w->post_w && w->post_b;
    for (int s = 0; s < VOC_STAGES && all; ++s) {
        all = w->up_w[s] && w->up_b[s];
        for (int b = 0; b < VOC_BLOCKS && all; ++b)
            for (int i = 0; i < 2 * VOC_PAIRS && all; ++i) all = w->res_w[s][b][i] && w->res_b[s][b][i];
    }
    if (!all) return fail(TTS_E_INVAL, "a weight pointer is null");
    const VocLayout lay = layout_of(*cfg);
    if (arena_bytes < lay.total) return fail(TTS_E_INVAL, "arena has %zu bytes, %zu needed", arena_bytes, lay.total);
    if ((uintptr_t)dev_arena % 256) return fail(TTS_E_INVAL, "arena must be 256-byte aligned");
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, dev_arena) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(TTS_E_INVAL, "arena is not device memory");
    }
    tts_vocoder* v = new (std::nothrow) tts_vocoder();
    if (!v) return fail(TTS_E_INVAL, "out of host memory");
    v->cfg = *cfg;
    v->stream = (hipStream_t)hip_stream;
    v->open.assign(cfg->max_requests, 0);
    char* base = (char*)dev_arena;
    const bool bf = cfg->weight_dtype == TTS_DTYPE_BF16;

    // a plain convolution [c_out][c_in][taps]: GEMM row = output channel, k = tap * c_in + channel
    auto put_conv = [&](size_t off, const ConvShape& sh, const float* src) {
        return upload(base + off, pack_fragments(sh.rows_pad, sh.k_pad, bf, [&](int r, int k) {
                          const int tap = k / sh.c_in, c = k - tap * sh.c_in;
                          return (r < sh.rows && tap < sh.taps) ? src[((size_t)r * sh.c_in + c) * sh.taps + tap] : 0.f;
                      }), bf);
    };
    // a transposed convolution [c_in][c_out][2u], stride u, padding u/2: output u p + phase takes input p + tap - 1
    // through kernel element j = phase + u/2 - (tap - 1) u, where that lies in [0, 2u); GEMM row = phase * c_out + channel
    auto put_up = [&](size_t off, int s, const float* src) {
        const ConvShape sh = up_shape(s, bf);
        const int u = voc_rate(s), c_out = voc_channels(s), c_in = sh.c_in;
        return upload(base + off, pack_fragments(sh.rows_pad, sh.k_pad, bf, [&](int r, int k) {
                          const int tap = k / c_in, c = k - tap * c_in;
                          if (r >= sh.rows || tap >= 3) return 0.f;
                          const int phase = r / c_out, co = r - phase * c_out;
                          const int j = phase + u / 2 - (tap - 1) * u;
                          return (j >= 0 && j < 2 * u) ? src[((size_t)c * c_out + co) * (2 * u) + j] : 0.f;
                      }), bf);
    };
    auto put_bias = [&](size_t off, const float* src, int n) { return upload(base + off, std::vector<float>(src, src + n), false); };

    rc = put_conv(lay.pre_w, pre_shape(bf), w->pre_w);
    if (rc == TTS_OK) rc = put_bias(lay.pre_b, w->pre_b, VOC_C0);
    for (int s = 0; s < VOC_STAGES && rc == TTS_OK; ++s) {
        rc = put_up(lay.up_w[s], s, w->up_w[s]);
        if (rc == TTS_OK) rc = put_bias(lay.up_b[s], w->up_b[s], voc_channels(s));
        for (int b = 0; b < VOC_BLOCKS && rc == TTS_OK; ++b)
            for (int i = 0; i < 2 * VOC_PAIRS && rc == TTS_OK; ++i) {
                rc = put_conv(lay.res_w[s][b][i], res_shape(s, b, bf), w->res_w[s][b][i]);
                if (rc == TTS_OK) rc = put_bias(lay.res_b[s][b][i], w->res_b[s][b][i], voc_channels(s));
            }
    }
    if (rc == TTS_OK) rc = put_conv(lay.post_w, post_shape(bf), w->post_w);
    if (rc == TTS_OK) rc = put_bias(lay.post_b, w->post_b, 1);
    if (rc == TTS_OK && cfg->overlap > 0) {
        // equal-power fade over the overlap: alpha^2 + beta^2 = 1, sampled at the mid-points
        const int N = cfg->overlap * VOC_HOP;
        std::vector<float> al(N), be(N);
        for (int i = 0; i < N; ++i) {
            const double u = (i + 0.5) / N, ph = 1.5707963267948966 * u;
            al[i] = (float)std::sin(ph);
            be[i] = (float)std::cos(ph);
        }
        rc = upload(base + lay.alpha, al, false);
        if (rc == TTS_OK) rc = upload(base + lay.beta, be, false);
    }
    if (rc == TTS_OK && hipMemset(base + lay.state_begin, 0, lay.total - lay.state_begin) != hipSuccess)
        rc = fail(TTS_E_HIP, "clearing the state and activation buffers failed");
    if (rc == TTS_OK && (hipEventCreate(&v->ev0) != hipSuccess || hipEventCreate(&v->ev1) != hipSuccess))
        rc = fail(TTS_E_HIP, "hipEventCreate failed");
    if (rc) {
        tts_vocoder_destroy(v);
        return rc;
    }
    VocoderPtrs& d = v->d;
    d.pre_w = base + lay.pre_w;
    d.pre_b = (const float*)(base + lay.pre_b);
    for (int s = 0; s < VOC_STAGES; ++s) {
        d.up_w[s] = base + lay.up_w[s];
        d.up_b[s] = (const float*)(base + lay.up_b[s]);
        for (int b = 0; b < VOC_BLOCKS; ++b)
            for (int i = 0; i < 2 * VOC_PAIRS; ++i) {
                d.res_w[s][b][i] = base + lay.res_w[s][b][i];
                d.res_b[s][b][i] = (const float*)(base + lay.res_b[s][b][i]);
            }
    }
    d.post_w = base + lay.post_w;
    d.post_b = (const float*)(base + lay.post_b);
    d.alpha = (const float*)(base + lay.alpha);
    d.beta = (const float*)(base + lay.beta);
    d.m_tail = (float*)(base + lay.m_tail);
    d.s_tail = (float*)(base + lay.s_tail);
    d.len = (int*)(base + lay.len);
    d.x_mel = (float*)(base + lay.x_mel);
    d.x0 = (float*)(base + lay.x0);
    d.y = (float*)(base + lay.y);
    for (int b = 0; b < VOC_BLOCKS; ++b) {
        d.r[b] = (float*)(base + lay.r[b]);
    }
    d.audio = (float*)(base + lay.audio);
    d.overlap = cfg->overlap;
    d.window = cfg->overlap + cfg->max_chunk;
    *out = v;
    return TTS_OK;
}

extern "C" int tts_vocoder_run(tts_vocoder* v, const float* d_mel, const int* n_frames, const int* state_slot,
                               const int* flags, int n, float* d_audio, int* out_samples)
{
    if (!v || !d_mel || !n_frames || !state_slot || !flags || !d_audio || !out_samples)
        return fail(TTS_E_INVAL, "null argument");
    if (n < 1 || n > v->cfg.max_batch) return fail(TTS_E_INVAL, "n = %d chunks, max_batch = %d", n, v->cfg.max_batch);
    const int ov = v->cfg.overlap;
    VocBatch b;
    b.n = n;
    int row = 0;
    long long off = 0;
    // validate everything before any state changes
    for (int i = 0; i < n; ++i) {
        const int nf = n_frames[i], slot = state_slot[i], fl = flags[i];
        if (fl & ~(TTS_VOCODER_FIRST | TTS_VOCODER_LAST)) return fail(TTS_E_INVAL, "chunk %d: flags = %d", i, fl);
        const bool first = fl & TTS_VOCODER_FIRST, last = fl & TTS_VOCODER_LAST;
        if (nf < 1 || nf > v->cfg.max_chunk) return fail(TTS_E_INVAL, "chunk %d has %d frames, max_chunk = %d", i, nf, v->cfg.max_chunk);
        if (!last && nf < ov) return fail(TTS_E_INVAL, "chunk %d has %d frames: fewer than the overlap (%d) and not the last", i, nf, ov);
        if (slot < 0 || slot >= v->cfg.max_requests) return fail(TTS_E_INVAL, "chunk %d: state slot %d outside 0..%d", i, slot, v->cfg.max_requests - 1);
        for (int k = 0; k < i; ++k)
            if (state_slot[k] == slot) return fail(TTS_E_INVAL, "state slot %d appears twice in one call", slot);
        if (!first && !v->open[slot]) return fail(TTS_E_INVAL, "chunk %d: state slot %d has no previous chunk", i, slot);
        const bool has_prev = !first;
        const int len = (has_prev ? ov : 0) + nf;
        const int emit = (last ? len : len - ov) * VOC_HOP;
        b.src_row[i] = row;
        b.out_off[i] = (int)off;
        b.n_frames[i] = (uint16_t)nf;
        b.slot[i] = (uint16_t)slot;
        b.has_prev[i] = has_prev ? 1 : 0;
        b.last[i] = last ? 1 : 0;
        out_samples[i] = emit;
        row += nf;
        off += emit;
        if (off > 0x7FFFFFFF) return fail(TTS_E_INVAL, "more than 2^31 samples in one call");
    }
    for (int i = 0; i < n; ++i) v->open[state_slot[i]] = (flags[i] & TTS_VOCODER_LAST) ? 0 : 1;
    HIP_TRY(hipEventRecord(v->ev0, v->stream));
    HIP_TRY(launch_vocoder_splice(v->d, b, d_mel, v->stream));
    HIP_TRY(launch_vocoder_generator(v->d, v->cfg.weight_dtype, n, v->stream));
    HIP_TRY(launch_vocoder_fade(v->d, b, d_audio, v->stream));
    HIP_TRY(hipEventRecord(v->ev1, v->stream));
    v->ev_valid = true;
    return TTS_OK;
}

extern "C" int tts_vocoder_elapsed_ms(tts_vocoder* v, float* out_ms)
{
    if (!v || !out_ms) return fail(TTS_E_INVAL, "null argument");
    if (!v->ev_valid) return fail(TTS_E_INVAL, "nothing has run yet");
    HIP_TRY(hipEventSynchronize(v->ev1));
    HIP_TRY(hipEventElapsedTime(out_ms, v->ev0, v->ev1));
    return TTS_OK;
}

extern "C" void tts_vocoder_destroy(tts_vocoder* v)
{
    if (!v) return;
    if (v->ev0) (void)hipEventDestroy(v->ev0);
    if (v->ev1) (void)hipEventDestroy(v->ev1);
    delete v;
}
