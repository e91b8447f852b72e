// Host side of the tts_encoder C ABI: argument checks, arena carve-up, weight re-layout (LSTM gate rows permuted
// to unit-major / gate-minor), the per-call request table and the upload of the id sequences.  All arithmetic is
// in encoder.hip and conv5_kernels.h.
#include "../../include/tts_encoder.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "encoder_kernels.h"
#include "hostutil.h"

using namespace tts;

namespace {

int check(const tts_encoder_config* c)
{
    if (!c) return fail(TTS_E_INVAL, "config is null");
    if (c->dim != ENC_DIM || c->hid != ENC_HID)
        return fail(TTS_E_UNSUPPORTED, "kernels are built for width %d and %d units per direction", ENC_DIM, ENC_HID);
    for (int t = 0; t < ENC_TABLES; ++t)
        if (c->vocab[t] < 1 || c->vocab[t] > (1 << 20)) return fail(TTS_E_INVAL, "vocab[%d] must be in 1..2^20", t);
    if (c->max_len < 1 || c->max_len > 0x7FFF) return fail(TTS_E_INVAL, "max_len must be in 1..32767");
    if (c->max_tokens < c->max_len || c->max_tokens > (1 << 22)) return fail(TTS_E_INVAL, "max_tokens must be in max_len..2^22");
    if (c->weight_dtype != TTS_DTYPE_F32 && c->weight_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "weight_dtype must be 0 (fp32) or 1 (bf16)");
    return TTS_OK;
}

struct EncLayout {
    size_t tables[ENC_TABLES], conv_w[ENC_CONVS], conv_b[ENC_CONVS], w_ih[2], w_hh[2], b[2];
    size_t act[2], cmeta, orow, ids, xproj, total;
    size_t scratch_begin;      // everything from here on is cleared at creation
};

EncLayout layout_of(const tts_encoder_config& c)
{
    const size_t ws = c.weight_dtype == TTS_DTYPE_BF16 ? 2 : 4;
    const size_t cols = (size_t)(c.max_tokens + 15) / 16 * 16;
    Carver a;
    EncLayout l;
    for (int t = 0; t < ENC_TABLES; ++t) l.tables[t] = a.take((size_t)c.vocab[t] * ENC_DIM * 4);
    for (int i = 0; i < ENC_CONVS; ++i) {
        l.conv_w[i] = a.take((size_t)ENC_DIM * PN_TAPS * ENC_DIM * ws);
        l.conv_b[i] = a.take(ENC_DIM * 4);
    }
    for (int d = 0; d < 2; ++d) {
        l.w_ih[d] = a.take((size_t)ENC_GATES * ENC_DIM * ws);
        l.w_hh[d] = a.take((size_t)ENC_GATES * ENC_HID * ws);
        l.b[d] = a.take(ENC_GATES * 4);
    }
    l.scratch_begin = a.off;
    for (int i = 0; i < 2; ++i) l.act[i] = a.take(cols * ENC_DIM * ws);
    l.cmeta = a.take(cols * 4);
    l.orow = a.take(cols * 4);
    l.ids = a.take((size_t)ENC_TABLES * c.max_tokens * 4);
    l.xproj = a.take((size_t)2 * c.max_tokens * ENC_GATES * 4);
    l.total = a.off;
    return l;
}

// gate row r of the permuted matrices = (unit r / 4, gate r % 4); the caller's rows are gate * hid + unit
inline int source_row(int r) { return (r % 4) * ENC_HID + r / 4; }

}  // namespace

struct tts_encoder {
    tts_encoder_config cfg;
    EncoderPtrs d;
    hipStream_t stream = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    bool ev_valid = false;
    int* h_ids = nullptr;            // pinned staging buffer [tables][max_tokens]: the caller's ids leave its memory at once
    hipEvent_t ev_copied = nullptr;  // the staging buffer has been read by the last call's copies
    bool copy_pending = false;
};

extern "C" size_t tts_encoder_workspace_bytes(const tts_encoder_config* cfg)
{
    if (check(cfg) != TTS_OK) return 0;
    return layout_of(*cfg).total;
}

extern "C" int tts_encoder_create(const tts_encoder_config* cfg, const tts_encoder_weights* w, void* dev_arena,
                                  size_t arena_bytes, void* hip_stream, tts_encoder** out)
{
    if (!out) return fail(TTS_E_INVAL, "out is null");
    *out = nullptr;
    int rc = check(cfg);
    if (rc) return rc;
    if (!w || !dev_arena) return fail(TTS_E_INVAL, "null argument");
    bool all = true;
    for (int t = 0; t < ENC_TABLES; ++t) all = all && w->tables[t];
    for (int i = 0; i < ENC_CONVS; ++i) all = all && w->conv_w[i] && w->conv_b[i];
    for (int d = 0; d < 2; ++d) all = all && w->w_ih[d] && w->w_hh[d] && w->b[d];
    if (!all) return fail(TTS_E_INVAL, "a weight pointer is null");
    const EncLayout lay = layout_of(*cfg);
    if (arena_bytes < lay.total) return fail(TTS_E_INVAL, "arena has %zu bytes, %zu needed", arena_bytes, lay.total);
    if ((uintptr_t)dev_arena % 256) return fail(TTS_E_INVAL, "arena must be 256-byte aligned");
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, dev_arena) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(TTS_E_INVAL, "arena is not device memory");
    }
    tts_encoder* e = new (std::nothrow) tts_encoder();
    if (!e) return fail(TTS_E_INVAL, "out of host memory");
    e->cfg = *cfg;
    e->stream = (hipStream_t)hip_stream;
    char* base = (char*)dev_arena;
    const bool bf = cfg->weight_dtype == TTS_DTYPE_BF16;
    for (int t = 0; t < ENC_TABLES && rc == TTS_OK; ++t)
        rc = upload(base + lay.tables[t], std::vector<float>(w->tables[t], w->tables[t] + (size_t)cfg->vocab[t] * ENC_DIM), false);
    for (int i = 0; i < ENC_CONVS && rc == TTS_OK; ++i) {
        const float* src = w->conv_w[i];
        // GEMM row = output channel, k = tap * dim + input channel
        rc = upload(base + lay.conv_w[i], pack_fragments(ENC_DIM, PN_TAPS * ENC_DIM, bf, [&](int r, int k) {
                        const int tap = k / ENC_DIM, c = k - tap * ENC_DIM;
                        return src[((size_t)r * ENC_DIM + c) * PN_TAPS + tap];
                    }), bf);
        if (rc == TTS_OK) rc = upload(base + lay.conv_b[i], std::vector<float>(w->conv_b[i], w->conv_b[i] + ENC_DIM), false);
    }
    for (int d = 0; d < 2 && rc == TTS_OK; ++d) {
        const float *ih = w->w_ih[d], *hh = w->w_hh[d], *bb = w->b[d];
        rc = upload(base + lay.w_ih[d], pack_fragments(ENC_GATES, ENC_DIM, bf, [&](int r, int k) { return ih[(size_t)source_row(r) * ENC_DIM + k]; }), bf);
        if (rc == TTS_OK)
            rc = upload(base + lay.w_hh[d], pack_fragments(ENC_GATES, ENC_HID, bf, [&](int r, int k) { return hh[(size_t)source_row(r) * ENC_HID + k]; }), bf);
        if (rc == TTS_OK) {
            std::vector<float> bp(ENC_GATES);
            for (int r = 0; r < ENC_GATES; ++r) bp[r] = bb[source_row(r)];
            rc = upload(base + lay.b[d], bp, false);
        }
    }
    if (rc == TTS_OK && hipMemset(base + lay.scratch_begin, 0, lay.total - lay.scratch_begin) != hipSuccess)
        rc = fail(TTS_E_HIP, "clearing the activation buffers failed");
    if (rc == TTS_OK && (hipEventCreate(&e->ev0) != hipSuccess || hipEventCreate(&e->ev1) != hipSuccess ||
                         hipEventCreate(&e->ev_copied) != hipSuccess))
        rc = fail(TTS_E_HIP, "hipEventCreate failed");
    if (rc == TTS_OK && hipHostMalloc((void**)&e->h_ids, (size_t)ENC_TABLES * cfg->max_tokens * 4, hipHostMallocDefault) != hipSuccess)
        rc = fail(TTS_E_HIP, "hipHostMalloc of the id staging buffer failed");
    if (rc) {
        tts_encoder_destroy(e);
        return rc;
    }
    EncoderPtrs& p = e->d;
    for (int t = 0; t < ENC_TABLES; ++t) p.tables[t] = (const float*)(base + lay.tables[t]);
    for (int i = 0; i < ENC_CONVS; ++i) {
        p.conv_w[i] = base + lay.conv_w[i];
        p.conv_b[i] = (const float*)(base + lay.conv_b[i]);
    }
    for (int d = 0; d < 2; ++d) {
        p.w_ih[d] = base + lay.w_ih[d];
        p.w_hh[d] = base + lay.w_hh[d];
        p.b[d] = (const float*)(base + lay.b[d]);
    }
    p.act[0] = base + lay.act[0];
    p.act[1] = base + lay.act[1];
    p.cmeta = (int*)(base + lay.cmeta);
    p.orow = (int*)(base + lay.orow);
    p.ids = (int*)(base + lay.ids);
    p.xproj = (float*)(base + lay.xproj);
    p.max_tokens = cfg->max_tokens;
    *out = e;
    return TTS_OK;
}

extern "C" int tts_encoder_run(tts_encoder* e, const int* ids, const int* lens, int n, float* d_out)
{
    if (!e || !ids || !lens || !d_out) return fail(TTS_E_INVAL, "null argument");
    if (n < 1 || n > ENC_MAX_BATCH) return fail(TTS_E_INVAL, "n = %d requests, at most %d per call", n, ENC_MAX_BATCH);
    PnWindows w;
    w.n = n;
    long long total = 0;
    for (int i = 0; i < n; ++i) {
        if (lens[i] < 1 || lens[i] > e->cfg.max_len) return fail(TTS_E_INVAL, "request %d has %d tokens, max_len = %d", i, lens[i], e->cfg.max_len);
        w.col0[i] = (int)total;
        w.row0[i] = (int)total;
        w.len[i] = (uint16_t)lens[i];
        w.keep[i] = 0;
        total += lens[i];
        if (total > e->cfg.max_tokens) return fail(TTS_E_INVAL, "more than max_tokens = %d tokens in one call", e->cfg.max_tokens);
    }
    const int n_col = (int)total;
    // every id must address a row of its table: the device does not check
    for (int t = 0; t < ENC_TABLES; ++t)
        for (int c = 0; c < n_col; ++c) {
            const int id = ids[(size_t)t * n_col + c];
            if (id < 0 || id >= e->cfg.vocab[t]) return fail(TTS_E_INVAL, "table %d, token %d: id %d outside [0, %d)", t, c, id, e->cfg.vocab[t]);
        }
    if (e->copy_pending) HIP_TRY(hipEventSynchronize(e->ev_copied));      // the previous call's copies have read the staging buffer
    for (int t = 0; t < ENC_TABLES; ++t) memcpy(e->h_ids + (size_t)t * e->cfg.max_tokens, ids + (size_t)t * n_col, (size_t)n_col * 4);
    HIP_TRY(hipEventRecord(e->ev0, e->stream));
    for (int t = 0; t < ENC_TABLES; ++t)
        HIP_TRY(hipMemcpyAsync(e->d.ids + (size_t)t * e->cfg.max_tokens, e->h_ids + (size_t)t * e->cfg.max_tokens, (size_t)n_col * 4,
                               hipMemcpyHostToDevice, e->stream));
    HIP_TRY(hipEventRecord(e->ev_copied, e->stream));
    e->copy_pending = true;
    HIP_TRY(launch_encoder(e->d, e->cfg.weight_dtype, w, n_col, d_out, e->stream));
    HIP_TRY(hipEventRecord(e->ev1, e->stream));
    e->ev_valid = true;
    return TTS_OK;
}

extern "C" int tts_encoder_elapsed_ms(tts_encoder* e, float* out_ms)
{
    if (!e || !out_ms) return fail(TTS_E_INVAL, "null argument");
    if (!e->ev_valid) return fail(TTS_E_INVAL, "nothing has run yet");
    HIP_TRY(hipEventSynchronize(e->ev1));
    HIP_TRY(hipEventElapsedTime(out_ms, e->ev0, e->ev1));
    return TTS_OK;
}

extern "C" void tts_encoder_destroy(tts_encoder* e)
{
    if (!e) return;
    if (e->ev0) (void)hipEventDestroy(e->ev0);
    if (e->ev1) (void)hipEventDestroy(e->ev1);
    if (e->ev_copied) (void)hipEventDestroy(e->ev_copied);
    if (e->h_ids) (void)hipHostFree(e->h_ids);
    delete e;
}
