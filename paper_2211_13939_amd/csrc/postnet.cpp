// Host side of the tts_postnet C ABI: argument checks, arena carve-up, weight re-layout, the
// per-call column tables.  All arithmetic is in postnet.hip.
#include "../../include/tts_postnet.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "hostutil.h"
#include "postnet_kernels.h"

using namespace tts;

namespace {

int check(const tts_postnet_config* c)
{
    if (!c) return fail(TTS_E_INVAL, "config is null");
    if (c->n_mel != PN_N_MEL || c->channels != PN_CHANNELS)
        return fail(TTS_E_UNSUPPORTED, "kernels are built for %d mel bins and %d channels", PN_N_MEL, PN_CHANNELS);
    if (c->max_columns < 1 || c->max_columns > (1 << 20)) return fail(TTS_E_INVAL, "max_columns must be in 1..2^20");
    if (c->weight_dtype != TTS_DTYPE_F32 && c->weight_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "weight_dtype must be 0 (fp32) or 1 (bf16)");
    return TTS_OK;
}

int c_in_of(int l) { return l == 0 ? PN_N_MEL : PN_CHANNELS; }
int c_in_padded(int l) { return l == 0 ? PN_CIN0 : PN_CHANNELS; }
int c_out_of(int l) { return l == PN_LAYERS - 1 ? PN_COUT_LAST : PN_CHANNELS; }

struct PnLayout {
    size_t W[PN_LAYERS], b[PN_LAYERS], act[2], cmeta, orow, total;
};

PnLayout layout_of(const tts_postnet_config& c)
{
    const size_t ws = c.weight_dtype == TTS_DTYPE_BF16 ? 2 : 4;
    const size_t cols = (size_t)(c.max_columns + 15) / 16 * 16;
    Carver a;
    PnLayout l;
    for (int i = 0; i < PN_LAYERS; ++i) {
        l.W[i] = a.take((size_t)c_out_of(i) * PN_TAPS * c_in_padded(i) * ws);
        l.b[i] = a.take((size_t)c_out_of(i) * 4);
    }
    for (int i = 0; i < 2; ++i) l.act[i] = a.take(cols * PN_CHANNELS * ws);
    l.cmeta = a.take(cols * 4);
    l.orow = a.take(cols * 4);
    l.total = a.off;
    return l;
}

}  // namespace

struct tts_postnet {
    tts_postnet_config cfg;
    PostnetPtrs d;
    int device = -1;              // the device the arena (hence the weights) lives on
    hipStream_t stream = nullptr;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    bool ev_valid = false;
};

// ---- scratch of the entry point that allocates nothing (tts_postnet_run_static): the activations between layers and
// the per-column tables of one call, for up to TTS_POSTNET_STATIC_MAX_COLUMNS columns of fp32 activations.  One copy
// per GPU, at its own address, held until the process ends; every call on a GPU uses it, so calls that overlap on one
// GPU race.  The array's name is only a host-side handle: the address the kernels get is looked up once per device.
namespace {
constexpr size_t PN_STATIC_COLS = TTS_POSTNET_STATIC_MAX_COLUMNS;
static_assert(PN_STATIC_COLS % 16 == 0, "whole column tiles");
constexpr size_t PN_STATIC_ACT = PN_STATIC_COLS * PN_CHANNELS * 4;     // one activation buffer, fp32 (bf16 uses half of it)
constexpr size_t PN_STATIC_TABLE = PN_STATIC_COLS * 4;
constexpr size_t PN_STATIC_BYTES = 2 * PN_STATIC_ACT + 2 * PN_STATIC_TABLE;
static_assert(PN_STATIC_BYTES == TTS_POSTNET_STATIC_BYTES, "the size the header states");
constexpr int PN_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[PN_STATIC_BYTES];
static unsigned char* g_scratch[PN_MAX_DEVICES];   // per device: where that GPU's copy of `scratch` lives (null: not looked up yet)

// the address of the current device's copy of `scratch` (looked up on the first call on that device)
static int static_scratch(int device, unsigned char** out)
{
    if (device < 0 || device >= PN_MAX_DEVICES) return fail(TTS_E_UNSUPPORTED, "device %d: at most %d devices", device, PN_MAX_DEVICES);
    if (!g_scratch[device]) {
        int cur = -1;
        HIP_TRY(hipGetDevice(&cur));
        if (cur != device) return fail(TTS_E_INVAL, "device %d is current, the PostNet lives on device %d", cur, device);
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(TTS_E_HIP, "no device address for the static scratch array");
        g_scratch[device] = static_cast<unsigned char*>(ptr);
    }
    *out = g_scratch[device];
    return TTS_OK;
}

extern "C" size_t tts_postnet_workspace_bytes(const tts_postnet_config* cfg)
{
    if (check(cfg) != TTS_OK) return 0;
    return layout_of(*cfg).total;
}

extern "C" int tts_postnet_create(const tts_postnet_config* cfg, const tts_postnet_weights* w, void* dev_arena,
                                  size_t arena_bytes, void* hip_stream, tts_postnet** out)
{
    if (!out) return fail(TTS_E_INVAL, "out is null");
    *out = nullptr;
    int rc = check(cfg);
    if (rc) return rc;
    if (!w || !dev_arena) return fail(TTS_E_INVAL, "null argument");
    for (int l = 0; l < PN_LAYERS; ++l)
        if (!w->conv_w[l] || !w->conv_b[l]) return fail(TTS_E_INVAL, "weights of layer %d are null", l);
    const PnLayout lay = layout_of(*cfg);
    if (arena_bytes < lay.total) return fail(TTS_E_INVAL, "arena has %zu bytes, %zu needed", arena_bytes, lay.total);
    if ((uintptr_t)dev_arena % 256) return fail(TTS_E_INVAL, "arena must be 256-byte aligned");
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, dev_arena) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(TTS_E_INVAL, "arena is not device memory");
    }
    tts_postnet* p = new (std::nothrow) tts_postnet();
    if (!p) return fail(TTS_E_INVAL, "out of host memory");
    p->cfg = *cfg;
    p->device = attr.device;
    p->stream = (hipStream_t)hip_stream;
    {
        // set-up is the place to look the static scratch array up (tts_postnet_run_static may run where nothing but
        // launches is allowed); if another device is current now, the first call on the arena's device does it
        int cur = -1;
        unsigned char* unused = nullptr;
        if (hipGetDevice(&cur) == hipSuccess && cur == attr.device) rc = static_scratch(attr.device, &unused);
    }
    char* base = (char*)dev_arena;
    const bool bf = cfg->weight_dtype == TTS_DTYPE_BF16;
    for (int l = 0; l < PN_LAYERS && rc == TTS_OK; ++l) {
        const int ci = c_in_of(l), cip = c_in_padded(l), co = c_out_of(l);
        const float* src = w->conv_w[l];
        // GEMM row = output channel, k = tap * (padded input channels) + input channel
        rc = upload(base + lay.W[l], pack_fragments(co, PN_TAPS * cip, bf, [&](int r, int k) {
                        const int tap = k / cip, c = k - tap * cip;
                        return c < ci ? src[((size_t)r * ci + c) * PN_TAPS + tap] : 0.f;
                    }), bf);
        if (rc == TTS_OK) rc = upload(base + lay.b[l], std::vector<float>(w->conv_b[l], w->conv_b[l] + co), false);
        p->d.W[l] = base + lay.W[l];
        p->d.b[l] = (const float*)(base + lay.b[l]);
    }
    if (rc == TTS_OK && hipMemset(base + lay.act[0], 0, lay.total - lay.act[0]) != hipSuccess)
        rc = fail(TTS_E_HIP, "clearing the activation buffers failed");
    if (rc == TTS_OK && (hipEventCreate(&p->ev0) != hipSuccess || hipEventCreate(&p->ev1) != hipSuccess))
        rc = fail(TTS_E_HIP, "hipEventCreate failed");
    if (rc) {
        tts_postnet_destroy(p);
        return rc;
    }
    p->d.act[0] = base + lay.act[0];
    p->d.act[1] = base + lay.act[1];
    p->d.cmeta = (int*)(base + lay.cmeta);
    p->d.orow = (int*)(base + lay.orow);
    p->d.n_mel = cfg->n_mel;
    *out = p;
    return TTS_OK;
}

// one dynamic batch with the scratch of `d` (the arena's, or the static array's); `timed`: HIP events around it
static int run_batch(tts_postnet* p, const PostnetPtrs& d, int max_columns, bool timed, const float* d_mel, const int* win_len,
                     const int* keep_from, int n, float* d_out)
{
    if (!p || !d_mel || !win_len || !keep_from || !d_out) return fail(TTS_E_INVAL, "null argument");
    if (n < 1) return fail(TTS_E_INVAL, "n = %d windows", n);
    long long cols = 0;
    for (int i = 0; i < n; ++i) {
        if (win_len[i] < 1 || win_len[i] > 0x7FFF) return fail(TTS_E_INVAL, "window %d has %d frames", i, win_len[i]);
        if (keep_from[i] < 0 || keep_from[i] >= win_len[i])
            return fail(TTS_E_INVAL, "window %d: keep_from = %d outside [0, %d)", i, keep_from[i], win_len[i]);
        cols += win_len[i];
    }
    if (cols > max_columns) return fail(TTS_E_INVAL, "%lld frames in one call, at most %d fit", cols, max_columns);
    const int n_col = (int)cols, n_pad = (n_col + 15) / 16 * 16;
    // the window list travels as kernel arguments, 256 windows at a time; the device expands it into the
    // per-column tables (position inside the window for the zero padding, output row of the column)
    if (timed) HIP_TRY(hipEventRecord(p->ev0, p->stream));
    int c = 0, r = 0;
    for (int i0 = 0; i0 < n; i0 += PN_META_WINDOWS) {
        PnWindows w;
        w.n = n - i0 < PN_META_WINDOWS ? n - i0 : PN_META_WINDOWS;
        for (int k = 0; k < w.n; ++k) {
            const int i = i0 + k;
            w.col0[k] = c;
            w.row0[k] = r;
            w.len[k] = (uint16_t)win_len[i];
            w.keep[k] = (uint16_t)keep_from[i];
            c += win_len[i];
            r += win_len[i] - keep_from[i];
        }
        HIP_TRY(launch_postnet_meta(d, w, n_col, n_pad, i0 == 0, p->stream));
    }
    HIP_TRY(launch_postnet(d, p->cfg.weight_dtype, d_mel, n_col, d_out, p->stream));
    if (timed) {
        HIP_TRY(hipEventRecord(p->ev1, p->stream));
        p->ev_valid = true;
    }
    return TTS_OK;
}

extern "C" int tts_postnet_run(tts_postnet* p, const float* d_mel, const int* win_len, const int* keep_from, int n,
                               float* d_out)
{
    if (!p) return fail(TTS_E_INVAL, "null argument");
    return run_batch(p, p->d, p->cfg.max_columns, true, d_mel, win_len, keep_from, n, d_out);
}

extern "C" int tts_postnet_run_static(tts_postnet* p, const float* d_mel, const int* win_len, const int* keep_from, int n,
                                      float* d_out)
{
    if (!p) return fail(TTS_E_INVAL, "null argument");
    unsigned char* base = nullptr;
    int rc = static_scratch(p->device, &base);
    if (rc) return rc;
    // the same kernels, their scratch in this GPU's copy of the static array instead of the arena.  A call writes every
    // word of it that it reads (tables and activations of all its column tiles, padding columns included), so nothing
    // has to start at zero and what the previous call left is never seen.
    PostnetPtrs d = p->d;
    d.act[0] = base;
    d.act[1] = base + PN_STATIC_ACT;
    d.cmeta = reinterpret_cast<int*>(base + 2 * PN_STATIC_ACT);
    d.orow = reinterpret_cast<int*>(base + 2 * PN_STATIC_ACT + PN_STATIC_TABLE);
    return run_batch(p, d, TTS_POSTNET_STATIC_MAX_COLUMNS, false, d_mel, win_len, keep_from, n, d_out);
}

extern "C" int tts_postnet_elapsed_ms(tts_postnet* p, float* out_ms)
{
    if (!p || !out_ms) return fail(TTS_E_INVAL, "null argument");
    if (!p->ev_valid) return fail(TTS_E_INVAL, "nothing has run yet");
    HIP_TRY(hipEventSynchronize(p->ev1));
    HIP_TRY(hipEventElapsedTime(out_ms, p->ev0, p->ev1));
    return TTS_OK;
}

extern "C" void tts_postnet_destroy(tts_postnet* p)
{
    if (!p) return;
    if (p->ev0) (void)hipEventDestroy(p->ev0);
    if (p->ev1) (void)hipEventDestroy(p->ev1);
    delete p;
}
