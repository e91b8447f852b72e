// Host side of the tts_pool C ABI: argument checks, arena carve-up, weight
// re-layout, pool bookkeeping, kernel / graph launches.  All arithmetic of the
// decoder step lives in kernels.hip.
#include "../../include/tts_pool.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "book.h"
#include "dev.h"
#include "hostutil.h"
#include "kernels.h"

using namespace tts;

// ------------------------------------------------------------------ errors
static thread_local std::string g_err;

int tts::fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

extern "C" const char* tts_last_error(void) { return g_err.c_str(); }

// ------------------------------------------------------------------ config
static int check_config(const tts_config* c)
{
    if (!c) return fail(TTS_E_INVAL, "config is null");
    if (c->n_mel != N_MEL || c->prenet_dim != PRENET || c->enc_dim != ENC || c->att_rnn_dim != HID ||
        c->dec_rnn_dim != HID || c->att_dim != ATT || c->loc_filters != LOC_F || c->loc_kernel != LOC_K ||
        (c->loc_in_channels != 1 && c->loc_in_channels != 2))
        return fail(TTS_E_UNSUPPORTED,
                    "kernels are built for dims 80/256/512/1024/1024/128, 32 filters, kernel 31, 1 or 2 channels");
    if (c->max_pool < 1 || c->max_pool > MAX_POOL) return fail(TTS_E_INVAL, "max_pool must be in 1..%d", MAX_POOL);
    if (c->max_enc_len < 1 || c->max_enc_len > MAX_ENC_LEN)
        return fail(TTS_E_INVAL, "max_enc_len must be in 1..%d", MAX_ENC_LEN);
    if (c->max_steps < 1 || c->max_steps > (1 << 20)) return fail(TTS_E_INVAL, "max_steps must be in 1..2^20");
    if (c->chunk_frames < 1) return fail(TTS_E_INVAL, "chunk_frames must be >= 1");
    if (c->weight_dtype != TTS_DTYPE_F32 && c->weight_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "weight_dtype must be 0 (fp32) or 1 (bf16)");
    if (c->memory_dtype != TTS_DTYPE_F32 && c->memory_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "memory_dtype must be 0 (fp32) or 1 (bf16)");
    if (c->memory_dtype == TTS_DTYPE_BF16 && c->weight_dtype != TTS_DTYPE_BF16)
        return fail(TTS_E_INVAL, "bf16 memory requires bf16 weights");
    // the cumulative attention weights (at most one per frame and position) are a half-precision MFMA operand there
    if (c->weight_dtype == TTS_DTYPE_BF16 && c->max_steps > 65504)
        return fail(TTS_E_INVAL, "max_steps must be at most 65504 with bf16 weights");
    return TTS_OK;
}

// ------------------------------------------------------------------ arena
namespace {

struct Layout {
    size_t Wa, Wd, ba, bd, Wq, Wq_epi, qpart, pre_att, pre_dec, pre_dec_b, proj_part, WmemT, lsa_kfrag, lsa_wfrag, v, Wmel, bmel, Wp1, Wp2;
    size_t xatt[2], xdec[2], c_att, c_dec, m_last, w_last[2], w_acc[2], Fmem, PM, mel_ring, stop_ring;
    size_t L, t, n_steps, done, failed, live, proj_seq, step_seq, lsa_x, hdec_x, p_x, pre_x, wg_seq, stage;
    size_t total, proj_part_bytes;
};

// Gate pre-sums: the projection kernel needs a handful of CUs, so its launch also contracts what the next step's LSTMs
// already have of their inputs ([A; H_att] of the attention LSTM; in pools of at most four tiles also H_dec of the
// decoder LSTM).  The attention LSTM, left with K = 256, then runs as tall tiles and hands the attention query over as
// 32 rank-32 partial products per slot (16 KB) instead of the attention kernel pulling W_q (256 KB in bf16) through
// each of its CUs.  Fixed per pool (it changes the order in which gates and query are summed): a request's bits do
// not depend on what else the pool holds.  Every bf16 pool has them; fp32 pools up to four tiles (the pre-sum
// workgroups of larger pools hold several row tiles' fragments in registers, which fp32 fragments do not fit).
bool pre_gates_for(const tts_config& c)
{
    return (c.max_pool + 15) / 16 <= PRESUM_SMALL_TILES || c.weight_dtype == TTS_DTYPE_BF16;
}
// the decoder LSTM's pre-sum too: only where the pre-sum workgroups still finish in the projection's shadow (beyond four
// tiles it saved the decoder LSTM 1.8 us and kept the projection's launch 5 us longer)
bool pre_dec_for(const tts_config& c) { return pre_gates_for(c) && (c.max_pool + 15) / 16 <= PRESUM_SMALL_TILES; }
// and its sums over H_att formed beside the attention kernel, in the same launch: that kernel is a chain of waits that
// leaves a CU's load path idle, and two of its workgroups fit a CU only with two-byte operands and memory
bool pre_dec_hatt_for(const tts_config& c) { return pre_dec_for(c) && c.weight_dtype == TTS_DTYPE_BF16 && c.memory_dtype == TTS_DTYPE_BF16; }
// pools whose last kernel's launch holds the decoder LSTM and hands H_dec to the projection as words: those, and pools of
// more than 64 slots with two-byte weights
bool hdec_words_for(const tts_config& c) { return pre_dec_hatt_for(c) || (pre_gates_for(c) && !pre_dec_for(c) && c.weight_dtype == TTS_DTYPE_BF16); }
// workgroups per pool tile in the projection kernel: with pre-sums they must fit XCD 0 (32 CUs)
int proj_group_for(const tts_config& c)
{
    const int tiles = (c.max_pool + 15) / 16;
    if (!pre_gates_for(c) || tiles <= 5) return 6;
    return tiles <= 10 ? 3 : 2;
}

Layout make_layout(const tts_config& c)
{
    const size_t ws = c.weight_dtype == TTS_DTYPE_BF16 ? 2 : 4;
    const size_t ms = c.memory_dtype == TTS_DTYPE_BF16 ? 2 : 4;
    const size_t S = (size_t)((c.max_pool + 15) / 16) * 16, ML = c.max_enc_len;   // slots padded to whole 16-slot tiles
    Carver a;
    Layout l;
    l.Wa = a.take((size_t)4 * HID * K_ATT * ws);
    l.Wd = a.take((size_t)4 * HID * K_DEC * ws);
    l.ba = a.take((size_t)4 * HID * 4);
    l.bd = a.take((size_t)4 * HID * 4);
    l.Wq = a.take((size_t)ATT * HID * ws);
    l.Wq_epi = a.take((size_t)ATT * HID * 4);
    l.WmemT = a.take((size_t)ENC * ATT * 4);
    l.lsa_kfrag = a.take((size_t)2 * 16 * 64 * 4);
    l.lsa_wfrag = a.take((size_t)16 * 64 * 16);
    l.v = a.take((size_t)ATT * 4);
    l.Wmel = a.take((size_t)96 * K_PROJ * ws);
    l.bmel = a.take((size_t)N_PROJ * 4);
    l.Wp1 = a.take((size_t)PRENET * 96 * ws);
    l.Wp2 = a.take((size_t)PRENET * PRENET * ws);
    for (int b = 0; b < 2; ++b) {
        l.xatt[b] = a.take(S * K_ATT * ws);
        l.xdec[b] = a.take(S * K_DEC * ws);
    }
    l.qpart = a.take((pre_gates_for(c) ? S : 0) * (size_t)QUERY_PARTIALS * ATT * 4);
    l.pre_att = a.take((pre_gates_for(c) ? S / 16 : 0) * (size_t)(HID / 4) * 64 * 16);
    l.pre_dec = a.take((pre_dec_for(c) ? S / 16 : 0) * (size_t)(HID / 4) * 64 * 16);
    l.pre_dec_b = a.take((pre_dec_hatt_for(c) ? S / 16 : 0) * (size_t)(HID / 4) * 64 * 16);
    l.proj_part_bytes = (S / 16) * (size_t)PROJ_GROUP * 96 * 16 * 8;   // (in the fused form every worker hands its sums over)
    l.proj_part = a.take(l.proj_part_bytes);
    l.c_att = a.take(S * HID * 4);
    l.c_dec = a.take(S * HID * 4);
    l.m_last = a.take(S * N_MEL * 4);
    for (int b = 0; b < 2; ++b) {
        l.w_last[b] = a.take(S * ML * 4);
        l.w_acc[b] = a.take(S * ML * 4);
    }
    l.Fmem = a.take(S * ML * ENC * ms);
    l.PM = a.take(S * ML * ATT * ms);
    l.mel_ring = a.take(S * (size_t)c.max_steps * N_MEL * 4);
    l.stop_ring = a.take(S * (size_t)c.max_steps * 4);
    l.L = a.take(S * 4);
    l.t = a.take(S * 4);
    l.n_steps = a.take(S * 4);
    l.done = a.take(S * 4);
    l.failed = a.take(S * 4);
    l.live = a.take(MAX_POOL * 4);
    l.proj_seq = a.take((size_t)MAX_TILES * PROJ_GROUP * 4);     // zeroed at creation with the counters above
    l.step_seq = a.take(4);
    l.lsa_x = a.take(S * ML * 8);                        // zeroed too: no word carries a step's number yet
    l.hdec_x = a.take((hdec_words_for(c) ? S / 16 : 0) * (size_t)(HID / 32) * 64 * 4 * 8);   // likewise
    l.p_x = a.take((pre_dec_hatt_for(c) ? S / 16 : 0) * (size_t)(PRENET / 32) * 64 * 4 * 8);
    l.pre_x = a.take((pre_dec_hatt_for(c) ? S / 16 : 0) * (size_t)(HID / 4) * 64 * 4 * 8);
    l.wg_seq = a.take(2 * 4);
    l.stage = a.take(ML * ENC * 4);
    l.total = a.off;
    return l;
}

// Gate matrix [W_ih | W_hh] (rows i,f,g,o blocks of HID): rows re-ordered
// unit-major/gate-minor so that one 16-row tile is the four gates of four units.
std::vector<float> gate_fragments(const float* w_ih, int in_dim, const float* w_hh, bool bf16)
{
    return pack_fragments(4 * HID, in_dim + HID, bf16, [&](int r, int k) {
        const int unit = r >> 2, gate = r & 3;
        const int src_row = gate * HID + unit;
        return k < in_dim ? w_ih[(size_t)src_row * in_dim + k] : w_hh[(size_t)src_row * HID + (k - in_dim)];
    });
}

// Location filters and W_loc as the per-lane constant A operands of the
// attention kernel.  Channel 0 of the kernel is W_last, channel 1 W_acc (a
// one-channel model convolves W_acc only); taps are padded from 31 to 32.
// Lane = (jl = lane%16, g = lane/16).
void lsa_fragments(const float* loc_conv, int C, const float* loc_w, bool bf16,
                   std::vector<float>* kfrag, std::vector<float>* wfrag)
{
    auto tap = [&](int f, int cd, int k) -> float {
        if (k >= LOC_K) return 0.f;
        if (C == 2) return loc_conv[((size_t)f * 2 + cd) * LOC_K + k];
        return cd == 1 ? loc_conv[(size_t)f * LOC_K + k] : 0.f;
    };
    auto wrow = [&](int at, int jl) { return 32 * (jl >> 2) + 4 * at + (jl & 3); };
    if (!bf16) {
        // kfrag[(mt*16 + c*8 + s)*64 + lane] = tap 4s+g of channel c, filter 16mt+jl
        kfrag->assign((size_t)32 * 64, 0.f);
        for (int mt = 0; mt < 2; ++mt)
            for (int cs = 0; cs < 16; ++cs)
                for (int lane = 0; lane < 64; ++lane)
                    (*kfrag)[((size_t)mt * 16 + cs) * 64 + lane] =
                        tap(16 * mt + (lane & 15), cs >> 3, 4 * (cs & 7) + (lane >> 4));
        // wfrag[((at*2 + mt)*64 + lane)*4 + i] = W_loc[row(at,jl)][16mt + 4g + i]
        wfrag->assign((size_t)16 * 64 * 4, 0.f);
        for (int at = 0; at < 8; ++at)
            for (int mt = 0; mt < 2; ++mt)
                for (int lane = 0; lane < 64; ++lane)
                    for (int i = 0; i < 4; ++i)
                        (*wfrag)[(((size_t)at * 2 + mt) * 64 + lane) * 4 + i] =
                            loc_w[(size_t)wrow(at, lane & 15) * LOC_F + 16 * mt + 4 * (lane >> 4) + i];
    } else {
        // kfrag[((mt*2 + c)*64 + lane)*8 + e] = tap 8g+e of channel c, filter 16mt+jl
        kfrag->assign((size_t)4 * 64 * 8, 0.f);
        for (int mt = 0; mt < 2; ++mt)
            for (int c = 0; c < 2; ++c)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e)
                        (*kfrag)[(((size_t)mt * 2 + c) * 64 + lane) * 8 + e] =
                            tap(16 * mt + (lane & 15), c, 8 * (lane >> 4) + e);
        // wfrag[(at*64 + lane)*8 + e] = W_loc[row(at,jl)][e < 4 ? 4g+e : 16+4g+e-4]
        wfrag->assign((size_t)8 * 64 * 8, 0.f);
        for (int at = 0; at < 8; ++at)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 8; ++e) {
                    const int g = lane >> 4;
                    const int f = e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4);
                    (*wfrag)[((size_t)at * 64 + lane) * 8 + e] = loc_w[(size_t)wrow(at, lane & 15) * LOC_F + f];
                }
    }
}

}  // namespace

extern "C" size_t tts_pool_workspace_bytes(const tts_config* cfg)
{
    if (check_config(cfg) != TTS_OK) return 0;
    return make_layout(*cfg).total;
}

// ------------------------------------------------------------------ pool
struct tts_pool {
    tts_config cfg;
    DevPtrs d;
    hipStream_t stream = nullptr;
    std::unique_ptr<PoolBook> book;
    int parity = 0;               // activation buffer half the next step reads
    long long n_moves = 0;        // requests moved to lower slots since creation
    int slot_span = 0;            // highest active slot + 1 (as last uploaded): what the per-slot grids must cover
    bool stop_enabled = false;
    bool timing = false;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    bool ev_valid = false;
    std::map<int, hipGraphExec_t> graphs;   // key = ((steps * 1024 + bucket) * 2 + parity
    std::vector<hipGraph_t> graph_defs;
    int* h_fault = nullptr;       // pinned, mapped: non-zero once a kernel's bounded wait has run out
    float* h_chunk = nullptr;     // pinned staging for one chunk on its way to the caller's (pageable) buffer: a copy from
                                  // the device into pinned memory is a plain DMA, one into pageable memory is staged by the
                                  // runtime at three times the cost
    int n_slots_padded = 0;       // slots the arena holds (max_pool rounded up to whole tiles)
    std::vector<int64_t> lost_ids; // requests the device ended early that tts_pool_sync has not reported yet
};

// After the stream has been waited for: did a workgroup's bounded wait run out since the last look?  The kernels froze
// the requests concerned on the device (no frame was stored for them from that step on, every other request went on);
// here the host's bookkeeping follows: each such request ends after the frames the device holds for it and is marked
// lost, the device's marks and the status word are cleared.  The ids wait in `lost_ids` for the next tts_pool_sync.
static int absorb_failures(tts_pool* p)
{
    if (!p->h_fault || !*p->h_fault) return TTS_OK;
    const int n = p->n_slots_padded;
    std::vector<int> failed(n), t(n);
    HIP_TRY(hipMemcpyAsync(failed.data(), p->d.failed, (size_t)n * 4, hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipMemcpyAsync(t.data(), p->d.t, (size_t)n * 4, hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipMemsetAsync(p->d.failed, 0, (size_t)n * 4, p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
    *p->h_fault = 0;
    for (int sl = 0; sl < n && sl < p->cfg.max_pool; ++sl) {
        if (!failed[sl] || p->book->slot(sl).state == SlotState::Free) continue;
        p->book->lose(sl, t[sl]);
        p->lost_ids.push_back(p->book->slot(sl).id);
    }
    return TTS_OK;
}

// what tts_pool_sync says about the requests lost since it last said so
static int report_lost(tts_pool* p)
{
    if (p->lost_ids.empty()) return TTS_OK;
    std::string ids;
    for (size_t i = 0; i < p->lost_ids.size() && i < 8; ++i) ids += (i ? ", " : "") + std::to_string((long long)p->lost_ids[i]);
    const size_t n = p->lost_ids.size();
    p->lost_ids.clear();
    return fail(TTS_E_LOST, "%zu request(s) ended early (id %s%s): a workgroup gave up waiting for the words of its partners; "
                "their frames so far are valid and can be drained, no further ones will come", n, ids.c_str(), n > 8 ? ", ..." : "");
}

static int upload_weights(tts_pool* p, const tts_weights* w, char* base, const Layout& l)
{
    const bool bf = p->cfg.weight_dtype == TTS_DTYPE_BF16;
    const int C = p->cfg.loc_in_channels;
    int rc;
    // LSTM gate matrices: attention LSTM sees [Pre(M_last); A] then H_att, decoder LSTM [H_att; A] then H_dec
    if ((rc = upload(base + l.Wa, gate_fragments(w->att_w_ih, PRENET + ENC, w->att_w_hh, bf), bf))) return rc;
    if ((rc = upload(base + l.Wd, gate_fragments(w->dec_w_ih, HID + ENC, w->dec_w_hh, bf), bf))) return rc;
    std::vector<float> ba(4 * HID), bd(4 * HID);
    for (int u = 0; u < HID; ++u)
        for (int g = 0; g < 4; ++g) {
            ba[u * 4 + g] = w->att_b[g * HID + u];
            bd[u * 4 + g] = w->dec_b[g * HID + u];
        }
    if ((rc = upload(base + l.ba, ba, false))) return rc;
    if ((rc = upload(base + l.bd, bd, false))) return rc;
    if ((rc = upload(base + l.Wq, pack_fragments(ATT, HID, bf, [&](int r, int k) { return w->q_w[(size_t)r * HID + k]; }), bf)))
        return rc;
    // W_q for the attention LSTM's epilogue: row tile rt of the gates = hidden units 4rt..4rt+3;
    // lane l of A operand `at` holds W_q[16 at + l%16][4 rt + l/16] (kept in fp32: the values of the
    // weight dtype; the product runs on the fp32 MFMA in both modes)
    std::vector<float> wq_epi((size_t)ATT * HID);
    for (int rt = 0; rt < HID / 4; ++rt)
        for (int at = 0; at < ATT / 16; ++at)
            for (int lane = 0; lane < 64; ++lane) {
                const float x = w->q_w[(size_t)(16 * at + (lane & 15)) * HID + 4 * rt + (lane >> 4)];
                wq_epi[((size_t)rt * (ATT / 16) + at) * 64 + lane] = bf ? host_bf2f(host_f2bf(x)) : x;
            }
    if ((rc = upload(base + l.Wq_epi, wq_epi, false))) return rc;
    std::vector<float> memT((size_t)ENC * ATT);
    for (int a = 0; a < ATT; ++a)
        for (int k = 0; k < ENC; ++k) memT[(size_t)k * ATT + a] = w->mem_w[(size_t)a * ENC + k];
    if ((rc = upload(base + l.WmemT, memT, false))) return rc;
    std::vector<float> kfrag, wfrag;
    lsa_fragments(w->loc_conv, C, w->loc_w, bf, &kfrag, &wfrag);
    if ((rc = upload(base + l.lsa_kfrag, kfrag, bf))) return rc;
    if ((rc = upload(base + l.lsa_wfrag, wfrag, bf))) return rc;
    if ((rc = upload(base + l.v, std::vector<float>(w->v, w->v + ATT), false))) return rc;
    // projection rows: 80 mel rows, the stop row, zero rows up to 96
    if ((rc = upload(base + l.Wmel, pack_fragments(96, K_PROJ, bf, [&](int r, int k) {
             return r < N_MEL ? w->mel_w[(size_t)r * K_PROJ + k] : (r == N_MEL ? w->stop_w[k] : 0.f);
         }), bf)))
        return rc;
    std::vector<float> bproj(N_PROJ);
    memcpy(bproj.data(), w->mel_b, N_MEL * 4);
    bproj[N_MEL] = w->stop_b[0];
    if ((rc = upload(base + l.bmel, bproj, false))) return rc;
    const int k1 = bf ? 96 : 80;   // the first prenet layer's K padded to whole fragments
    if ((rc = upload(base + l.Wp1, pack_fragments(PRENET, k1, bf, [&](int r, int k) {
             return k < N_MEL ? w->prenet1[(size_t)r * N_MEL + k] : 0.f;
         }), bf)))
        return rc;
    if ((rc = upload(base + l.Wp2, pack_fragments(PRENET, PRENET, bf, [&](int r, int k) {
             return w->prenet2[(size_t)r * PRENET + k];
         }), bf)))
        return rc;
    return TTS_OK;
}

extern "C" int tts_pool_create(const tts_config* cfg, const tts_weights* w, void* dev_arena, size_t arena_bytes,
                               void* hip_stream, tts_pool** out)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !out) return fail(TTS_E_INVAL, "weights / out is null");
    const float* const* wp = reinterpret_cast<const float* const*>(w);
    for (size_t i = 0; i < sizeof(tts_weights) / sizeof(float*); ++i)
        if (!wp[i]) return fail(TTS_E_INVAL, "weight tensor %zu is null", i);
    const Layout l = make_layout(*cfg);
    if (!dev_arena || ((uintptr_t)dev_arena & 255)) return fail(TTS_E_ARENA, "arena is null or not 256-byte aligned");
    if (arena_bytes < l.total) return fail(TTS_E_ARENA, "arena has %zu bytes, %zu needed", arena_bytes, l.total);
    if (cfg->use_graph && !hip_stream)
        return fail(TTS_E_INVAL, "graph capture needs a stream other than the default (null) stream");
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, dev_arena) != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(TTS_E_ARENA, "arena is not device memory");
    }
    // Workgroups of one launch wait for each other's words (the projection's helpers and leader, the attention
    // workgroups of a slot): every launch is laid out so that all its workgroups are resident at once on the 256 CUs
    // of an MI355X, one per CU.  On a device (or partition) with fewer they would wait for partners that cannot start.
    {
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, attr.device) != hipSuccess) {
            (void)hipGetLastError();
            return fail(TTS_E_HIP, "cannot read the device's CU count");
        }
        if (n_cu < MIN_DEVICE_CUS)
            return fail(TTS_E_UNSUPPORTED, "the device has %d CUs; the step kernels are laid out for %d", n_cu, MIN_DEVICE_CUS);
    }

    tts_pool* p = new (std::nothrow) tts_pool();
    if (!p) return fail(TTS_E_INVAL, "out of host memory");
    p->cfg = *cfg;
    p->stream = (hipStream_t)hip_stream;
    p->stop_enabled = cfg->stop_threshold >= 0.f && cfg->stop_threshold <= 1.f;
    p->book.reset(new PoolBook(cfg->max_pool, cfg->max_enc_len, cfg->max_steps, cfg->chunk_frames));
    p->n_slots_padded = (cfg->max_pool + 15) / 16 * 16;

    char* base = (char*)dev_arena;
    DevPtrs& d = p->d;
    d.Wa = (const uint4*)(base + l.Wa);
    d.Wd = (const uint4*)(base + l.Wd);
    d.ba = (const float*)(base + l.ba);
    d.bd = (const float*)(base + l.bd);
    d.Wq = base + l.Wq;
    d.Wq_epi = reinterpret_cast<const float*>(base + l.Wq_epi);
    d.qpart = pre_gates_for(*cfg) ? reinterpret_cast<float*>(base + l.qpart) : nullptr;
    d.pre_att = pre_gates_for(*cfg) ? reinterpret_cast<float*>(base + l.pre_att) : nullptr;
    d.pre_dec = pre_dec_for(*cfg) ? reinterpret_cast<float*>(base + l.pre_dec) : nullptr;
    d.pre_dec_b = pre_dec_hatt_for(*cfg) ? reinterpret_cast<float*>(base + l.pre_dec_b) : nullptr;
    d.proj_part = reinterpret_cast<unsigned long long*>(base + l.proj_part);
    d.proj_seq = reinterpret_cast<unsigned*>(base + l.proj_seq);
    d.step_seq = reinterpret_cast<unsigned*>(base + l.step_seq);
    d.lsa_x = reinterpret_cast<unsigned long long*>(base + l.lsa_x);
    d.hdec_x = hdec_words_for(*cfg) ? reinterpret_cast<unsigned long long*>(base + l.hdec_x) : nullptr;
    d.p_x = pre_dec_hatt_for(*cfg) ? reinterpret_cast<unsigned long long*>(base + l.p_x) : nullptr;
    d.pre_x = pre_dec_hatt_for(*cfg) ? reinterpret_cast<unsigned long long*>(base + l.pre_x) : nullptr;
    d.wg_seq = reinterpret_cast<unsigned*>(base + l.wg_seq);
    // one pinned word the kernels can reach: a projection leader that gives up on its helpers says so here
    {
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&p->h_fault), sizeof(int), hipHostMallocMapped);
        if (e == hipSuccess) {
            *p->h_fault = 0;
            e = hipHostGetDevicePointer(reinterpret_cast<void**>(&d.fault), p->h_fault, 0);
        }
        if (e != hipSuccess) {
            const int rc0 = fail(TTS_E_HIP, "pinned status word: %s", hipGetErrorString(e));
            tts_pool_destroy(p);
            return rc0;
        }
    }
    if (hipHostMalloc(reinterpret_cast<void**>(&p->h_chunk), (size_t)cfg->chunk_frames * N_MEL * 4, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        p->h_chunk = nullptr;     // drains then copy straight into the caller's buffer
    }
    d.WmemT = (const float*)(base + l.WmemT);
    d.lsa_kfrag = base + l.lsa_kfrag;
    d.lsa_wfrag = base + l.lsa_wfrag;
    d.v = (const float*)(base + l.v);
    d.Wmel = base + l.Wmel;
    d.bmel = (const float*)(base + l.bmel);
    d.Wp1 = base + l.Wp1;
    d.Wp2 = base + l.Wp2;
    for (int b = 0; b < 2; ++b) {
        d.xatt[b] = base + l.xatt[b];
        d.xdec[b] = base + l.xdec[b];
    }
    d.c_att = (float*)(base + l.c_att);
    d.c_dec = (float*)(base + l.c_dec);
    d.m_last = (float*)(base + l.m_last);
    for (int b = 0; b < 2; ++b) {
        d.w_last[b] = (float*)(base + l.w_last[b]);
        d.w_acc[b] = (float*)(base + l.w_acc[b]);
    }
    d.Fmem = base + l.Fmem;
    d.PM = base + l.PM;
    d.mel_ring = (float*)(base + l.mel_ring);
    d.stop_ring = (float*)(base + l.stop_ring);
    d.L = (int*)(base + l.L);
    d.t = (int*)(base + l.t);
    d.n_steps = (int*)(base + l.n_steps);
    d.done = (int*)(base + l.done);
    d.failed = (int*)(base + l.failed);
    d.live = (int*)(base + l.live);
    d.stage = (float*)(base + l.stage);
    d.wait_polls = DEFAULT_WAIT_POLLS;
    d.max_enc_len = cfg->max_enc_len;
    d.max_steps = cfg->max_steps;
    d.stop_threshold = p->stop_enabled ? cfg->stop_threshold : -1.f;

    rc = upload_weights(p, w, base, l);
    if (rc == TTS_OK) {
        // slot counters and flags start defined: nothing live, no frames produced
        hipError_t e = hipMemset(base + l.L, 0, l.stage - l.L);
        // no word of the projection's hand-over buffer may carry a sequence number a leader could wait for
        if (e == hipSuccess && d.proj_part) e = hipMemset(base + l.proj_part, 0, l.proj_part_bytes);
        if (e == hipSuccess) e = hipEventCreate(&p->ev0);
        if (e == hipSuccess) e = hipEventCreate(&p->ev1);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) rc = fail(TTS_E_HIP, "pool setup: %s", hipGetErrorString(e));
    }
    if (rc) {
        tts_pool_destroy(p);
        return rc;
    }
    *out = p;
    return TTS_OK;
}

extern "C" void tts_pool_destroy(tts_pool* p)
{
    if (!p) return;
    (void)hipStreamSynchronize(p->stream);
    for (auto& kv : p->graphs) (void)hipGraphExecDestroy(kv.second);
    for (auto g : p->graph_defs) (void)hipGraphDestroy(g);
    if (p->ev0) (void)hipEventDestroy(p->ev0);
    if (p->ev1) (void)hipEventDestroy(p->ev1);
    if (p->h_fault) (void)hipHostFree(p->h_fault);
    if (p->h_chunk) (void)hipHostFree(p->h_chunk);
    delete p;
}

static bool is_device_pointer(const void* ptr)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, ptr) == hipSuccess) return attr.type == hipMemoryTypeDevice;
    (void)hipGetLastError();
    return false;
}

extern "C" int tts_pool_add_requests(tts_pool* p, int n, const float* const* enc_out, const int* L, const int* n_steps, int64_t* out_ids)
{
    if (!p || n < 0 || (n > 0 && (!enc_out || !L || !n_steps || !out_ids))) return fail(TTS_E_INVAL, "null argument");
    for (int i = 0; i < n; ++i) {
        if (!enc_out[i]) return fail(TTS_E_INVAL, "request %d: null encoder output", i);
        if (L[i] < 1 || L[i] > p->cfg.max_enc_len) return fail(TTS_E_INVAL, "request %d: L = %d outside 1..%d", i, L[i], p->cfg.max_enc_len);
        if (n_steps[i] < 1 || n_steps[i] > p->cfg.max_steps)
            return fail(TTS_E_INVAL, "request %d: n_steps = %d outside 1..%d", i, n_steps[i], p->cfg.max_steps);
    }
    if (p->book->size() + n > p->cfg.max_pool)
        return fail(TTS_E_FULL, "pool holds %d of max_pool = %d requests, %d more do not fit", p->book->size(), p->cfg.max_pool, n);

    JoinArgs ja;
    memset(&ja, 0, sizeof ja);
    int nb = 0;
    auto flush = [&]() -> int {
        if (nb) HIP_TRY(launch_join(p->d, p->cfg.weight_dtype, p->cfg.memory_dtype, ja, nb, p->stream));
        nb = 0;
        return TTS_OK;
    };
    for (int i = 0; i < n; ++i) {
        const bool on_device = is_device_pointer(enc_out[i]);
        int slot;
        int rc = p->book->add(L[i], n_steps[i], &out_ids[i], &slot);
        if (rc) return fail(rc == -2 ? TTS_E_FULL : TTS_E_INVAL, "request rejected");
        if (!on_device) {
            // one staging buffer: what is queued goes first, then this request alone; the caller may free a host
            // buffer on return, so the copy is finished before returning
            if ((rc = flush())) return rc;
            HIP_TRY(hipMemcpyAsync(p->d.stage, enc_out[i], (size_t)L[i] * ENC * 4, hipMemcpyHostToDevice, p->stream));
            HIP_TRY(hipStreamSynchronize(p->stream));
        }
        ja.F[nb] = on_device ? enc_out[i] : p->d.stage;
        ja.slot[nb] = slot;
        ja.L[nb] = L[i];
        ja.n_steps[nb] = n_steps[i];
        ++nb;
        if (!on_device || nb == JOIN_BATCH)
            if ((rc = flush())) return rc;
    }
    return flush();
}

extern "C" int tts_pool_add_request(tts_pool* p, const float* enc_out, int L, int n_steps, int64_t* out_id)
{
    if (!p || !enc_out || !out_id) return fail(TTS_E_INVAL, "null argument");
    return tts_pool_add_requests(p, 1, &enc_out, &L, &n_steps, out_id);
}

// workgroups per request in the attention kernel: more when the pool alone cannot fill the chip
static int lsa_split_for(int n_blocks) { return n_blocks <= 64 ? 4 : (n_blocks <= 128 ? 2 : 1); }

// LSTM tiling by the slots spanned: with one pool tile a workgroup takes one row tile, up to 8 tiles two row
// tiles and half of the pool tiles (32 slots: 32.1 -> 31.0 us per step against one row tile), above that the
// decoder LSTM takes four row tiles and a
// quarter (the attention LSTM, with its shorter K, stays at two: its four-row variant measured slower)
static int lstm_rows_for(int n_blocks) { return n_blocks > 128 ? 4 : (n_blocks > 16 ? 2 : 1); }

// most steps captured into one graph
static const int MAX_GRAPH_STEPS = 32;
static const bool CHAIN_ATT_LSTM = true;
// a whole chunk of at most this many steps is one graph of its own
static const int MAX_CHUNK_GRAPH_STEPS = 64;

// Span classes that launch shapes and graphs are keyed by: whole pool tiles, and powers of two within the first tile.
static int bucket_for(int n) { return PoolBook::span_class(n); }

// The step kernels cover every slot below the highest running one, so after requests have left the pool is packed into
// fewer pool tiles when that is possible (Sec. 2.2.2 rebuilds its batch tensors every iteration; here a request's
// state moves only when that shrinks the launch).  Launches over 16 slots and fewer take the same time.
static const int COMPACT_MIN_SPAN = 16;
static int compact(tts_pool* p)
{
    const std::vector<std::pair<int, int>> moves = p->book->plan_moves(COMPACT_MIN_SPAN);
    for (size_t i0 = 0; i0 < moves.size(); i0 += MOVE_BATCH) {
        MoveArgs mv;
        memset(&mv, 0, sizeof mv);
        const int n = (int)std::min(moves.size() - i0, (size_t)MOVE_BATCH);
        for (int i = 0; i < n; ++i) {
            const SlotInfo& si = p->book->slot(moves[i0 + i].first);
            mv.from[i] = moves[i0 + i].first;
            mv.to[i] = moves[i0 + i].second;
            mv.L[i] = si.L;
            mv.t[i] = si.t;
        }
        HIP_TRY(launch_move_slots(p->d, p->cfg.weight_dtype, p->cfg.memory_dtype, mv, n, p->stream));
        for (int i = 0; i < n; ++i) p->book->move(mv.from[i], mv.to[i]);
        p->n_moves += n;
    }
    return TTS_OK;
}

// Tell the device which slots the next steps advance (only when the membership changed).
static int push_membership(tts_pool* p)
{
    if (!p->book->dirty()) return TTS_OK;
    int rcc = compact(p);
    if (rcc) return rcc;
    LiveArgs a;
    memset(&a, 0, sizeof a);
    int span = 0;
    for (int sl : p->book->active()) {
        a.bits[sl >> 5] |= 1u << (sl & 31);
        if (sl + 1 > span) span = sl + 1;
    }
    p->slot_span = span;
    HIP_TRY(launch_set_live(p->d, a, p->stream));
    p->book->clear_dirty();
    return TTS_OK;
}

// Launch shape for a pool whose active slots lie below `span`: the attention kernel gets `lsa_split`
// workgroups per slot, the projection kernel one per 16-slot tile; slots and tiles without a running
// request are computed and dropped, so the grids may cover more than is active but never more than
// the arena holds.
static void shape_for(const tts_pool* p, int span, StepLaunch* sl)
{
    const int padded = (p->cfg.max_pool + 15) / 16 * 16;
    if (span > padded) span = padded;
    if (span < 1) span = 1;
    sl->n_blocks = span;
    sl->n_tiles = (span + 15) / 16;
    sl->lsa_split = lsa_split_for(span);
    sl->lstm_rows = lstm_rows_for(span);
    sl->pre_gates = !pre_gates_for(p->cfg) ? 0 : (pre_dec_for(p->cfg) ? 2 : 1);
    sl->proj_group = proj_group_for(p->cfg);
    sl->att_lead = 1;
    sl->att_tail = 0;
}

// Step i of `nsteps` consecutive steps of one call: in pools whose last launch can form the next step's attention LSTM
// (d.p_x) every step but the last does, and every step but the first therefore has no attention-LSTM launch of its own.
// Nothing can change between two steps of one call: joins, retirements and state accesses happen between calls, and the
// first step of a call always launches its own attention LSTM.
static void chain_steps(const tts_pool* p, StepLaunch* sl, int i, int nsteps)
{
    const bool chain = p->d.p_x != nullptr && CHAIN_ATT_LSTM;
    sl->att_lead = !(chain && i > 0);
    sl->att_tail = chain && i + 1 < nsteps;
}

// Queue `nsteps` consecutive steps for the current membership.  With graphs the
// steps are one hipGraph launch (captured once per (nsteps, pool bucket,
// parity)); requests that reach their end inside the graph are skipped by the
// kernels through their device-side done flag.
static int launch_steps(tts_pool* p, int n_active, int nsteps)
{
    StepLaunch sl;
    sl.wdtype = p->cfg.weight_dtype;
    sl.mdtype = p->cfg.memory_dtype;
    (void)n_active;
    if (!p->cfg.use_graph) {
        shape_for(p, p->slot_span, &sl);
        for (int i = 0; i < nsteps; ++i) {
            chain_steps(p, &sl, i, nsteps);
            HIP_TRY(launch_step(p->d, sl, p->parity ^ (i & 1), p->stream));
        }
        return TTS_OK;
    }
    const int bucket = bucket_for(p->slot_span);
    const int key = (nsteps * 1024 + bucket) * 2 + p->parity;
    auto it = p->graphs.find(key);
    if (it == p->graphs.end()) {
        shape_for(p, bucket, &sl);
        hipGraph_t g = nullptr;
        hipGraphExec_t ge = nullptr;
        HIP_TRY(hipStreamBeginCapture(p->stream, hipStreamCaptureModeThreadLocal));
        hipError_t le = hipSuccess;
        for (int i = 0; i < nsteps && le == hipSuccess; ++i) {
            chain_steps(p, &sl, i, nsteps);
            le = launch_step(p->d, sl, p->parity ^ (i & 1), p->stream);
        }
        hipError_t ce = hipStreamEndCapture(p->stream, &g);
        if (le != hipSuccess || ce != hipSuccess) {
            if (ce == hipSuccess && g) (void)hipGraphDestroy(g);
            if (le != hipSuccess) return fail(TTS_E_HIP, "capture of the step failed: %s", hipGetErrorString(le));
            return fail(TTS_E_HIP, "hipStreamEndCapture: %s", hipGetErrorString(ce));
        }
        const hipError_t ie = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
        if (ie != hipSuccess) {
            (void)hipGraphDestroy(g);
            return fail(TTS_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(ie));
        }
        p->graph_defs.push_back(g);
        it = p->graphs.emplace(key, ge).first;
    }
    HIP_TRY(hipGraphLaunch(it->second, p->stream));
    return TTS_OK;
}

static int step_impl(tts_pool* p, int n, int64_t* out_frames, int* out_last_active)
{
    int64_t frames = 0;
    int last = 0;
    if (p->timing) HIP_TRY(hipEventRecord(p->ev0, p->stream));
    int i = 0;
    while (i < n) {
        const int n_active = (int)p->book->active().size();
        last = n_active;
        if (n_active == 0) break;
        int rc = push_membership(p);
        if (rc) return rc;
        // graphs exist for powers of two up to MAX_GRAPH_STEPS and for one whole chunk (the paper's iteration: a
        // segment of 40 steps as one graph measured 0.05 - 0.2 us per step faster than as graphs of 32 and 8)
        int g = 1;
        if (p->cfg.use_graph) {
            while (g * 2 <= n - i && g * 2 <= MAX_GRAPH_STEPS) g *= 2;
            const int chunk = p->cfg.chunk_frames;
            if (chunk > g && chunk <= n - i && chunk <= MAX_CHUNK_GRAPH_STEPS) g = chunk;
        }
        rc = launch_steps(p, n_active, g);
        if (rc) return rc;
        for (int k = 0; k < g; ++k) {
            p->parity ^= 1;
            frames += p->book->step(p->parity);
        }
        i += g;
    }
    if (p->timing) {
        HIP_TRY(hipEventRecord(p->ev1, p->stream));
        p->ev_valid = true;
    }
    if (out_frames) *out_frames = frames;
    if (out_last_active) *out_last_active = last;
    return TTS_OK;
}

extern "C" int tts_pool_step(tts_pool* p, int* out_n_active)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    return step_impl(p, 1, nullptr, out_n_active);
}

extern "C" int tts_pool_step_n(tts_pool* p, int n, int64_t* out_frames)
{
    if (!p || n < 0) return fail(TTS_E_INVAL, "bad argument");
    return step_impl(p, n, out_frames, nullptr);
}

// n un-graphed steps with an event between consecutive kernels, queued back to
// back (one wait at the end); average device time of each kernel in
// microseconds.  An event costs device time of its own: that cost is measured
// with pairs of adjacent events and subtracted.  The steps are launched as one
// call of n steps launches them: the membership is uploaded once, and where a
// step's last launch forms the next step's attention LSTM it does so here.
extern "C" int tts_pool_kernel_times(tts_pool* p, int n, float* out_us, int cap, int* out_n_kernels)
{
    if (!p || !out_us || n < 1 || n > 4096) return fail(TTS_E_INVAL, "bad argument");
    if (out_n_kernels) *out_n_kernels = N_STEP_KERNELS;
    if (cap < N_STEP_KERNELS) return fail(TTS_E_INVAL, "room for %d kernels, %d needed", cap, N_STEP_KERNELS);
    const int per = N_STEP_KERNELS + 2;          // events per step: one before, one after each kernel, one more for calibration
    std::vector<hipEvent_t> ev((size_t)n * per, nullptr);
    int rc = TTS_OK;
    for (auto& e : ev)
        if (hipEventCreate(&e) != hipSuccess) { rc = fail(TTS_E_HIP, "hipEventCreate failed"); break; }
    int done = 0;
    StepLaunch sl;
    sl.wdtype = p->cfg.weight_dtype;
    sl.mdtype = p->cfg.memory_dtype;
    if (rc == TTS_OK && !p->book->active().empty()) {
        rc = push_membership(p);
        shape_for(p, p->slot_span, &sl);
    }
    for (int i = 0; i < n && rc == TTS_OK; ++i) {
        // (a pool that empties on the way: the step before formed an attention LSTM in which no request took part)
        if (p->book->active().empty()) break;
        chain_steps(p, &sl, i, n);
        hipEvent_t* e = &ev[(size_t)i * per];
        hipError_t he = launch_step(p->d, sl, p->parity, p->stream, e);
        // an empty interval right after the step: the cost of the event itself
        if (he == hipSuccess) he = hipEventRecord(e[N_STEP_KERNELS + 1], p->stream);
        if (he != hipSuccess) { rc = fail(TTS_E_HIP, "timed step: %s", hipGetErrorString(he)); break; }
        p->parity ^= 1;
        p->book->step(p->parity);
        ++done;
    }
    // per kernel: the steps that launched it.  The last kernel is averaged apart for the steps in which it also formed
    // the next step's attention LSTM (all but the last, in pools that do this) and for those in which it did not.
    const bool chained = n > 1 && p->d.p_x != nullptr && CHAIN_ATT_LSTM;
    double acc[N_STEP_KERNELS + 1] = {0}, last_plain = 0;
    int cnt[N_STEP_KERNELS + 1] = {0}, n_plain = 0;
    if (rc == TTS_OK && done > 0) {
        hipError_t he = hipStreamSynchronize(p->stream);
        for (int i = 0; i < done && he == hipSuccess; ++i)
            for (int k = 0; k <= N_STEP_KERNELS && he == hipSuccess; ++k) {
                float ms = 0.f;
                he = hipEventElapsedTime(&ms, ev[(size_t)i * per + k], ev[(size_t)i * per + k + 1]);
                if (k == 0 && chained && i > 0) continue;                  // no attention-LSTM launch of its own
                if (k == N_STEP_KERNELS - 1 && chained && i == n - 1) {    // the call's last step: nothing formed for a next one
                    last_plain += ms;
                    ++n_plain;
                    continue;
                }
                acc[k] += ms;
                ++cnt[k];
            }
        if (he != hipSuccess) rc = fail(TTS_E_HIP, "timed step: %s", hipGetErrorString(he));
    }
    for (auto& e : ev)
        if (e) (void)hipEventDestroy(e);
    if (rc) return rc;
    if (done == 0) return fail(TTS_E_INVAL, "the pool is empty");
    const double ev_cost = acc[N_STEP_KERNELS] / cnt[N_STEP_KERNELS];
    for (int k = 0; k < N_STEP_KERNELS; ++k) {
        const double us = cnt[k] ? (acc[k] / cnt[k] - ev_cost) * 1e3 : 0.0;
        out_us[k] = (float)(us > 0 ? us : 0);
    }
    // a pool whose last kernel holds the decoder LSTM launches no kernel between its third and fourth event
    // (pools of more than 64 slots: while they span more than 16 slots)
    if (p->d.hdec_x && (p->d.pre_dec_b || lstm_rows_for(p->slot_span) > 1)) out_us[2] = 0.f;
    if (cap > N_STEP_KERNELS) out_us[N_STEP_KERNELS] = (float)(ev_cost * 1e3);
    // the last kernel without the next step's attention LSTM (0: every timed step's was of one kind)
    if (cap > N_STEP_KERNELS + 1) {
        const double us = n_plain ? (last_plain / n_plain - ev_cost) * 1e3 : 0.0;
        out_us[N_STEP_KERNELS + 1] = (float)(us > 0 ? us : 0);
    }
    return TTS_OK;
}

// with a stop threshold the device may have ended a request before its cap
static int refresh_slot(tts_pool* p, int slot)
{
    if (!p->stop_enabled) return TTS_OK;
    int td[2] = {0, 0};
    HIP_TRY(hipMemcpyAsync(&td[0], p->d.t + slot, 4, hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipMemcpyAsync(&td[1], p->d.done + slot, 4, hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
    if (td[1] && td[0] <= p->book->slot(slot).t) p->book->finish_early(slot, td[0]);
    return TTS_OK;
}

extern "C" int tts_pool_drain_chunk(tts_pool* p, int64_t id, float* dst, int* out_frames, int* out_finished)
{
    if (!p || !dst || !out_frames || !out_finished) return fail(TTS_E_INVAL, "null argument");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int rc = refresh_slot(p, slot);
    if (rc) return rc;
    int first, count, fin;
    p->book->drain_plan(slot, &first, &count, &fin);
    if (count > 0) {
        float* via = p->h_chunk ? p->h_chunk : dst;      // count <= chunk_frames: the staging buffer holds it
        const float* src = p->d.mel_ring + ((size_t)slot * p->cfg.max_steps + first) * N_MEL;
        HIP_TRY(hipMemcpyAsync(via, src, (size_t)count * N_MEL * 4, hipMemcpyDeviceToHost, p->stream));
        HIP_TRY(hipStreamSynchronize(p->stream));
        if (*p->h_fault) {
            // some request was frozen since the last look: if it is this one, the plan above counted frames that were
            // never made; plan again from what the device holds (the copy above is then repeated for the right range)
            if ((rc = absorb_failures(p))) return rc;
            p->book->drain_plan(slot, &first, &count, &fin);
            if (count > 0) {
                src = p->d.mel_ring + ((size_t)slot * p->cfg.max_steps + first) * N_MEL;
                HIP_TRY(hipMemcpyAsync(via, src, (size_t)count * N_MEL * 4, hipMemcpyDeviceToHost, p->stream));
                HIP_TRY(hipStreamSynchronize(p->stream));
            }
        }
        if (via != dst && count > 0) memcpy(dst, via, (size_t)count * N_MEL * 4);
        p->book->drain_commit(slot, count);
    }
    *out_frames = count;
    *out_finished = fin;
    return TTS_OK;
}

extern "C" int tts_pool_chunk_window(tts_pool* p, int64_t id, int context, float* d_dst, int* out_context,
                                     int* out_frames, int* out_finished)
{
    if (!p || !d_dst || !out_context || !out_frames || !out_finished) return fail(TTS_E_INVAL, "null argument");
    if (context < 0) return fail(TTS_E_INVAL, "context = %d", context);
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int rc = refresh_slot(p, slot);
    if (rc) return rc;
    // a request frozen by steps that have already run must not hand out frames it never made (steps still in flight
    // are the caller's to wait for: tts_pool_sync reports what they lost)
    if (*p->h_fault) {
        HIP_TRY(hipStreamSynchronize(p->stream));
        if ((rc = absorb_failures(p))) return rc;
    }
    int first, count, fin;
    p->book->drain_plan(slot, &first, &count, &fin);
    const int ctx = count > 0 ? (first < context ? first : context) : 0;
    if (count > 0) {
        const float* src = p->d.mel_ring + ((size_t)slot * p->cfg.max_steps + (first - ctx)) * N_MEL;
        HIP_TRY(hipMemcpyAsync(d_dst, src, (size_t)(ctx + count) * N_MEL * 4, hipMemcpyDeviceToDevice, p->stream));
        p->book->drain_commit(slot, count);
    }
    *out_context = ctx;
    *out_frames = count;
    *out_finished = fin;
    return TTS_OK;
}

extern "C" int tts_pool_get_stop_logits(tts_pool* p, int64_t id, int first, int count, float* dst)
{
    if (!p || !dst) return fail(TTS_E_INVAL, "null argument");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int rc = refresh_slot(p, slot);
    if (rc) return rc;
    if (first < 0 || count < 0 || first + count > p->book->slot(slot).t)
        return fail(TTS_E_INVAL, "frames [%d, %d) not produced yet", first, first + count);
    if (count == 0) return TTS_OK;
    HIP_TRY(hipMemcpyAsync(dst, p->d.stop_ring + (size_t)slot * p->cfg.max_steps + first, (size_t)count * 4,
                           hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
    return TTS_OK;
}

extern "C" int tts_pool_retire(tts_pool* p, int64_t id)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    if (p->book->retire(id)) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    return TTS_OK;
}

extern "C" int tts_pool_frames(tts_pool* p, int64_t id, int* out_frames, int* out_finished)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int rc = refresh_slot(p, slot);
    if (rc) return rc;
    if (*p->h_fault) {
        HIP_TRY(hipStreamSynchronize(p->stream));
        if ((rc = absorb_failures(p))) return rc;
    }
    if (out_frames) *out_frames = p->book->slot(slot).t;
    if (out_finished) *out_finished = p->book->slot(slot).state == SlotState::Finished;
    return TTS_OK;
}

extern "C" int tts_pool_size(const tts_pool* p) { return p ? p->book->size() : 0; }
extern "C" int tts_pool_n_active(const tts_pool* p) { return p ? (int)p->book->active().size() : 0; }
extern "C" int tts_pool_span(const tts_pool* p) { return p ? p->book->span() : 0; }
extern "C" long long tts_pool_moves(const tts_pool* p) { return p ? p->n_moves : 0; }

extern "C" int tts_pool_sync(tts_pool* p)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    HIP_TRY(hipStreamSynchronize(p->stream));
    int rc = absorb_failures(p);
    return rc ? rc : report_lost(p);
}

extern "C" int tts_pool_lost(tts_pool* p, int64_t id, int* out_lost)
{
    if (!p || !out_lost) return fail(TTS_E_INVAL, "null argument");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int rc = TTS_OK;
    if (*p->h_fault) {
        HIP_TRY(hipStreamSynchronize(p->stream));
        if ((rc = absorb_failures(p))) return rc;
    }
    *out_lost = p->book->slot(slot).lost ? 1 : 0;
    return TTS_OK;
}

extern "C" int tts_pool_set_wait_polls(tts_pool* p, int polls)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    if (polls < 0) return fail(TTS_E_INVAL, "polls = %d is negative", polls);
    HIP_TRY(hipStreamSynchronize(p->stream));
    p->d.wait_polls = polls;
    // captured graphs hold the old value among their kernel arguments
    for (auto& kv : p->graphs) (void)hipGraphExecDestroy(kv.second);
    for (auto g : p->graph_defs) (void)hipGraphDestroy(g);
    p->graphs.clear();
    p->graph_defs.clear();
    return TTS_OK;
}

extern "C" int tts_pool_timing(tts_pool* p, int enable)
{
    if (!p) return fail(TTS_E_INVAL, "pool is null");
    p->timing = enable != 0;
    p->ev_valid = false;
    return TTS_OK;
}

extern "C" int tts_pool_elapsed_ms(tts_pool* p, float* out_ms)
{
    if (!p || !out_ms) return fail(TTS_E_INVAL, "null argument");
    if (!p->ev_valid) return fail(TTS_E_INVAL, "no timed step yet (enable tts_pool_timing first)");
    HIP_TRY(hipEventSynchronize(p->ev1));
    HIP_TRY(hipEventElapsedTime(out_ms, p->ev0, p->ev1));
    return TTS_OK;
}

// ------------------------------------------------------------------ state access
namespace {
// where one carried state lives: either plain fp32 arrays (up to two copies) or
// pieces of the slot-tiled activation arrays (up to four copies)
struct StateLoc {
    int n = 0;
    int n_plain = 0;
    float* plain[2];
    int n_x = 0;
    void* x[4];
    int xK[4];
    int xoff[4];
};
}  // namespace

static int locate_state(tts_pool* p, int slot, int which, StateLoc* s)
{
    const DevPtrs& d = p->d;
    const int rd = p->book->slot(slot).parity;   // buffer half holding the newest state of this request
    const size_t ml = d.max_enc_len;
    auto addx = [&](void* X, int K, int off) { s->x[s->n_x] = X; s->xK[s->n_x] = K; s->xoff[s->n_x] = off; ++s->n_x; };
    switch (which) {
    case TTS_STATE_M_LAST: s->n = N_MEL; s->plain[s->n_plain++] = d.m_last + (size_t)slot * N_MEL; break;
    case TTS_STATE_A:
        s->n = ENC;
        addx(d.xatt[rd], K_ATT, XA_A); addx(d.xatt[rd ^ 1], K_ATT, XA_A);
        addx(d.xdec[rd], K_DEC, XD_A); addx(d.xdec[rd ^ 1], K_DEC, XD_A);
        break;
    case TTS_STATE_W_LAST:
        s->n = p->book->slot(slot).L;
        s->plain[s->n_plain++] = d.w_last[rd] + slot * ml; s->plain[s->n_plain++] = d.w_last[rd ^ 1] + slot * ml;
        break;
    case TTS_STATE_W_ACC:
        s->n = p->book->slot(slot).L;
        s->plain[s->n_plain++] = d.w_acc[rd] + slot * ml; s->plain[s->n_plain++] = d.w_acc[rd ^ 1] + slot * ml;
        break;
    case TTS_STATE_H_ATT:
        s->n = HID;
        addx(d.xatt[rd], K_ATT, XA_H); addx(d.xatt[rd ^ 1], K_ATT, XA_H);
        addx(d.xdec[rd], K_DEC, XD_HA); addx(d.xdec[rd ^ 1], K_DEC, XD_HA);
        break;
    case TTS_STATE_C_ATT: s->n = HID; s->plain[s->n_plain++] = d.c_att + (size_t)slot * HID; break;
    case TTS_STATE_H_DEC:
        s->n = HID;
        addx(d.xdec[rd], K_DEC, XD_HD); addx(d.xdec[rd ^ 1], K_DEC, XD_HD);
        break;
    case TTS_STATE_C_DEC: s->n = HID; s->plain[s->n_plain++] = d.c_dec + (size_t)slot * HID; break;
    default: return fail(TTS_E_INVAL, "unknown state %d", which);
    }
    return TTS_OK;
}

extern "C" int tts_pool_get_state(tts_pool* p, int64_t id, int which, float* dst, int cap, int* out_n)
{
    if (!p || !dst) return fail(TTS_E_INVAL, "null argument");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    StateLoc s;
    int rc = locate_state(p, slot, which, &s);
    if (rc) return rc;
    if (out_n) *out_n = s.n;
    if (cap < s.n) return fail(TTS_E_INVAL, "room for %d elements, %d needed", cap, s.n);
    const float* src = s.n_plain ? s.plain[0] : p->d.stage;
    if (!s.n_plain) HIP_TRY(launch_x_get(p->cfg.weight_dtype, s.x[0], s.xK[0], slot, s.xoff[0], s.n, p->d.stage, p->stream));
    HIP_TRY(hipMemcpyAsync(dst, src, (size_t)s.n * 4, hipMemcpyDeviceToHost, p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
    return TTS_OK;
}

extern "C" int tts_pool_set_state(tts_pool* p, int64_t id, int which, const float* src, int n)
{
    if (!p || !src) return fail(TTS_E_INVAL, "null argument");
    const int slot = p->book->find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    StateLoc s;
    int rc = locate_state(p, slot, which, &s);
    if (rc) return rc;
    if (n != s.n) return fail(TTS_E_INVAL, "state %d has %d elements, %d given", which, s.n, n);
    for (int i = 0; i < s.n_plain; ++i)
        HIP_TRY(hipMemcpyAsync(s.plain[i], src, (size_t)n * 4, hipMemcpyHostToDevice, p->stream));
    if (s.n_x) {
        HIP_TRY(hipMemcpyAsync(p->d.stage, src, (size_t)n * 4, hipMemcpyHostToDevice, p->stream));
        for (int i = 0; i < s.n_x; ++i)
            HIP_TRY(launch_x_set(p->cfg.weight_dtype, s.x[i], s.xK[i], slot, s.xoff[i], n, p->d.stage, p->stream));
    }
    if (which == TTS_STATE_M_LAST) HIP_TRY(launch_prenet_slot(p->d, p->cfg.weight_dtype, slot, p->stream));
    // the next step's gate pre-sums were formed from the old state: redo the slot's tile from the half that step reads
    if (pre_gates_for(p->cfg) && (which == TTS_STATE_A || which == TTS_STATE_H_ATT || (which == TTS_STATE_H_DEC && pre_dec_for(p->cfg))))
        HIP_TRY(launch_presum_tile(p->d, p->cfg.weight_dtype, slot >> 4, p->parity, p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
    return TTS_OK;
}

// ------------------------------------------------------------------ host-only bookkeeping model
struct tts_book {
    PoolBook book;
    tts_book(int a, int b, int c, int d) : book(a, b, c, d) {}
};

extern "C" tts_book* tts_book_create(int max_pool, int max_enc_len, int max_steps, int chunk_frames)
{
    if (max_pool < 1 || max_enc_len < 1 || max_steps < 1 || chunk_frames < 1) return nullptr;
    return new (std::nothrow) tts_book(max_pool, max_enc_len, max_steps, chunk_frames);
}

extern "C" int tts_book_add(tts_book* b, int L, int n_steps, int64_t* out_id)
{
    if (!b || !out_id) return fail(TTS_E_INVAL, "null argument");
    int rc = b->book.add(L, n_steps, out_id, nullptr);
    if (rc == -1) return fail(TTS_E_INVAL, "L or n_steps out of range");
    if (rc == -2) return fail(TTS_E_FULL, "pool is full");
    return TTS_OK;
}

extern "C" int tts_book_step(tts_book* b, int64_t* out_ids, int* out_n_active)
{
    if (!b) return fail(TTS_E_INVAL, "null argument");
    std::vector<int> adv;
    int n = b->book.step(0, &adv);
    // ids must be read before a finished slot could be reused; slots keep their info until retired
    if (out_ids)
        for (int i = 0; i < n; ++i) out_ids[i] = b->book.slot(adv[i]).id;
    if (out_n_active) *out_n_active = n;
    return TTS_OK;
}

extern "C" int tts_book_drain(tts_book* b, int64_t id, int* out_first, int* out_frames, int* out_finished)
{
    if (!b) return fail(TTS_E_INVAL, "null argument");
    int slot = b->book.find(id);
    if (slot < 0) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    int first, count, fin;
    b->book.drain_plan(slot, &first, &count, &fin);
    b->book.drain_commit(slot, count);
    if (out_first) *out_first = first;
    if (out_frames) *out_frames = count;
    if (out_finished) *out_finished = fin;
    return TTS_OK;
}

extern "C" int tts_book_slot(const tts_book* b, int64_t id) { return b ? b->book.find(id) : -1; }

extern "C" int tts_book_compact(tts_book* b, int min_span, int* out_from, int* out_to, int cap)
{
    if (!b || cap < 0 || (cap > 0 && (!out_from || !out_to))) return fail(TTS_E_INVAL, "null argument");
    int n = 0;
    for (const std::pair<int, int>& m : b->book.plan_moves(min_span)) {
        if (n < cap) { out_from[n] = m.first; out_to[n] = m.second; }
        b->book.move(m.first, m.second);
        ++n;
    }
    return n;
}

extern "C" int tts_book_retire(tts_book* b, int64_t id)
{
    if (!b) return fail(TTS_E_INVAL, "null argument");
    if (b->book.retire(id)) return fail(TTS_E_NOTFOUND, "no request with id %lld", (long long)id);
    return TTS_OK;
}

extern "C" void tts_book_destroy(tts_book* b) { delete b; }
