// Acoustic encoder kernels (Sec. 2.1.2, Eq. 1) for a ragged batch of requests whose tokens are packed back to back:
//   k_enc_embed   E_all = sum of the four embedding rows of every token, stored as the first convolution's input
//   (conv5_kernels.h: three kernel-5 convolutions with ReLU, "same" padding inside each request)
//   k_enc_xproj   W_ih x + b for every token and both directions: the part of the LSTM that has no recurrence
//   k_enc_lstm    the recurrence, one workgroup per direction and group of 16 requests (fp32 weights);
//                 k_enc_lstm_dot: two-byte weights, one workgroup per direction and request
//
// The recurrence is a chain of L dependent steps of a 1024 x 256 matrix-vector product: latency, not bandwidth.
// With two-byte weights the matrix of one direction (512 KB) is resident in ONE compute unit per request -- registers
// and LDS of k_enc_lstm_dot's workgroup -- so a step touches no memory beyond the request's precomputed input projection.
// fp32 matrices (1 MB) do not fit a compute unit: they stream from L2 every step through MFMAs whose 16 columns are 16
// requests, the hidden state going round through LDS in B-fragment order.  Gate rows are stored unit-major / gate-minor,
// so the four gate sums of a unit are contiguous.
#include "encoder_kernels.h"

#include "conv5_kernels.h"

namespace tts {
namespace {

struct EncTables { const float* t[ENC_TABLES]; };
constexpr int ENC_COMPACT_UP_TO = 2;       // requests per call up to which the recurrence compacts its cell update

template <typename XT>
__global__ __launch_bounds__(256) void k_enc_embed(EncTables tb, const int* __restrict__ ids, int max_tokens, int n_col,
                                                   int n_col_pad, XT* __restrict__ X)
{
    constexpr int KB = Frag<XT>::KB;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int col = idx / ENC_DIM, ch = idx - col * ENC_DIM;
    if (col >= n_col_pad) return;
    float v = 0.f;
    if (col < n_col) {
#pragma unroll
        for (int t = 0; t < ENC_TABLES; ++t) v += tb.t[t][(size_t)ids[(size_t)t * max_tokens + col] * ENC_DIM + ch];
    }
    X[xoff<XT>(ENC_DIM / KB, col, ch)] = from_float<XT>(v);
}

// grid = (row tiles / 4, column tiles, 2 directions); a wave = one 16-row tile x one 16-column tile, K = dim
template <typename XT>
__global__ __launch_bounds__(256) void k_enc_xproj(const uint4* __restrict__ W0, const uint4* __restrict__ W1, const float* __restrict__ b0,
                                                   const float* __restrict__ b1, const uint4* __restrict__ X, int n_col, int max_tokens,
                                                   float* __restrict__ Y)
{
    constexpr int NKF = ENC_DIM / Frag<XT>::KB;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
    const int rt = blockIdx.x * 4 + wave, ct = blockIdx.y, dir = blockIdx.z;
    const uint4* W = dir ? W1 : W0;
    const float* b = dir ? b1 : b0;
    floatx4 acc = *reinterpret_cast<const floatx4*>(b + rt * 16 + 4 * g);
#pragma unroll 4
    for (int kf = 0; kf < NKF; ++kf) acc = mfma_frag<XT>(W[xfrag(NKF, rt, kf, lane)], X[xfrag(NKF, ct, kf, lane)], acc);
    const int col = ct * 16 + n;
    if (col < n_col) *reinterpret_cast<floatx4*>(Y + ((size_t)dir * max_tokens + col) * ENC_GATES + rt * 16 + 4 * g) = acc;
}

template <typename XT> struct EncLstmGeom {
    static constexpr int KB = Frag<XT>::KB, EPL = Frag<XT>::EPL;
    static constexpr int NK = ENC_HID / KB;                       // k fragments of W_hh (it streams from L2 every step)
    static constexpr int ROW_TILES = ENC_GATES / 16;              // 64
    static constexpr int TILES_PER_WAVE = ROW_TILES / 4;          // 16: a wave owns 64 units
    static constexpr int GCOLS = 2;                               // requests whose gate sums pass through LDS: the most a call may have
    static_assert(GCOLS >= ENC_COMPACT_UP_TO, "the compacting kernel serves calls of up to ENC_COMPACT_UP_TO requests");
    static constexpr int H_VECS = NK * 64;                        // h of the 16 requests, B-fragment order
    static constexpr int C_VECS = ENC_HID * 16 / 4;               // the cell state of 256 units x 16 requests, fp32
    static constexpr int G_VECS = GCOLS * ENC_GATES / 4;          // W_hh h of GCOLS requests, fp32
    static constexpr int LDS_BYTES = (H_VECS + C_VECS + G_VECS) * 16;
};

// grid = (2 directions, 1), 256 threads; for calls of at most GCOLS requests.
// One step:  (1) every wave: its 16 row tiles of W_hh h on MFMA, the requests as the first of the 16 columns;
//            (2) the lanes that hold those columns put the sums into LDS;
//            (3) thread u = hidden unit u takes the four gate sums of its unit, adds the precomputed input
//                projection, updates the cell and writes h (B-fragment order in LDS for the next step, fp32 to F_enc).
// The cell update runs on compacted data: with one request in flight the MFMA columns are 1/16 full, and so would
// every vector instruction be that worked on the accumulators where they are.
template <typename XT>
__global__ __launch_bounds__(256) void k_enc_lstm(const uint4* __restrict__ Whh0, const uint4* __restrict__ Whh1,
                                                  const float* __restrict__ xproj, PnWindows w, int max_tokens, float* __restrict__ out)
{
    using G = EncLstmGeom<XT>;
    constexpr int NK = G::NK, TPW = G::TILES_PER_WAVE, GCOLS = G::GCOLS;
    extern __shared__ uint4 lds_enc[];
    uint4* hb = lds_enc;                                          // [NK][64 lanes]
    float* cl = reinterpret_cast<float*>(hb + G::H_VECS);         // [unit][request]
    float* gl = cl + ENC_HID * 16;                                // [GCOLS][gate row]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
    const int dir = blockIdx.x, req0 = blockIdx.y * 16;
    const int nact = min(GCOLS, w.n - req0);                      // requests of this call
    // lengths and first tokens once, into registers: the request table is a kernel argument, and indexing it inside
    // the step loop would cost a memory round trip per use
    int len_of[GCOLS], col0_of[GCOLS], lmax = 0;
#pragma unroll
    for (int j = 0; j < GCOLS; ++j) {
        const int jj = min(j, nact - 1);
        len_of[j] = w.len[req0 + jj];
        col0_of[j] = w.col0[req0 + jj];
        if (j < nact) lmax = max(lmax, len_of[j]);
    }
    const uint4* Whh = dir ? Whh1 : Whh0;

    for (int idx = tid; idx < G::H_VECS + G::C_VECS; idx += 256) hb[idx] = make_uint4(0, 0, 0, 0);    // h = 0, c = 0

    // token of request j at step s: forwards from 0, backwards from the request's own last token
    auto token = [&](int j, int s) { return dir ? len_of[j] - 1 - s : s; };
    // this thread's unit: four gate sums of a request are 16 contiguous bytes of the input projection
    const float* xp = xproj + (size_t)dir * max_tokens * ENC_GATES + 4 * tid;
    // the first two requests' input projections are requested a step ahead (a batch at join time is that small)
    floatx4 xnext[GCOLS];
#pragma unroll
    for (int j = 0; j < GCOLS; ++j) {
        const int t0 = min(max(token(j, 0), 0), len_of[j] - 1);
        xnext[j] = *reinterpret_cast<const floatx4*>(xp + (size_t)(col0_of[j] + t0) * ENC_GATES);
    }
    __syncthreads();

    for (int s = 0; s < lmax; ++s) {
        // ---- (1) W_hh h: the matrix streams from L2, one k fragment of the wave's row tiles at a time;
        //      (2) the sums of this call's (at most GCOLS) requests into LDS
        float* dst = gl + (n % GCOLS) * ENC_GATES + (TPW * wave) * 16 + 4 * g;
        floatx4 acc[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int kf = 0; kf < NK; ++kf) {
            const uint4 bv = hb[kf * 64 + lane];
#pragma unroll
            for (int i = 0; i < TPW; ++i) acc[i] = mfma_frag<XT>(Whh[xfrag(NK, TPW * wave + i, kf, lane)], bv, acc[i]);
        }
        if (n < GCOLS) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) *reinterpret_cast<floatx4*>(dst + i * 16) = acc[i];
        }
        __syncthreads();                                   // the sums are in LDS and every wave has read h
        // ---- (3) thread = hidden unit
#pragma unroll
        for (int j = 0; j < GCOLS; ++j) {
            if (j >= nact) break;                          // uniform over the workgroup
            const int len = len_of[j], col0 = col0_of[j];
            if (s >= len) continue;                        // this request has ended
            const int t = token(j, s);
            const floatx4 gs = *reinterpret_cast<const floatx4*>(gl + j * ENC_GATES + 4 * tid) + xnext[j];
            const float gi = sigmoidf_(gs[0]), gf = sigmoidf_(gs[1]), gg = tanhf_(gs[2]), go = sigmoidf_(gs[3]);
            const float cn = gf * cl[tid * 16 + j] + gi * gg;
            cl[tid * 16 + j] = cn;
            const float h = go * tanhf_(cn);
            reinterpret_cast<XT*>(hb)[(((tid / G::KB) * 64 + j + 16 * ((tid % G::KB) / G::EPL)) * G::EPL) + (tid % G::EPL)] = from_float<XT>(h);
            out[(size_t)(col0 + t) * (2 * ENC_HID) + dir * ENC_HID + tid] = h;
            const int tn = min(max(token(j, s + 1), 0), len - 1);      // next step's input projection, clamped to the request
            xnext[j] = *reinterpret_cast<const floatx4*>(xp + (size_t)(col0 + tn) * ENC_GATES);
        }
        __syncthreads();                                   // h is complete and the gate buffer free for the next step
    }
}

// The recurrence with two-byte weights, on the vector units: one workgroup per direction and REQUEST (a call has at most
// ENC_MAX_BATCH = 256 requests, so at most two workgroups per CU's worth of the chip, and the usual call at join time
// has one).  A request's steps are a chain, and a chain is as fast alone on a CU as it gets: sixteen requests side by
// side as the columns of one workgroup's MFMAs take 6 us per step, sixteen workgroups 1.9 us.  Every workgroup reads
// the direction's 512 KB of W_hh once, from L2 after the first.  The recurrence of a request does not depend on its
// companions in the call.
// 512 threads: a pair of threads is one hidden unit, each holding one half of k of the unit's four gate rows - the even
// one the even pieces of eight consecutive k, the odd one the odd pieces - (512 halves a thread: 192 registers' worth and
// 64 LDS words, the same split of k as above, straight from the fragment-ordered matrix; at two waves per SIMD a lane has
// 256 registers, all of them operands of vector instructions).  A thread forms its half of the four gate sums as chains
// of two-element dot products (v_dot2_f32_f16, fp32 accumulation) over its half of h, which it reads from LDS as a
// broadcast (a wave reads two neighbouring pieces at a time: no bank is asked twice); the pair adds its halves and both
// update the cell.  With one request in flight an MFMA's sixteen columns are 1/16 full - 32 cycles of the matrix
// pipe for 512 useful products - while a dot-product instruction does 128 useful products in 4 cycles, and the gate sums
// never pass through LDS.
// grid = (2 directions, requests), 512 threads.  LDS: [16][512] uint4 of weights, h as halves [2 buffers][256].
constexpr int ENC_DOT_THREADS = 2 * ENC_HID;
constexpr int ENC_DOT_W_VECS = 16 * ENC_DOT_THREADS;
constexpr int ENC_DOT_LDS_BYTES = ENC_DOT_W_VECS * 16 + 2 * ENC_HID * 2;

__device__ __forceinline__ float dot8(uint4 w, uint4 h, float acc)
{
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2, w.x), __builtin_bit_cast(halfx2, h.x), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2, w.y), __builtin_bit_cast(halfx2, h.y), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2, w.z), __builtin_bit_cast(halfx2, h.z), acc, false);
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2, w.w), __builtin_bit_cast(halfx2, h.w), acc, false);
}

__global__ __launch_bounds__(ENC_DOT_THREADS) void k_enc_lstm_dot(const uint4* __restrict__ Whh0, const uint4* __restrict__ Whh1,
                                                                  const float* __restrict__ xproj, PnWindows w, int max_tokens, float* __restrict__ out)
{
    typedef h16_t XT;
    constexpr int KB = Frag<XT>::KB, NK = ENC_HID / KB;
    static_assert(KB == 32 && NK == 8, "k = 32 kf + 8 q + e: a lane's 16 bytes are 8 consecutive k");
    extern __shared__ uint4 lds_enc[];
    uint4* wl = lds_enc;                                                        // [gate * 4 + piece / 4][thread]
    uint16_t* hs = reinterpret_cast<uint16_t*>(lds_enc + ENC_DOT_W_VECS);       // [buffer][unit]
    const int tid = threadIdx.x, dir = blockIdx.x, req = blockIdx.y, unit = tid >> 1, half = tid & 1;
    const int len = w.len[req], col0 = w.col0[req];
    const uint4* Whh = dir ? Whh1 : Whh0;
    // gate row 4 u + g lies in row tile u / 4 at row 4 (u % 4) + g; its k = 32 kf + 8 q .. + 7 in lane row + 16 q;
    // this thread's pieces are q = half and half + 2
    const int rt = unit >> 2, r0 = 4 * (unit & 3);
    // of its 16 pieces (piece i: kf = i / 2, q = half + 2 (i % 2)) every fourth lives in LDS, the others in registers: the
    // LDS reads are spread evenly over a step
    constexpr int NP = 2 * NK, NP_LDS = NP / 4, NP_REG = NP - NP_LDS;
    static_assert(NP_LDS * 4 * ENC_DOT_THREADS == ENC_DOT_W_VECS, "the LDS share of the weights");
    uint4 wr[4][NP_REG];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const uint4 v = Whh[xfrag(NK, rt, i >> 1, r0 + g + 16 * (half + 2 * (i & 1)))];
            if ((i & 3) == 3) wl[(g * NP_LDS + (i >> 2)) * ENC_DOT_THREADS + tid] = v;
            else wr[g][i - (i >> 2)] = v;
        }
    hs[tid] = 0;                                                                // h = 0, both buffers

    auto token = [&](int s) { return dir ? len - 1 - s : s; };
    const float* xp = xproj + ((size_t)dir * max_tokens + col0) * ENC_GATES + 4 * unit;
    floatx4 xnext = *reinterpret_cast<const floatx4*>(xp + (size_t)min(max(token(0), 0), len - 1) * ENC_GATES);
    float c = 0.f;
    __syncthreads();

    for (int s = 0; s < len; ++s) {
        const uint4* hr = reinterpret_cast<const uint4*>(hs + (s & 1) * ENC_HID);               // 32 pieces of 8 halves
        uint16_t* hx = hs + ((s + 1) & 1) * ENC_HID;
        asm volatile("" ::: "memory");                    // (the LDS-resident weights are read again every step, not kept in registers)
        // one chain per gate over this thread's half of k, a piece of eight k at a time; the next piece's LDS words (h, and
        // the weights that live there) are requested before the current piece's products, and no further ahead: few live
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        uint4 hv = hr[half], wv[4];
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            uint4 hn = hv, wn[4];
            if (i + 1 < NP) {
                hn = hr[((i + 1) >> 1) * 4 + half + 2 * ((i + 1) & 1)];
                if (((i + 1) & 3) == 3) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) wn[g] = wl[(g * NP_LDS + ((i + 1) >> 2)) * ENC_DOT_THREADS + tid];
                }
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) acc[g] = dot8((i & 3) == 3 ? wv[g] : wr[g][(i & 3) == 3 ? 0 : i - (i >> 2)], hv, acc[g]);
            hv = hn;
            if (i + 1 < NP && ((i + 1) & 3) == 3) {
#pragma unroll
                for (int g = 0; g < 4; ++g) wv[g] = wn[g];
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
        // the pair adds its halves: both threads hold all four gate sums, bit for bit the same
        const int t = token(s);
        floatx4 gs;
#pragma unroll
        for (int g = 0; g < 4; ++g) gs[g] = acc[g] + __shfl_xor(acc[g], 1, 64);
        gs += xnext;
        const float gi = sigmoidf_(gs[0]), gf = sigmoidf_(gs[1]), gg = tanhf_(gs[2]), go = sigmoidf_(gs[3]);
        c = gf * c + gi * gg;
        const float h = go * tanhf_(c);
        if (half == 0) {
            hx[unit] = from_float<XT>(h).bits;
            out[(size_t)(col0 + t) * (2 * ENC_HID) + dir * ENC_HID + unit] = h;
        }
        const int tn = min(max(token(s + 1), 0), len - 1);             // next step's input projection, clamped to the request
        xnext = *reinterpret_cast<const floatx4*>(xp + (size_t)tn * ENC_GATES);
        __syncthreads();                                   // h is complete (the other buffer is free for the next step)
    }
}

template <typename XT> struct EncLstmWideGeom {
    static constexpr int KB = Frag<XT>::KB, EPL = Frag<XT>::EPL;
    static constexpr int NK = ENC_HID / KB;                       // k fragments of W_hh (it streams from L2 every step)
    static constexpr int ROW_TILES = ENC_GATES / 16;              // 64
    static constexpr int TILES_PER_WAVE = ROW_TILES / 4;          // 16: a wave owns 64 units
    static constexpr int H_VECS = NK * 64;                        // one copy of h; there are two (read one, write the other)
    static constexpr int C_VECS = ENC_HID * 16 / 4;              // the cell state of 256 units x 16 requests, fp32
    static constexpr int LDS_BYTES = (2 * H_VECS + C_VECS) * 16;
};

// The recurrence for well-filled groups (more than ENC_COMPACT_UP_TO requests in the call): the cell update runs where
// the accumulators are -- a lane owns the four gates of one unit for its request's column -- so nothing passes through
// LDS but h, and the next step's input projection lands in the accumulators half a step ahead.
// grid = (2 directions, groups of 16 requests), 256 threads
template <typename XT>
__global__ __launch_bounds__(256) void k_enc_lstm_wide(const uint4* __restrict__ Whh0, const uint4* __restrict__ Whh1,
                                                  const float* __restrict__ xproj, PnWindows w, int max_tokens, float* __restrict__ out)
{
    using G = EncLstmWideGeom<XT>;
    constexpr int NK = G::NK, TPW = G::TILES_PER_WAVE;
    extern __shared__ uint4 lds_enc[];
    uint4* hb = lds_enc;                     // h of the 16 requests, B-fragment order, [NK][64 lanes]
    float* cl = reinterpret_cast<float*>(hb + 2 * G::H_VECS); // cell state [unit][request]: only its owner lane touches an entry
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
    const int dir = blockIdx.x, req = blockIdx.y * 16 + n;
    const bool active = req < w.n;
    const int len = active ? (int)w.len[req] : 0, col0 = active ? w.col0[req] : 0;
    int lmax = len;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) lmax = max(lmax, __shfl_xor(lmax, o, 64));
    const uint4* Whh = dir ? Whh1 : Whh0;

    for (int idx = tid; idx < 2 * G::H_VECS; idx += 256) hb[idx] = make_uint4(0, 0, 0, 0);

    // token of this lane's request at step s: forwards from 0, backwards from its own last token; clamped so that
    // a request that has ended keeps reading (and computing on) valid memory -- its results are not stored
    auto token = [&](int s) { return min(max(dir ? len - 1 - s : s, 0), max(len - 1, 0)); };
    const float* xp = xproj + ((size_t)dir * max_tokens + col0) * ENC_GATES + (TPW * wave) * 16 + 4 * g;
    floatx4 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        acc[i] = *reinterpret_cast<const floatx4*>(xp + (size_t)token(0) * ENC_GATES + i * 16);
        cl[(4 * (TPW * wave + i) + g) * 16 + n] = 0.f;
    }
    __syncthreads();

    // A step in two halves of eight row tiles.  h is read from one buffer and written to the other, so a half's cell
    // update can follow its MFMAs at once (and overlap the other half's MFMAs); when a half's accumulators have been
    // consumed, the next step's input projection for those tiles is requested into them: half a step ahead of its use.
    constexpr int HALF = TPW / 2;
    for (int s = 0; s < lmax; ++s) {
        const uint4* hr = hb + (s & 1) * G::H_VECS;
        XT* hx = reinterpret_cast<XT*>(hb + ((s + 1) & 1) * G::H_VECS);
        const int t_cur = dir ? len - 1 - s : s;
        const bool store = active && s < len;
        const int tn = token(s + 1);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // the matrix streams from L2, one k fragment of the half's row tiles at a time
#pragma unroll 1
            for (int kf = 0; kf < NK; ++kf) {
                const uint4 bv = hr[kf * 64 + lane];
#pragma unroll
                for (int j = 0; j < HALF; ++j)
                    acc[half * HALF + j] = mfma_frag<XT>(Whh[xfrag(NK, TPW * wave + half * HALF + j, kf, lane)], bv, acc[half * HALF + j]);
            }
#pragma unroll
            for (int j = 0; j < HALF; ++j) {
                const int i = half * HALF + j;
                const float gi = sigmoidf_(acc[i][0]), gf = sigmoidf_(acc[i][1]), gg = tanhf_(acc[i][2]), go = sigmoidf_(acc[i][3]);
                const int u = 4 * (TPW * wave + i) + g;           // this lane's unit of tile i
                const float cn = gf * cl[u * 16 + n] + gi * gg;
                cl[u * 16 + n] = cn;
                const float h = go * tanhf_(cn);
                hx[(((u / G::KB) * 64 + n + 16 * ((u % G::KB) / G::EPL)) * G::EPL) + (u % G::EPL)] = from_float<XT>(h);
                if (store) out[(size_t)(col0 + t_cur) * (2 * ENC_HID) + dir * ENC_HID + u] = h;
                acc[i] = *reinterpret_cast<const floatx4*>(xp + (size_t)tn * ENC_GATES + i * 16);
            }
        }
        __syncthreads();                       // the new h is complete; the old one is free to be overwritten next step
    }
}

template <typename XT>
hipError_t run_typed(const EncoderPtrs& d, const PnWindows& w, int n_col, float* out, hipStream_t s)
{
    constexpr int C = ENC_DIM;
    const int n_ctiles = (n_col + 15) / 16, n_col_pad = n_ctiles * 16;
    const bool wide = n_ctiles >= PN_WIDE_FROM;
    XT* x0 = reinterpret_cast<XT*>(d.act[0]);
    XT* x1 = reinterpret_cast<XT*>(d.act[1]);
    PostnetPtrs tables{};                     // the shared per-column table kernel only needs these two
    tables.cmeta = d.cmeta;
    tables.orow = d.orow;
    hipError_t e = launch_postnet_meta(tables, w, n_col, n_col_pad, true, s);
    if (e != hipSuccess) return e;
    EncTables tb;
    for (int t = 0; t < ENC_TABLES; ++t) tb.t[t] = d.tables[t];
    hipLaunchKernelGGL((k_enc_embed<XT>), dim3((n_col_pad * C + 255) / 256), dim3(256), 0, s, tb, d.ids, d.max_tokens, n_col, n_col_pad, x0);
    e = hipGetLastError();
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_RELU>(wide, d.conv_w[0], d.conv_b[0], x0, x1, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_RELU>(wide, d.conv_w[1], d.conv_b[1], x1, x0, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_RELU>(wide, d.conv_w[2], d.conv_b[2], x0, x1, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_enc_xproj<XT>), dim3(ENC_GATES / 16 / 4, n_ctiles, 2), dim3(256), 0, s, (const uint4*)d.w_ih[0], (const uint4*)d.w_ih[1],
                       d.b[0], d.b[1], (const uint4*)x1, n_col, d.max_tokens, d.xproj);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if constexpr (sizeof(XT) == 2) {
        // two-byte weights: the recurrence on the vector units, a workgroup per direction and request
        static bool dot_attr_set = false;
        if (!dot_attr_set) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_enc_lstm_dot), hipFuncAttributeMaxDynamicSharedMemorySize, ENC_DOT_LDS_BYTES);
            if (e != hipSuccess) return e;
            dot_attr_set = true;
        }
        hipLaunchKernelGGL(k_enc_lstm_dot, dim3(2, w.n), dim3(ENC_DOT_THREADS), ENC_DOT_LDS_BYTES, s, (const uint4*)d.w_hh[0], (const uint4*)d.w_hh[1], d.xproj, w,
                           d.max_tokens, out);
    } else {
        // fp32 weights: a call with a few requests takes the kernel that compacts the cell update
        const bool compact = w.n <= ENC_COMPACT_UP_TO;
        const int lds = compact ? EncLstmGeom<XT>::LDS_BYTES : EncLstmWideGeom<XT>::LDS_BYTES;
        auto kern = compact ? k_enc_lstm<XT> : k_enc_lstm_wide<XT>;
        static bool attr_set[2] = {false, false};   // dynamic LDS above 64 KB has to be allowed once per kernel
        if (!attr_set[compact]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
            attr_set[compact] = true;
        }
        hipLaunchKernelGGL(kern, dim3(2, (w.n + 15) / 16), dim3(256), lds, s, (const uint4*)d.w_hh[0], (const uint4*)d.w_hh[1], d.xproj, w,
                           d.max_tokens, out);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_encoder(const EncoderPtrs& d, int wdtype, const PnWindows& w, int n_col, float* out, hipStream_t s)
{
    if (n_col < 1 || w.n < 1) return hipSuccess;
    return wdtype == 0 ? run_typed<float>(d, w, n_col, out, s) : run_typed<h16_t>(d, w, n_col, out, s);
}

}  // namespace tts
