// Decoder-step kernels for gfx950 (MI355X).  One step of paper Eq. 2 for a pool
// of requests is four kernels:
//   k_lstm<att>   gates GEMM on MFMA + fused cell        (Eq. 2 line 1)
//   k_lsa         query, location features, energies, ragged softmax, context,
//                 W_acc update                            (Eq. 2 lines 2 and 4)
//   k_lstm<dec>   gates GEMM on MFMA + fused cell        (Eq. 2 line 3)
//   k_proj        mel + stop projection, ring write, prenet of the new frame
//                                                         (Eq. 2 line 5, Pre() of line 1)
#include "kernels.h"

namespace tts {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// round to nearest even; inputs are finite here
__device__ __forceinline__ uint16_t f2bf_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { bf16_t r; r.bits = f2bf_bits(x); return r; }

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }
// 1 - 2/(1+e^{2x}): absolute error ~1e-7, saturates cleanly at +-1
__device__ __forceinline__ float tanhf_(float x) { return 1.0f - 2.0f / (1.0f + __expf(2.0f * x)); }

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// 16 bytes of T -> floats (4 for fp32, 8 for bf16)
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void unpack(const uint4& u, float* f)
    {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void unpack(const uint4& u, float* f)
    {
        f[0] = bf16_lo(u.x); f[1] = bf16_hi(u.x); f[2] = bf16_lo(u.y); f[3] = bf16_hi(u.y);
        f[4] = bf16_lo(u.z); f[5] = bf16_hi(u.z); f[6] = bf16_lo(u.w); f[7] = bf16_hi(u.w);
    }
};

// D(16x16) += A(16 x 64B of k) * B(64B of k x 16): one fragment pair.
// Lane l of A holds row l%16, bytes [16*(l/16), +16) of that row's 64-byte k chunk;
// lane l of B the same for column l%16.  A and B use the same k <-> (lane group,
// element) map, so the contraction is over the whole chunk whatever order the
// instruction walks it in.  D: lane l holds column l%16, rows 4*(l/16)..+3.
template <typename T> __device__ __forceinline__ floatx4 mfma_frag(const uint4& a, const uint4& b, floatx4 acc);
template <> __device__ __forceinline__ floatx4 mfma_frag<bf16_t>(const uint4& a, const uint4& b, floatx4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mfma_frag<float>(const uint4& a, const uint4& b, floatx4 acc)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    return acc;
}

// ---------------------------------------------------------------------------
// LSTM gates + cell.  Workgroup b owns hidden units 4b..4b+3 (16 gate rows in
// unit-major, gate-minor order) for the whole pool; its waves split K.
//   gates = W [x] + b;  c <- sig(f) c + sig(i) tanh(g);  h <- sig(o) tanh(c)
// ---------------------------------------------------------------------------
constexpr int LSTM_WAVES = 8;

template <typename XT, int K>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_lstm(
    const uint4* __restrict__ Wfrag, const float* __restrict__ bias, const XT* __restrict__ X,
    float* __restrict__ c_state, XT* __restrict__ hout0, int stride0, int off0,
    XT* __restrict__ hout1, int stride1, int off1,
    const int* __restrict__ table, const int* __restrict__ done)
{
    constexpr int NW = LSTM_WAVES;
    constexpr int KB = 64 / (int)sizeof(XT);   // k elements per fragment
    constexpr int NK = K / KB;
    constexpr int NF = NK / NW;
    static_assert(NK % NW == 0, "K must split evenly over the waves");
    constexpr int EPL = 16 / (int)sizeof(XT);  // elements per lane per fragment

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rt = blockIdx.x;
    const int P = table[0];
    if (P <= 0) return;

    uint4 a[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) a[f] = Wfrag[((size_t)rt * NK + (wave + f * NW)) * 64 + lane];

    __shared__ floatx4 red[NW][4][64];

    for (int pc = 0; pc < P; pc += 64) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int p0 = pc + nt * 16;
            if (p0 < P) {
                const int pi = p0 + (lane & 15);
                const bool valid = pi < P;
                const int slot = valid ? table[TABLE_HDR + pi] : 0;
                const XT* xrow = X + (size_t)slot * K + (lane >> 4) * EPL;
                uint4 b[NF];
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    b[f] = make_uint4(0, 0, 0, 0);
                    if (valid) b[f] = *reinterpret_cast<const uint4*>(xrow + (wave + f * NW) * KB);
                }
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NF; ++f) acc = mfma_frag<XT>(a[f], b[f], acc);
                red[wave][nt][lane] = acc;
            }
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            const int nt = threadIdx.x >> 6;
            const int pi = pc + nt * 16 + (lane & 15);
            if (pi < P) {
                const int slot = table[TABLE_HDR + pi];
                if (!done[slot]) {
                    const int unit = rt * 4 + (lane >> 4);
                    floatx4 g = *reinterpret_cast<const floatx4*>(bias + unit * 4);
#pragma unroll
                    for (int w = 0; w < NW; ++w) g += red[w][nt][lane];
                    const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
                    const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
                    const size_t ci = (size_t)slot * HID + unit;
                    const float c = gf * c_state[ci] + gi * gg;
                    c_state[ci] = c;
                    const XT h = from_float<XT>(go * tanhf_(c));
                    hout0[(size_t)slot * stride0 + off0 + unit] = h;
                    hout1[(size_t)slot * stride1 + off1 + unit] = h;
                }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Location-sensitive attention, one workgroup per request.
//   q = W_q h_att
//   loc[j][f] = sum_c sum_k Kc[f][c][k] u_c[j+k-15]      (u = W_last, W_acc; zero outside [0,L))
//   e_j = v . tanh(q + W_loc loc[j] + PM[j])
//   w = softmax_{j<L}(e);  A = sum_j w_j F[j];  W_last <- w;  W_acc <- W_acc + w
// ---------------------------------------------------------------------------
template <typename XT, typename MT>
__global__ __launch_bounds__(256) void k_lsa(DevPtrs d, int cur)
{
    const int pi = blockIdx.x;
    if (pi >= d.table[0]) return;
    const int slot = d.table[TABLE_HDR + pi];
    if (d.done[slot]) return;
    const int L = d.L[slot];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    __shared__ float s_q[ATT];
    __shared__ float s_v[ATT];
    __shared__ __attribute__((aligned(16))) float s_K[2 * LOC_K * LOC_F];
    __shared__ __attribute__((aligned(16))) float s_Wl[ATT * LOC_F];
    __shared__ float s_u[2][MAX_ENC_LEN + 2 * LOC_PAD + 2];
    __shared__ float s_e[MAX_ENC_LEN];
    __shared__ float s_red[8];
    __shared__ __attribute__((aligned(16))) float s_ctx[4][ENC];

    // ---- stage small weights and the two weight histories
    for (int i = tid; i < 2 * LOC_K * LOC_F; i += 256) s_K[i] = d.KcT[i];
    for (int i = tid; i < ATT * LOC_F; i += 256) s_Wl[i] = d.Wloc[i];
    if (tid < ATT) s_v[tid] = d.v[tid];
    const float* wl = d.w_last + (size_t)slot * d.max_enc_len;
    const float* wa = d.w_acc + (size_t)slot * d.max_enc_len;
    for (int i = tid; i < L + 2 * LOC_PAD; i += 256) {
        const int j = i - LOC_PAD;
        const bool in = (j >= 0 && j < L);
        s_u[0][i] = in ? wl[j] : 0.f;
        s_u[1][i] = in ? wa[j] : 0.f;
    }

    // ---- q = W_q h_att: each wave 32 outputs, lanes stride k in 16-byte pieces
    {
        constexpr int N = Vec16<XT>::N;
        constexpr int CH = HID / N / 64;     // 16-byte chunks per lane
        const XT* h = reinterpret_cast<const XT*>(d.xdec[cur]) + (size_t)slot * K_DEC + XD_HA;
        float hv[CH][N];
#pragma unroll
        for (int c = 0; c < CH; ++c)
            Vec16<XT>::unpack(*reinterpret_cast<const uint4*>(h + (lane + 64 * c) * N), hv[c]);
        const XT* Wq = reinterpret_cast<const XT*>(d.Wq);
        for (int o = wave * 32; o < wave * 32 + 32; ++o) {
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                float wv[N];
                Vec16<XT>::unpack(*reinterpret_cast<const uint4*>(Wq + (size_t)o * HID + (lane + 64 * c) * N), wv);
#pragma unroll
                for (int i = 0; i < N; ++i) acc += wv[i] * hv[c][i];
            }
            acc = wave_sum(acc);
            if (lane == 0) s_q[o] = acc;
        }
    }
    __syncthreads();

    // ---- energies, one position per thread
    const MT* PMs = reinterpret_cast<const MT*>(d.PM) + (size_t)slot * d.max_enc_len * ATT;
    for (int j = tid; j < L; j += 256) {
        float loc[LOC_F];
#pragma unroll
        for (int f = 0; f < LOC_F; ++f) loc[f] = 0.f;
        for (int c = 0; c < 2; ++c)
            for (int k = 0; k < LOC_K; ++k) {
                const float u = s_u[c][j + k];
                const float4* kk = reinterpret_cast<const float4*>(&s_K[(c * LOC_K + k) * LOC_F]);
#pragma unroll
                for (int f4 = 0; f4 < LOC_F / 4; ++f4) {
                    const float4 kv = kk[f4];
                    loc[4 * f4 + 0] += kv.x * u; loc[4 * f4 + 1] += kv.y * u;
                    loc[4 * f4 + 2] += kv.z * u; loc[4 * f4 + 3] += kv.w * u;
                }
            }
        constexpr int N = Vec16<MT>::N;
        const MT* pm = PMs + (size_t)j * ATT;
        float e = 0.f;
        for (int a0 = 0; a0 < ATT; a0 += N) {
            float pv[N];
            Vec16<MT>::unpack(*reinterpret_cast<const uint4*>(pm + a0), pv);
#pragma unroll
            for (int i = 0; i < N; ++i) {
                const int a = a0 + i;
                const float4* wr = reinterpret_cast<const float4*>(&s_Wl[a * LOC_F]);
                float pl = 0.f;
#pragma unroll
                for (int f4 = 0; f4 < LOC_F / 4; ++f4) {
                    const float4 wv = wr[f4];
                    pl += wv.x * loc[4 * f4 + 0] + wv.y * loc[4 * f4 + 1] + wv.z * loc[4 * f4 + 2] + wv.w * loc[4 * f4 + 3];
                }
                e += s_v[a] * tanhf_(s_q[a] + pl + pv[i]);
            }
        }
        s_e[j] = e;
    }
    __syncthreads();

    // ---- ragged softmax over j < L
    float mx = -INFINITY;
    for (int j = tid; j < L; j += 256) mx = fmaxf(mx, s_e[j]);
    mx = wave_max(mx);
    if (lane == 0) s_red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    float sum = 0.f;
    for (int j = tid; j < L; j += 256) {
        const float p = __expf(s_e[j] - mx);
        s_e[j] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) s_red[4 + wave] = sum;
    __syncthreads();
    const float inv = 1.0f / (s_red[4] + s_red[5] + s_red[6] + s_red[7]);
    float* wl_out = d.w_last + (size_t)slot * d.max_enc_len;
    float* wa_out = d.w_acc + (size_t)slot * d.max_enc_len;
    for (int j = tid; j < L; j += 256) {
        const float w = s_e[j] * inv;
        s_e[j] = w;
        wl_out[j] = w;
        wa_out[j] = s_u[1][j + LOC_PAD] + w;
    }
    __syncthreads();

    // ---- context: wave w takes rows j = w, w+4, ...; lane takes 8 columns
    {
        const MT* Fm = reinterpret_cast<const MT*>(d.Fmem) + (size_t)slot * d.max_enc_len * ENC;
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int j = wave; j < L; j += 4) {
            const float w = s_e[j];
            const MT* row = Fm + (size_t)j * ENC + lane * 8;
            float fv[8];
            if constexpr (sizeof(MT) == 2) {
                Vec16<MT>::unpack(*reinterpret_cast<const uint4*>(row), fv);
            } else {
                Vec16<MT>::unpack(*reinterpret_cast<const uint4*>(row), fv);
                Vec16<MT>::unpack(*reinterpret_cast<const uint4*>(row + 4), fv + 4);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += w * fv[i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) s_ctx[wave][lane * 8 + i] = acc[i];
    }
    __syncthreads();
    XT* xa = reinterpret_cast<XT*>(d.xatt[cur ^ 1]) + (size_t)slot * K_ATT + XA_A;
    XT* xd = reinterpret_cast<XT*>(d.xdec[cur]) + (size_t)slot * K_DEC + XD_A;
    for (int k = tid; k < ENC; k += 256) {
        const XT a = from_float<XT>(s_ctx[0][k] + s_ctx[1][k] + s_ctx[2][k] + s_ctx[3][k]);
        xa[k] = a;
        xd[k] = a;
    }
}

// ---------------------------------------------------------------------------
// Prenet of one frame held in LDS: p = relu(W2 relu(W1 m)), thread o < 256
// computes output o.  Both matrices are stored transposed so lanes read
// consecutive addresses.
// ---------------------------------------------------------------------------
template <typename XT>
__device__ __forceinline__ float prenet_thread(const DevPtrs& d, const float* s_mel, float* s_hid, int o)
{
    const XT* W1 = reinterpret_cast<const XT*>(d.Wp1T);
    const XT* W2 = reinterpret_cast<const XT*>(d.Wp2T);
    float acc = 0.f;
    for (int k = 0; k < N_MEL; ++k) acc += to_float(W1[k * PRENET + o]) * s_mel[k];
    s_hid[o] = fmaxf(acc, 0.f);
    __syncthreads();
    acc = 0.f;
    for (int k = 0; k < PRENET; ++k) acc += to_float(W2[k * PRENET + o]) * s_hid[k];
    return fmaxf(acc, 0.f);
}

// mel/stop projection of [H_dec; A], ring write, frame counter, prenet of the new frame
template <typename XT>
__global__ __launch_bounds__(256) void k_proj(DevPtrs d, int cur)
{
    const int pi = blockIdx.x;
    if (pi >= d.table[0]) return;
    const int slot = d.table[TABLE_HDR + pi];
    if (d.done[slot]) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    __shared__ float s_mel[N_PROJ + 3];
    __shared__ float s_hid[PRENET];

    constexpr int N = Vec16<XT>::N;
    constexpr int CH = K_PROJ / N / 64;   // 16-byte chunks per lane: 3 (bf16) or 6 (fp32)
    const XT* hd = reinterpret_cast<const XT*>(d.xdec[cur ^ 1]) + (size_t)slot * K_DEC + XD_HD;
    const XT* av = reinterpret_cast<const XT*>(d.xdec[cur]) + (size_t)slot * K_DEC + XD_A;
    float yv[CH][N];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int k = (lane + 64 * c) * N;
        const XT* src = (k < HID) ? (hd + k) : (av + (k - HID));
        Vec16<XT>::unpack(*reinterpret_cast<const uint4*>(src), yv[c]);
    }
    const XT* W = reinterpret_cast<const XT*>(d.Wmel);
    for (int o = wave; o < N_PROJ; o += 4) {
        float acc = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float wv[N];
            Vec16<XT>::unpack(*reinterpret_cast<const uint4*>(W + (size_t)o * K_PROJ + (lane + 64 * c) * N), wv);
#pragma unroll
            for (int i = 0; i < N; ++i) acc += wv[i] * yv[c][i];
        }
        acc = wave_sum(acc);
        if (lane == 0) s_mel[o] = acc + d.bmel[o];
    }
    __syncthreads();

    const int t = d.t[slot];
    if (tid < N_MEL) {
        d.mel_ring[((size_t)slot * d.max_steps + t) * N_MEL + tid] = s_mel[tid];
        d.m_last[(size_t)slot * N_MEL + tid] = s_mel[tid];
    }
    if (tid == N_MEL) d.stop_ring[(size_t)slot * d.max_steps + t] = s_mel[N_MEL];

    const float p = prenet_thread<XT>(d, s_mel, s_hid, tid);
    reinterpret_cast<XT*>(d.xatt[cur ^ 1])[(size_t)slot * K_ATT + XA_P + tid] = from_float<XT>(p);

    if (tid == 0) {
        const int tn = t + 1;
        d.t[slot] = tn;
        bool fin = tn >= d.n_steps[slot];
        if (d.stop_threshold >= 0.f && sigmoidf_(s_mel[N_MEL]) > d.stop_threshold) fin = true;
        if (fin) d.done[slot] = 1;
    }
}

// p = Pre(m_last) of one slot into both activation buffers
template <typename XT>
__global__ __launch_bounds__(256) void k_prenet_slot(DevPtrs d, int slot)
{
    __shared__ float s_mel[N_MEL];
    __shared__ float s_hid[PRENET];
    if (threadIdx.x < N_MEL) s_mel[threadIdx.x] = d.m_last[(size_t)slot * N_MEL + threadIdx.x];
    __syncthreads();
    const XT p = from_float<XT>(prenet_thread<XT>(d, s_mel, s_hid, threadIdx.x));
    reinterpret_cast<XT*>(d.xatt[0])[(size_t)slot * K_ATT + XA_P + threadIdx.x] = p;
    reinterpret_cast<XT*>(d.xatt[1])[(size_t)slot * K_ATT + XA_P + threadIdx.x] = p;
}

// ---------------------------------------------------------------------------
// Pool bookkeeping on the device
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_set_table(TableArgs a, int* table)
{
    if (threadIdx.x == 0) table[0] = a.n_active;
    if ((int)threadIdx.x < a.n_active) table[TABLE_HDR + threadIdx.x] = a.slot[threadIdx.x];
}

// a joining request starts from all-zero state
template <typename XT>
__global__ __launch_bounds__(256) void k_slot_init(DevPtrs d, int slot, int L, int n_steps)
{
    const int tid = threadIdx.x;
    const XT z = from_float<XT>(0.f);
    for (int b = 0; b < 2; ++b) {
        XT* xa = reinterpret_cast<XT*>(d.xatt[b]) + (size_t)slot * K_ATT;
        XT* xd = reinterpret_cast<XT*>(d.xdec[b]) + (size_t)slot * K_DEC;
        for (int i = tid; i < K_ATT; i += 256) xa[i] = z;
        for (int i = tid; i < K_DEC; i += 256) xd[i] = z;
    }
    for (int i = tid; i < HID; i += 256) {
        d.c_att[(size_t)slot * HID + i] = 0.f;
        d.c_dec[(size_t)slot * HID + i] = 0.f;
    }
    if (tid < N_MEL) d.m_last[(size_t)slot * N_MEL + tid] = 0.f;
    for (int i = tid; i < d.max_enc_len; i += 256) {
        d.w_last[(size_t)slot * d.max_enc_len + i] = 0.f;
        d.w_acc[(size_t)slot * d.max_enc_len + i] = 0.f;
    }
    if (tid == 0) {
        d.L[slot] = L;
        d.t[slot] = 0;
        d.n_steps[slot] = n_steps;
        d.done[slot] = 0;
    }
}

// one workgroup per encoder position: store the row, PM[j] = W_mem F[j]
template <typename MT>
__global__ __launch_bounds__(ATT) void k_join_memory(DevPtrs d, const float* __restrict__ F, int slot)
{
    const int j = blockIdx.x, tid = threadIdx.x;
    __shared__ float s_f[ENC];
    MT* Fm = reinterpret_cast<MT*>(d.Fmem) + ((size_t)slot * d.max_enc_len + j) * ENC;
    for (int k = tid; k < ENC; k += ATT) {
        const float x = F[(size_t)j * ENC + k];
        s_f[k] = x;
        Fm[k] = from_float<MT>(x);
    }
    __syncthreads();
    float acc = 0.f;
    for (int k = 0; k < ENC; ++k) acc += d.WmemT[k * ATT + tid] * s_f[k];
    reinterpret_cast<MT*>(d.PM)[((size_t)slot * d.max_enc_len + j) * ATT + tid] = from_float<MT>(acc);
}

// ---------------------------------------------------------------------------
// launch wrappers
// ---------------------------------------------------------------------------
template <typename XT, typename MT>
static hipError_t step_typed(const DevPtrs& d, int nb, int cur, hipStream_t s, hipEvent_t* ev)
{
    auto mark = [&](int i) { if (ev) (void)hipEventRecord(ev[i], s); };
    mark(0);
    XT* xatt_cur = reinterpret_cast<XT*>(d.xatt[cur]);
    XT* xatt_nxt = reinterpret_cast<XT*>(d.xatt[cur ^ 1]);
    XT* xdec_cur = reinterpret_cast<XT*>(d.xdec[cur]);
    XT* xdec_nxt = reinterpret_cast<XT*>(d.xdec[cur ^ 1]);
    // H_att(t): consumed by this step's decoder LSTM / LSA and by the next step's attention LSTM
    hipLaunchKernelGGL((k_lstm<XT, K_ATT>), dim3(HID / 4), dim3(LSTM_WAVES * 64), 0, s,
                       d.Wa, d.ba, xatt_cur, d.c_att, xdec_cur, K_DEC, XD_HA, xatt_nxt, K_ATT, XA_H,
                       d.table, d.done);
    mark(1);
    hipLaunchKernelGGL((k_lsa<XT, MT>), dim3(nb), dim3(256), 0, s, d, cur);
    mark(2);
    // H_dec(t): consumed by this step's projection and the next step's decoder LSTM (same buffer)
    hipLaunchKernelGGL((k_lstm<XT, K_DEC>), dim3(HID / 4), dim3(LSTM_WAVES * 64), 0, s,
                       d.Wd, d.bd, xdec_cur, d.c_dec, xdec_nxt, K_DEC, XD_HD, xdec_nxt, K_DEC, XD_HD,
                       d.table, d.done);
    mark(3);
    hipLaunchKernelGGL((k_proj<XT>), dim3(nb), dim3(256), 0, s, d, cur);
    mark(4);
    return hipGetLastError();
}

hipError_t launch_step(const DevPtrs& d, const StepLaunch& cfg, int cur, hipStream_t s, hipEvent_t* ev)
{
    if (cfg.n_blocks < 1) return hipSuccess;
    if (cfg.wdtype == 0 && cfg.mdtype == 0) return step_typed<float, float>(d, cfg.n_blocks, cur, s, ev);
    if (cfg.wdtype == 1 && cfg.mdtype == 1) return step_typed<bf16_t, bf16_t>(d, cfg.n_blocks, cur, s, ev);
    if (cfg.wdtype == 1 && cfg.mdtype == 0) return step_typed<bf16_t, float>(d, cfg.n_blocks, cur, s, ev);
    return hipErrorInvalidValue;
}

hipError_t launch_set_table(const DevPtrs& d, const TableArgs& args, hipStream_t s)
{
    hipLaunchKernelGGL(k_set_table, dim3(1), dim3(256), 0, s, args, d.table);
    return hipGetLastError();
}

hipError_t launch_slot_init(const DevPtrs& d, int wdtype, int slot, int L, int n_steps, hipStream_t s)
{
    if (wdtype == 0) hipLaunchKernelGGL((k_slot_init<float>), dim3(1), dim3(256), 0, s, d, slot, L, n_steps);
    else hipLaunchKernelGGL((k_slot_init<bf16_t>), dim3(1), dim3(256), 0, s, d, slot, L, n_steps);
    return hipGetLastError();
}

hipError_t launch_join_memory(const DevPtrs& d, int mdtype, const float* F_dev, int slot, int L, hipStream_t s)
{
    if (mdtype == 0) hipLaunchKernelGGL((k_join_memory<float>), dim3(L), dim3(ATT), 0, s, d, F_dev, slot);
    else hipLaunchKernelGGL((k_join_memory<bf16_t>), dim3(L), dim3(ATT), 0, s, d, F_dev, slot);
    return hipGetLastError();
}

hipError_t launch_prenet_slot(const DevPtrs& d, int wdtype, int slot, hipStream_t s)
{
    if (wdtype == 0) hipLaunchKernelGGL((k_prenet_slot<float>), dim3(1), dim3(256), 0, s, d, slot);
    else hipLaunchKernelGGL((k_prenet_slot<bf16_t>), dim3(1), dim3(256), 0, s, d, slot);
    return hipGetLastError();
}

}  // namespace tts
