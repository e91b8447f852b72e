// Vocoder kernels (Sec. 2.1.4, Eq. 3, Eq. 4): the generator G as a chain of one-dimensional convolutions on
// MFMA, the splice of [tail(M_pre), M_cur] and the equal-power fade of the overlapping audio.
//
// Every convolution of G -- plain, dilated or transposed -- is one GEMM  Y[row][p] = sum_k W[row][k] X[k][p]
// over the positions p of a window, with k = tap * C_in + channel and X[k][p] = act(x[p + (tap - half) * dil][channel]):
//   plain / dilated   rows = output channels, taps = the kernel's taps
//   transposed        stride u, kernel 2u, padding u/2: output u p + r depends on inputs p - 1, p, p + 1 only, so it is
//                     a 3-tap convolution with rows = (phase r, output channel) and one zero tap per phase
// Activations live in HBM as fp32 [position][channel]; a workgroup stages the positions of its tile plus the halo
// in LDS (leaky ReLU and the conversion to the MFMA operand type happen there, once per element), so that a lane's
// B operand -- consecutive channels of one tap at one position -- is one 16-byte LDS read.  Rows of LDS are padded
// to an odd number of 16-byte pieces.  The weights are stored in A-fragment order and stream from L2.
// Windows of different requests lie at a fixed stride; positions outside a window's own length read as zero, which
// is the zero padding of every layer.
#include "vocoder_kernels.h"

#include "mfma.h"

namespace tts {
namespace {

constexpr int VC_THREADS = 256;
constexpr int VC_WAVES = VC_THREADS / 64;
constexpr float VC_SLOPE = 0.1f;
constexpr int VC_LDS_BYTES = 48 * 1024;
constexpr int VC_AHEAD = 4;                  // k steps between the request for a weight fragment and its use

enum { EPI_PLAIN = 0, EPI_UP = 2, EPI_POST = 3 };

template <typename XT, int CIN> struct VcGeom {
    static constexpr int EPL = Frag<XT>::EPL;
    static constexpr int GP = CIN / EPL;         // 16-byte pieces per position
    static constexpr int GPP = GP | 1;           // ... padded to an odd count
    static constexpr int CINP = GPP * EPL;
    static_assert(CIN % EPL == 0, "channels must fill whole 16-byte pieces");
};

// positions per workgroup: as many as the accumulators (64 registers) and 48 KB of LDS allow
template <typename XT, int CIN, int ROWS, int HALO, bool SHORT = false> constexpr int vc_tp()
{
    constexpr int RT = ROWS / 16, RG = RT < 4 ? RT : 4;
    int tp = SHORT ? 64 : 1024 / RG;
    while (tp > 64 && (tp + 2 * HALO) * VcGeom<XT, CIN>::GPP * 16 > VC_LDS_BYTES) tp /= 2;
    return tp;
}

struct VcArgs {
    const float* in0;     // input activations [position][C_in]
    const float* in1;     // with SRC3 the input is the mean of in0, in1, in2 (the three residual blocks of a stage)
    const float* in2;
    float* out;
    const uint4* W;
    const float* bias;
    int dil;
};

// slope < 1: the larger of x and slope * x
__device__ __forceinline__ float lrelu(float x) { return fmaxf(x, VC_SLOPE * x); }

template <typename XT> __device__ __forceinline__ void lds_put4(uint4* lds, int elem, float4 v);
template <> __device__ __forceinline__ void lds_put4<float>(uint4* lds, int elem, float4 v)
{
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(lds) + elem) = v;
}
template <> __device__ __forceinline__ void lds_put4<h16_t>(uint4* lds, int elem, float4 v)
{
    uint2 u;
    u.x = pack2<h16_t>(v.x, v.y);
    u.y = pack2<h16_t>(v.z, v.w);
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(lds) + elem) = u;
}

// One tile of TP positions of one window, all ROWS output rows.
//   valid  positions of this window that exist (input side); wbase = first position of the window in the arrays
//   p0     first position of the tile inside the window
template <typename XT, int CIN, int ROWS, int COUT, int KS, int TP, int EPI, bool PRE_ACT, bool SRC3, int U>
__device__ __forceinline__ void conv_tile(const VcArgs& a, int valid, size_t wbase, int p0, uint4* lds)
{
    using G = VcGeom<XT, CIN>;
    constexpr int KB = Frag<XT>::KB;
    constexpr int RT = ROWS / 16, RG = RT < 4 ? RT : 4, CT = TP / (16 * VC_WAVES);
    constexpr int NK = (KS * CIN + KB - 1) / KB;     // K fragments (the weights are zero padded to whole fragments)
    constexpr int NQ = KS * G::GP;                   // 16-byte pieces of k that exist
    constexpr int C4 = CIN / 4;
    static_assert(ROWS % 16 == 0 && RT % RG == 0 && TP % (16 * VC_WAVES) == 0, "tile shape");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int halo = (KS - 1) / 2 * a.dil;
    const int nrows = TP + 2 * halo;

    // ---- stage positions [p0 - halo, p0 + TP + halo): activation and operand type applied once per element
    for (int idx = tid; idx < nrows * C4; idx += VC_THREADS) {
        const int row = idx / C4, c4 = idx - row * C4;
        const int p = p0 - halo + row;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p >= 0 && p < valid) {
            const size_t off = (wbase + p) * CIN + 4 * c4;
            v = *reinterpret_cast<const float4*>(a.in0 + off);
            if constexpr (SRC3) {
                const float4 v1 = *reinterpret_cast<const float4*>(a.in1 + off);
                const float4 v2 = *reinterpret_cast<const float4*>(a.in2 + off);
                constexpr float third = 1.0f / 3.0f;
                v.x = ((v.x + v1.x) + v2.x) * third; v.y = ((v.y + v1.y) + v2.y) * third;
                v.z = ((v.z + v1.z) + v2.z) * third; v.w = ((v.w + v1.w) + v2.w) * third;
            }
            if constexpr (PRE_ACT) { v.x = lrelu(v.x); v.y = lrelu(v.y); v.z = lrelu(v.z); v.w = lrelu(v.w); }
        }
        lds_put4<XT>(lds, row * G::CINP + 4 * c4, v);
    }
    __syncthreads();

    const int colbase = wave * (TP / VC_WAVES);
    // The workgroup's share of the output rows: row group blockIdx.z.  Its weights stream from L2 / HBM through a
    // ring of registers, requested VC_AHEAD k steps before they are used.
    {
        const int rt0 = blockIdx.z * RG;
        floatx4 acc[RG][CT];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[rg][ct] = floatx4{0.f, 0.f, 0.f, 0.f};
        const uint4* Wl = a.W + (size_t)rt0 * NK * 64 + lane;
        constexpr int AHEAD = NK < VC_AHEAD ? NK : VC_AHEAD;
        uint4 ring[AHEAD][RG];
#pragma unroll
        for (int d = 0; d < AHEAD; ++d)
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) ring[d][rg] = Wl[((size_t)rg * NK + d) * 64];
#pragma unroll
        for (int kf = 0; kf < NK; ++kf) {
            uint4 af[RG];
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                af[rg] = ring[kf % AHEAD][rg];
                if (kf + AHEAD < NK) ring[kf % AHEAD][rg] = Wl[((size_t)rg * NK + kf + AHEAD) * 64];
            }
            // this lane's 16 bytes of k: piece q = (tap, channel group); pieces past the end meet zero weights
            const int q = min(kf * 4 + g, NQ - 1);
            const int tap = q / G::GP, cg = q - tap * G::GP;
            const uint4* bl = lds + (colbase + n + tap * a.dil) * G::GPP + cg;
            uint4 bv[CT];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) bv[ct] = bl[ct * 16 * G::GPP];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) acc[rg][ct] = mfma_frag<XT>(af[rg], bv[ct], acc[rg][ct]);
        }
        // ---- epilogue: lane holds rows row0 .. row0 + 3 of column n of every tile
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
            const int row0 = (rt0 + rg) * 16 + 4 * g;
            if (row0 >= (EPI == EPI_UP ? ROWS : COUT)) continue;
            if constexpr (EPI == EPI_POST) {
                if (row0 != 0) continue;
                const float b0 = a.bias[0];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const int p = p0 + colbase + ct * 16 + n;
                    if (p < valid) a.out[wbase + p] = tanhf_(acc[rg][ct][0] + b0);
                }
            } else {
                const int co = EPI == EPI_UP ? row0 % COUT : row0;
                const int phase = EPI == EPI_UP ? row0 / COUT : 0;
                const float4 bv = *reinterpret_cast<const float4*>(a.bias + co);
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const int p = p0 + colbase + ct * 16 + n;
                    if (p >= valid) continue;
                    const size_t o = ((wbase + p) * U + phase) * COUT + co;
                    const float4 r = make_float4(acc[rg][ct][0] + bv.x, acc[rg][ct][1] + bv.y, acc[rg][ct][2] + bv.z, acc[rg][ct][3] + bv.w);
                    *reinterpret_cast<float4*>(a.out + o) = r;
                }
            }
        }
    }
}

// grid = (tiles of a window, windows): one convolution of one kind
template <typename XT, int CIN, int ROWS, int COUT, int KS, int EPI, bool PRE_ACT, bool SRC3, int U, bool SHORT>
__global__ __launch_bounds__(VC_THREADS) void k_vconv(VcArgs a, const int* __restrict__ len, int rate, int window)
{
    constexpr int TP = vc_tp<XT, CIN, ROWS, (KS - 1) / 2, SHORT>();
    __shared__ uint4 lds[(TP + 2 * ((KS - 1) / 2)) * VcGeom<XT, CIN>::GPP];
    const int w = blockIdx.y, valid = len[w] * rate, p0 = blockIdx.x * TP;
    if (p0 >= valid) return;
    conv_tile<XT, CIN, ROWS, COUT, KS, TP, EPI, PRE_ACT, SRC3, U>(a, valid, (size_t)w * window * rate, p0, lds);
}

// ---------------------------------------------------------------------------
// One residual block, all three convolution pairs, on one tile of positions without leaving the CU:
//   for d in (1, 3, 5):  x += conv_{k,1}(lrelu(conv_{k,d}(lrelu(x))))
// The residual stream x of the tile -- TP positions plus the halo H = (k-1)/2 * 12 that the six convolutions
// eat on each side -- stays in registers in the MFMA accumulator layout (lane = one position, four channels
// per row tile), so the second convolution of a pair accumulates straight onto it.  The operand of the next
// convolution (leaky ReLU applied, operand type, zero outside the request's window) goes through one LDS
// buffer: written by the lanes that own the values, read as B fragments by every wave.  Values near the
// edge of the region are wrong after a convolution (their neighbours were not staged); the error front moves
// inwards by one halo per convolution and stops exactly at the TP positions that are written out.
// ---------------------------------------------------------------------------
struct VrArgs {
    const float* in;                         // the stage's upsampled activations
    float* out;                              // the block's output
    const uint4* W[2 * VOC_PAIRS];           // [2 pair + {0: dilated, 1: plain}]
    const float* bias[2 * VOC_PAIRS];
};
struct VrArgs3 { VrArgs b[VOC_BLOCKS]; };

constexpr int VR_LDS_MAX = 160 * 1024;

template <typename XT, int C, int KS, int TP> struct VrGeom {
    static constexpr int HALF = (KS - 1) / 2;
    static constexpr int H = HALF * 12;                       // sum over d = 1, 3, 5 of (d + 1) * HALF
    static constexpr int NCOL = (TP + 2 * H + 63) / 64;       // column tiles per wave
    static constexpr int W = 64 * NCOL;                       // positions of the region
    static constexpr int PADR = HALF * 5;                     // zero rows on each side: the widest tap offset
    static constexpr int OPERAND_VECS = (W + 2 * PADR) * VcGeom<XT, C>::GPP;     // 16-byte pieces of the operand buffer
    // one convolution's weights (A-fragment order) as 16-byte pieces; they go through LDS when both fit
    static constexpr int W_VECS = ((C < 16 ? 16 : C) / 16) * ((KS * C + Frag<XT>::KB - 1) / Frag<XT>::KB) * 64;
    static constexpr bool W_LDS = (OPERAND_VECS + W_VECS) * 16 <= VR_LDS_MAX;
    static constexpr int BYTES = (OPERAND_VECS + (W_LDS ? W_VECS : 0)) * 16;
};

// Positions per workgroup of the fused kernel.  Up to 32 channels the region's accumulators (x and one convolution's
// output) and the operand buffer are small enough for two workgroups to share a CU: while one is in a convolution
// (MFMA) the other can be preparing an operand (VALU).  Small batches take half of that, a request or two a quarter:
// more workgroups, each with a shorter chain (and a larger share of halo: the sum of their work grows).
template <int C, int LEVEL> constexpr int vr_tp() { return (C >= 32 ? 256 : 512) >> LEVEL; }
constexpr int VR_SMALL_BELOW = 1024;             // workgroups of the large tiling below which the half tiles are used
constexpr int VR_TINY_BELOW = 128;               // ... and the quarter tiles

// acc[rt][ct] += W (rows rt, all k) * operand(columns of tile ct shifted by the taps)
template <typename XT, int C, int KS, int NCOL, int PADR>
__device__ __forceinline__ void conv_regs(const uint4* __restrict__ Wf, int dil, const uint4* lds, int col0, int lane,
                                          floatx4 (&acc)[(C < 16 ? 16 : C) / 16][NCOL])
{
    using G = VcGeom<XT, C>;
    constexpr int KB = Frag<XT>::KB;
    constexpr int RT = (C < 16 ? 16 : C) / 16;
    constexpr int NK = (KS * C + KB - 1) / KB;
    constexpr int NQ = KS * G::GP;
    const int n = lane & 15, g = lane >> 4;
    const uint4* Wl = Wf + lane;
#pragma unroll 2
    for (int kf = 0; kf < NK; ++kf) {
        uint4 af[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) af[rt] = Wl[((size_t)rt * NK + kf) * 64];
        const int q = min(kf * 4 + g, NQ - 1);
        const int tap = q / G::GP, cg = q - tap * G::GP;
        const uint4* bl = lds + (col0 + n + PADR + (tap - (KS - 1) / 2) * dil) * G::GPP + cg;
        // all B fragments of this k step are requested before the first MFMA waits for one
        uint4 bv[NCOL];
#pragma unroll
        for (int ct = 0; ct < NCOL; ++ct) bv[ct] = bl[ct * 16 * G::GPP];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ct = 0; ct < NCOL; ++ct)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[rt][ct] = mfma_frag<XT>(af[rt], bv[ct], acc[rt][ct]);
    }
}

template <typename XT, int C, int KS, int TP>
__device__ __forceinline__ void resblock_tile(const VrArgs& a, int valid, size_t wbase, int p0, uint4* lds)
{
    using G = VcGeom<XT, C>;
    using R = VrGeom<XT, C, KS, TP>;
    constexpr int RT = (C < 16 ? 16 : C) / 16, NCOL = R::NCOL;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int col0 = wave * 16 * NCOL;           // this wave's first position of the region
    const int pbase = p0 - R::H;                 // the region's first position inside the window
    const bool rows_ok = 4 * g < C;              // C = 8: the upper half of the 16-row tile is padding

    // zero rows in front of and behind the region: never written again
    for (int idx = tid; idx < 2 * R::PADR * G::GPP; idx += VC_THREADS) {
        const int r = idx / G::GPP, c = idx - r * G::GPP;
        lds[(r < R::PADR ? r : R::W + r) * G::GPP + c] = make_uint4(0, 0, 0, 0);
    }
    // The weights of the next convolution are fetched into registers while the current one computes and
    // handed to LDS together with its operand, so no MFMA loop waits for L2 (where they fit beside the operand).
    constexpr int W_PER = (R::W_VECS + VC_THREADS - 1) / VC_THREADS;
    uint4* wbuf = lds + R::OPERAND_VECS;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 wreg[R::W_LDS ? W_PER : 1];
    auto fetch = [&](const uint4* __restrict__ Wg) __attribute__((always_inline)) {
        if constexpr (R::W_LDS) {
#pragma unroll
            for (int i = 0; i < W_PER; ++i) wreg[i] = reinterpret_cast<const u32x4*>(Wg)[min(tid + i * VC_THREADS, R::W_VECS - 1)];
        }
    };
    auto stash = [&]() __attribute__((always_inline)) {
        if constexpr (R::W_LDS) {
#pragma unroll
            for (int i = 0; i < W_PER; ++i)
                if (tid + i * VC_THREADS < R::W_VECS) reinterpret_cast<u32x4*>(wbuf)[tid + i * VC_THREADS] = wreg[i];
        }
    };
    fetch(a.W[0]);
    floatx4 x[RT][NCOL];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < NCOL; ++ct) {
            const int p = pbase + col0 + ct * 16 + n;
            floatx4 v = {0.f, 0.f, 0.f, 0.f};
            if (p >= 0 && p < valid && rows_ok) v = *reinterpret_cast<const floatx4*>(a.in + (wbase + p) * C + rt * 16 + 4 * g);
            x[rt][ct] = v;
        }
    // operand of the next convolution: lrelu, zero outside the window, operand type
    const bool edge = pbase < 0 || pbase + R::W > valid;        // only tiles at a window's ends need the mask
    auto put = [&](const floatx4 (&v)[RT][NCOL]) __attribute__((always_inline)) {
        if (!rows_ok) return;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ct = 0; ct < NCOL; ++ct) {
                const int j = col0 + ct * 16 + n, p = pbase + j;
                const bool in = !edge || (p >= 0 && p < valid);
                const float4 o = make_float4(in ? lrelu(v[rt][ct][0]) : 0.f, in ? lrelu(v[rt][ct][1]) : 0.f,
                                             in ? lrelu(v[rt][ct][2]) : 0.f, in ? lrelu(v[rt][ct][3]) : 0.f);
                lds_put4<XT>(lds, (j + R::PADR) * G::CINP + rt * 16 + 4 * g, o);
            }
    };
    auto bias_of = [&](const float* b, int rt) __attribute__((always_inline)) {
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (rows_ok) v = *reinterpret_cast<const floatx4*>(b + rt * 16 + 4 * g);
        return v;
    };
    put(x);
    stash();
    __syncthreads();
#pragma unroll 1
    for (int pair = 0; pair < VOC_PAIRS; ++pair) {
        fetch(a.W[2 * pair + 1]);
        floatx4 t[RT][NCOL];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const floatx4 b1 = bias_of(a.bias[2 * pair], rt);
#pragma unroll
            for (int ct = 0; ct < NCOL; ++ct) t[rt][ct] = b1;
        }
        conv_regs<XT, C, KS, NCOL, R::PADR>(R::W_LDS ? wbuf : a.W[2 * pair], 2 * pair + 1, lds, col0, lane, t);
        __syncthreads();                          // every wave has read the old operand and the old weights
        put(t);
        stash();
        __syncthreads();
        if (pair + 1 < VOC_PAIRS) fetch(a.W[2 * pair + 2]);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const floatx4 b2 = bias_of(a.bias[2 * pair + 1], rt);
#pragma unroll
            for (int ct = 0; ct < NCOL; ++ct) x[rt][ct] += b2;
        }
        conv_regs<XT, C, KS, NCOL, R::PADR>(R::W_LDS ? wbuf : a.W[2 * pair + 1], 1, lds, col0, lane, x);
        if (pair + 1 < VOC_PAIRS) {
            __syncthreads();
            put(x);
            stash();
            __syncthreads();
        }
    }
    if (!rows_ok) return;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < NCOL; ++ct) {
            const int j = col0 + ct * 16 + n, p = pbase + j;
            if (j >= R::H && j < R::H + TP && p < valid)
                *reinterpret_cast<floatx4*>(a.out + (wbase + p) * C + rt * 16 + 4 * g) = x[rt][ct];
        }
}

// grid = (tiles, windows, 3): the three residual blocks (kernels 3, 7, 11) of a stage
template <typename XT, int C, int TP>
__global__ __launch_bounds__(VC_THREADS) void k_vres(VrArgs3 a3, const int* __restrict__ len, int rate, int window)
{
    extern __shared__ uint4 lds_dyn[];
    const int w = blockIdx.y, valid = len[w] * rate, p0 = blockIdx.x * TP;
    if (p0 >= valid) return;
    const size_t wbase = (size_t)w * window * rate;
    if (blockIdx.z == 0) resblock_tile<XT, C, 3, TP>(a3.b[0], valid, wbase, p0, lds_dyn);
    else if (blockIdx.z == 1) resblock_tile<XT, C, 7, TP>(a3.b[1], valid, wbase, p0, lds_dyn);
    else resblock_tile<XT, C, 11, TP>(a3.b[2], valid, wbase, p0, lds_dyn);
}

// One workgroup per window: rows [0, ov) <- tail(M_pre) of the slot (if the request has a previous chunk), then M_cur;
// the slot's tail becomes M_cur's last ov frames (Eq. 4) unless this was the request's last chunk.
__global__ __launch_bounds__(256) void k_voc_splice(VocBatch b, const float* __restrict__ d_mel, float* __restrict__ x_mel,
                                                    float* __restrict__ m_tail, int* __restrict__ len, int ov, int window)
{
    const int w = blockIdx.x, tid = threadIdx.x;
    const int nf = b.n_frames[w], hp = b.has_prev[w], last = b.last[w];
    const float* src = d_mel + (size_t)b.src_row[w] * VOC_N_MEL;
    float* dst = x_mel + (size_t)w * window * VOC_N_MEL;
    float* tail = m_tail + (size_t)b.slot[w] * ov * VOC_N_MEL;
    const int ovw = hp ? ov : 0;
    for (int e = tid; e < ov * VOC_N_MEL; e += 256) {
        if (hp) dst[e] = tail[e];
        if (!last) tail[e] = src[(size_t)(nf - ov) * VOC_N_MEL + e];
    }
    for (int e = tid; e < nf * VOC_N_MEL; e += 256) dst[(size_t)ovw * VOC_N_MEL + e] = src[e];
    if (tid == 0) len[w] = ovw + nf;
}

// grid = (frames of a window, windows), one sample per thread.  The thread that owns sample i of the overlap
// region reads the slot's old tail(S_pre)[i] before it writes the new one, so nothing races.
__global__ __launch_bounds__(VOC_HOP) void k_voc_fade(VocBatch b, const float* __restrict__ audio, const float* __restrict__ alpha,
                                                      const float* __restrict__ beta, float* __restrict__ s_tail,
                                                      float* __restrict__ d_audio, int ov, int window)
{
    const int w = blockIdx.y, i = blockIdx.x * VOC_HOP + threadIdx.x;
    const int hp = b.has_prev[w], last = b.last[w];
    const int N = ov * VOC_HOP;
    const int L = ((hp ? ov : 0) + b.n_frames[w]) * VOC_HOP;
    if (i >= L) return;
    const float* S = audio + (size_t)w * window * VOC_HOP;
    float v = S[i];
    if (i < N) {
        float* tail = s_tail + (size_t)b.slot[w] * N;
        if (hp) v = alpha[i] * v + beta[i] * tail[i];
        if (!last) tail[i] = S[L - N + i];
    }
    const int emit = last ? L : L - N;
    if (i < emit) d_audio[(size_t)b.out_off[w] + i] = v;
}

// grid = (tiles of a window, windows, row groups).  SHORT: tiles of 64 positions - for the layer that runs at one position
// per frame, where a window is a few dozen positions long, and for every layer of a batch so small that the large tiles
// would leave most of the chip idle (an output's sum does not depend on the tile it falls in).
constexpr int VC_SHORT_BELOW = 512;              // workgroups of the large tiling below which the short one is used
template <typename XT, int CIN, int ROWS, int COUT, int KS, int EPI, bool PRE_ACT, bool SRC3, int U, bool SHORT>
void conv_launch(const VcArgs& a, const int* len, int rate, int window, int n_windows, hipStream_t s)
{
    constexpr int TP = vc_tp<XT, CIN, ROWS, (KS - 1) / 2, SHORT>();
    constexpr int RT = ROWS / 16, RG = RT < 4 ? RT : 4;
    const dim3 grid((window * rate + TP - 1) / TP, n_windows, RT / RG);
    if constexpr (!SHORT) {
        if ((long)grid.x * grid.y * grid.z < VC_SHORT_BELOW) {
            conv_launch<XT, CIN, ROWS, COUT, KS, EPI, PRE_ACT, SRC3, U, true>(a, len, rate, window, n_windows, s);
            return;
        }
    }
    hipLaunchKernelGGL((k_vconv<XT, CIN, ROWS, COUT, KS, EPI, PRE_ACT, SRC3, U, SHORT>), grid, dim3(VC_THREADS), 0, s, a, len, rate, window);
}

template <typename XT, int C, int LEVEL>
hipError_t blocks_launch_tp(const VrArgs3& a, const int* len, int rate, int window, int n_windows, hipStream_t s)
{
    constexpr int TP = vr_tp<C, LEVEL>();
    constexpr int L3 = VrGeom<XT, C, 3, TP>::BYTES, L7 = VrGeom<XT, C, 7, TP>::BYTES, L11 = VrGeom<XT, C, 11, TP>::BYTES;
    constexpr int LDS = L3 > L7 ? (L3 > L11 ? L3 : L11) : (L7 > L11 ? L7 : L11);      // the three kernels share a launch
    auto kern = k_vres<XT, C, TP>;
    static bool attr_set = false;                            // dynamic LDS above 64 KB has to be allowed once per kernel
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid((window * rate + TP - 1) / TP, n_windows, VOC_BLOCKS);
    hipLaunchKernelGGL(kern, grid, dim3(VC_THREADS), LDS, s, a, len, rate, window);
    return hipSuccess;
}

template <typename XT, int C>
hipError_t blocks_launch(const VrArgs3& a, const int* len, int rate, int window, int n_windows, hipStream_t s)
{
    const long wgs = (long)((window * rate + vr_tp<C, 0>() - 1) / vr_tp<C, 0>()) * n_windows * VOC_BLOCKS;
    return wgs < VR_TINY_BELOW    ? blocks_launch_tp<XT, C, 2>(a, len, rate, window, n_windows, s)
           : wgs < VR_SMALL_BELOW ? blocks_launch_tp<XT, C, 1>(a, len, rate, window, n_windows, s)
                                  : blocks_launch_tp<XT, C, 0>(a, len, rate, window, n_windows, s);
}

template <typename XT, int S>
hipError_t stage_launch(const VocoderPtrs& d, int n_windows, hipStream_t s)
{
    constexpr int CIN = VOC_C0 >> S, C = CIN / 2, U = voc_rate(S);
    constexpr int rate_in = S == 0 ? 1 : voc_cum_rate(S - 1), rate = voc_cum_rate(S);
    VcArgs up{};
    up.in0 = S == 0 ? d.x0 : d.r[0];
    up.in1 = d.r[1];
    up.in2 = d.r[2];
    up.out = d.y;
    up.W = reinterpret_cast<const uint4*>(d.up_w[S]);
    up.bias = d.up_b[S];
    up.dil = 1;
    conv_launch<XT, CIN, U * C, C, 3, EPI_UP, true, (S > 0), U, (S == 0)>(up, d.len, rate_in, d.window, n_windows, s);
    VrArgs3 rb{};
    for (int b = 0; b < VOC_BLOCKS; ++b) {
        rb.b[b].in = d.y;
        rb.b[b].out = d.r[b];
        for (int i = 0; i < 2 * VOC_PAIRS; ++i) {
            rb.b[b].W[i] = reinterpret_cast<const uint4*>(d.res_w[S][b][i]);
            rb.b[b].bias[i] = d.res_b[S][b][i];
        }
    }
    return blocks_launch<XT, C>(rb, d.len, rate, d.window, n_windows, s);
}

template <typename XT>
hipError_t generator_typed(const VocoderPtrs& d, int n_windows, hipStream_t s)
{
    VcArgs pre{};
    pre.in0 = d.x_mel;
    pre.out = d.x0;
    pre.W = reinterpret_cast<const uint4*>(d.pre_w);
    pre.bias = d.pre_b;
    pre.dil = 1;
    conv_launch<XT, VOC_N_MEL, VOC_C0, VOC_C0, VOC_K_PRE, EPI_PLAIN, false, false, 1, true>(pre, d.len, 1, d.window, n_windows, s);
    hipError_t e = stage_launch<XT, 0>(d, n_windows, s);
    if (e == hipSuccess) e = stage_launch<XT, 1>(d, n_windows, s);
    if (e == hipSuccess) e = stage_launch<XT, 2>(d, n_windows, s);
    if (e == hipSuccess) e = stage_launch<XT, 3>(d, n_windows, s);
    if (e != hipSuccess) return e;
    VcArgs post{};
    post.in0 = d.r[0];
    post.in1 = d.r[1];
    post.in2 = d.r[2];
    post.out = d.audio;
    post.W = reinterpret_cast<const uint4*>(d.post_w);
    post.bias = d.post_b;
    post.dil = 1;
    conv_launch<XT, voc_channels(VOC_STAGES - 1), 16, 1, VOC_K_POST, EPI_POST, true, true, 1, false>(post, d.len, VOC_HOP, d.window, n_windows, s);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_vocoder_splice(const VocoderPtrs& d, const VocBatch& b, const float* d_mel, hipStream_t s)
{
    hipLaunchKernelGGL(k_voc_splice, dim3(b.n), dim3(256), 0, s, b, d_mel, d.x_mel, d.m_tail, d.len, d.overlap, d.window);
    return hipGetLastError();
}

hipError_t launch_vocoder_generator(const VocoderPtrs& d, int wdtype, int n_windows, hipStream_t s)
{
    return wdtype == 0 ? generator_typed<float>(d, n_windows, s) : generator_typed<h16_t>(d, n_windows, s);
}

hipError_t launch_vocoder_fade(const VocoderPtrs& d, const VocBatch& b, float* d_audio, hipStream_t s)
{
    hipLaunchKernelGGL(k_voc_fade, dim3(d.window, b.n), dim3(VOC_HOP), 0, s, b, d.audio, d.alpha, d.beta, d.s_tail, d_audio,
                       d.overlap, d.window);
    return hipGetLastError();
}

}  // namespace tts
