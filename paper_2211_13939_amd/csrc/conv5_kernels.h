// Kernel-5 convolution over time on a ragged batch of windows, on MFMA: shared by the PostNet (windows = chunks with
// context, tanh) and the acoustic encoder (windows = the token sequences of requests, ReLU).
//
// A convolution layer is a GEMM  Y[c_out][column] = W[c_out][tap * C_in + c_in] * X[c_in][column + tap - 2]
// with the columns of all windows packed back to back; a column that would leave its own window
// reads zero ("same" padding per window).  It runs on MFMA with 16 columns as N:
//   * activations between layers live in HBM in the same MFMA B-operand fragment order as the
//     decoder's activations (16 columns form a tile, 64 bytes of channels per fragment), so a
//     layer's output is stored exactly as the next layer loads it;
//   * a workgroup owns one 16-row tile of output channels and one or two column tiles; it stages the
//     columns it needs (its tiles plus two columns on either side) in LDS once, and its eight
//     waves split K = 5 * C_in: every wave keeps its share of the weight fragments in registers,
//     builds the five shifted B operands from LDS, and the partial sums meet in LDS;
//   * bias, the activation, the residual sum of the PostNet's last layer and the selection of the chunk's own
//     frames are fused into the epilogue.
#pragma once
#include "postnet_kernels.h"
#include "mfma.h"

namespace tts {

constexpr int PN_THREADS = 512;
constexpr int PN_WAVES = PN_THREADS / 64;
constexpr int PN_HALO = PN_TAPS / 2;             // columns needed on either side of a tile
// column tiles per workgroup: what fits 64 KB of LDS next to the reduction buffer
template <typename XT> struct PnCT { static constexpr int value = sizeof(XT) == 2 ? 2 : 1; };

// epilogue of a layer: tanh / ReLU into the next layer's input, or the PostNet's last layer
enum { PN_EPI_TANH = 0, PN_EPI_LAST = 1, PN_EPI_RELU = 2 };
template <int EPI> __device__ __forceinline__ float pn_act(float x) { return EPI == PN_EPI_RELU ? fmaxf(x, 0.f) : tanhf_(x); }

// One layer.  grid = (COUT / 16, ceil(column tiles / PnCT)).
//   cmeta[col] = (frames in the column's window << 16) | the column's index inside its window
//   PN_EPI_LAST: out[orow[col]][*] = mel[col][*] + bias + sum  for columns with orow >= 0 (the chunk's own frames)
template <typename XT, int CIN, int COUT, int EPI>
__global__ __launch_bounds__(PN_THREADS) void k_pn_conv(
    const uint4* __restrict__ Wfrag, const float* __restrict__ bias, const uint4* __restrict__ Xin, XT* __restrict__ Xout,
    const int* __restrict__ cmeta, int n_ctiles, const float* __restrict__ mel, int n_mel, const int* __restrict__ orow,
    float* __restrict__ out)
{
    constexpr int KB = Frag<XT>::KB, EPL = Frag<XT>::EPL;
    constexpr int PN_CT = PnCT<XT>::value;
    constexpr int NKF = CIN / KB;                      // channel fragments per column tile
    constexpr int NKT = PN_TAPS * NKF;                 // K fragments of the GEMM
    constexpr int NFW = (NKT + PN_WAVES - 1) / PN_WAVES;   // per wave
    constexpr int ROWS = PN_CT * 16 + 2 * PN_HALO;     // staged columns
    constexpr int LD = CIN * (int)sizeof(XT) + 16;     // bytes per staged column: an odd number of 16-byte pieces
    static_assert(CIN % KB == 0 && COUT % 16 == 0, "channel counts must fill whole fragments / row tiles");

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jl = lane & 15, g = lane >> 4;
    const int rt = blockIdx.x;
    const int ct0 = blockIdx.y * PN_CT;

    __shared__ __attribute__((aligned(16))) unsigned char s_x[ROWS * LD];
    __shared__ floatx4 red[PN_WAVES][PN_CT][64];

    // this wave's share of the weights: fragments wave, wave + 8, ... of row tile rt (k = tap * CIN + channel)
    uint4 a[NFW];
#pragma unroll
    for (int i = 0; i < NFW; ++i) {
        const int f = wave + i * PN_WAVES;
        a[i] = f < NKT ? Wfrag[xfrag(NKT, rt, f, lane)] : make_uint4(0, 0, 0, 0);
    }
    // the columns of this workgroup's tiles and two more on either side, once, into LDS:
    // piece (row, channel fragment cf, lane group gg) = 16 bytes of channels cf * KB + gg * EPL ..
    const int col_first = ct0 * 16 - PN_HALO;
    const int n_col_pad = n_ctiles * 16;
    for (int p = tid; p < ROWS * NKF * 4; p += PN_THREADS) {
        const int row = p / (NKF * 4), rem = p - row * (NKF * 4);
        const int cf = rem >> 2, gg = rem & 3;
        const int col = col_first + row;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (col >= 0 && col < n_col_pad) v = Xin[xfrag(NKF, col >> 4, cf, (col & 15) + 16 * gg)];
        *reinterpret_cast<uint4*>(&s_x[row * LD + (cf * KB + gg * EPL) * (int)sizeof(XT)]) = v;
    }
    // which taps stay inside the column's own window (bit d+2 for column offset d)
    int tapmask[PN_CT];
#pragma unroll
    for (int c = 0; c < PN_CT; ++c) {
        const int col = min((ct0 + c) * 16 + jl, n_col_pad - 1);
        const int m = cmeta[col];
        const int t = m & 0xFFFF, T = m >> 16;
        int bits = 0;
#pragma unroll
        for (int d = -PN_HALO; d <= PN_HALO; ++d) bits |= (t + d >= 0 && t + d < T) ? (1 << (d + PN_HALO)) : 0;
        tapmask[c] = bits;
    }
    floatx4 bias4 = {0.f, 0.f, 0.f, 0.f};
    if (wave < PN_CT) bias4 = *reinterpret_cast<const floatx4*>(bias + rt * 16 + 4 * g);
    __syncthreads();

#pragma unroll
    for (int c = 0; c < PN_CT; ++c) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        if (ct0 + c < n_ctiles) {
#pragma unroll
            for (int i = 0; i < NFW; ++i) {
                const int f = wave + i * PN_WAVES;           // = tap * NKF + cf
                if (f < NKT) {
                    const int tap = f / NKF, cf = f - tap * NKF;
                    uint4 b = *reinterpret_cast<const uint4*>(&s_x[(c * 16 + jl + tap) * LD + (cf * KB + g * EPL) * (int)sizeof(XT)]);
                    if (!((tapmask[c] >> tap) & 1)) b = make_uint4(0, 0, 0, 0);
                    acc = mfma_frag<XT>(a[i], b, acc);
                }
            }
        }
        red[wave][c][lane] = acc;
    }
    __syncthreads();
    if (wave < PN_CT && ct0 + wave < n_ctiles) {
        floatx4 y = bias4;
#pragma unroll
        for (int w = 0; w < PN_WAVES; ++w) y += red[w][wave][lane];
        const int col = (ct0 + wave) * 16 + jl;
        const int ch = rt * 16 + 4 * g;                  // the lane holds channels ch .. ch + 3 of its column
        if constexpr (EPI != PN_EPI_LAST) {
            const float y0 = pn_act<EPI>(y[0]), y1 = pn_act<EPI>(y[1]), y2 = pn_act<EPI>(y[2]), y3 = pn_act<EPI>(y[3]);
            XT* dst = Xout + xoff<XT>(COUT / KB, col, ch);
            if constexpr (sizeof(XT) == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(pack2<XT>(y0, y1), pack2<XT>(y2, y3));
            else *reinterpret_cast<float4*>(dst) = make_float4(y0, y1, y2, y3);
        } else {
            const int r = orow[col];
            if (r >= 0 && ch < n_mel) {
                const float4 m = *reinterpret_cast<const float4*>(mel + (size_t)col * n_mel + ch);
                *reinterpret_cast<float4*>(out + (size_t)r * n_mel + ch) = make_float4(m.x + y[0], m.y + y[1], m.z + y[2], m.w + y[3]);
            }
        }
    }
}

// The same layer for large batches.  The kernel above spreads a small batch over many workgroups (one
// row tile each, K split over the waves) but pulls 80 KB of weights per 160 MFMAs; here a workgroup owns
// 8 row tiles (one per wave, no K split, no reduction) and PN_WCT column tiles, whose staged columns in LDS
// serve all eight waves: 8 x 80 KB of weights for 8 x 80 x PN_WCT MFMAs.
constexpr int PN_WCT = 4;
template <typename XT, int CIN, int COUT, int EPI>
__global__ __launch_bounds__(PN_THREADS) void k_pn_conv_wide(
    const uint4* __restrict__ Wfrag, const float* __restrict__ bias, const uint4* __restrict__ Xin, XT* __restrict__ Xout,
    const int* __restrict__ cmeta, int n_ctiles, const float* __restrict__ mel, int n_mel, const int* __restrict__ orow,
    float* __restrict__ out)
{
    constexpr int KB = Frag<XT>::KB, EPL = Frag<XT>::EPL;
    constexpr int NKF = CIN / KB, NKT = PN_TAPS * NKF;
    constexpr int ROWS = PN_WCT * 16 + 2 * PN_HALO;
    constexpr int LD = CIN * (int)sizeof(XT) + 16;
    constexpr int NRT = COUT / 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];   // ROWS * LD bytes
    unsigned char* s_x = s_dyn;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jl = lane & 15, g = lane >> 4;
    const int rt = blockIdx.x * PN_WAVES + wave;           // this wave's row tile (may lie beyond the last one)
    const bool row_on = rt < NRT;
    const int rtc = row_on ? rt : NRT - 1;
    const int ct0 = blockIdx.y * PN_WCT;
    const int n_col_pad = n_ctiles * 16;
    const int col_first = ct0 * 16 - PN_HALO;

    for (int p = tid; p < ROWS * NKF * 4; p += PN_THREADS) {
        const int row = p / (NKF * 4), rem = p - row * (NKF * 4);
        const int cf = rem >> 2, gg = rem & 3;
        const int col = col_first + row;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (col >= 0 && col < n_col_pad) v = Xin[xfrag(NKF, col >> 4, cf, (col & 15) + 16 * gg)];
        *reinterpret_cast<uint4*>(&s_x[row * LD + (cf * KB + gg * EPL) * (int)sizeof(XT)]) = v;
    }
    int tapmask[PN_WCT];
#pragma unroll
    for (int c = 0; c < PN_WCT; ++c) {
        const int col = min((ct0 + c) * 16 + jl, n_col_pad - 1);
        const int m = cmeta[col];
        const int t = m & 0xFFFF, T = m >> 16;
        int bits = 0;
#pragma unroll
        for (int d = -PN_HALO; d <= PN_HALO; ++d) bits |= (t + d >= 0 && t + d < T) ? (1 << (d + PN_HALO)) : 0;
        tapmask[c] = bits;
    }
    const floatx4 bias4 = *reinterpret_cast<const floatx4*>(bias + rtc * 16 + 4 * g);
    __syncthreads();

    floatx4 acc[PN_WCT];
#pragma unroll
    for (int c = 0; c < PN_WCT; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
    // weights of the wave's row tile stream through registers, PF fragments ahead
    constexpr int PF = 16;
    uint4 a[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) a[i] = Wfrag[xfrag(NKT, rtc, i < NKT ? i : NKT - 1, lane)];
#pragma unroll 1
    for (int f0 = 0; f0 < NKT; f0 += PF) {
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int f = f0 + i;
            const uint4 af = a[i];
            a[i] = Wfrag[xfrag(NKT, rtc, min(f + PF, NKT - 1), lane)];   // unconditional: past the end it re-reads the last one
            if (f < NKT) {
                const int tap = f / NKF, cf = f - tap * NKF;
#pragma unroll
                for (int c = 0; c < PN_WCT; ++c) {
                    uint4 b = *reinterpret_cast<const uint4*>(&s_x[(c * 16 + jl + tap) * LD + (cf * KB + g * EPL) * (int)sizeof(XT)]);
                    if (!((tapmask[c] >> tap) & 1)) b = make_uint4(0, 0, 0, 0);
                    acc[c] = mfma_frag<XT>(af, b, acc[c]);
                }
            }
        }
    }
    if (!row_on) return;
#pragma unroll
    for (int c = 0; c < PN_WCT; ++c) {
        if (ct0 + c >= n_ctiles) break;
        const floatx4 y = acc[c] + bias4;
        const int col = (ct0 + c) * 16 + jl;
        const int ch = rt * 16 + 4 * g;
        if constexpr (EPI != PN_EPI_LAST) {
            const float y0 = pn_act<EPI>(y[0]), y1 = pn_act<EPI>(y[1]), y2 = pn_act<EPI>(y[2]), y3 = pn_act<EPI>(y[3]);
            XT* dst = Xout + xoff<XT>(COUT / KB, col, ch);
            if constexpr (sizeof(XT) == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(pack2<XT>(y0, y1), pack2<XT>(y2, y3));
            else *reinterpret_cast<float4*>(dst) = make_float4(y0, y1, y2, y3);
        } else {
            const int r = orow[col];
            if (r >= 0 && ch < n_mel) {
                const float4 m = *reinterpret_cast<const float4*>(mel + (size_t)col * n_mel + ch);
                *reinterpret_cast<float4*>(out + (size_t)r * n_mel + ch) = make_float4(m.x + y[0], m.y + y[1], m.z + y[2], m.w + y[3]);
            }
        }
    }
}

template <typename XT, int CIN, int COUT, int EPI>
inline hipError_t conv_layer(bool wide, const void* W, const float* b, const void* xin, XT* xout, const int* cmeta, int n_ctiles,
                             const float* mel, int n_mel, const int* orow, float* out, hipStream_t s)
{
    // fewer row tiles than a wide workgroup has waves (the PostNet's last layer, 512 -> 80): the wide kernel would run on a
    // few dozen workgroups with idle waves; the narrow one spreads the layer over the chip whatever the batch
    if (COUT / 16 < PN_WAVES) wide = false;
    if (wide) {
        constexpr int LDS = (PN_WCT * 16 + 2 * PN_HALO) * (CIN * (int)sizeof(XT) + 16);
        auto kern = k_pn_conv_wide<XT, CIN, COUT, EPI>;
        static bool attr_set = false;             // dynamic LDS above 64 KB has to be allowed once per kernel
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        const dim3 grid((COUT / 16 + PN_WAVES - 1) / PN_WAVES, (n_ctiles + PN_WCT - 1) / PN_WCT);
        hipLaunchKernelGGL(kern, grid, dim3(PN_THREADS), LDS, s, (const uint4*)W, b, (const uint4*)xin, xout, cmeta, n_ctiles,
                           mel, n_mel, orow, out);
    } else {
        constexpr int CT = PnCT<XT>::value;
        const dim3 grid(COUT / 16, (n_ctiles + CT - 1) / CT);
        hipLaunchKernelGGL((k_pn_conv<XT, CIN, COUT, EPI>), grid, dim3(PN_THREADS), 0, s, (const uint4*)W, b, (const uint4*)xin,
                           xout, cmeta, n_ctiles, mel, n_mel, orow, out);
    }
    return hipGetLastError();
}

// batches of at least this many column tiles take the wide kernel (measured with 50-column windows, two-byte mode: the narrow
// kernel is the faster one up to 75 column tiles - 25 tiles 43 against 71 us per PostNet round -, the wide one from 100)
constexpr int PN_WIDE_FROM = 80;

}  // namespace tts
