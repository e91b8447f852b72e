// PostNet of the acoustic decoder on a ragged batch of windows (one window = the frames of one request's chunk plus the
// context in front of it): the per-column tables, the packing of the mel input and the five-layer stack.  The
// convolution kernels themselves are in conv5_kernels.h.
#include "conv5_kernels.h"

namespace tts {

// Per-column tables from the call's window list: one workgroup per window; the first launch of a call
// also marks the columns that pad the last tile.
__global__ __launch_bounds__(64) void k_pn_meta(PnWindows w, int n_col, int n_col_pad, int clear_pad, int* __restrict__ cmeta,
                                                int* __restrict__ orow)
{
    const int i = blockIdx.x;
    if (i < w.n) {
        const int T = w.len[i], keep = w.keep[i];
        for (int t = threadIdx.x; t < T; t += 64) {
            cmeta[w.col0[i] + t] = (T << 16) | t;
            orow[w.col0[i] + t] = t >= keep ? w.row0[i] + (t - keep) : -1;
        }
    }
    if (clear_pad && i == 0)
        for (int c = n_col + threadIdx.x; c < n_col_pad; c += 64) {
            cmeta[c] = 0;
            orow[c] = -1;
        }
}

hipError_t launch_postnet_meta(const PostnetPtrs& d, const PnWindows& w, int n_col, int n_col_pad, bool first, hipStream_t s)
{
    hipLaunchKernelGGL(k_pn_meta, dim3(w.n > 0 ? w.n : 1), dim3(64), 0, s, w, n_col, n_col_pad, first ? 1 : 0, d.cmeta, d.orow);
    return hipGetLastError();
}

// mel fp32 [n_col][n_mel] -> layer-1 input in fragment order, channels zero-padded to CIN
template <typename XT, int CIN>
__global__ __launch_bounds__(256) void k_pn_pack(const float* __restrict__ mel, int n_mel, int n_col, int n_col_pad, XT* __restrict__ X)
{
    constexpr int KB = Frag<XT>::KB;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int col = idx / CIN, ch = idx - col * CIN;
    if (col >= n_col_pad) return;
    const float v = (col < n_col && ch < n_mel) ? mel[(size_t)col * n_mel + ch] : 0.f;
    X[xoff<XT>(CIN / KB, col, ch)] = from_float<XT>(v);
}

template <typename XT>
static hipError_t run_typed(const PostnetPtrs& d, const float* mel, int n_col, int n_ctiles, float* out, hipStream_t s)
{
    constexpr int C1 = PN_CIN0, C = PN_CHANNELS, CO = PN_COUT_LAST;
    const int n_col_pad = n_ctiles * 16;
    const bool wide = n_ctiles >= PN_WIDE_FROM;
    XT* x0 = reinterpret_cast<XT*>(d.act[0]);
    XT* x1 = reinterpret_cast<XT*>(d.act[1]);
    hipLaunchKernelGGL((k_pn_pack<XT, C1>), dim3((n_col_pad * C1 + 255) / 256), dim3(256), 0, s, mel, d.n_mel, n_col, n_col_pad, x0);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = conv_layer<XT, C1, C, PN_EPI_TANH>(wide, d.W[0], d.b[0], x0, x1, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_TANH>(wide, d.W[1], d.b[1], x1, x0, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_TANH>(wide, d.W[2], d.b[2], x0, x1, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, C, PN_EPI_TANH>(wide, d.W[3], d.b[3], x1, x0, d.cmeta, n_ctiles, nullptr, 0, nullptr, nullptr, s);
    if (e == hipSuccess) e = conv_layer<XT, C, CO, PN_EPI_LAST>(wide, d.W[4], d.b[4], x0, (XT*)nullptr, d.cmeta, n_ctiles, mel, d.n_mel, d.orow, out, s);
    return e;
}

hipError_t launch_postnet(const PostnetPtrs& d, int wdtype, const float* mel, int n_col, float* out, hipStream_t s)
{
    const int n_ctiles = (n_col + 15) / 16;
    if (n_ctiles < 1) return hipSuccess;
    return wdtype == 0 ? run_typed<float>(d, mel, n_col, n_ctiles, out, s) : run_typed<h16_t>(d, mel, n_col, n_ctiles, out, s);
}

}  // namespace tts
