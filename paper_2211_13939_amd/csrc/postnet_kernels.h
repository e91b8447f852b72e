// Host-visible launch wrapper of the PostNet kernels (postnet.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tts {

constexpr int PN_LAYERS = 5;
constexpr int PN_TAPS = 5;
constexpr int PN_N_MEL = 80;
constexpr int PN_CIN0 = 96;          // the mel channels padded to whole 64-byte fragments in both dtypes
constexpr int PN_CHANNELS = 512;
constexpr int PN_COUT_LAST = 80;

struct PostnetPtrs {
    const void* W[PN_LAYERS];   // weight dtype, MFMA A-fragment order, k = tap * C_in(padded) + channel
    const float* b[PN_LAYERS];  // [c_out]
    void* act[2];               // activations between layers, fragment order, [column tile][channel fragment][lane][16 B]
    int* cmeta;                 // [columns padded to 16] (window length << 16) | index inside the window; 0 for padding
    int* orow;                  // [columns padded to 16] output row of the column, -1 = context or padding
    int n_mel;
};

// Up to PN_META_WINDOWS windows of one call, as a kernel argument (no host-to-device copy): the device
// expands it into the per-column tables.
constexpr int PN_META_WINDOWS = 256;
struct PnWindows {
    int n;
    int col0[PN_META_WINDOWS];        // first column of the window
    int row0[PN_META_WINDOWS];        // output row of the window's first kept frame
    uint16_t len[PN_META_WINDOWS];    // frames in the window
    uint16_t keep[PN_META_WINDOWS];   // frames of context in front of the chunk
};
// n_col_pad: columns rounded up to whole tiles; `first` clears the padding columns too
hipError_t launch_postnet_meta(const PostnetPtrs& d, const PnWindows& w, int n_col, int n_col_pad, bool first, hipStream_t s);

// mel: device fp32 [n_col][n_mel]; out: device fp32 [kept rows][n_mel]
hipError_t launch_postnet(const PostnetPtrs& d, int wdtype, const float* mel, int n_col, float* out, hipStream_t s);

}  // namespace tts
