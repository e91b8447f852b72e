// Host-visible launch wrapper of the encoder kernels (encoder.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "postnet_kernels.h"

namespace tts {

constexpr int ENC_TABLES = 4;
constexpr int ENC_CONVS = 3;
constexpr int ENC_DIM = 512;
constexpr int ENC_HID = 256;
constexpr int ENC_GATES = 4 * ENC_HID;      // gate rows per direction
constexpr int ENC_MAX_BATCH = 256;

struct EncoderPtrs {
    const float* tables[ENC_TABLES];        // fp32 [vocab][dim]
    const void* conv_w[ENC_CONVS];          // weight dtype, A-fragment order, k = tap * dim + channel
    const float* conv_b[ENC_CONVS];
    const void* w_ih[2];                    // weight dtype, A-fragment order, rows permuted to unit-major / gate-minor
    const void* w_hh[2];
    const float* b[2];                      // permuted like the rows
    void* act[2];                           // activations of the convolution stack, fragment order
    int* cmeta;                             // per column: (request length << 16) | position inside the request
    int* orow;                              // written by the shared table kernel, unused here
    int* ids;                               // [tables][max_tokens]
    float* xproj;                           // [2][max_tokens][ENC_GATES]: W_ih x + b of every token, both directions
    int max_tokens;
};

// ids are already in d.ids; w lists the requests (PnWindows: col0 = first token, len); out fp32 [n_col][2 hid]
hipError_t launch_encoder(const EncoderPtrs& d, int wdtype, const PnWindows& w, int n_col, float* out, hipStream_t s);

}  // namespace tts
