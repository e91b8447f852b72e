// Host-visible launch wrappers of the vocoder kernels (vocoder.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tts {

constexpr int VOC_STAGES = 4;
constexpr int VOC_BLOCKS = 3;
constexpr int VOC_PAIRS = 3;
constexpr int VOC_N_MEL = 80;
constexpr int VOC_C0 = 128;
constexpr int VOC_HOP = 256;
constexpr int VOC_K_PRE = 7;
constexpr int VOC_K_POST = 7;
constexpr int VOC_MAX_BATCH = 256;
constexpr int VOC_MAX_OVERLAP = 16;
constexpr int voc_rate(int s) { return s < 2 ? 8 : 2; }
constexpr int voc_block_k(int b) { return b == 0 ? 3 : (b == 1 ? 7 : 11); }
constexpr int voc_dil(int p) { return 2 * p + 1; }
constexpr int voc_channels(int s) { return VOC_C0 >> (s + 1); }              // channels after stage s
constexpr int voc_cum_rate(int s) { return s == 0 ? 8 : (s == 1 ? 64 : (s == 2 ? 128 : 256)); }   // positions per frame after stage s

struct VocoderPtrs {
    // weights in MFMA A-fragment order (weight dtype), k = tap * C_in + channel; biases fp32
    const void* pre_w;  const float* pre_b;
    const void* up_w[VOC_STAGES];  const float* up_b[VOC_STAGES];     // rows = phase * C_out + channel, taps = input offsets -1, 0, +1
    const void* res_w[VOC_STAGES][VOC_BLOCKS][2 * VOC_PAIRS];
    const float* res_b[VOC_STAGES][VOC_BLOCKS][2 * VOC_PAIRS];
    const void* post_w; const float* post_b;
    const float* alpha; const float* beta;    // [overlap * 256] fade-in / fade-out
    float* m_tail;      // [max_requests][overlap][n_mel]   tail(M_pre) of every state slot
    float* s_tail;      // [max_requests][overlap * 256]    tail(S_pre)
    int* len;           // [max_batch] frames in window i of this call (overlap frames in front included)
    float* x_mel;       // [max_batch * window][n_mel]      the spliced windows
    float* x0;          // [max_batch * window][c0]         conv_pre output
    float* y;           // upsampled activations of the current stage, [positions][channels]
    float* r[VOC_BLOCKS];   // output of every residual block of the current stage
    float* audio;       // [max_batch * window * 256]       S_cur of every window
    int overlap, window;    // window = overlap + max_chunk frames: the stride between windows, in frames
};

// The batch as a kernel argument (no host-to-device copy).
struct VocBatch {
    int n;
    int src_row[VOC_MAX_BATCH];      // first row of the chunk in d_mel
    int out_off[VOC_MAX_BATCH];      // first sample of the response in d_audio
    uint16_t n_frames[VOC_MAX_BATCH];
    uint16_t slot[VOC_MAX_BATCH];
    uint8_t has_prev[VOC_MAX_BATCH];
    uint8_t last[VOC_MAX_BATCH];
};

// splice [tail(M_pre), M_cur] into the windows, write tail(M_cur) back (Eq. 3 line 1, Eq. 4), publish the window lengths
hipError_t launch_vocoder_splice(const VocoderPtrs& d, const VocBatch& b, const float* d_mel, hipStream_t s);
// G on every window: x_mel -> audio
hipError_t launch_vocoder_generator(const VocoderPtrs& d, int wdtype, int n_windows, hipStream_t s);
// fade the heads against tail(S_pre), write the responses, write tail(S_cur) back (Eq. 3 line 2, Eq. 4)
hipError_t launch_vocoder_fade(const VocoderPtrs& d, const VocBatch& b, float* d_audio, hipStream_t s);

}  // namespace tts
