// Device-side view of a pool: plain pointers into the caller's arena, passed to
// every kernel by value.  Shared by the host code and the kernels of this
// library only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tts {

// Fixed decoder geometry the kernels are specialised for (Tacotron-2 decoder,
// paper Sec. 2.1.3 / 3.1).
constexpr int N_MEL = 80;
constexpr int PRENET = 256;
constexpr int ENC = 512;
constexpr int HID = 1024;           // both LSTMs
constexpr int ATT = 128;
constexpr int LOC_F = 32;
constexpr int LOC_K = 31;
constexpr int LOC_PAD = 15;
constexpr int K_ATT = PRENET + ENC + HID;   // 1792: [Pre(M_last); A; H_att]
constexpr int K_DEC = HID + ENC + HID;      // 2560: [H_att; A; H_dec]
constexpr int K_PROJ = HID + ENC;           // 1536: [H_dec; A]
constexpr int N_PROJ = N_MEL + 1;           // mel rows + stop row
constexpr int MAX_POOL = 256;
constexpr int MAX_ENC_LEN = 1024;
constexpr int TABLE_HDR = 4;                // table[0] = n_active, slots follow at [4..]

// offsets inside the activation rows
constexpr int XA_P = 0, XA_A = PRENET, XA_H = PRENET + ENC;       // x_att = [p | a | h_att]
constexpr int XD_HA = 0, XD_A = HID, XD_HD = HID + ENC;           // x_dec = [h_att | a | h_dec]

struct DevPtrs {
    // weights (WT = float or bf16 as configured)
    const uint4* Wa;      // attention-LSTM gate matrix, MFMA fragment order
    const uint4* Wd;      // decoder-LSTM gate matrix, MFMA fragment order
    const float* ba;      // [HID][4] gate-interleaved merged bias
    const float* bd;
    const void* Wq;       // [ATT][HID] WT
    const float* WmemT;   // [ENC][ATT] fp32 (join time only)
    const float* KcT;     // [2][LOC_K][LOC_F] fp32, channel 0 = W_last, 1 = W_acc
    const float* Wloc;    // [ATT][LOC_F] fp32
    const float* v;       // [ATT] fp32
    const void* Wmel;     // [N_PROJ][K_PROJ] WT, last row = stop
    const float* bmel;    // [N_PROJ]
    const void* Wp1T;     // [N_MEL][PRENET] WT (transposed)
    const void* Wp2T;     // [PRENET][PRENET] WT (transposed)
    // per-slot state
    void* xatt[2];        // [slots][K_ATT] WT, double buffered
    void* xdec[2];        // [slots][K_DEC] WT, double buffered
    float* c_att;         // [slots][HID]
    float* c_dec;         // [slots][HID]
    float* m_last;        // [slots][N_MEL]
    float* w_last;        // [slots][max_enc_len]
    float* w_acc;         // [slots][max_enc_len]
    void* Fmem;           // [slots][max_enc_len][ENC] MT
    void* PM;             // [slots][max_enc_len][ATT] MT
    float* mel_ring;      // [slots][max_steps][N_MEL]
    float* stop_ring;     // [slots][max_steps]
    int* L;               // [slots]
    int* t;               // [slots] frames produced
    int* n_steps;         // [slots]
    int* done;            // [slots]
    int* table;           // [TABLE_HDR + MAX_POOL]
    float* stage;         // [max_enc_len][ENC] fp32 staging for host-side encoder outputs
    int max_enc_len;
    int max_steps;
    float stop_threshold; // < 0: disabled
};

struct TableArgs {
    int n_active;
    uint16_t slot[MAX_POOL];
};

}  // namespace tts
