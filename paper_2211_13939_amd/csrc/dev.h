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
constexpr int MAX_TILES = MAX_POOL / 16;     // a pool tile = 16 consecutive slots = the 16 columns of one MFMA
// offsets inside the activation rows
constexpr int XA_P = 0, XA_A = PRENET, XA_H = PRENET + ENC;       // x_att = [p | a | h_att]
constexpr int XD_HA = 0, XD_A = HID, XD_HD = HID + ENC;           // x_dec = [h_att | a | h_dec]

// bound of the in-kernel waits: about a quarter of a second of polling
constexpr int DEFAULT_WAIT_POLLS = 1 << 18;

struct DevPtrs {
    // weights (WT = float or bf16 as configured)
    const uint4* Wa;      // attention-LSTM gate matrix, MFMA fragment order
    const uint4* Wd;      // decoder-LSTM gate matrix, MFMA fragment order
    const float* ba;      // [HID][4] gate-interleaved merged bias
    const float* bd;
    const void* Wq;       // [ATT][HID] WT, MFMA fragment order (8 row tiles): pools that compute q in the attention kernel
    const float* Wq_epi;  // W_q as fp32 16x16x4 MFMA A operands, [HID/4][8][64 lanes]: entry (u, a, l) = W_q[16 a + l % 16][4 u + l / 16]
                          // (the attention LSTM's query partials, pools with gate pre-sums)
    float* qpart;         // [slots][32][ATT] rank-32 partial sums of q = W_q h_att, written and read within one step (null without pre-sums)
    float* pre_att;       // [tiles][HID/4 row tiles][64 lanes][4]: the attention LSTM's gate sums over [A; H_att], MFMA accumulator layout,
                          // written by the projection kernel's launch for the next step (null: the LSTM kernels contract all of K)
    float* pre_dec;       // same for the decoder LSTM's sums over H_dec
    float* pre_dec_b;     // same layout: the decoder LSTM's sums over H_att, formed inside the attention kernel's launch of the same step
                          // (null: the decoder LSTM contracts H_att itself)
    unsigned long long* proj_part; // [tiles][5][96 * 16] (sequence number << 32 | float bits): partial sums of the projection's helper
                          // workgroups (pools with pre-sums), written and read within one kernel.  Fused form: [tiles][6][96 * 16]
                          // 4-byte words in the same space (float bits, the low four mantissa bits replaced by the count's)
    unsigned* proj_seq;   // [tiles][6]: steps each of a tile's projection workgroups has taken part in (zero at creation)
    unsigned long long* lsa_x; // [slots][max_enc_len] (step number << 32 | float bits): the energies the workgroups of a request hand each other
    unsigned* step_seq;   // [1] steps taken (zero at creation; advanced by the projection kernel)
    unsigned long long* hdec_x; // [tiles][HID / 32 fragments][64 lanes][2] (four halves, bit 14 of each = a bit of the count): H_dec of the
                          // step as the projection's B operand, handed from the decoder LSTM's part of the fused last kernel to the
                          // projection's workgroups of the same launch (two-byte pools of at most 64 slots; pools of more than 64
                          // slots with two-byte weights from 17 slots spanned; null: the decoder LSTM is always a kernel of its own)
    unsigned long long* p_x;    // [tiles][PRENET / 32 fragments][4][64 lanes] (bit 63: the slot takes no further step | sequence number << 32 |
                          // two halves): the prenet output of the step as the attention LSTM's B operand, handed from a tile's leader to
                          // the workgroups that form the NEXT step's attention LSTM inside the same launch (steps that are followed
                          // by another step of the same call; null: the attention LSTM is always a kernel of its own)
    unsigned long long* pre_x;  // [tiles][HID / 4 row tiles][4][64 lanes] (sequence number << 32 | float bits): the attention LSTM's
                          // gate pre-sums, handed to those workgroups by the ones that form them
    unsigned* wg_seq;     // [2]: launches of the fused last kernel so far, double buffered by the steps' parity (a launch reads one
                          // and writes the other; zero at creation): the stamp of the words in p_x and pre_x
    int* fault;           // pinned host memory: set by a workgroup whose bounded wait for another's words ran out (with `failed` of the slots it froze)
    const void* lsa_kfrag; // location filters as per-lane MFMA A operands (layout depends on WT)
    const void* lsa_wfrag; // W_loc as per-lane MFMA A operands (layout depends on WT)
    const float* WmemT;   // [ENC][ATT] fp32 (join time only)
    const float* v;       // [ATT] fp32
    const void* Wmel;     // [96][K_PROJ] WT in MFMA fragment order: 80 mel rows, the stop row, zero rows
    const float* bmel;    // [N_PROJ]
    const void* Wp1;      // [PRENET][80 (fp32) or 96 (bf16, zero padded)] WT in MFMA fragment order
    const void* Wp2;      // [PRENET][PRENET] WT in MFMA fragment order
    // per-slot state
    void* xatt[2];        // [tiles][K_ATT / KB fragments][64 lanes][16 B] WT: slot-tiled MFMA B-operand order, double buffered
    void* xdec[2];        // same for K_DEC
    float* c_att;         // [slots][HID]
    float* c_dec;         // [slots][HID]
    float* m_last;        // [slots][N_MEL]
    float* w_last[2];     // [slots][max_enc_len], double buffered like the activations
    float* w_acc[2];      // [slots][max_enc_len]
    void* Fmem;           // [slots][max_enc_len][ENC] MT
    void* PM;             // [slots][max_enc_len][ATT] MT
    float* mel_ring;      // [slots][max_steps][N_MEL]
    float* stop_ring;     // [slots][max_steps]
    int* L;               // [slots]
    int* t;               // [slots] frames produced
    int* n_steps;         // [slots]
    int* done;            // [slots] reached its last frame (or tripped the stop threshold, or failed)
    int* failed;          // [slots] frozen by a workgroup whose bounded wait for its partners' words ran out (cleared when a request joins)
    int* live;            // [MAX_POOL] 1 = the slot's request is advanced by the next step (set by the host's membership upload)
    float* stage;         // [max_enc_len][ENC] fp32 staging for host-side encoder outputs
    int wait_polls;       // how often a workgroup polls another's words before it gives up and raises `fault` (DEFAULT_WAIT_POLLS)
    int max_enc_len;
    int max_steps;
    float stop_threshold; // < 0: disabled
};

// membership upload: which slots the next steps advance (kernel argument, 40 bytes)
struct LiveArgs {
    uint32_t bits[MAX_POOL / 32];
};

// one launch's worth of slot moves (kernel argument): request i goes from slot from[i] to slot to[i]; L = its encoder
// length, t = frames it has produced so far (an upper bound is fine)
constexpr int MOVE_BATCH = 32;
constexpr int MOVE_WGS = 32;     // workgroups per move
struct MoveArgs {
    int from[MOVE_BATCH], to[MOVE_BATCH], L[MOVE_BATCH], t[MOVE_BATCH];
};

// one launch's worth of joining requests (kernel argument): encoder outputs F[i] (fp32 [L][ENC], device) go to slot[i]
constexpr int JOIN_BATCH = 64;
constexpr int JOIN_POS = 8;      // encoder positions per workgroup
struct JoinArgs {
    const float* F[JOIN_BATCH];
    int slot[JOIN_BATCH], L[JOIN_BATCH], n_steps[JOIN_BATCH];
};

}  // namespace tts
