// Launch wrappers of the decoder-step kernels (definitions in kernels.hip).
#pragma once
#include "dev.h"

namespace tts {

// dtype codes as in the public header: 0 = fp32, 1 = bf16
struct StepLaunch {
    int wdtype;     // weights / activations
    int mdtype;     // encoder memory
    int n_blocks;   // the attention grid covers slots 0 .. n_blocks - 1 (all active slots lie below)
    int n_tiles;    // the projection grid covers 16-slot tiles 0 .. n_tiles - 1
    int lsa_split;  // workgroups per request in the attention kernel (1, 2 or 4; they split the context columns)
    int lstm_rows;  // row tiles per LSTM workgroup: 1 (all pool tiles each), 2 or 4 (1/2 or 1/4 of the pool tiles each)
    int proj_group; // workgroups per pool tile in the projection kernel: 6, 3 or 2 (fixed per pool; with pre_gates, n_tiles * proj_group <= 32)
    int att_lead;   // 1: the step begins with the attention LSTM's own launch (always, except in pools with d.p_x for a step
                    // whose predecessor in the same call formed it already); 0: it does not
    int att_tail;   // 1 (pools with d.p_x only): the step's last launch also forms the attention LSTM of the next step, which then
                    // has att_lead = 0.  The membership and the requests' states must not change between the two steps.
    int pre_gates;  // 2: the projection's launch also forms the next step's gate pre-sums (d.pre_att / d.pre_dec; fp32: n_tiles <= PRESUM_SMALL_TILES),
                    // 1: the attention LSTM's only (pools of more than PRESUM_SMALL_TILES tiles: d.pre_dec is null);
                    // either way the attention LSTM hands the query to the attention kernel as rank-32 partial products (d.qpart)
};

// CUs the launches count on: the projection's launch of a pool with gate pre-sums has this many workgroups, one per CU,
// and the attention kernel at most this many
constexpr int MIN_DEVICE_CUS = 256;

// up to this many 16-slot tiles a pre-sum workgroup holds all its pool tiles' sums at once (both dtypes); beyond, it walks
// them with its row tiles' weights in registers (bf16 only)
constexpr int PRESUM_SMALL_TILES = 4;
// such a pool's attention LSTM writes this many partial products of the attention query per slot (d.qpart)
constexpr int QUERY_PARTIALS = 32;
// and its projection runs as this many workgroups per tile: d.proj_seq holds one sequence number for each, d.proj_part
// the 96 x 16 partial sums of all but the first (of all of them, and one more sequence number for the tile's leader, in
// the fused form of the last kernel: d.hdec_x)
constexpr int PROJ_GROUP = 6;       // the largest group

// One decoder step (paper Eq. 2) for every request whose slot is flagged in d.live.
// `cur` selects which half of the double-buffered activations is read.
// If `ev` is given it holds N_STEP_KERNELS + 1 events: ev[0] is recorded before the
// first kernel and ev[i + 1] after kernel i (per-kernel device times).
// (Pools with d.hdec_x launch three kernels - the decoder LSTM is part of the last one - and record ev[3] right after ev[2].)
constexpr int N_STEP_KERNELS = 4;
hipError_t launch_step(const DevPtrs& d, const StepLaunch& cfg, int cur, hipStream_t s, hipEvent_t* ev = nullptr);

hipError_t launch_set_live(const DevPtrs& d, const LiveArgs& args, hipStream_t s);
// the whole per-slot state of `n` (<= MOVE_BATCH) running requests, each from its slot to a free one; the slots moved
// from and the slots moved to are disjoint
hipError_t launch_move_slots(const DevPtrs& d, int wdtype, int mdtype, const MoveArgs& mv, int n, hipStream_t s);
// `n` (<= JOIN_BATCH) requests join: state zeroed, F_enc (fp32, device) -> slot memory, processed memory PM = F W_mem^T
hipError_t launch_join(const DevPtrs& d, int wdtype, int mdtype, const JoinArgs& ja, int n, hipStream_t s);
// the gate pre-sums of one pool tile from activation half `nxt` (after a state overwrite between steps)
hipError_t launch_presum_tile(const DevPtrs& d, int wdtype, int tile, int nxt, hipStream_t s);
// p = Pre(m_last) into both activation buffers of one slot (after a state overwrite)
hipError_t launch_prenet_slot(const DevPtrs& d, int wdtype, int slot, hipStream_t s);

// one slot's piece [off, off+n) of a slot-tiled activation array with K elements per slot <-> fp32 device buffer
hipError_t launch_x_get(int wdtype, const void* X, int K, int slot, int off, int n, float* out, hipStream_t s);
hipError_t launch_x_set(int wdtype, void* X, int K, int slot, int off, int n, const float* in, hipStream_t s);

}  // namespace tts
