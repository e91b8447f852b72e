// Decoder-step kernels for gfx950 (MI355X).  One step of paper Eq. 2 for a pool
// of requests is four kernels (every extra kernel costs a launch gap plus a chain
// of dependent memory round trips, about 4-6 us on this machine):
//   k_lstm<att>   gates GEMM on MFMA + fused cell        (Eq. 2 line 1)
//   k_lsa         query, location features, energies, ragged softmax, context,
//                 W_acc update                            (Eq. 2 lines 2 and 4)
//   k_lstm<dec>   gates GEMM on MFMA + fused cell        (Eq. 2 line 3)
//   k_proj        mel + stop projection, ring write, prenet of the new frame
//                                                         (Eq. 2 line 5, Pre() of line 1)
// Two-byte pools of at most 64 slots run three: what is left of the decoder LSTM
// there (K = 512 of 2560, the rest arrives as gate pre-sums) is formed by the
// workgroups of k_proj's launch before they turn to their own parts.  And two
// for a step that follows another step of the same call: its attention LSTM
// (K = 256 left) was formed at the end of that step's k_proj launch.  Pools of
// more than 64 slots with two-byte weights run three as well from 17 slots
// spanned: the decoder LSTM (all of its K, k_lstm_stream's tiles) is the first
// part of k_proj's launch there.
//
// Activations (the vectors multiplied by weight matrices) live in HBM in MFMA
// B-operand order, tiled by pool slot: 16 slots form a tile, and a tile's
// [K x 16] block is stored fragment by fragment (64 bytes of k per column),
// lane l = column l%16, 16-byte piece l/16.  One wave-wide 16-byte load is then
// one contiguous kilobyte, for the weights (A operand) and the activations (B
// operand) alike, and building / splitting the dynamic batch is pure indexing.
#include "kernels.h"
#include "mfma.h"
#include <type_traits>


namespace tts {

// ---------------------------------------------------------------------------
// LSTM gates + cell.  Workgroup b owns hidden units 4b..4b+3 (16 gate rows in
// unit-major, gate-minor order) for every pool tile; its waves split K.
//   gates = W [x] + b;  c <- sig(f) c + sig(i) tanh(g);  h <- sig(o) tanh(c)
// The accumulator of lane l is (column l%16, gates i,f,g,o of unit l/16): the
// cell update needs no data movement beyond the cross-wave reduction.
//
// With PRE only the early part of K is contracted here and the rest arrives as
// pre-sums (below).
// ---------------------------------------------------------------------------
constexpr int LSTM_WAVES = 8;

// Gate pre-sums (PRE).  Part of an LSTM's input is known long before the kernel runs: [A; H_att] of the attention
// LSTM's input is complete once the attention kernel of the previous step has finished, H_dec of the decoder LSTM's
// input once the previous step's decoder LSTM has.  The projection kernel leaves almost every CU idle (a few
// workgroups per 16 slots), so that launch carries extra workgroups which contract those parts
// with their columns of the gate matrices and store the sums in accumulator layout:
//   pre[pool tile][row tile][lane] (floatx4) = sum over the late fragments of W[row tile] x[pool tile].
// The LSTM kernels of the next step then contract only the early fragments -- Pre(M_last) (K = 256 of 1792) and
// [H_att; A] (K = 1536 of 2560) -- and add pre in the cell update.  With HA the decoder LSTM's leading fragments (H_att,
// K = 1024) are summed too, beside the attention kernel in its launch (dec_hatt_presums), and arrive in pre_b.  Wave w owns fragments w, w + 8, ...: the early part
// is the first lstm_main_frags() of them, for both matrices.
template <typename XT, int K> constexpr int lstm_main_frags()
{
    static_assert(K == K_ATT || K == K_DEC, "the two gate matrices");
    return (K == K_ATT ? PRENET : HID + ENC) / Frag<XT>::KB / LSTM_WAVES;
}
static_assert(XA_P == 0 && XD_HA == 0 && XD_A == HID, "the early parts lead the activation rows");
// the leading fragments of a wave that hold H_att in the decoder LSTM's input
template <typename XT> constexpr int lstm_hatt_frags() { return HID / Frag<XT>::KB / LSTM_WAVES; }

template <typename XT, int K, bool PRE, bool HA = false>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_lstm(
    const uint4* __restrict__ Wfrag, const uint4* __restrict__ X, const float* __restrict__ bias, float* __restrict__ c_state,
    const int* __restrict__ live, const int* __restrict__ done, const floatx4* __restrict__ pre, const floatx4* __restrict__ pre_b,
    XT* __restrict__ hout0, int nk0, int off0, XT* __restrict__ hout1, int nk1, int off1, int n_tiles)
{
    constexpr int NW = LSTM_WAVES;
    constexpr int NK = K / Frag<XT>::KB;      // fragments per row tile / per pool tile
    constexpr int F0 = HA ? lstm_hatt_frags<XT>() : 0;             // with HA the sums over H_att arrive in pre_b
    constexpr int NF = (PRE ? lstm_main_frags<XT, K>() : NK / NW) - F0;   // fragments per wave (the early ones only with PRE)
    static_assert(!HA || (PRE && K == K_DEC), "H_att leads the decoder LSTM's input");
    static_assert(NK % NW == 0, "K must split evenly over the waves");
    constexpr int TIF = sizeof(XT) == 2 ? 4 : 1;   // pool tiles whose activations are in flight together

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rt = blockIdx.x;

    // The pool tiles 0 .. n_tiles - 1 (a launch argument: all active slots lie below) are walked
    // directly, not through a list of active tiles: nothing has to be read before the activations
    // can be requested, they go out together with this workgroup's slice of the gate matrix (the
    // only HBM stream).  A tile without a running request is computed and dropped.
    uint4 a[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) a[f] = Wfrag[xfrag(NK, rt, wave + (F0 + f) * NW, lane)];
    // the first four waves also own the cell update of (pool tile in flight = wave, lane)
    const int unit = rt * 4 + (lane >> 4);
    floatx4 bias4 = {0.f, 0.f, 0.f, 0.f};
    if (wave < 4) bias4 = *reinterpret_cast<const floatx4*>(bias + unit * 4);

    __shared__ floatx4 red[NW][4][64];

#pragma unroll
    for (int tg = 0; tg < MAX_TILES; tg += 4) {
        if (tg >= n_tiles) break;
        // The cell update's inputs: three independent, unconditional loads (a load inside a branch
        // makes the compiler wait for every load in flight, the weights included, where the branch
        // rejoins).  Waves without a cell update load the same words as wave % 4 and drop them.
        const int my_tile = min(tg + (wave & 3), n_tiles - 1);
        const int sl = my_tile * 16 + (lane & 15);
        const int lv = live[sl], dn = done[sl];
        const float c_old = c_state[(size_t)sl * HID + unit];
        floatx4 pre4 = {0.f, 0.f, 0.f, 0.f};
        floatx4 pre4b = {0.f, 0.f, 0.f, 0.f};
        if constexpr (PRE) pre4 = pre[((size_t)my_tile * (HID / 4) + rt) * 64 + lane];
        if constexpr (HA) pre4b = pre_b[((size_t)my_tile * (HID / 4) + rt) * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);   // issued here, looked at after the products
#pragma unroll
        for (int t0 = 0; t0 < 4; t0 += TIF) {
            uint4 b[TIF][NF];
#pragma unroll
            for (int t = 0; t < TIF; ++t) {
                if (tg + t0 + t < n_tiles) {
                    const int tile = tg + t0 + t;
#pragma unroll
                    for (int f = 0; f < NF; ++f) b[t][f] = X[xfrag(NK, tile, wave + (F0 + f) * NW, lane)];
                }
            }
#pragma unroll
            for (int t = 0; t < TIF; ++t) {
                if (tg + t0 + t < n_tiles) {
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int f = 0; f < NF; ++f) acc = mfma_frag<XT>(a[f], b[t][f], acc);
                    red[wave][t0 + t][lane] = acc;
                }
            }
        }
        __syncthreads();
        const int slotE = (wave < 4 && tg + wave < n_tiles && lv && !dn) ? sl : -1;
        if (slotE >= 0) {
            floatx4 g = bias4;
#pragma unroll
            for (int w = 0; w < NW; ++w) g += red[w][wave][lane];
            if constexpr (PRE) g += pre4;
            if constexpr (HA) g += pre4b;
            const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
            const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
            const float c = gf * c_old + gi * gg;
            c_state[(size_t)slotE * HID + unit] = c;
            const XT h = from_float<XT>(go * tanhf_(c));
            hout0[xoff<XT>(nk0, slotE, off0 + unit)] = h;
            hout1[xoff<XT>(nk1, slotE, off1 + unit)] = h;
        }
        __syncthreads();
    }
}

// Variants for pools of many tiles: a workgroup owns R row tiles (4 R hidden units) and 1/R of the pool
// tiles, grid = (256 / R) row groups x R pool groups = 256 workgroups.  What bounds the kernel once the
// pool is large is the bytes that pass through one CU (the activations come from L2, and a CU's load path,
// not HBM, is the bottleneck): per workgroup R row tiles of weights + (tiles / R) tiles of activations,
// against 1 + tiles for the one-row-tile kernel.  R = 2 is the minimum at 4 tiles, R = 4 at 16.  The
// workgroups that share rows sit on the same XCD (their blockIdx differ by a multiple of 64), so the
// repeated reads of the weights hit that XCD's L2.  The sums are taken in the same order as in k_lstm.
template <typename XT, int K, int R, bool PRE = false, bool HA = false>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_lstm_rc(
    const uint4* __restrict__ Wfrag, const uint4* __restrict__ X, const float* __restrict__ bias, float* __restrict__ c_state,
    const int* __restrict__ live, const int* __restrict__ done, const floatx4* __restrict__ pre, const floatx4* __restrict__ pre_b,
    XT* __restrict__ hout0, int nk0, int off0, XT* __restrict__ hout1, int nk1, int off1, int n_tiles)
{
    constexpr int NW = LSTM_WAVES;
    constexpr int NK = K / Frag<XT>::KB;
    constexpr int F0 = HA ? lstm_hatt_frags<XT>() : 0;
    constexpr int NF = (PRE ? lstm_main_frags<XT, K>() : NK / NW) - F0;
    static_assert(!HA || (PRE && K == K_DEC), "H_att leads the decoder LSTM's input");
    constexpr int TP = 4 / R;                      // pool tiles per round: R x TP = 4 cell-update waves
    constexpr int NRG = HID / 4 / R;               // row groups
    static_assert(R == 2 || R == 4, "two or four row tiles per workgroup");

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = blockIdx.x % NRG, cg = blockIdx.x / NRG;

    __shared__ floatx4 red[NW][4][64];
    uint4 a[R][NF];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int f = 0; f < NF; ++f) a[r][f] = Wfrag[xfrag(NK, R * rg + r, wave + (F0 + f) * NW, lane)];
    const int per = (n_tiles + R - 1) / R;
    const int c0 = min(cg * per, n_tiles), c1 = min(c0 + per, n_tiles);

    // waves 0 .. 3 also own a cell update: (pool tile of the round = wave / R, row tile = wave % R)
    const int er = wave % R, et = (wave / R) % TP;
    const int unit = (R * rg + er) * 4 + (lane >> 4);
    floatx4 bias4 = {0.f, 0.f, 0.f, 0.f};
    if (wave < 4) bias4 = *reinterpret_cast<const floatx4*>(bias + unit * 4);
    for (int tp = c0; tp < c1; tp += TP) {
        // cell update inputs: independent, unconditional loads (see k_lstm)
        const int sl = min(tp + et, c1 - 1) * 16 + (lane & 15);
        const int lv = live[sl], dn = done[sl];
        const float c_old = c_state[(size_t)sl * HID + unit];
        floatx4 pre4 = {0.f, 0.f, 0.f, 0.f};
        floatx4 pre4b = {0.f, 0.f, 0.f, 0.f};
        if constexpr (PRE) pre4 = pre[((size_t)min(tp + et, c1 - 1) * (HID / 4) + R * rg + er) * 64 + lane];
        if constexpr (HA) pre4b = pre_b[((size_t)min(tp + et, c1 - 1) * (HID / 4) + R * rg + er) * 64 + lane];
        __builtin_amdgcn_sched_barrier(0);
        uint4 b[TP][NF];
#pragma unroll
        for (int t = 0; t < TP; ++t) {
            if (tp + t < c1) {
                const int tile = tp + t;
#pragma unroll
                for (int f = 0; f < NF; ++f) b[t][f] = X[xfrag(NK, tile, wave + (F0 + f) * NW, lane)];
            }
        }
#pragma unroll
        for (int t = 0; t < TP; ++t) {
            if (tp + t < c1) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int f = 0; f < NF; ++f) acc = mfma_frag<XT>(a[r][f], b[t][f], acc);
                    red[wave][R * t + r][lane] = acc;
                }
            }
        }
        __syncthreads();
        const int slotE = (wave < 4 && tp + et < c1 && lv && !dn) ? sl : -1;
        if (slotE >= 0) {
            floatx4 g = bias4;
#pragma unroll
            for (int w = 0; w < NW; ++w) g += red[w][wave][lane];
            if constexpr (PRE) g += pre4;
            if constexpr (HA) g += pre4b;
            const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
            const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
            const float c = gf * c_old + gi * gg;
            c_state[(size_t)slotE * HID + unit] = c;
            const XT h = from_float<XT>(go * tanhf_(c));
            hout0[xoff<XT>(nk0, slotE, off0 + unit)] = h;
            hout1[xoff<XT>(nk1, slotE, off1 + unit)] = h;
        }
        __syncthreads();
    }
}

// The same tile (R row tiles x up to C pool tiles per workgroup, all of K) as one stream over K: wave w walks its
// fragments w, w + 8, ... once, each step fetching the R weight fragments and the C activation fragments of that k
// and chaining them into R x C accumulators, with WIN steps of loads in flight.  Nothing waits for a whole matrix
// slice or a whole pool tile any more: k_lstm_rc requests its weights in one burst and then pays one round trip to L2
// per round of pool tiles; here the loads leave at the rate the products consume them.  Every (row tile, pool tile) sum
// is formed as in k_lstm (wave w chains w + 8 f in increasing f; bias, then the eight waves' sums in wave order), so the
// gates are the same bits.  The R x C sums are reduced through LDS eight at a time, one cell update per wave.
// hx (may be null): H_dec is also handed, as 8-byte words of four halves whose exponent top bits carry the low four bits
// of the tile's step count (proj_seq[tile * pg] + 1, as DecUnit does), to the projection's workgroups of the same launch:
// the form in which this tile is the first thing every workgroup of the last kernel's launch does (pools of more than 64
// slots with two-byte weights).  A slot without a running request hands over zeros.
typedef floatx4 (*StreamRed)[LSTM_WAVES][64];      // [wave][sum of the phase][lane]: 64 KB
template <typename XT, int K, int R, int C>
__device__ __forceinline__ void lstm_stream_unit(
    const uint4* __restrict__ Wfrag, const uint4* __restrict__ X, const float* __restrict__ bias, float* __restrict__ c_state,
    const int* __restrict__ live, const int* __restrict__ done,
    XT* __restrict__ hout0, int nk0, int off0, XT* __restrict__ hout1, int nk1, int off1, int n_tiles, int blk, StreamRed red,
    unsigned long long* __restrict__ hx, const unsigned* __restrict__ proj_seq, int pg)
{
    constexpr int NW = LSTM_WAVES;
    constexpr int NK = K / Frag<XT>::KB;
    constexpr int NF = NK / NW;                    // k steps per wave
    constexpr int NRG = HID / 4 / R;               // row groups; R groups of pool tiles
    constexpr int WIN = 3;                         // k steps in flight
    constexpr int PH = R * C / NW;                 // reduction phases of eight sums
    static_assert(NK % NW == 0 && (R * C) % NW == 0 && WIN <= NF, "shape");

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = blk % NRG, cg = blk / NRG;
    const int per = (n_tiles + R - 1) / R;         // <= C (checked by the launcher)
    const int c0 = min(cg * per, n_tiles), c1 = min(c0 + per, n_tiles);
    if (c0 >= c1) return;                          // the whole workgroup: no pool tile in this group

    // a pool tile past the group's last repeats it (the line is in L2 already) and is dropped
    int tb[C];
#pragma unroll
    for (int t = 0; t < C; ++t) tb[t] = min(c0 + t, c1 - 1);

    uint4 a[WIN][R], b[WIN][C];
    auto issue = [&](int f) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < R; ++r) a[f % WIN][r] = Wfrag[xfrag(NK, R * rg + r, wave + f * NW, lane)];
#pragma unroll
        for (int t = 0; t < C; ++t) b[f % WIN][t] = X[xfrag(NK, tb[t], wave + f * NW, lane)];
    };
#pragma unroll
    for (int f = 0; f < WIN - 1; ++f) issue(f);

    // the cell updates this wave owns: sum 8 p + wave of phase p = (row tile er[p], pool tile et[p])
    int sl[PH], unit[PH], lv[PH], dn[PH];
    float c_old[PH];
    floatx4 bias4[PH];
    unsigned seq[PH];
    bool mine[PH];
#pragma unroll
    for (int p = 0; p < PH; ++p) {
        const int idx = NW * p + wave, er = idx / C, et = idx % C;
        mine[p] = c0 + et < c1;
        sl[p] = tb[et] * 16 + (lane & 15);
        unit[p] = (R * rg + er) * 4 + (lane >> 4);
        lv[p] = live[sl[p]];
        dn[p] = done[sl[p]];
        c_old[p] = c_state[(size_t)sl[p] * HID + unit[p]];
        bias4[p] = *reinterpret_cast<const floatx4*>(bias + unit[p] * 4);
        seq[p] = hx ? proj_seq[tb[et] * pg] + 1u : 0u;
    }

    floatx4 acc[R][C];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < C; ++t) acc[r][t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        if (f + WIN - 1 < NF) issue(f + WIN - 1);
        __builtin_amdgcn_sched_barrier(0);         // the step ahead is requested before this one's products wait for theirs
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < C; ++t) acc[r][t] = mfma_frag<XT>(a[f % WIN][r], b[f % WIN][t], acc[r][t]);
    }

#pragma unroll
    for (int p = 0; p < PH; ++p) {
        if (p) __syncthreads();
#pragma unroll
        for (int j = 0; j < NW; ++j) red[wave][j][lane] = acc[(NW * p + j) / C][(NW * p + j) % C];
        __syncthreads();
        if (mine[p]) {                              // (the same for the whole wave)
            floatx4 g = bias4[p];
#pragma unroll
            for (int w = 0; w < NW; ++w) g += red[w][wave][lane];
            const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
            const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
            const float c = gf * c_old[p] + gi * gg;
            const bool on = lv[p] && !dn[p];
            XT h = from_float<XT>(go * tanhf_(c));
            if (on) {
                c_state[(size_t)sl[p] * HID + unit[p]] = c;
                hout0[xoff<XT>(nk0, sl[p], off0 + unit[p])] = h;
                hout1[xoff<XT>(nk1, sl[p], off1 + unit[p])] = h;
            }
            if constexpr (sizeof(XT) == 2) {
                if (hx) {
                    // lanes l, l + 16, l + 32, l + 48 hold the row tile's four units of one slot: the first stores all four
                    const int mineb = on ? (int)h.bits : 0;
                    const unsigned long long u0 = (unsigned)mineb, u1 = (unsigned)__shfl(mineb, (lane & 15) + 16, 64);
                    const unsigned long long u2 = (unsigned)__shfl(mineb, (lane & 15) + 32, 64), u3 = (unsigned)__shfl(mineb, (lane & 15) + 48, 64);
                    if (lane < 16) {
                        const int rt = unit[p] >> 2;                       // row tile: two of them are a 16-byte piece, eight a fragment
                        const size_t w = (((size_t)(sl[p] >> 4) * (HID / 32) + rt / 8) * 64 + (rt / 2 % 4) * 16 + lane) * 2 + (rt & 1);
                        const unsigned sq = seq[p];
                        const unsigned long long mark = (unsigned long long)(sq & 1u) << 14 | (unsigned long long)(sq >> 1 & 1u) << 30 |
                                                        (unsigned long long)(sq >> 2 & 1u) << 46 | (unsigned long long)(sq >> 3 & 1u) << 62;
                        __hip_atomic_store(&hx[w], u0 | u1 << 16 | u2 << 32 | u3 << 48 | mark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
    }
}

template <typename XT, int K, int R, int C>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_lstm_stream(
    const uint4* __restrict__ Wfrag, const uint4* __restrict__ X, const float* __restrict__ bias, float* __restrict__ c_state,
    const int* __restrict__ live, const int* __restrict__ done,
    XT* __restrict__ hout0, int nk0, int off0, XT* __restrict__ hout1, int nk1, int off1, int n_tiles)
{
    __shared__ floatx4 red[LSTM_WAVES][LSTM_WAVES][64];
    lstm_stream_unit<XT, K, R, C>(Wfrag, X, bias, c_state, live, done, hout0, nk0, off0, hout1, nk1, off1, n_tiles, blockIdx.x, red, nullptr, nullptr, 0);
}

// ---------------------------------------------------------------------------
// Attention LSTM of pools with gate pre-sums.  What is left of its gates is K = 256 (the prenet output), so the shape
// of a workgroup's tile no longer matters for the bytes it pulls, and the tile is chosen for the attention query
// instead: a workgroup owns 8 row tiles (32 hidden units, one row tile per wave, no split of K) of one pool tile and
// hands q = W_q h over as rank-32 partial products, 32 per slot (16 KB) instead of W_q itself (256 KB in bf16) through
// every workgroup of the attention kernel.  Wave w forms the rows 16 w .. 16 w + 15 of the partial from the 32 units
// of h the workgroup has just produced (eight chained 16x16x4 fp32 MFMAs, h through LDS).
//   grid = 32 row groups x pool tiles; qpart[slot][row group][a]
// ---------------------------------------------------------------------------
constexpr int TALL_RT = 8;                      // row tiles per workgroup
constexpr int QP_TALL = HID / 4 / TALL_RT;      // partials per slot
static_assert(QP_TALL == QUERY_PARTIALS, "the arena holds QUERY_PARTIALS partials per slot");

// TP: pool tiles per workgroup.  With more than eight pool tiles one tile per workgroup would be more workgroups than
// compute units, each pulling the same 80 KB of weights; then a workgroup keeps its weights for two tiles.
template <typename XT, int TP>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_lstm_att_tall(
    const uint4* __restrict__ Wfrag, const uint4* __restrict__ X, const float* __restrict__ bias, float* __restrict__ c_state,
    const int* __restrict__ live, const int* __restrict__ done, const floatx4* __restrict__ pre, const float* __restrict__ wq_epi,
    XT* __restrict__ hout0, int nk0, int off0, XT* __restrict__ hout1, int nk1, int off1, float* __restrict__ qpart, int n_tiles)
{
    static_assert(TALL_RT == LSTM_WAVES, "one row tile per wave");
    constexpr int NK = K_ATT / Frag<XT>::KB;
    constexpr int NF = PRENET / Frag<XT>::KB;       // the early fragments: all of them in every wave
    constexpr int BPW = NF / LSTM_WAVES;            // of the pool tile's, fetched per wave
    static_assert(NF % LSTM_WAVES == 0, "the activations' fragments split evenly over the waves");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = blockIdx.x % QP_TALL, tile0 = (blockIdx.x / QP_TALL) * TP;
    const int rt = rg * TALL_RT + wave;
    const int unit = rt * 4 + (lane >> 4);

    // everything is requested at once, for all of the workgroup's tiles (a tile past the last repeats it and is dropped)
    uint4 a[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) a[f] = Wfrag[xfrag(NK, rt, f, lane)];
    uint4 bw[TP][BPW];
    floatx4 pre4[TP];
    int lv[TP], dn[TP];
    float c_old[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int tile = min(tile0 + j, n_tiles - 1), sl = tile * 16 + (lane & 15);
#pragma unroll
        for (int i = 0; i < BPW; ++i) bw[j][i] = X[xfrag(NK, tile, wave + i * LSTM_WAVES, lane)];
        pre4[j] = pre[((size_t)tile * (HID / 4) + rt) * 64 + lane];
        lv[j] = live[sl];
        dn[j] = done[sl];
        c_old[j] = c_state[(size_t)sl * HID + unit];
    }
    const floatx4 bias4 = *reinterpret_cast<const floatx4*>(bias + unit * 4);
    // W_q[16 wave + lane % 16][32 rg + 4 s + lane / 16]: the A operands of the query partial's eight k steps
    float wq[TALL_RT];
#pragma unroll
    for (int s = 0; s < TALL_RT; ++s) wq[s] = wq_epi[((size_t)(rg * TALL_RT + s) * 8 + wave) * 64 + lane];
    __builtin_amdgcn_sched_barrier(0);

    __shared__ uint4 s_b[TP][NF][64];
    __shared__ float s_h[TP][4 * TALL_RT][16];
#pragma unroll
    for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int i = 0; i < BPW; ++i) s_b[j][wave + i * LSTM_WAVES][lane] = bw[j][i];
    __syncthreads();
    bool active[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int sl = (tile0 + j) * 16 + (lane & 15);
        floatx4 g = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < NF; ++f) g = mfma_frag<XT>(a[f], s_b[j][f][lane], g);
        g += bias4;
        g += pre4[j];
        active[j] = lv[j] && !dn[j] && tile0 + j < n_tiles;
        const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
        const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
        const float c = gf * c_old[j] + gi * gg;
        const XT h = from_float<XT>(go * tanhf_(c));
        if (active[j]) {
            c_state[(size_t)sl * HID + unit] = c;
            hout0[xoff<XT>(nk0, sl, off0 + unit)] = h;
            hout1[xoff<XT>(nk1, sl, off1 + unit)] = h;
        }
        s_h[j][4 * wave + (lane >> 4)][lane & 15] = active[j] ? to_float(h) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int sl = (tile0 + j) * 16 + (lane & 15);
        floatx4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < TALL_RT; ++s)
            part = __builtin_amdgcn_mfma_f32_16x16x4f32(wq[s], s_h[j][4 * s + (lane >> 4)][lane & 15], part, 0, 0, 0);
        if (active[j])
            *reinterpret_cast<floatx4*>(qpart + ((size_t)sl * QP_TALL + rg) * ATT + 16 * wave + 4 * (lane >> 4)) = part;
    }
}

// ---------------------------------------------------------------------------
// The pre-sums themselves: one workgroup contracts the late fragments of NR <= 3 row tiles (from r0) with those of
// NT <= 2 pool tiles (from t0), first for the attention LSTM, then for the decoder LSTM, as one stream of chunks (two
// fragments per wave, row tile and pool tile) with PG_WIN chunks in flight: the loads never pause between the two
// matrices.  Every (row tile, pool tile) sum is formed the same way whatever the split: wave w chains its fragments
// w + 8 f in increasing f, the eight waves' sums are added in wave order.  `red` is 48 KB of LDS.
// ---------------------------------------------------------------------------
constexpr int PG_R = 3, PG_T = 2;
constexpr int PG_CH = 2, PG_WIN = 4;
typedef floatx4 (*PresumRed)[PG_R * PG_T][64];

// What the projection kernel's launch requests first, as kernel arguments of their own (the leading 16 dwords of a
// kernel's arguments arrive in scalar registers with the wave; the rest has to be read from memory first).
struct ProjHot {
    const uint4 *Wa, *Wd;           // the gate matrices
    const void *xatt_nxt, *xdec_nxt; // the activation halves the next step reads
    const void* xdec_cur;           // a of this step
    const void* Wmel;
    const int* live;
    unsigned* proj_seq;
};

// DEC: the decoder LSTM's pre-sums too (pools of at most four tiles; larger pools keep all of its K in its own kernel
// and have no buffer for them)
// With `stamp` non-zero the attention LSTM's sums go to pre_x as 8-byte words that carry the stamp instead of to pre_att:
// the next step's attention LSTM is then formed inside this launch (att_tail_unit) and polls them.
template <typename XT, int NR, int NT, bool DEC>
__device__ __forceinline__ void gate_presums_rt(const DevPtrs& d, const ProjHot& hot, int r0, int t0, PresumRed red, unsigned stamp)
{
    constexpr int NW = LSTM_WAVES, KB = Frag<XT>::KB;
    constexpr int NK_A = K_ATT / KB, NK_D = K_DEC / KB;
    constexpr int F0_A = lstm_main_frags<XT, K_ATT>(), F0_D = lstm_main_frags<XT, K_DEC>();
    constexpr int NA = (NK_A / NW - F0_A) / PG_CH, ND = DEC ? (NK_D / NW - F0_D) / PG_CH : 0, N = NA + ND;   // chunks
    static_assert((NK_A / NW - F0_A) % PG_CH == 0 && (NK_D / NW - F0_D) % PG_CH == 0, "the late fragments split evenly into chunks");
    static_assert(NR * NT <= NW, "one wave adds up one (row tile, pool tile) sum");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint4* __restrict__ Wa = hot.Wa;
    const uint4* __restrict__ Wd = hot.Wd;
    const uint4* __restrict__ xa = reinterpret_cast<const uint4*>(hot.xatt_nxt);
    const uint4* __restrict__ xd = reinterpret_cast<const uint4*>(hot.xdec_nxt);

    uint4 a[PG_WIN][NR][PG_CH], b[PG_WIN][NT][PG_CH];
    floatx4 acc[NR][NT];
    // chunk i (a compile-time number once the loops below are unrolled) into window slot i % PG_WIN
    auto issue = [&](int i) __attribute__((always_inline)) {
        const bool att = i < NA;
        const uint4* W = att ? Wa : Wd;
        const uint4* X = att ? xa : xd;
        const int NK = att ? NK_A : NK_D;
        const int f0 = att ? F0_A + i * PG_CH : F0_D + (i - NA) * PG_CH;
#pragma unroll
        for (int c = 0; c < PG_CH; ++c) {
#pragma unroll
            for (int r = 0; r < NR; ++r) a[i % PG_WIN][r][c] = W[xfrag(NK, r0 + r, wave + (f0 + c) * NW, lane)];
#pragma unroll
            for (int t = 0; t < NT; ++t) b[i % PG_WIN][t][c] = X[xfrag(NK, t0 + t, wave + (f0 + c) * NW, lane)];
        }
    };
    auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[r][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    };
    auto finish = [&](float* out, bool as_words) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t) red[wave][r * NT + t][lane] = acc[r][t];
        __syncthreads();
        if (wave < NR * NT) {
            floatx4 g = red[0][wave][lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) g += red[w][wave][lane];
            const size_t at = (size_t)(t0 + wave % NT) * (HID / 4) + r0 + wave / NT;
            if (as_words) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    __hip_atomic_store(&d.pre_x[(at * 4 + i) * 64 + lane], ((unsigned long long)stamp << 32) | __float_as_uint(g[i]),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                reinterpret_cast<floatx4*>(out)[at * 64 + lane] = g;
            }
        }
        __syncthreads();
    };
#pragma unroll
    for (int i = 0; i < PG_WIN - 1 && i < N; ++i) issue(i);
    clear();
#pragma unroll
    for (int i = 0; i < N; ++i) {
        if (i + PG_WIN - 1 < N) issue(i + PG_WIN - 1);
        __builtin_amdgcn_sched_barrier(0);       // the next chunk is requested before this one's products wait for theirs
#pragma unroll
        for (int c = 0; c < PG_CH; ++c)
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[r][t] = mfma_frag<XT>(a[i % PG_WIN][r][c], b[i % PG_WIN][t][c], acc[r][t]);
        if (i == NA - 1) {
            finish(d.pre_att, stamp != 0u);
            clear();
        }
    }
    if constexpr (DEC) finish(d.pre_dec, false);
}

template <typename XT, bool DEC>
__device__ __forceinline__ void gate_presums_sel(const DevPtrs& d, const ProjHot& hot, int r0, int nr, int t0, int nt, PresumRed red, unsigned stamp = 0u)
{
    if (nt == 1) {
        if (nr == 1) gate_presums_rt<XT, 1, 1, DEC>(d, hot, r0, t0, red, stamp);
        else if (nr == 2) gate_presums_rt<XT, 2, 1, DEC>(d, hot, r0, t0, red, stamp);
        else gate_presums_rt<XT, 3, 1, DEC>(d, hot, r0, t0, red, stamp);
    } else {
        if (nr == 1) gate_presums_rt<XT, 1, 2, DEC>(d, hot, r0, t0, red, stamp);
        else if (nr == 2) gate_presums_rt<XT, 2, 2, DEC>(d, hot, r0, t0, red, stamp);
        else gate_presums_rt<XT, 3, 2, DEC>(d, hot, r0, t0, red, stamp);
    }
}

// The pre-sums of the next step, from the activation halves that step will read (cur ^ 1 of the step that is running),
// for nr in 1 .. PG_R row tiles and nt in 1 .. PG_T pool tiles (the same for the whole workgroup).
template <typename XT>
__device__ __forceinline__ void gate_presums(const DevPtrs& d, const ProjHot& hot, int r0, int nr, int t0, int nt, PresumRed red)
{
    if (d.pre_dec) gate_presums_sel<XT, true>(d, hot, r0, nr, t0, nt, red);
    else gate_presums_sel<XT, false>(d, hot, r0, nr, t0, nt, red);
}

// Pools that span more than four tiles: a workgroup has up to PG_WALK_R row tiles and up to four pool tiles.  Its row
// tiles' late fragments stay in registers and the pool tiles are walked one at a time, the next tile's activations
// requested before the current tile's products (the loop of the decoder LSTM's large-pool kernel without the cell).
// Each (row tile, pool tile) sum is formed in the same order as above.  bf16 only (fp32 fragments of five row tiles
// do not fit the register file).
constexpr int PG_WALK_R = 5;
typedef floatx4 (*WalkRed)[PG_WALK_R][64];

template <typename XT, int K, int NR>
__device__ __forceinline__ void gate_presum_walk(const uint4* __restrict__ W, const uint4* __restrict__ X, floatx4* __restrict__ pre,
                                                 int r0, int t0, int nt, WalkRed red)
{
    constexpr int NW = LSTM_WAVES;
    constexpr int NK = K / Frag<XT>::KB;
    constexpr int F0 = lstm_main_frags<XT, K>();
    constexpr int NFP = NK / NW - F0;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint4 a[NR][NFP];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int f = 0; f < NFP; ++f) a[r][f] = W[xfrag(NK, r0 + r, wave + (F0 + f) * NW, lane)];
    auto fetch = [&](int t, uint4 (&b)[NFP]) __attribute__((always_inline)) {
        const int tile = t0 + min(t, nt - 1);            // past the end: the last tile again, never used
#pragma unroll
        for (int f = 0; f < NFP; ++f) b[f] = X[xfrag(NK, tile, wave + (F0 + f) * NW, lane)];
    };
    auto round = [&](int t, const uint4 (&b)[NFP]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int f = 0; f < NFP; ++f) acc = mfma_frag<XT>(a[r][f], b[f], acc);
            red[wave][r][lane] = acc;
        }
        __syncthreads();
        if (wave < NR) {
            floatx4 g = red[0][wave][lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) g += red[w][wave][lane];
            pre[((size_t)(t0 + t) * (HID / 4) + r0 + wave) * 64 + lane] = g;
        }
        __syncthreads();
    };
    uint4 b0[NFP], b1[NFP];
    fetch(0, b0);
    for (int t = 0; t < nt; t += 2) {
        fetch(t + 1, b1);
        __builtin_amdgcn_sched_barrier(0);
        round(t, b0);
        if (t + 1 >= nt) break;
        fetch(t + 2, b0);
        __builtin_amdgcn_sched_barrier(0);
        round(t + 1, b1);
    }
}

template <typename XT>
__device__ __forceinline__ void gate_presums_walk(const DevPtrs& d, const ProjHot& hot, int r0, int nr, int t0, int nt, WalkRed red)
{
    const uint4* xa = reinterpret_cast<const uint4*>(hot.xatt_nxt);
    const uint4* xd = reinterpret_cast<const uint4*>(hot.xdec_nxt);
    floatx4* pa = reinterpret_cast<floatx4*>(d.pre_att);
    floatx4* pd = reinterpret_cast<floatx4*>(d.pre_dec);
    if constexpr (sizeof(XT) == 2) {
        switch (nr) {
        case 1: gate_presum_walk<XT, K_ATT, 1>(hot.Wa, xa, pa, r0, t0, nt, red); if (pd) gate_presum_walk<XT, K_DEC, 1>(hot.Wd, xd, pd, r0, t0, nt, red); break;
        case 2: gate_presum_walk<XT, K_ATT, 2>(hot.Wa, xa, pa, r0, t0, nt, red); if (pd) gate_presum_walk<XT, K_DEC, 2>(hot.Wd, xd, pd, r0, t0, nt, red); break;
        case 3: gate_presum_walk<XT, K_ATT, 3>(hot.Wa, xa, pa, r0, t0, nt, red); if (pd) gate_presum_walk<XT, K_DEC, 3>(hot.Wd, xd, pd, r0, t0, nt, red); break;
        case 4: gate_presum_walk<XT, K_ATT, 4>(hot.Wa, xa, pa, r0, t0, nt, red); if (pd) gate_presum_walk<XT, K_DEC, 4>(hot.Wd, xd, pd, r0, t0, nt, red); break;
        default: gate_presum_walk<XT, K_ATT, 5>(hot.Wa, xa, pa, r0, t0, nt, red); if (pd) gate_presum_walk<XT, K_DEC, 5>(hot.Wd, xd, pd, r0, t0, nt, red); break;
        }
    }
}

// The pre-sums of one pool tile outside a step (after a state overwrite): one row tile per workgroup.
template <typename XT>
__global__ __launch_bounds__(LSTM_WAVES * 64) void k_presum_tile(DevPtrs d, int nxt, int tile)
{
    __shared__ floatx4 red[LSTM_WAVES][PG_R * PG_T][64];
    static_assert(PG_WALK_R <= PG_R * PG_T, "either form's reduction buffer");
    const ProjHot hot = {d.Wa, d.Wd, d.xatt[nxt], d.xdec[nxt], nullptr, d.Wmel, d.live, d.proj_seq};
    if (d.pre_dec) gate_presums<XT>(d, hot, blockIdx.x, 1, tile, 1, red);
    else gate_presums_walk<XT>(d, hot, blockIdx.x, 1, tile, 1, reinterpret_cast<WalkRed>(&red[0][0][0]));   // the attention LSTM's only
}

// ---------------------------------------------------------------------------
// Location-sensitive attention, one workgroup (8 waves) per request:
//   q = W_q h_att
//   loc[j][f] = sum_c sum_k Kc[f][c][k] u_c[j+k-15]         (u = W_last, W_acc; zero outside [0,L))
//   e_j = v . tanh(q + W_loc loc[j] + PM[j])
//   w = softmax_{j<L}(e);  A = sum_j w_j F[j];  W_last <- w;  W_acc <- W_acc + w
// The contractions run on MFMA with 16 positions (or, for q, 16 copies of h_att)
// as the columns (pools with gate pre-sums get q as partial sums from the
// attention LSTM's epilogue instead):
//   q      (128 x 16, K split over the waves) = W_q * h_att
//   loc^T  (32 x 16)          = Kc (32 x 64 taps) * U^T (64 taps x 16 positions)
//   pl^T   (128 x 16)         = W_loc (128 x 32)  * loc^T
// The accumulator layout of loc^T is exactly the B-operand layout of the next
// product once the filter index is walked in the order the lanes hold it, so
// nothing moves between the two.  The rows of W_loc are permuted so that lane
// group g ends up with attention dims 32g..32g+31: its slice of PM[j] is one
// contiguous run.  The constant A operands come pre-arranged per lane.
// ---------------------------------------------------------------------------
constexpr int LSA_THREADS = 512;
constexpr int LSA_WAVES = LSA_THREADS / 64;
constexpr int LSA_UPAD = MAX_ENC_LEN + 48;

template <typename XT> struct LsaTile;

// fp32: v_mfma_f32_16x16x4_f32, lane group g supplies k = g of each 4-wide step
template <> struct LsaTile<float> {
    float kA[2][16];   // [mt][c*8+s]: filter 16 mt + jl, tap 4 s + g of channel c
    float4 wA[8][2];   // [at][mt]: W_loc row 32 (jl/4) + 4 at + jl%4, filters 16 mt + 4 g .. +3
    __device__ __forceinline__ void load(const DevPtrs& d, int lane)
    {
        const float* kf = reinterpret_cast<const float*>(d.lsa_kfrag);
        const float4* wf = reinterpret_cast<const float4*>(d.lsa_wfrag);
#pragma unroll
        for (int i = 0; i < 32; ++i) kA[i >> 4][i & 15] = kf[i * 64 + lane];
#pragma unroll
        for (int i = 0; i < 16; ++i) wA[i >> 1][i & 1] = wf[i * 64 + lane];
    }
    // x0 = index into s_u of this lane's position at tap 0
    // pl[at] = q[at] + W_loc loc: the query rides in as the accumulator's start value
    __device__ __forceinline__ void run(const float* u0, const float* u1, int x0, int g, const floatx4* q, floatx4* pl) const
    {
        floatx4 loc0 = {0.f, 0.f, 0.f, 0.f}, loc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cs = 0; cs < 16; ++cs) {
            const float b = (cs < 8 ? u0 : u1)[x0 + g + 4 * (cs & 7)];
            loc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(kA[0][cs], b, loc0, 0, 0, 0);
            loc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(kA[1][cs], b, loc1, 0, 0, 0);
        }
#pragma unroll
        for (int at = 0; at < 8; ++at) {
            floatx4 p = q[at];
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][0].x, loc0[0], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][0].y, loc0[1], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][0].z, loc0[2], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][0].w, loc0[3], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][1].x, loc1[0], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][1].y, loc1[1], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][1].z, loc1[2], p, 0, 0, 0);
            p = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[at][1].w, loc1[3], p, 0, 0, 0);
            pl[at] = p;
        }
    }
};

// two-byte operands: v_mfma_f32_16x16x32_f16, lane group g supplies 8 k values per step
template <> struct LsaTile<h16_t> {
    uint4 kA[2][2];    // [mt][c]: filter 16 mt + jl, taps 8 g .. 8 g + 7 of channel c
    uint4 wA[8];       // [at]: W_loc row 32 (jl/4) + 4 at + jl%4, filters {4g..4g+3, 16+4g..16+4g+3}
    static constexpr int LDS_VECS = 12 * 64;   // the operands of all 64 lanes, as 16-byte pieces
    // the operands are the same for every wave: the workgroup fetches them once into LDS ...
    __device__ static __forceinline__ uint4 fetch(const DevPtrs& d, int i)
    {
        const uint4* kf = reinterpret_cast<const uint4*>(d.lsa_kfrag);
        const uint4* wf = reinterpret_cast<const uint4*>(d.lsa_wfrag);
        return i < 4 * 64 ? kf[i] : wf[i - 4 * 64];
    }
    // ... and every wave takes its lanes' share from there
    __device__ __forceinline__ void load(const uint4* lds, int lane)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) kA[i >> 1][i & 1] = lds[i * 64 + lane];
#pragma unroll
        for (int i = 0; i < 8; ++i) wA[i] = lds[(4 + i) * 64 + lane];
    }
    __device__ __forceinline__ void run(const float* u0, const float* u1, int x0, int g, const floatx4* q, floatx4* pl) const
    {
        floatx4 loc0 = {0.f, 0.f, 0.f, 0.f}, loc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const float* u = (c == 0 ? u0 : u1) + x0 + 8 * g;
            uint4 b;
            b.x = pack2<h16_t>(u[0], u[1]); b.y = pack2<h16_t>(u[2], u[3]);
            b.z = pack2<h16_t>(u[4], u[5]); b.w = pack2<h16_t>(u[6], u[7]);
            loc0 = mfma_frag<h16_t>(kA[0][c], b, loc0);
            loc1 = mfma_frag<h16_t>(kA[1][c], b, loc1);
        }
        uint4 bl;
        bl.x = pack2<h16_t>(loc0[0], loc0[1]); bl.y = pack2<h16_t>(loc0[2], loc0[3]);
        bl.z = pack2<h16_t>(loc1[0], loc1[1]); bl.w = pack2<h16_t>(loc1[2], loc1[3]);
#pragma unroll
        for (int at = 0; at < 8; ++at) pl[at] = mfma_frag<h16_t>(wA[at], bl, q[at]);
    }
};

// The decoder LSTM's gate sums over H_att (K = HID of its 2560), formed inside the attention kernel's launch.  H_att(t) is
// complete when that launch begins, and the attention itself is a chain of waits (exchange of energies, dependent round
// trips) that leaves the load path of its compute units idle: workgroups j = 0 .. 255 behind the attention's own share a
// CU with one of them each and contract two row tiles (2 (j % 128), + 1) with half of the pool tiles (j / 128), K split
// over the waves as in k_lstm_rc; wave w chains its fragments w + 8 f in increasing f, the eight waves' sums are added
// in wave order.  The sums land in pre_dec_b in accumulator layout and are read by the decoder LSTM of the same step.
typedef floatx4 (*HattRed)[2][64];               // [wave][row tile][lane]: 16 KB
// HD: the sums over H_dec of the step before (the trailing K = HID, into pre_dec) are formed here as well, after those
// over H_att; that part's weights are requested before the first part's products.  (Pools whose last kernel holds the
// decoder LSTM: its launch can no longer form them for the next step, H_dec being complete only when it ends.)
template <typename XT, bool HD>
__device__ __forceinline__ void dec_hatt_presums(const uint4* __restrict__ Wd, const uint4* __restrict__ X, floatx4* __restrict__ out,
                                                 floatx4* __restrict__ out_hd, int j, int n_tiles, HattRed red)
{
    constexpr int NW = LSTM_WAVES, R = 2, TP = 2;
    constexpr int NK = K_DEC / Frag<XT>::KB;
    constexpr int NF = lstm_hatt_frags<XT>();
    constexpr int F_HD = lstm_main_frags<XT, K_DEC>();      // a wave's fragments that hold H_dec follow its early ones
    static_assert(NK / NW - F_HD == NF, "H_dec is as long as H_att");
    constexpr int NRG = HID / 4 / R;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = j % NRG, cg = j / NRG;
    uint4 a[R][NF];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int f = 0; f < NF; ++f) a[r][f] = Wd[xfrag(NK, R * rg + r, wave + f * NW, lane)];
    const int per = (n_tiles + R - 1) / R;
    const int c0 = min(cg * per, n_tiles), c1 = min(c0 + per, n_tiles);
    static_assert(PRESUM_SMALL_TILES <= R * TP, "one round of pool tiles per workgroup");
    if (c0 >= c1) return;
    auto part = [&](int F0, floatx4* __restrict__ dst, bool prefetch) __attribute__((always_inline)) {
        uint4 b[TP][NF];
#pragma unroll
        for (int t = 0; t < TP; ++t) {
            const int tile = min(c0 + t, c1 - 1);
#pragma unroll
            for (int f = 0; f < NF; ++f) b[t][f] = X[xfrag(NK, tile, wave + (F0 + f) * NW, lane)];
        }
        floatx4 acc[TP][R];
#pragma unroll
        for (int t = 0; t < TP; ++t)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc[t][r] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[t][r] = mfma_frag<XT>(a[r][f], b[t][f], acc[t][r]);
            }
        if (prefetch) {
            // the next part's weights: on their way during this part's reduction
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int f = 0; f < NF; ++f) a[r][f] = Wd[xfrag(NK, R * rg + r, wave + (F_HD + f) * NW, lane)];
        }
#pragma unroll
        for (int t = 0; t < TP; ++t) {
#pragma unroll
            for (int r = 0; r < R; ++r) red[wave][r][lane] = acc[t][r];
            __syncthreads();
            if (wave < R && c0 + t < c1) {
                floatx4 g = red[0][wave][lane];
#pragma unroll
                for (int w = 1; w < NW; ++w) g += red[w][wave][lane];
                dst[((size_t)(c0 + t) * (HID / 4) + R * rg + wave) * 64 + lane] = g;
            }
            __syncthreads();
        }
    };
    part(0, out, HD);
    if constexpr (HD) part(F_HD, out_hd, false);
}
constexpr int DEC_HATT_WGS = HID / 4 / 2;        // per half of the pool tiles

// The first eight arguments repeat pointers that are also in `d_all`: the leading 16 dwords of a kernel's arguments
// arrive in scalar registers with the wave, so the prologue's loads can go out before the argument block has been read.
// CO: the launch carries the workgroups of dec_hatt_presums behind the attention's own; two workgroups then share a CU
// (four waves per SIMD: at most 128 registers).
template <typename XT, typename MT, int S, bool QP, bool CO = false>
__global__ __launch_bounds__(LSA_THREADS, CO ? 4 : 1) void k_lsa(int* L_first, int* live_first, int* done_first, unsigned* seq_first, float* qpart_first,
                                                    float* w_last_first, float* w_acc_first, void* PM_first, DevPtrs d, int cur, int n_slots)
{
    __shared__ __attribute__((aligned(16))) float s_ctx[LSA_WAVES][ENC];
    if constexpr (CO) {
        static_assert(sizeof(floatx4) * LSTM_WAVES * 2 * 64 <= sizeof(float) * LSA_WAVES * ENC && LSA_WAVES == LSTM_WAVES, "the pre-sums' reduction fits s_ctx");
        const int n_lsa = (n_slots + 7) / 8 * 8 * S;
        if ((int)blockIdx.x >= n_lsa) {
            dec_hatt_presums<XT, true>(d.Wd, reinterpret_cast<const uint4*>(d.xdec[cur]), reinterpret_cast<floatx4*>(d.pre_dec_b),
                                       reinterpret_cast<floatx4*>(d.pre_dec), blockIdx.x - n_lsa, (n_slots + 15) / 16,
                                       reinterpret_cast<HattRed>(&s_ctx[0][0]));
            return;
        }
    }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jl = lane & 15, g = lane >> 4;
    // Workgroups are laid over the pool's SLOTS, not over a list of active requests: a list would
    // cost a dependent round trip (about a microsecond from a cold L2) before anything else could be
    // requested.  Whether the slot holds a running request, and its encoder length, arrive with the
    // rest of the prologue's loads.  There is deliberately no early exit in this kernel either: the
    // compiler moves loads below a branch that may leave the kernel, which would serialise them
    // behind that branch's condition.  A workgroup with nothing to do computes on whatever its
    // slot holds (all reads stay inside the slot's arrays) and writes nothing.
    // A slot's S workgroups sit on one XCD (workgroup b runs on XCD b % 8): what they all read - the query's partial
    // products, the words they hand each other - then crosses into that XCD's L2 once.  Slots are dealt to the XCDs in
    // eights; the grid is padded to whole eights, and a workgroup past the last slot repeats the last slot's work
    // (every read stays inside the arrays), stores nothing and waits for nobody.
    const int xcd = blockIdx.x & 7, kx = blockIdx.x >> 3;
    const int slot_raw = (kx / S) * 8 + xcd, sp = kx % S;
    const int slot = min(slot_raw, n_slots - 1);
    const int live_w = live_first[slot], done_w = done_first[slot], L_w = L_first[slot];
    const bool twin = slot_raw >= n_slots;
    // the request's S workgroups share the energies (below): this step's number marks the words they exchange
    constexpr bool XCH = S > 1;
    unsigned seq = 0;
    if constexpr (XCH) seq = seq_first[0] + 1u;
    // q = W_q h_att, one of two ways.
    // QP (pools with gate pre-sums): it arrives as QP_TALL rank-32 partial products written by this step's attention
    // LSTM.  Thread (a = tid % 128, quarter = tid / 128) adds up its quarter's pair sums P[2i] + P[2i+1] in
    // increasing i; then q[a] = (s0 + s1) + (s2 + s3).
    // Otherwise: on MFMA here, wave w contracting k in [128 w, 128 w + 128) for all 128 outputs
    // with 16 copies of h_att as the columns; the weights do not depend on the request.
    constexpr int QN = QP ? QP_TALL / 4 : 1;      // partials per thread: QP_TALL partial products per slot, four quarters
    constexpr int NKQ = HID / Frag<XT>::KB;       // fragments per row tile of W_q
    constexpr int NKW = NKQ / LSA_WAVES;          // fragments per wave
    constexpr int MG = QP ? 1 : (sizeof(XT) == 2 ? 8 : 2);   // row tiles whose fragments are in flight together
    float qv[QN];
    uint4 qa[MG][QP ? 1 : NKW];
    const uint4* Wq = reinterpret_cast<const uint4*>(d.Wq) + (size_t)(wave * NKW) * 64 + lane;
    if constexpr (QP) {
        const float* qp = qpart_first + ((size_t)slot * QP_TALL + (tid >> 7) * QN) * ATT + (tid & (ATT - 1));
#pragma unroll
        for (int i = 0; i < QN; ++i) qv[i] = qp[(size_t)i * ATT];
    } else {
#pragma unroll
        for (int m = 0; m < MG; ++m)
#pragma unroll
            for (int f = 0; f < NKW; ++f) qa[m][f] = Wq[((size_t)m * NKQ + f) * 64];
    }

    __shared__ __attribute__((aligned(16))) float s_q[ATT];
    __shared__ __attribute__((aligned(16))) float s_v[ATT];
    __shared__ float s_u[2][LSA_UPAD];            // s_u[c][x] = u_c[x - 15]
    __shared__ float s_e[MAX_ENC_LEN];
    __shared__ float s_red[2 * LSA_WAVES];
    __shared__ int s_fail;                        // a wait for another workgroup's words ran out

    constexpr int KB = Frag<XT>::KB;
    constexpr int NPM = Vec16<MT>::N;
    constexpr int NV = 32 / NPM;                  // 16-byte pieces of a lane's 32 attention dims of PM[j]
    const int ML = d.max_enc_len;
    const MT* PMs = reinterpret_cast<const MT*>(PM_first) + (size_t)slot * ML * ATT + 32 * g;
    const float* wl = w_last_first + (size_t)slot * ML;
    const float* wa = w_acc_first + (size_t)slot * ML;

    // ---- everything the prologue needs is requested before anything is consumed
    constexpr int UPT = (LSA_UPAD + LSA_THREADS - 1) / LSA_THREADS;
    float ul[UPT], ua[UPT];
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        // unconditional loads from a clamped index (a load inside a branch makes the compiler wait
        // for every outstanding load where the branch rejoins)
        // (the index is clamped to the slot's array, not to the length, which is still on its way)
        const int jc = min(max(tid + i * LSA_THREADS - LOC_PAD, 0), ML - 1);
        ul[i] = wl[jc];
        ua[i] = wa[jc];
    }
    const float vreg = d.v[tid & (ATT - 1)];
    // every column of the B operand of the query product is this request's h_att (column slot%16 of its tile)
    uint4 hb[QP ? 1 : NKW];
    if constexpr (!QP) {
        const uint4* hx = reinterpret_cast<const uint4*>(d.xdec[cur]) +
                          xfrag(K_DEC / KB, slot >> 4, XD_HA / KB + wave * NKW, (slot & 15) + 16 * g);
#pragma unroll
        for (int f = 0; f < NKW; ++f) hb[f] = hx[(size_t)f * 64];
    }
    LsaTile<XT> tile;
    // bf16: the constant MFMA operands go through LDS once per workgroup (straight from global every
    // wave would pull its own 12 KB copy through the CU's one load path)
    constexpr bool TILE_LDS = sizeof(XT) == 2;
    constexpr int TILE_VECS = TILE_LDS ? 12 * 64 : 1;
    __shared__ uint4 s_tile[TILE_VECS];
    uint4 tv0 = make_uint4(0, 0, 0, 0), tv1 = make_uint4(0, 0, 0, 0);
    if constexpr (TILE_LDS) {
        tv0 = LsaTile<XT>::fetch(d, tid);
        tv1 = LsaTile<XT>::fetch(d, LSA_THREADS + (tid & 255));   // 768 pieces: the upper half of the threads repeats the lower's
    }
    constexpr bool PM_AHEAD = sizeof(XT) == 2;    // fp32 operands leave no registers for a second PM row
    uint4 pmv[NV];
    if constexpr (PM_AHEAD) {
        const MT* pm = PMs + (size_t)min((sp + S * wave) * 16 + jl, ML - 1) * ATT;
#pragma unroll
        for (int i = 0; i < NV; ++i) pmv[i] = *reinterpret_cast<const uint4*>(pm + i * NPM);
    }
    __builtin_amdgcn_sched_barrier(0);            // everything above is in flight before anything below waits
    const bool active = live_w && !done_w && !twin;
    const int L = active ? L_w : 1;
    const int ntile = (L + 15) >> 4;
    if constexpr (QP) {
        float sq = qv[0] + qv[1];
#pragma unroll
        for (int i = 2; i < QN; i += 2) sq += qv[i] + qv[i + 1];
        s_ctx[tid >> 7][tid & (ATT - 1)] = sq;    // s_ctx doubles as the partial-q buffer
    } else {
#pragma unroll
        for (int m0 = 0; m0 < 8; m0 += MG) {
            if (m0 > 0) {
#pragma unroll
                for (int m = 0; m < MG; ++m)
#pragma unroll
                    for (int f = 0; f < NKW; ++f) qa[m][f] = Wq[((size_t)(m0 + m) * NKQ + f) * 64];
            }
#pragma unroll
            for (int m = 0; m < MG; ++m) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NKW; ++f) acc = mfma_frag<XT>(qa[m][f], hb[f], acc);
                // every column holds the same h: take column 0
                if (jl == 0) *reinterpret_cast<floatx4*>(&s_ctx[wave][16 * (m0 + m) + 4 * g]) = acc;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int x = tid + i * LSA_THREADS;
        if (x < ntile * 16 + 32) {
            const bool in = (x >= LOC_PAD && x < L + LOC_PAD);
            s_u[0][x] = in ? ul[i] : 0.f;
            s_u[1][x] = in ? ua[i] : 0.f;
        }
    }
    if (tid < ATT) s_v[tid] = -2.0f * vreg;       // v . tanh(x) = sum(v) - 2 sum(v / (1 + e^{2x}))
    if (tid == 0) s_fail = 0;
    if constexpr (TILE_LDS) {
        s_tile[tid] = tv0;
        if (tid < 256) s_tile[LSA_THREADS + tid] = tv1;
    } else {
        tile.load(d, lane);                      // fp32: too many registers to hold through the prologue
    }
    __syncthreads();
    if (tid < ATT) {
        float q;
        if constexpr (QP) {
            q = (s_ctx[0][tid] + s_ctx[1][tid]) + (s_ctx[2][tid] + s_ctx[3][tid]);
        } else {
            q = 0.f;
#pragma unroll
            for (int w = 0; w < LSA_WAVES; ++w) q += s_ctx[w][tid];
        }
        s_q[tid] = q;
    }
    __syncthreads();
    if constexpr (TILE_LDS) tile.load(s_tile, lane);

    // this lane's share of sum(v): its 32 attention dims (s_v holds -2 v)
    float vsum = 0.f;
#pragma unroll
    for (int at = 0; at < 8; ++at) {
        const float4 vv = *reinterpret_cast<const float4*>(&s_v[32 * g + 4 * at]);
        vsum += (vv.x + vv.y) + (vv.z + vv.w);
    }
    vsum *= -0.5f;
    // |e_j| <= sum |v| =: bound.  The softmax does not care which constant is subtracted from the
    // energies, so when the bound is small enough for exp(e - bound) to stay far from underflow
    // (exp(-2 * 30) = 9e-27) it replaces the maximum: the weights' numerators and their sum are then
    // formed right here in the energy loop, and the two passes over s_e (maximum, exponentials) with
    // their barriers fall away.  A model with a larger bound takes those passes.
    float bound = 0.f;
#pragma unroll
    for (int at = 0; at < 8; ++at) {
        const float4 vv = *reinterpret_cast<const float4*>(&s_v[32 * g + 4 * at]);
        bound += (fabsf(vv.x) + fabsf(vv.y)) + (fabsf(vv.z) + fabsf(vv.w));
    }
    bound += __shfl_xor(bound, 16, 64);
    bound += __shfl_xor(bound, 32, 64);
    bound *= 0.5f;
    const bool fast_softmax = bound <= 30.f;        // the same in every lane of every wave
    float psum = 0.f;
    // ---- energies, one 16-position tile per wave at a time; PM of the next tile is already in flight.
    // The request's S workgroups share them: workgroup sp takes tiles sp, sp + S, ... and stores every energy
    // (numerator) beside this step's number as one 8-byte word; the others' words are fetched below.  The
    // energies are VALU work (128 exp + 128 rcp per position): computing all of them in each of the S
    // workgroups held the request's longest workgroup for 3 us at 300 positions.
    unsigned long long* ex = d.lsa_x + (size_t)slot * ML;
    for (int tt = sp + S * wave; tt < ntile; tt += S * LSA_WAVES) {
        const int j = tt * 16 + jl;
        uint4 pmc[NV];
        if constexpr (PM_AHEAD) {
#pragma unroll
            for (int i = 0; i < NV; ++i) pmc[i] = pmv[i];
            // unconditional: past the end it re-reads the last row, which is never used
            const MT* pm = PMs + (size_t)min(j + S * LSA_WAVES * 16, L - 1) * ATT;
#pragma unroll
            for (int i = 0; i < NV; ++i) pmv[i] = *reinterpret_cast<const uint4*>(pm + i * NPM);
        } else {
            const MT* pm = PMs + (size_t)min(j, L - 1) * ATT;
#pragma unroll
            for (int i = 0; i < NV; ++i) pmc[i] = *reinterpret_cast<const uint4*>(pm + i * NPM);
        }
        // rows 4g..4g+3 of tile `at` are attention dims 32 g + 4 at + i
        floatx4 pl[8], qv[8];
#pragma unroll
        for (int at = 0; at < 8; ++at) qv[at] = *reinterpret_cast<const floatx4*>(&s_q[32 * g + 4 * at]);
        tile.run(s_u[0], s_u[1], tt * 16 + jl, g, qv, pl);
        float e = vsum;
#pragma unroll
        for (int at = 0; at < 8; ++at) {
            const float4 vv = *reinterpret_cast<const float4*>(&s_v[32 * g + 4 * at]);
            float pv[4];
            if constexpr (sizeof(MT) == 2) {
                const uint4& u = pmc[at >> 1];
                const uint32_t w0 = (at & 1) ? u.z : u.x, w1 = (at & 1) ? u.w : u.y;
                pv[0] = bf16_lo(w0); pv[1] = bf16_hi(w0); pv[2] = bf16_lo(w1); pv[3] = bf16_hi(w1);
            } else {
                Vec16<float>::unpack(pmc[at], pv);
            }
            e = fmaf(vv.x, half_one_minus_tanh(pl[at][0] + pv[0]), e);
            e = fmaf(vv.y, half_one_minus_tanh(pl[at][1] + pv[1]), e);
            e = fmaf(vv.z, half_one_minus_tanh(pl[at][2] + pv[2]), e);
            e = fmaf(vv.w, half_one_minus_tanh(pl[at][3] + pv[3]), e);
        }
        e += __shfl_xor(e, 16, 64);
        e += __shfl_xor(e, 32, 64);
        if (fast_softmax) e = __expf(e - bound);
        if (g == 0 && j < L) {
            s_e[j] = e;
            if constexpr (XCH) {
                if (!twin) __hip_atomic_store(&ex[j], ((unsigned long long)seq << 32) | __float_as_uint(e), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                psum += e;
            }
        }
    }

    // ---- context over this workgroup's ENC / S columns: a wave-wide load covers S encoder rows
    // (64 / S lanes x 8 columns each), NR loads in flight per wave.  The first batch is requested
    // before the softmax needs its barriers.
    // The sum over positions is taken in an order that does not depend on S: position x belongs to
    // class x % 32 = 4 * wave + r, each class is summed in increasing x, then
    // a = sum_{wave = 0..7} ((c[0] + c[1]) + (c[2] + c[3])), so that a request's result is bit-identical
    // whatever the pool size (and hence S) happens to be.
    constexpr int FS = ENC / S;                     // columns of this workgroup
    constexpr int LPR = 64 / S;                     // lanes per encoder row
    constexpr int NA = 4 / S;                       // position classes per lane
    // rows in flight per lane.  CO: the kernel has 128 registers.  S = 1 (pools of more than 128 slots): the kernel streams
    // from HBM on every CU at once, and eight rows per lane in flight moved more bytes per second than sixteen or four.
    constexpr int NR = sizeof(MT) == 2 ? (CO ? 12 : (S == 1 ? 8 : 16)) : 8;
    constexpr int NP = NR / NA;                     // 32-position passes in flight
    constexpr int VPR = 8 * (int)sizeof(MT) / 16;   // 16-byte loads per row per lane
    const int xw = wave * 4 + (lane / LPR) * NA;    // this lane's first class
    // Rows are fetched through a buffer descriptor that ends at the request's last row: a row past the end comes back
    // as zeros without a memory access, so all NR loads per lane can be issued whatever the length, at no traffic.
    const MT* Fslot = reinterpret_cast<const MT*>(d.Fmem) + (size_t)slot * d.max_enc_len * ENC;
    const __amdgpu_buffer_rsrc_t f_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<MT*>(Fslot), 0, L * ENC * (int)sizeof(MT), BUFFER_RSRC_RAW);
    const int f_col = (sp * FS + (lane % LPR) * 8) * (int)sizeof(MT);     // this lane's columns inside a row, in bytes
    uint4 rows[NP][NA][VPR];
#pragma unroll
    for (int pp = 0; pp < NP; ++pp)
#pragma unroll
        for (int c = 0; c < NA; ++c) {
#pragma unroll
            for (int v = 0; v < VPR; ++v)
                rows[pp][c][v] = buffer_load16(f_rsrc, (pp * 32 + xw + c) * ENC * (int)sizeof(MT) + f_col + 16 * v);
        }
    if constexpr (XCH) {
        // the other workgroups' energies: every thread polls its own words until they carry this step's number
        // (bounded: the request's workgroups are resident together, S * slots <= 256 = one per CU)
        for (int x = tid; x < L; x += LSA_THREADS) {
            if (!twin && (x >> 4) % S != sp) {
                unsigned long long w = 0;
                bool in = false;
                for (int spin = 0; spin < d.wait_polls && !in; ++spin) {
                    w = __hip_atomic_load(&ex[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    in = (unsigned)(w >> 32) == seq;
                }
                if (!in) s_fail = 1;
                s_e[x] = __uint_as_float((unsigned)w);
            }
        }
        __syncthreads();
        // the sum in the order the one-workgroup form takes it: wave w adds tiles w, w + 8, ...
        for (int tt = wave; tt < ntile; tt += LSA_WAVES) {
            const int j = tt * 16 + jl;
            if (g == 0 && j < L) psum += s_e[j];
        }
    }
    psum = wave_sum(psum);
    if (lane == 0) s_red[LSA_WAVES + wave] = psum;
    __syncthreads();

    // ---- ragged softmax over j < L: s_e holds the numerators already, or the energies
    float sum;
    if (!fast_softmax) {
        float mx = -INFINITY;
        for (int x = tid; x < L; x += LSA_THREADS) mx = fmaxf(mx, s_e[x]);
        mx = wave_max(mx);
        if (lane == 0) s_red[wave] = mx;
        __syncthreads();
        mx = s_red[0];
#pragma unroll
        for (int w = 1; w < LSA_WAVES; ++w) mx = fmaxf(mx, s_red[w]);
        sum = 0.f;
        for (int x = tid; x < L; x += LSA_THREADS) {
            const float p = __expf(s_e[x] - mx);
            s_e[x] = p;
            sum += p;
        }
        sum = wave_sum(sum);
        if (lane == 0) s_red[LSA_WAVES + wave] = sum;
        __syncthreads();
    }
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < LSA_WAVES; ++w) sum += s_red[LSA_WAVES + w];
    const float inv = 1.0f / sum;

    {
        float acc[NA][8];
#pragma unroll
        for (int c = 0; c < NA; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[c][i] = 0.f;
        for (int x0 = 0; x0 < L; x0 += 32 * NP) {
#pragma unroll
            for (int pp = 0; pp < NP; ++pp) {
                // a pass of 32 positions that lies wholly past the end adds exact zeros: skipped (the same for the whole
                // workgroup; no load sits inside the branch)
                if (x0 + pp * 32 < L) {
#pragma unroll
                    for (int c = 0; c < NA; ++c) {
                        const int x = x0 + pp * 32 + xw + c;
                        const float w = x < L ? s_e[x] : 0.f;
                        float fv[8];
#pragma unroll
                        for (int v = 0; v < VPR; ++v) Vec16<MT>::unpack(rows[pp][c][v], fv + v * NPM);
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[c][i] = fmaf(w, fv[i], acc[c][i]);
                    }
                }
                // refill these register rows with the rows NP passes ahead (unconditional: past the end the loads
                // return zeros and move nothing)
#pragma unroll
                for (int c = 0; c < NA; ++c)
#pragma unroll
                    for (int v = 0; v < VPR; ++v)
                        rows[pp][c][v] = buffer_load16(f_rsrc, (x0 + pp * 32 + xw + c + 32 * NP) * ENC * (int)sizeof(MT) + f_col + 16 * v);
            }
        }
        // classes held by one lane are paired here: (c0 + c1) [+ (c2 + c3)]
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float t = acc[0][i];
            if constexpr (NA >= 2) t = acc[0][i] + acc[1][i];
            if constexpr (NA == 4) t = t + (acc[2][i] + acc[3][i]);
            s_ctx[wave][lane * 8 + i] = t;
        }
    }
    __syncthreads();

    // A wait that ran out: the request cannot be advanced any further (its partners' energies never came).  It is
    // frozen where it stands - marked done, so that every later kernel leaves it alone, and failed, so that the host
    // can tell its owner - and nothing of this step is stored for it; every other request goes on.  (s_fail was last
    // written before the barrier that follows the polling.)
    const bool failed = XCH && s_fail != 0;
    if (failed && tid == 0 && active) {
        d.done[slot] = 1;
        d.failed[slot] = 1;
        *d.fault = 1;
    }
    const bool store = active && !failed;
    XT* xa = reinterpret_cast<XT*>(d.xatt[cur ^ 1]);
    XT* xd = reinterpret_cast<XT*>(d.xdec[cur]);
    for (int f = tid; f < FS; f += LSA_THREADS) {
        // column f of this workgroup: lane f/8 of each row group, element f%8
        const int e0 = (f / 8) * 8 + (f & 7);
        float c = 0.f;
#pragma unroll
        for (int w = 0; w < LSA_WAVES; ++w) {
            float t;
            if constexpr (S == 1) t = s_ctx[w][e0];
            else if constexpr (S == 2) t = s_ctx[w][e0] + s_ctx[w][LPR * 8 + e0];
            else t = (s_ctx[w][e0] + s_ctx[w][LPR * 8 + e0]) + (s_ctx[w][2 * LPR * 8 + e0] + s_ctx[w][3 * LPR * 8 + e0]);
            c += t;
        }
        const XT a = from_float<XT>(c * inv);
        const int k = sp * FS + f;
        if (store) {
            xa[xoff<XT>(K_ATT / KB, slot, XA_A + k)] = a;
            xd[xoff<XT>(K_DEC / KB, slot, XD_A + k)] = a;
        }
    }
    // the new weights: every workgroup of the request holds all of them, each writes its share
    float* wl_out = d.w_last[cur ^ 1] + (size_t)slot * d.max_enc_len;
    float* wa_out = d.w_acc[cur ^ 1] + (size_t)slot * d.max_enc_len;
    for (int x = sp + S * tid; x < L; x += S * LSA_THREADS) {
        const float w = s_e[x] * inv;
        if (store) {
            wl_out[x] = w;
            wa_out[x] = s_u[1][x + LOC_PAD] + w;
        }
    }
}

// ---------------------------------------------------------------------------
// Mel + stop projection of [H_dec; A] (Eq. 2 line 5), ring write, frame counter
// and the prenet of the new frame (the Pre(M_last) of the next step), per pool
// tile (16 slots).  Three chained MFMA products with the slots as the 16 columns:
//   mel^T (96 x 16)  = W_proj (81 rows padded to 96, K = 1536, split over the waves) * Y^T
//   hid^T (256 x 16) = relu(W_p1 (K = 80, zero padded) * mel^T)
//   p^T   (256 x 16) = relu(W_p2 * hid^T)
// What bounds it is the weights that pass through one CU (475 KB in bf16 at 60 - 85 GB/s).  Pools without gate
// pre-sums run one workgroup per tile.  With pre-sums the launch fills the chip anyway and XCD 0 is reserved for the
// projection, so a tile gets G workgroups there (six, or fewer in pools of many tiles) that split the K of the first product: the helpers store their
// 96 x 16 partial sums and raise a sequence number each, the leader (which meanwhile pulls the prenet weights) waits
// for those numbers, adds the partials in helper order and goes on alone.  The wait is bounded: a leader that gives
// up raises d.fault and finishes with whatever it has, so the grid always drains.
// ---------------------------------------------------------------------------
constexpr int PROJ_THREADS = 512;
constexpr int PROJ_WAVES = PROJ_THREADS / 64;
constexpr int PROJ_ROWS = 96;
constexpr int PROJ_MEL_LD = PROJ_ROWS + 4, PROJ_HID_LD = PRENET + 4;
constexpr int PROJ_GROUP_K = PROJ_GROUP;   // workgroups that split K of the projection in pools of at most five tiles
constexpr int PROJ_WIN = 6;      // weight loads per wave in flight (the fused form)

template <typename XT> struct PrenetK1 { static constexpr int value = 80; };
template <> struct PrenetK1<h16_t> { static constexpr int value = 96; };

// B fragment (16 bytes of XT) from 16/sizeof(XT) consecutive fp32 values in LDS
template <typename XT> __device__ __forceinline__ uint4 frag_from_f32(const float* p);
template <> __device__ __forceinline__ uint4 frag_from_f32<float>(const float* p)
{
    return make_uint4(__float_as_uint(p[0]), __float_as_uint(p[1]), __float_as_uint(p[2]), __float_as_uint(p[3]));
}
template <> __device__ __forceinline__ uint4 frag_from_f32<h16_t>(const float* p)
{
    return make_uint4(pack2<h16_t>(p[0], p[1]), pack2<h16_t>(p[2], p[3]), pack2<h16_t>(p[4], p[5]), pack2<h16_t>(p[6], p[7]));
}

// The decoder LSTM inside the projection kernel's launch (two-byte pools of at most four tiles, where what is left of its
// gates is K = ENC: the sums over H_att and H_dec arrive as pre-sums).  Every one of the launch's 256 workgroups first
// forms one of the 256 pieces k_lstm_rc<dec, 2> would (two row tiles x half of the pool tiles, the same sums in the same
// order), stores H_dec where the next step reads it, and hands it to the projection's workgroups of the same launch as
// 8-byte words of four halves, laid out as the projection's B operand (hdec_x); the exponent's top bit of each half, never
// set for |h| <= 1, carries one of the low four bits of the step's number.  The number is the tile's leader's count of
// steps (the last of the tile's PROJ_GROUP_K + 1 counters), which the leader advances only after all of the tile's
// words have been consumed: a word of the step before carries the number before, one of sixteen steps ago cannot exist.
// (Polls of another workgroup's words pass through a CU's load path at 25-30 GB/s: the denser the words, the shorter a
// round of polls.)
// A slot without a running request hands over zeros (its projection is dropped).  issue() requests, finish() consumes:
// what a workgroup requests for its own part in between arrives behind the decoder LSTM's operands, not in front of them.
typedef floatx4 (*DecRed)[4][64];                // [wave][sum][lane]: 32 KB
template <typename XT>
struct DecUnit {
    static constexpr int NW = LSTM_WAVES, R = 2, TP = 2;
    static constexpr int NK = K_DEC / Frag<XT>::KB;
    static constexpr int F0 = lstm_hatt_frags<XT>();
    static constexpr int NF = lstm_main_frags<XT, K_DEC>() - F0;
    static constexpr int NRG = HID / 4 / R;
    static_assert(sizeof(XT) == 2 && Frag<XT>::KB == 32, "two-byte operands: a row group's eight units are one 16-byte piece");
    uint4 a[R][NF], b[TP][NF];
    floatx4 pre4, pre4b, bias4;
    float c_old;
    int lv, dn, sl, unit, c0, c1, rg;
    unsigned seq;
    bool mine;

    __device__ __forceinline__ void issue(const DevPtrs& d, const ProjHot& hot, int blk, int n_tiles)
    {
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const uint4* __restrict__ Wd = hot.Wd;
        const uint4* __restrict__ X = reinterpret_cast<const uint4*>(hot.xdec_cur);
        rg = blk % NRG;
        const int cg = blk / NRG;
        const int per = (n_tiles + R - 1) / R;
        c0 = min(cg * per, n_tiles);
        c1 = min(c0 + per, n_tiles);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int f = 0; f < NF; ++f) a[r][f] = Wd[xfrag(NK, R * rg + r, wave + (F0 + f) * NW, lane)];
#pragma unroll
        for (int t = 0; t < TP; ++t) {
            const int tile = max(min(c0 + t, c1 - 1), 0);
#pragma unroll
            for (int f = 0; f < NF; ++f) b[t][f] = X[xfrag(NK, tile, wave + (F0 + f) * NW, lane)];
        }
        // waves 0 .. 3 own a cell update: (pool tile c0 + wave / R, row tile wave % R); the others load the same words and drop them
        const int er = wave % R, et = (wave / R) % TP;
        const int tile_e = max(min(c0 + et, c1 - 1), 0);
        mine = wave < 4 && c0 + et < c1;
        sl = tile_e * 16 + (lane & 15);
        unit = (R * rg + er) * 4 + (lane >> 4);
        lv = hot.live[sl];
        dn = d.done[sl];
        c_old = d.c_dec[(size_t)sl * HID + unit];
        pre4 = reinterpret_cast<const floatx4*>(d.pre_dec)[((size_t)tile_e * (HID / 4) + R * rg + er) * 64 + lane];
        pre4b = reinterpret_cast<const floatx4*>(d.pre_dec_b)[((size_t)tile_e * (HID / 4) + R * rg + er) * 64 + lane];
        bias4 = *reinterpret_cast<const floatx4*>(d.bd + unit * 4);
        seq = hot.proj_seq[tile_e * (PROJ_GROUP_K + 1) + PROJ_GROUP_K] + 1u;
    }

    __device__ __forceinline__ void finish(const DevPtrs& d, const ProjHot& hot, DecRed red)
    {
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        if (c0 >= c1) return;                     // the whole workgroup: no pool tile in its half
#pragma unroll
        for (int t = 0; t < TP; ++t)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NF; ++f) acc = mfma_frag<XT>(a[r][f], b[t][f], acc);
                red[wave][R * t + r][lane] = acc;
            }
        __syncthreads();
        if (mine) {
            floatx4 g = bias4;
#pragma unroll
            for (int w = 0; w < NW; ++w) g += red[w][wave][lane];
            g += pre4;
            g += pre4b;
            const float gi = sigmoidf_(g[0]), gf = sigmoidf_(g[1]);
            const float gg = tanhf_(g[2]), go = sigmoidf_(g[3]);
            const float c = gf * c_old + gi * gg;
            const bool on = lv && !dn;
            XT h = from_float<XT>(go * tanhf_(c));
            if (on) {
                d.c_dec[(size_t)sl * HID + unit] = c;
                reinterpret_cast<XT*>(const_cast<void*>(hot.xdec_nxt))[xoff<XT>(NK, sl, XD_HD + unit)] = h;
            } else {
                h.bits = 0;
            }
            // lanes l, l + 16, l + 32, l + 48 hold the row tile's four units of one slot: the first stores all four as one
            // 8-byte word.  |h| <= 1, so bit 14 of a half (the exponent's top bit) is free: the four of them carry the
            // low four bits of the count.
            const int mineb = (int)h.bits;
            const unsigned long long u0 = (unsigned)mineb, u1 = (unsigned)__shfl(mineb, (lane & 15) + 16, 64);
            const unsigned long long u2 = (unsigned)__shfl(mineb, (lane & 15) + 32, 64), u3 = (unsigned)__shfl(mineb, (lane & 15) + 48, 64);
            if (lane < 16) {
                const int er = wave % R;
                const size_t w = (((size_t)(sl >> 4) * (HID / 32) + rg / 4) * 64 + (rg % 4) * 16 + lane) * 2 + er;
                const unsigned long long mark = (unsigned long long)(seq & 1u) << 14 | (unsigned long long)(seq >> 1 & 1u) << 30 |
                                                (unsigned long long)(seq >> 2 & 1u) << 46 | (unsigned long long)(seq >> 3 & 1u) << 62;
                __hip_atomic_store(&d.hdec_x[w], u0 | u1 << 16 | u2 << 32 | u3 << 48 | mark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
    }
};

struct ProjShared {
    float* big;                          // PROJ_WAVES * PROJ_ROWS * 16 floats: partial sums, later hid
    float (*mel)[PROJ_MEL_LD];           // [16][PROJ_MEL_LD]
    int *slot, *t, *cap;                 // [16] each
    int* ok;
};

// One workgroup's part of a tile: workgroup `kp` of G contracts fragments [kp, kp + 1) * NK / G of K; kp = 0 leads.
template <typename XT, int G, bool LEADER>
__device__ __forceinline__ void proj_tile(const DevPtrs& d, const ProjHot& hot, int cur, int tile, int kp, const ProjShared& sh, bool hand = false)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jl = lane & 15, g = lane >> 4;
    constexpr int KB = Frag<XT>::KB;
    constexpr int EPL = Frag<XT>::EPL;
    constexpr int NKD = K_DEC / KB;
    constexpr int NK = K_PROJ / KB;
    constexpr int NKW = NK / G / PROJ_WAVES;
    static_assert(NK % (G * PROJ_WAVES) == 0, "K must split evenly over the workgroups' waves");
    constexpr int NM = PROJ_ROWS / 16;
    // Everything is requested at once, small things first: the activations and the slots' bookkeeping words (a
    // workgroup serves the 16 slots tile * 16 ..: no list of active tiles to wait for), the biases, then the
    // weights.  A wave's whole share of W_proj (all row tiles of its K range) is in flight together, except for fp32
    // fragments of the whole K: there the row tiles go one at a time.  A tile without a running request is computed
    // and dropped (there is no early exit: the compiler would move the loads below it).
    constexpr bool W_EARLY = sizeof(XT) == 2 || G > 1;
    constexpr int MH = W_EARLY ? NM : 1;          // row tiles whose fragments are in flight together
    // the leader's prenet weights go out before the first product when its share of W_proj is small
    constexpr bool PRENET_FIRST = false;

    float (*s_part)[PROJ_ROWS][16] = reinterpret_cast<float (*)[PROJ_ROWS][16]>(sh.big);
    float (*s_hid)[PROJ_HID_LD] = reinterpret_cast<float (*)[PROJ_HID_LD]>(sh.big);
    static_assert(16 * PROJ_HID_LD <= PROJ_WAVES * PROJ_ROWS * 16, "hid must fit the partial-sum buffer it aliases");

    const uint4* xnew = reinterpret_cast<const uint4*>(hot.xdec_nxt);      // h_dec of this step
    const uint4* xcur = reinterpret_cast<const uint4*>(hot.xdec_cur);      // a of this step
    const int ks0 = (kp * PROJ_WAVES + wave) * NKW;
    uint4 b[NKW];
#pragma unroll
    for (int f = 0; f < NKW; ++f) {
        const int ks = ks0 + f;
        // (hand: h_dec is formed inside this launch and arrives as words, below; the load is of the step before's and dropped)
        b[f] = ks < HID / KB ? xnew[xfrag(NKD, tile, XD_HD / KB + ks, lane)]
                             : xcur[xfrag(NKD, tile, XD_A / KB + ks - HID / KB, lane)];
    }
    // this workgroup's sequence number: the steps it has taken part in
    unsigned my_seq = 0;
    if constexpr (G > 1) my_seq = hot.proj_seq[tile * G + kp];
    // slot bookkeeping of the 16 columns and this thread's biases of the reduction phase
    const int my_sl = tile * 16 + (tid & 15);
    int my_live = 0, my_done = 0, my_t = 0, my_cap = 0;
    constexpr int RED_IT = 16 * PROJ_ROWS / PROJ_THREADS;
    static_assert(16 * PROJ_ROWS % PROJ_THREADS == 0, "the reduction phase splits evenly");
    float bias_r[RED_IT];
    unsigned step_no = 0;
    if constexpr (LEADER) {
        step_no = d.step_seq[0];
        my_live = hot.live[my_sl]; my_done = d.done[my_sl]; my_t = d.t[my_sl]; my_cap = d.n_steps[my_sl];
#pragma unroll
        for (int it = 0; it < RED_IT; ++it) bias_r[it] = d.bmel[min((tid + it * PROJ_THREADS) >> 4, N_PROJ - 1)];
    }

    const uint4* W = reinterpret_cast<const uint4*>(hot.Wmel) + lane;
    uint4 a[MH][NKW];
    auto load_proj_weights = [&](int m0) __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < MH; ++m)
#pragma unroll
            for (int f = 0; f < NKW; ++f) {
                // the last row tile holds the stop row and 15 rows of zeros: do not fetch the zeros
                a[m][f] = make_uint4(0, 0, 0, 0);
                if (m0 + m < NM - 1 || jl == 0) a[m][f] = W[((size_t)(m0 + m) * NK + ks0 + f) * 64];
            }
    };
    if constexpr (W_EARLY) load_proj_weights(0);
    // weights of the two prenet layers for this wave's row tiles (w and w + 8), used after the two reduction phases
    constexpr int NK3 = PrenetK1<XT>::value / KB;
    constexpr int NK4 = PRENET / KB;
    uint4 a3[LEADER ? 2 : 1][NK3], a4[LEADER ? 2 : 1][NK4];
    auto load_prenet_weights = [&]() __attribute__((always_inline)) {
        const uint4* W1 = reinterpret_cast<const uint4*>(d.Wp1) + lane;
        const uint4* W2 = reinterpret_cast<const uint4*>(d.Wp2) + lane;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int mt = wave + m * PROJ_WAVES;
#pragma unroll
            for (int f = 0; f < NK3; ++f) a3[m][f] = W1[((size_t)mt * NK3 + f) * 64];
#pragma unroll
            for (int f = 0; f < NK4; ++f) a4[m][f] = W2[((size_t)mt * NK4 + f) * 64];
        }
    };
    if constexpr (PRENET_FIRST) load_prenet_weights();
    // keep the loads in this order: left alone, the scheduler issues the activation loads one at a
    // time between the MFMAs, each a full round trip
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (sizeof(XT) == 2) {
        if (hand) {
            // the wave's fragments of h_dec from the words the decoder LSTM's part of this launch hands over: every lane
            // polls its two words per fragment (a bounded number of times); a fragment that lies in `a` waits for nobody
            constexpr unsigned long long MARK = 0x4000400040004000ull;
            const unsigned cnt4 = (my_seq + 1u) & 15u;
            const unsigned long long expect = (unsigned long long)(cnt4 & 1u) << 14 | (unsigned long long)(cnt4 >> 1 & 1u) << 30 |
                                              (unsigned long long)(cnt4 >> 2 & 1u) << 46 | (unsigned long long)(cnt4 >> 3 & 1u) << 62;
            unsigned long long w[NKW][2];
            bool all_in = false;
            for (int spin = 0; spin < d.wait_polls && !all_in; ++spin) {
                all_in = true;
#pragma unroll
                for (int f = 0; f < NKW; ++f) {
                    const unsigned long long* hx = d.hdec_x + (((size_t)tile * (HID / KB) + min(ks0 + f, HID / KB - 1)) * 64 + lane) * 2;
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        w[f][i] = __hip_atomic_load(&hx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        all_in = all_in && (ks0 + f >= HID / KB || (w[f][i] & MARK) == expect);
                    }
                }
            }
            if (!all_in) *sh.ok = 0;                       // looked at after the next barrier
#pragma unroll
            for (int f = 0; f < NKW; ++f)
                if (ks0 + f < HID / KB) {
                    const unsigned long long w0 = w[f][0] & ~MARK, w1 = w[f][1] & ~MARK;
                    b[f] = all_in ? make_uint4((unsigned)w0, (unsigned)(w0 >> 32), (unsigned)w1, (unsigned)(w1 >> 32)) : make_uint4(0, 0, 0, 0);
                }
        }
    }

    // ---- phase 1: projection of [h_dec; a], K split over the waves
#pragma unroll
    for (int m0 = 0; m0 < NM; m0 += MH) {
        if constexpr (!W_EARLY) load_proj_weights(m0);
#pragma unroll
        for (int m = 0; m < MH; ++m) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int f = 0; f < NKW; ++f) acc = mfma_frag<XT>(a[m][f], b[f], acc);
#pragma unroll
            for (int i = 0; i < 4; ++i) s_part[wave][16 * (m0 + m) + 4 * g + i][jl] = acc[i];
        }
    }

    if constexpr (LEADER) {
        if (tid < 16) {
            const bool on = my_live && !my_done;
            sh.slot[tid] = on ? my_sl : -1;
            sh.t[tid] = on ? my_t : 0;
            sh.cap[tid] = on ? my_cap : 0;
        }
        // requested now that the projection fragments have left the registers
        if constexpr (!PRENET_FIRST) load_prenet_weights();
    }
    __syncthreads();

    // ---- phase 2: reduce over the waves ...
    float v[RED_IT];
#pragma unroll
    for (int it = 0; it < RED_IT; ++it) {
        const int idx = tid + it * PROJ_THREADS;
        const int o = idx >> 4, r = idx & 15;
        v[it] = 0.f;
        if (o < N_PROJ) {
            if constexpr (LEADER) v[it] = bias_r[it];
#pragma unroll
            for (int w = 0; w < PROJ_WAVES; ++w) v[it] += s_part[w][o][r];
        }
    }
    if constexpr (!LEADER) {
        // ... a helper hands its sums over, each word with the sequence number beside it in one 8-byte store: the
        // leader knows a word is this step's from the number it carries, no flag and no fence are needed
        // (a helper whose wait for h_dec ran out hands nothing over: the leader's wait for its sums then runs out as well)
        unsigned long long* mine = d.proj_part + (size_t)(tile * (G - 1) + kp - 1) * (16 * PROJ_ROWS);
        if (*sh.ok) {
#pragma unroll
            for (int it = 0; it < RED_IT; ++it)
                __hip_atomic_store(&mine[tid + it * PROJ_THREADS], ((unsigned long long)(my_seq + 1u) << 32) | __float_as_uint(v[it]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid == 0) hot.proj_seq[tile * G + kp] = my_seq + 1u;
        return;
    } else {
        if constexpr (G > 1) {
            // ... the leader takes the helpers' words as they arrive (every thread polls its own, a bounded number of
            // times) and adds them in helper order
            unsigned long long w[G - 1][RED_IT];
            bool all_in = false;
            for (int spin = 0; spin < d.wait_polls && !all_in; ++spin) {
                all_in = true;
#pragma unroll
                for (int h = 0; h < G - 1; ++h) {
                    const unsigned long long* theirs = d.proj_part + (size_t)(tile * (G - 1) + h) * (16 * PROJ_ROWS);
#pragma unroll
                    for (int it = 0; it < RED_IT; ++it) {
                        w[h][it] = __hip_atomic_load(&theirs[tid + it * PROJ_THREADS], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        all_in = all_in && (unsigned)(w[h][it] >> 32) == my_seq + 1u;
                    }
                }
            }
            if (!all_in) *sh.ok = 0;
#pragma unroll
            for (int h = 0; h < G - 1; ++h)
#pragma unroll
                for (int it = 0; it < RED_IT; ++it) v[it] += __uint_as_float((unsigned)w[h][it]);
            if (tid == 0) hot.proj_seq[tile * G] = my_seq + 1u;
        }
        // ... bias is in; hand the frame out
#pragma unroll
        for (int it = 0; it < RED_IT; ++it) {
            const int idx = tid + it * PROJ_THREADS;
            sh.mel[idx & 15][idx >> 4] = v[it];
        }
        __syncthreads();
        // A wait that ran out: the helpers' sums never came, so this tile's frames cannot be formed.  Its requests are
        // frozen where they stand (done: every later kernel leaves them alone; failed: the host tells their owners) and
        // nothing of this step is stored for them; the step counter below still advances for everyone else.
        const bool gave_up = *sh.ok == 0;
        __syncthreads();
        if (gave_up && tid < 16 && sh.slot[tid] >= 0) {
            d.done[sh.slot[tid]] = 1;
            d.failed[sh.slot[tid]] = 1;
            *d.fault = 1;
            sh.slot[tid] = -1;
        }
        if (gave_up) __syncthreads();
        for (int idx = tid; idx < 16 * N_PROJ; idx += PROJ_THREADS) {
            const int r = idx / N_PROJ, o = idx - r * N_PROJ;
            const int sl = sh.slot[r];
            if (sl >= 0) {
                const float m = sh.mel[r][o];
                if (o < N_MEL) {
                    d.mel_ring[((size_t)sl * d.max_steps + sh.t[r]) * N_MEL + o] = m;
                    d.m_last[(size_t)sl * N_MEL + o] = m;
                } else {
                    d.stop_ring[(size_t)sl * d.max_steps + sh.t[r]] = m;
                }
            }
        }

        // ---- phase 3: hid^T = relu(W_p1 mel^T); wave w owns row tiles w and w + 8
        {
            uint4 bm[NK3];
#pragma unroll
            for (int f = 0; f < NK3; ++f) bm[f] = frag_from_f32<XT>(&sh.mel[jl][f * KB + g * EPL]);
            floatx4 acc[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NK3; ++f) acc[m] = mfma_frag<XT>(a3[m][f], bm[f], acc[m]);
            }
            // s_hid aliases the partial sums: every read of those finished before the last barrier
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int i = 0; i < 4; ++i) s_hid[jl][16 * (wave + m * PROJ_WAVES) + 4 * g + i] = fmaxf(acc[m][i], 0.f);
        }
        __syncthreads();

        // ---- phase 4: p^T = relu(W_p2 hid^T)
        {
            uint4 bh[NK4];
#pragma unroll
            for (int f = 0; f < NK4; ++f) bh[f] = frag_from_f32<XT>(&s_hid[jl][f * KB + g * EPL]);
            const int sl = sh.slot[jl];
            XT* xa = reinterpret_cast<XT*>(d.xatt[cur ^ 1]);
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int mt = wave + m * PROJ_WAVES;
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NK4; ++f) acc = mfma_frag<XT>(a4[m][f], bh[f], acc);
                if (sl >= 0) {
                    // four consecutive k inside one 16-byte piece: one store
                    XT* dst = xa + xoff<XT>(K_ATT / KB, sl, XA_P + 16 * mt + 4 * g);
                    const float p0 = fmaxf(acc[0], 0.f), p1 = fmaxf(acc[1], 0.f), p2 = fmaxf(acc[2], 0.f), p3 = fmaxf(acc[3], 0.f);
                    if constexpr (sizeof(XT) == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(pack2<XT>(p0, p1), pack2<XT>(p2, p3));
                    else *reinterpret_cast<float4*>(dst) = make_float4(p0, p1, p2, p3);
                }
            }
        }

        // one step further: the number the attention kernel's workgroups mark their exchanged words with
        if (tile == 0 && tid == 0) d.step_seq[0] = step_no + 1u;
        if (tid < 16 && sh.slot[tid] >= 0) {
            const int sl = sh.slot[tid];
            const int tn = sh.t[tid] + 1;
            d.t[sl] = tn;
            bool fin = tn >= sh.cap[tid];
            if (d.stop_threshold >= 0.f && sigmoidf_(sh.mel[tid][N_MEL]) > d.stop_threshold) fin = true;
            if (fin) d.done[sl] = 1;
        }
    }
}

// The fused form of a tile's workgroups (two-byte pools of at most four tiles; the launch holds the decoder LSTM too,
// DecUnit).  Every workgroup first forms its piece of the decoder LSTM - other tiles' workgroups wait for it as well - and
// only then requests its weights.  G workers contract one G-th of K of the projection each, as in the plain form, with
// H_dec taken as words from hdec_x once every piece of a wave's K range is in, and hand their partial sums over as 4-byte
// words (the count's low four bits in the mantissa's); worker 0's start from the bias.  A further workgroup leads: it pulls nothing but the prenet's weights (with a
// short window of loads per wave in flight: a wave that asks for all of them at once gets less than half the rate out of
// the CU's load path), polls the G partial sums, adds them in worker order - the plain form's order - and runs the prenet.  The last worker, whose fragments of K lie in `a` and which is therefore done early,
// collects the sums as well and keeps the books meanwhile: frame and stop value into the rings, frame counters, end of a
// request.  (All G + 1 workgroups adding the sums themselves and sharing the prenet's second layer was tried: six times
// the polls, and a word took 3 us to be seen instead of 1.)
constexpr int FUSED_GROUP = PROJ_GROUP_K + 1;    // workgroups per tile: the workers and the leader
// row groups of the next step's attention LSTM per workgroup that forms them (two: half as many workgroups polling, but
// twice the weights through each one's load path, which is what the tail of the launch then waits for: + 0.5 us)
constexpr int TAIL_RG = 1;
template <typename XT>
__device__ __forceinline__ void proj_tile_fused(const DevPtrs& d, const ProjHot& hot, int cur, int tile, int kp, const ProjShared& sh, int n_tiles,
                                                unsigned tail_stamp)
{
    constexpr int G = PROJ_GROUP_K;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jl = lane & 15, g = lane >> 4;
    constexpr int KB = Frag<XT>::KB;
    constexpr int EPL = Frag<XT>::EPL;
    constexpr int NKD = K_DEC / KB;
    constexpr int NK = K_PROJ / KB;
    static_assert(NK == G * PROJ_WAVES, "one fragment of K per wave");
    constexpr int NM = PROJ_ROWS / 16;
    constexpr int NK3 = PrenetK1<XT>::value / KB;
    constexpr int NK4 = PRENET / KB;
    constexpr int RED_IT = 16 * PROJ_ROWS / PROJ_THREADS;
    static_assert(16 * PROJ_ROWS % PROJ_THREADS == 0, "the reduction phase splits evenly");
    const bool leader = kp == G;

    DecUnit<XT> dec;
    dec.issue(d, hot, blockIdx.x, n_tiles);
    if (tid == 0) *sh.ok = 1;
    float (*s_part)[PROJ_ROWS][16] = reinterpret_cast<float (*)[PROJ_ROWS][16]>(sh.big);
    float (*s_hid)[PROJ_HID_LD] = reinterpret_cast<float (*)[PROJ_HID_LD]>(sh.big);
    static_assert(16 * PROJ_HID_LD <= PROJ_WAVES * PROJ_ROWS * 16, "hid must fit the partial-sum buffer it aliases");
    // this workgroup's count of the steps it has taken part in: the number its words carry, and the one it expects
    const unsigned my_seq = hot.proj_seq[tile * FUSED_GROUP + kp];

    // slot bookkeeping of the 16 columns: the leader (which stores p) and the keeper of the books (the last worker) need it
    const bool keeper = kp == G - 1;
    const int my_sl = tile * 16 + (tid & 15);
    const int my_live = hot.live[my_sl], my_done = d.done[my_sl];
    const int my_t = d.t[my_sl], my_cap = d.n_steps[my_sl];
    const unsigned step_no = d.step_seq[0];

    // The workers' sums as they arrive (every thread polls its own words, a bounded number of times), added in worker
    // order; then the frame into LDS.  A wait that ran out: the tile's frames cannot be formed; its requests are frozen
    // where they stand (done: every later kernel leaves them alone; failed: the host tells their owners) and the
    // workgroup stores nothing of this step for them.  Leader and keeper each do this for themselves.
    auto collect_frame = [&]() __attribute__((always_inline)) {
        float v[RED_IT];
        unsigned w[G][RED_IT];
        // A word is a partial sum rounded to 20 bits of mantissa with the low four bits of the step count in the freed
        // bits (sum_word): four bytes instead of eight.  Polls of words that another workgroup writes pass through the
        // CU's load path at 25-30 GB/s, so a round of them takes as long as its bytes: 18 loads per thread of eight-byte
        // words took 2.9 us.  The workers whose fragments lie in `a` wait for nobody and are done first: their words
        // are asked for first and those of the workers that wait for h_dec last.
        const unsigned phase = (my_seq + 1u) & 15u;
        const unsigned* part32 = reinterpret_cast<const unsigned*>(d.proj_part);
        bool all_in = false;
        for (int spin = 0; spin < d.wait_polls && !all_in; ++spin) {
            all_in = true;
#pragma unroll
            for (int q = 0; q < G; ++q) {
                constexpr int H_WORKERS = HID / KB / PROJ_WAVES;      // workers 0 .. H_WORKERS - 1 contract h_dec
                const int h = (q + H_WORKERS) % G;
                const unsigned* theirs = part32 + (size_t)(tile * G + h) * (16 * PROJ_ROWS);
                // (a lane whose word lies in the zero rows beyond the stop row asks for the worker's first word instead: a
                // wave of such lanes is one request, and no branch surrounds the load)
#pragma unroll
                for (int it = 0; it < RED_IT; ++it) {
                    const int idx = tid + it * PROJ_THREADS;
                    w[h][it] = __hip_atomic_load(&theirs[(idx >> 4) < N_PROJ ? idx : 0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int it = 0; it < RED_IT; ++it) all_in = all_in && (w[h][it] & 15u) == phase;
        }
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int it = 0; it < RED_IT; ++it)
                if (((tid + it * PROJ_THREADS) >> 4) >= N_PROJ) w[h][it] = 0u;
        if (!all_in) *sh.ok = 0;
#pragma unroll
        for (int it = 0; it < RED_IT; ++it) {
            v[it] = __uint_as_float(w[0][it] & ~15u);
#pragma unroll
            for (int h = 1; h < G; ++h) v[it] += __uint_as_float(w[h][it] & ~15u);
            const int idx = tid + it * PROJ_THREADS;
            sh.mel[idx & 15][idx >> 4] = v[it];
        }
        __syncthreads();
        const bool gave_up = *sh.ok == 0;
        __syncthreads();
        if (gave_up && tid < 16 && sh.slot[tid] >= 0) {
            d.done[sh.slot[tid]] = 1;
            d.failed[sh.slot[tid]] = 1;
            *d.fault = 1;
            sh.slot[tid] = -1;
        }
        if (gave_up) __syncthreads();
    };

    if (!leader) {
        // ---- a worker: fragment ks of K = [h_dec; a] in wave `wave`
        const uint4* xcur = reinterpret_cast<const uint4*>(hot.xdec_cur);
        const int ks = kp * PROJ_WAVES + wave;
        const bool from_h = ks < HID / KB;
        uint4 b = xcur[xfrag(NKD, tile, XD_A / KB + max(ks - HID / KB, 0), lane)];
        float bias_r[RED_IT];
#pragma unroll
        for (int it = 0; it < RED_IT; ++it) bias_r[it] = d.bmel[min((tid + it * PROJ_THREADS) >> 4, N_PROJ - 1)];
        // The wave's fragments of the projection's weights are requested here, behind the piece's operands (they arrive in
        // the order of the requests, so the piece is not held up) and before the piece is formed: requested after it, these
        // 48 KB per workgroup were what a worker waited for, half a microsecond after its words of h_dec were in.
        // (all six row tiles' fragments, the zero rows of the last included: a branch around a load would make the
        // compiler wait for every load in flight where it rejoins)
        const uint4* W = reinterpret_cast<const uint4*>(hot.Wmel) + lane;
        uint4 a[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) a[m] = W[((size_t)m * NK + ks) * 64];
        __builtin_amdgcn_sched_barrier(0);
        dec.finish(d, hot, reinterpret_cast<DecRed>(sh.big));
        if (tid < 16) {
            const bool on = my_live && !my_done;
            sh.slot[tid] = on ? my_sl : -1;
            sh.t[tid] = on ? my_t : 0;
            sh.cap[tid] = on ? my_cap : 0;
        }
        __syncthreads();                                   // (a piece without pool tiles has no barrier of its own)
        // the wave's fragment of h_dec: every lane polls its four words (a bounded number of times)
        bool all_in = !from_h;                             // a wave whose fragment lies in `a` waits for nobody
        unsigned long long w[2];
        const unsigned long long* hx = d.hdec_x + (((size_t)tile * (HID / KB) + min(ks, HID / KB - 1)) * 64 + lane) * 2;
        constexpr unsigned long long MARK = 0x4000400040004000ull;
        const unsigned cnt4 = (my_seq + 1u) & 15u;
        const unsigned long long expect = (unsigned long long)(cnt4 & 1u) << 14 | (unsigned long long)(cnt4 >> 1 & 1u) << 30 |
                                          (unsigned long long)(cnt4 >> 2 & 1u) << 46 | (unsigned long long)(cnt4 >> 3 & 1u) << 62;
        for (int spin = 0; spin < d.wait_polls && !all_in; ++spin) {
            all_in = true;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                w[i] = __hip_atomic_load(&hx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                all_in = all_in && (w[i] & MARK) == expect;
            }
        }
        if (!all_in) *sh.ok = 0;                           // looked at after the next barrier
        if (from_h && all_in) {
            const unsigned long long w0 = w[0] & ~MARK, w1 = w[1] & ~MARK;
            b = make_uint4((unsigned)w0, (unsigned)(w0 >> 32), (unsigned)w1, (unsigned)(w1 >> 32));
        }
        // the projection, one fragment of K per wave ...
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const floatx4 acc = mfma_frag<XT>(a[m], b, floatx4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int i = 0; i < 4; ++i) s_part[wave][16 * m + 4 * g + i][jl] = acc[i];
        }
        __syncthreads();
        // ... reduced over the waves and handed over, each word with the step count beside it in one 8-byte store (a
        // worker whose wait for h_dec ran out hands nothing over: the waits for its sums then run out as well)
        if (*sh.ok) {
            unsigned* mine = reinterpret_cast<unsigned*>(d.proj_part) + (size_t)(tile * G + kp) * (16 * PROJ_ROWS);
#pragma unroll
            for (int it = 0; it < RED_IT; ++it) {
                const int idx = tid + it * PROJ_THREADS;
                const int o = idx >> 4, r = idx & 15;
                float v = 0.f;
                if (o < N_PROJ) {
                    if (kp == 0) v = bias_r[it];
#pragma unroll
                    for (int wv = 0; wv < PROJ_WAVES; ++wv) v += s_part[wv][o][r];
                }
                // sum_word: the magnitude rounded to the nearest multiple of 16 units in the last place, the count's
                // low four bits in their stead (a worker that hands nothing over in a step falls one count behind what
                // its readers expect, and stays recognisable for sixteen steps)
                __hip_atomic_store(&mine[idx], ((__float_as_uint(v) + 8u) & ~15u) | ((my_seq + 1u) & 15u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (tid == 0) hot.proj_seq[tile * FUSED_GROUP + kp] = my_seq + 1u;
        if (!keeper) return;

        // ---- the keeper of the books (the last worker, whose fragments lie in `a`: it is done early): the frame out, one
        // step further, while the leader runs the prenet
        collect_frame();
        for (int idx = tid; idx < 16 * N_PROJ; idx += PROJ_THREADS) {
            const int r = idx / N_PROJ, o = idx - r * N_PROJ;
            const int sl = sh.slot[r];
            if (sl >= 0) {
                const float m = sh.mel[r][o];
                if (o < N_MEL) {
                    d.mel_ring[((size_t)sl * d.max_steps + sh.t[r]) * N_MEL + o] = m;
                    d.m_last[(size_t)sl * N_MEL + o] = m;
                } else {
                    d.stop_ring[(size_t)sl * d.max_steps + sh.t[r]] = m;
                }
            }
        }
        // the number the attention kernel's workgroups mark their exchanged words with
        if (tile == 0 && tid == 0) d.step_seq[0] = step_no + 1u;
        if (tid < 16 && sh.slot[tid] >= 0) {
            const int sl = sh.slot[tid];
            const int tn = sh.t[tid] + 1;
            d.t[sl] = tn;
            bool fin = tn >= sh.cap[tid];
            if (d.stop_threshold >= 0.f && sigmoidf_(sh.mel[tid][N_MEL]) > d.stop_threshold) fin = true;
            if (fin) d.done[sl] = 1;
        }
        return;
    }

    // ---- the leader
    __builtin_amdgcn_sched_barrier(0);
    dec.finish(d, hot, reinterpret_cast<DecRed>(sh.big));
    if (tid < 16) {
        const bool on = my_live && !my_done;
        sh.slot[tid] = on ? my_sl : -1;
        sh.t[tid] = on ? my_t : 0;
        sh.cap[tid] = on ? my_cap : 0;
    }
    // weights of the two prenet layers for this wave's row tiles (w and w + 8)
    const uint4* W1 = reinterpret_cast<const uint4*>(d.Wp1) + lane;
    const uint4* W2 = reinterpret_cast<const uint4*>(d.Wp2) + lane;
    uint4 a3[2][NK3], a4[2][NK4];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int mt = wave + m * PROJ_WAVES;
#pragma unroll
        for (int f = 0; f < NK3; ++f) {
            a3[m][f] = W1[((size_t)mt * NK3 + f) * 64];
            vm_in_flight_at_most<PROJ_WIN>();
        }
#pragma unroll
        for (int f = 0; f < NK4; ++f) {
            a4[m][f] = W2[((size_t)mt * NK4 + f) * 64];
            vm_in_flight_at_most<PROJ_WIN>();
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    collect_frame();

    // hid^T = relu(W_p1 mel^T); wave w owns row tiles w and w + 8
    {
        uint4 bm[NK3];
#pragma unroll
        for (int f = 0; f < NK3; ++f) bm[f] = frag_from_f32<XT>(&sh.mel[jl][f * KB + g * EPL]);
        floatx4 acc[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int f = 0; f < NK3; ++f) acc[m] = mfma_frag<XT>(a3[m][f], bm[f], acc[m]);
        }
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int i = 0; i < 4; ++i) s_hid[jl][16 * (wave + m * PROJ_WAVES) + 4 * g + i] = fmaxf(acc[m][i], 0.f);
    }
    __syncthreads();
    // p^T = relu(W_p2 hid^T)
    {
        uint4 bh[NK4];
#pragma unroll
        for (int f = 0; f < NK4; ++f) bh[f] = frag_from_f32<XT>(&s_hid[jl][f * KB + g * EPL]);
        const int sl = sh.slot[jl];
        XT* xa = reinterpret_cast<XT*>(d.xatt[cur ^ 1]);
        // handed over as words (tail_stamp != 0): does the slot take the next step?  The rule the keeper of the books applies.
        bool goes_on = sl >= 0 && sh.t[jl] + 1 < sh.cap[jl];
        if (d.stop_threshold >= 0.f && sigmoidf_(sh.mel[jl][N_MEL]) > d.stop_threshold) goes_on = false;
        const unsigned long long mark = (unsigned long long)((goes_on ? 0u : 0x80000000u) | tail_stamp) << 32;
        // (both row tiles' products before the first store: the wait the compiler places in front of the second tile's
        // weights counts every memory operation issued before it, the first tile's stores included)
        floatx4 acc[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            acc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int f = 0; f < NK4; ++f) acc[m] = mfma_frag<XT>(a4[m][f], bh[f], acc[m]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int mt = wave + m * PROJ_WAVES;
            const float p0 = fmaxf(acc[m][0], 0.f), p1 = fmaxf(acc[m][1], 0.f), p2 = fmaxf(acc[m][2], 0.f), p3 = fmaxf(acc[m][3], 0.f);
            const unsigned lo = sl >= 0 ? pack2<XT>(p0, p1) : 0u, hi = sl >= 0 ? pack2<XT>(p2, p3) : 0u;
            if (tail_stamp != 0u) {
                // rows 16 mt + 4 g .. + 3 of p = half of the 16-byte piece (mt % 2) * 2 + g / 2 of fragment mt / 2, column jl
                const int piece = (mt & 1) * 2 + (g >> 1);
                unsigned long long* px = d.p_x + (((size_t)tile * (PRENET / KB) + (mt >> 1)) * 4 + 2 * (g & 1)) * 64 + piece * 16 + jl;
                __hip_atomic_store(px, mark | lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(px + 64, mark | hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (sl >= 0) {
                // four consecutive k inside one 16-byte piece: one store
                XT* dst = xa + xoff<XT>(K_ATT / KB, sl, XA_P + 16 * mt + 4 * g);
                *reinterpret_cast<uint2*>(dst) = make_uint2(lo, hi);
            }
        }
    }
    // (last: a store in front of the prenet's products would be counted by the waits in front of their operands)
    if (tid == 0) hot.proj_seq[tile * FUSED_GROUP + kp] = my_seq + 1u;
}

// ---------------------------------------------------------------------------
// The attention LSTM of the NEXT step inside the last kernel's launch (steps followed by another step of the same
// call): one of k_lstm_att_tall's units - 8 row tiles of one pool tile, one per wave - formed by a workgroup that has
// finished its gate pre-sums.  The prenet output of the frame just produced arrives from the tile's leader as words
// (p_x), the gate pre-sums from the workgroups that formed them (pre_x); every other operand is requested first.  Same
// products and sums in the same order as the kernel, so the state is the same bits.  `cur` is the running step's
// parity: the unit reads and writes what the next step's own kernel would (c_att, H_att into both activation halves,
// the query partials).  A wait that runs out freezes the tile's requests as the projection's do.
// ---------------------------------------------------------------------------
template <typename XT, int RG>
__device__ __forceinline__ void att_tail_unit(const DevPtrs& d, const ProjHot& hot, int cur, int tile, int rg0, unsigned stamp, float* lds)
{
    // RG row groups (rg0 .. rg0 + RG - 1) of 8 row tiles each: wave w owns row tile w of every one of them
    constexpr int KB = Frag<XT>::KB;
    constexpr int NK = K_ATT / KB;
    constexpr int NF = PRENET / KB;
    static_assert(NF == LSTM_WAVES && TALL_RT == LSTM_WAVES && PROJ_WAVES == LSTM_WAVES, "one fragment of p and one row tile per wave");
    static_assert((NF * 64 * 4 + RG * 4 * TALL_RT * 16 + 1) * 4 <= (int)sizeof(float) * PROJ_WAVES * PROJ_ROWS * 16, "fits the launch's LDS");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sl = tile * 16 + (lane & 15);
    const uint4* __restrict__ Wfrag = hot.Wa;

    uint4 a[RG][NF];
    float c_old[RG], wq[RG][TALL_RT];
    floatx4 bias4[RG];
    int unit[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const int rt = (rg0 + r) * TALL_RT + wave;
        unit[r] = rt * 4 + (lane >> 4);
#pragma unroll
        for (int f = 0; f < NF; ++f) a[r][f] = Wfrag[xfrag(NK, rt, f, lane)];
    }
    const int lv = hot.live[sl], dn = d.done[sl];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        c_old[r] = d.c_att[(size_t)sl * HID + unit[r]];
        bias4[r] = *reinterpret_cast<const floatx4*>(d.ba + unit[r] * 4);
#pragma unroll
        for (int s = 0; s < TALL_RT; ++s) wq[r][s] = d.Wq_epi[((size_t)((rg0 + r) * TALL_RT + s) * 8 + wave) * 64 + lane];
    }
    __builtin_amdgcn_sched_barrier(0);

    uint4 (*s_b)[64] = reinterpret_cast<uint4 (*)[64]>(lds);                                   // [NF][64]
    float (*s_h)[4 * TALL_RT][16] = reinterpret_cast<float (*)[4 * TALL_RT][16]>(lds + NF * 64 * 4);   // [RG][4 * TALL_RT][16]
    int* s_ok = reinterpret_cast<int*>(lds + NF * 64 * 4 + RG * 4 * TALL_RT * 16);
    if (threadIdx.x == 0) *s_ok = 1;
    __syncthreads();

    // The wave's row tiles of the pre-sums, long there; then its fragment of p: every lane polls its four words.
    unsigned long long wp[RG][4], wb[4] = {0ull, 0ull, 0ull, 0ull};
    bool all_in = false;
    for (int spin = 0; spin < d.wait_polls && !all_in; ++spin) {
        all_in = true;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const unsigned long long* qx = d.pre_x + (((size_t)tile * (HID / 4) + (rg0 + r) * TALL_RT + wave) * 4) * 64 + lane;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wp[r][i] = __hip_atomic_load(&qx[i * 64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                all_in = all_in && (unsigned)(wp[r][i] >> 32) == stamp;
            }
        }
    }
    const unsigned long long* px = d.p_x + (((size_t)tile * NF + wave) * 4) * 64 + lane;
    bool p_in = false;
    for (int spin = 0; spin < d.wait_polls && all_in && !p_in; ++spin) {
        p_in = true;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            wb[i] = __hip_atomic_load(&px[i * 64], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            p_in = p_in && ((unsigned)(wb[i] >> 32) & 0x7fffffffu) == stamp;
        }
    }
    if (!p_in) *s_ok = 0;
    s_b[wave][lane] = make_uint4((unsigned)wb[0], (unsigned)wb[1], (unsigned)wb[2], (unsigned)wb[3]);
    // (the words of lane l belong to column l % 16: the lane's own slot)
    const bool goes_on = p_in && (wb[0] >> 63) == 0;
    __syncthreads();
    if (*s_ok == 0) {
        if (threadIdx.x < 16 && lv && !dn) {
            d.done[sl] = 1;
            d.failed[sl] = 1;
            *d.fault = 1;
        }
        return;
    }
    const bool active = lv && !dn && goes_on;
    float c_new[RG];
    XT h_new[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const floatx4 pre4 = {__uint_as_float((unsigned)wp[r][0]), __uint_as_float((unsigned)wp[r][1]), __uint_as_float((unsigned)wp[r][2]),
                              __uint_as_float((unsigned)wp[r][3])};
        floatx4 g4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < NF; ++f) g4 = mfma_frag<XT>(a[r][f], s_b[f][lane], g4);
        g4 += bias4[r];
        g4 += pre4;
        const float gi = sigmoidf_(g4[0]), gf = sigmoidf_(g4[1]);
        const float gg = tanhf_(g4[2]), go = sigmoidf_(g4[3]);
        c_new[r] = gf * c_old[r] + gi * gg;
        h_new[r] = from_float<XT>(go * tanhf_(c_new[r]));
        s_h[r][4 * wave + (lane >> 4)][lane & 15] = active ? to_float(h_new[r]) : 0.f;
    }
    __syncthreads();
    // (every store after the last product: the wait the compiler places in front of a product's operands counts the
    // stores issued before it, and an acknowledged store is half a microsecond away)
    floatx4 part[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        part[r] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < TALL_RT; ++s)
            part[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(wq[r][s], s_h[r][4 * s + (lane >> 4)][lane & 15], part[r], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (active) {
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            // the next step's halves: its `cur` is this step's cur ^ 1
            d.c_att[(size_t)sl * HID + unit[r]] = c_new[r];
            reinterpret_cast<XT*>(d.xdec[cur ^ 1])[xoff<XT>(K_DEC / KB, sl, XD_HA + unit[r])] = h_new[r];
            reinterpret_cast<XT*>(d.xatt[cur])[xoff<XT>(NK, sl, XA_H + unit[r])] = h_new[r];
            *reinterpret_cast<floatx4*>(d.qpart + ((size_t)sl * QP_TALL + rg0 + r) * ATT + 16 * wave + 4 * (lane >> 4)) = part[r];
        }
    }
}

// G: workgroups per pool tile (fixed per pool: it sets the order in which the mel projection is summed)
template <typename XT, bool PRE, int G, bool FUSE = false>
__global__ __launch_bounds__(PROJ_THREADS) void k_proj(const uint4* Wa_first, const uint4* Wd_first, const void* xatt_nxt_first, const void* xdec_nxt_first,
                                                      const void* xdec_cur_first, const void* Wmel_first, const int* live_first, unsigned* proj_seq_first,
                                                      DevPtrs d, int cur, int n_tiles, int tail, int dec_rows)
{
    const ProjHot hot = {Wa_first, Wd_first, xatt_nxt_first, xdec_nxt_first, xdec_cur_first, Wmel_first, live_first, proj_seq_first};
    constexpr int BIG_FLOATS = PROJ_WAVES * PROJ_ROWS * 16 > LSTM_WAVES * LSTM_WAVES * 64 * 4 ? PROJ_WAVES * PROJ_ROWS * 16 : LSTM_WAVES * LSTM_WAVES * 64 * 4;
    __shared__ __attribute__((aligned(16))) float s_big[BIG_FLOATS];   // (the decoder LSTM's reduction buffer is the larger use: 64 KB)
    // row strides of 100 and 260 floats (an odd number of 16-byte pieces): the 16 columns of a
    // fragment read then fall into 16 different bank groups instead of one
    __shared__ __attribute__((aligned(16))) float s_mel[16][PROJ_MEL_LD];
    __shared__ int s_slot[16], s_t[16], s_cap[16], s_ok;
    const ProjShared sh = {s_big, s_mel, s_slot, s_t, s_cap, &s_ok};
    if (threadIdx.x == 0) s_ok = 1;

    // dec_rows != 0 (pools of more than 64 slots with two-byte weights, from 17 slots spanned): the decoder LSTM is the first
    // thing the launch's 256 workgroups do, each its k_lstm_stream tile, and the projection's workgroups take H_dec from the
    // words those tiles hand over (d.hdec_x) instead of a kernel boundary: a boundary costs the gap, the next kernel's
    // start-up and its first cold round trip, the hand-over one store-to-poll hop.
    if constexpr (PRE && !FUSE && sizeof(XT) == 2) {
        constexpr int KB = Frag<XT>::KB;
        XT* xdec_nxt = reinterpret_cast<XT*>(const_cast<void*>(xdec_nxt_first));
        const uint4* xdec_in = reinterpret_cast<const uint4*>(xdec_cur_first);
        if (dec_rows == 4)
            lstm_stream_unit<XT, K_DEC, 4, 4>(Wd_first, xdec_in, d.bd, d.c_dec, live_first, d.done, xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD,
                                              n_tiles, blockIdx.x, reinterpret_cast<StreamRed>(s_big), d.hdec_x, proj_seq_first, G);
        else if (dec_rows == 2)
            lstm_stream_unit<XT, K_DEC, 2, 4>(Wd_first, xdec_in, d.bd, d.c_dec, live_first, d.done, xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD,
                                              n_tiles, blockIdx.x, reinterpret_cast<StreamRed>(s_big), d.hdec_x, proj_seq_first, G);
        if (dec_rows) __syncthreads();
    }

    // tail: the launch also forms the next step's attention LSTM.  The words handed over for it carry a stamp: the number
    // of launches of this kernel so far, kept as a pair of counters.  A launch reads the one of its parity and workgroup 0
    // stores the next value into the other, which nobody reads before the next launch (the steps' parities alternate).
    unsigned tail_stamp = 0u;
    if constexpr (FUSE) {
        const unsigned c = d.wg_seq[cur];
        if (blockIdx.x == 0 && threadIdx.x == 0) d.wg_seq[cur ^ 1] = c + 1u;
        if (tail) tail_stamp = c % 0x7ffffffeu + 1u;               // never zero, bit 31 free
    }

    if constexpr (PRE) {
        // The launch has 256 workgroups, one per CU; workgroup b runs on XCD b % 8.  XCD 0 holds the projection's own
        // workgroups (b = 8 * (G * tile + part)) and is otherwise left idle: beside workgroups that stream at full
        // rate, the projection's loads took a quarter longer.  The other seven XCDs form the next step's gate pre-sums:
        // XCD x takes row tiles 256 (x - 1) / 7 .. 256 x / 7 of both matrices (every weight is fetched from HBM once),
        // its 32 workgroups split into groups by pool tiles and a group's workgroups share the XCD's 36 or 37 row tiles
        // evenly.  Up to four tiles: one or two groups (two from three tiles on: 32 x 32 is the shape that moves the
        // fewest bytes through a CU), two or three row tiles each (one or two without the split).  Above: groups of at
        // most four tiles, two to five row tiles each, the tiles walked one at a time.
        const int x = blockIdx.x & 7, i = blockIdx.x >> 3;
        static_assert(!FUSE || PRE, "the fused form is a form of the 256-workgroup launch");
        if constexpr (FUSE) {
            // Every workgroup forms its piece of the decoder LSTM first (the projection's own weave it into their start).
            // The pre-sum workgroups request nothing of their own before the piece is done: with their first chunks
            // on the way beside the pieces' operands, the pieces - which the projection waits for - finished 1.8 us later.
            if (x != 0 || i >= n_tiles * FUSED_GROUP) {
                DecUnit<XT> dec;
                dec.issue(d, hot, blockIdx.x, n_tiles);
                __builtin_amdgcn_sched_barrier(0);
                dec.finish(d, hot, reinterpret_cast<DecRed>(s_big));
            }
        }
        if (x != 0) {
            static_assert(sizeof(floatx4) * LSTM_WAVES * PG_R * PG_T * 64 <= sizeof(s_big), "the reduction buffer aliases the partial sums");
            static_assert(sizeof(floatx4) * LSTM_WAVES * PG_WALK_R * 64 <= sizeof(s_big), "the reduction buffer aliases the partial sums");
            static_assert(PROJ_WAVES == LSTM_WAVES, "the pre-sums split K over eight waves");
            const int rx0 = (HID / 4) * (x - 1) / 7, rx1 = (HID / 4) * x / 7;
            if (n_tiles <= 4) {
                int k = i, Mc = 32, t0 = 0, nt = n_tiles;
                if (n_tiles > 2) {
                    const int per = (n_tiles + 1) / 2;
                    Mc = 16;
                    if (k < 16) nt = per;
                    else { k -= 16; t0 = per; nt = n_tiles - per; }
                }
                const int lo = rx0 + (rx1 - rx0) * k / Mc, hi = rx0 + (rx1 - rx0) * (k + 1) / Mc;
                // (fused: the decoder LSTM's sums over H_dec are formed beside the attention kernel of the next step)
                if constexpr (FUSE) {
                    gate_presums_sel<XT, false>(d, hot, lo, hi - lo, t0, nt, reinterpret_cast<PresumRed>(s_big), tail_stamp);
                    // the next step's attention LSTM: unit c of 32 row groups x pool tiles, dealt over the seven XCDs
                    const int c = i * 7 + (x - 1);
                    constexpr int RG = TAIL_RG, per = QP_TALL / RG;
                    if (tail_stamp != 0u && c < per * n_tiles) att_tail_unit<XT, RG>(d, hot, cur, c / per, c % per * RG, tail_stamp, s_big);
                } else gate_presums<XT>(d, hot, lo, hi - lo, t0, nt, reinterpret_cast<PresumRed>(s_big));
            } else {
                const int CG = (n_tiles + 3) / 4, Mc = 32 / CG;          // 2, 3 or 4 groups of 16, 10 or 8 workgroups
                const int cg = i / Mc, k = i - cg * Mc;
                if (cg >= CG) return;                                     // 32 = 3 * 10 + 2: two workgroups stay idle
                const int per = (n_tiles + CG - 1) / CG, t0 = cg * per;
                const int nt = min(per, n_tiles - t0);
                const int lo = rx0 + (rx1 - rx0) * k / Mc, hi = rx0 + (rx1 - rx0) * (k + 1) / Mc;
                if (nt > 0) gate_presums_walk<XT>(d, hot, lo, hi - lo, t0, nt, reinterpret_cast<WalkRed>(s_big));
            }
            return;
        }
        if constexpr (FUSE) {
            static_assert(!FUSE || G == PROJ_GROUP_K, "the workers split K as the plain form's workgroups do");
            if (i < n_tiles * FUSED_GROUP) proj_tile_fused<XT>(d, hot, cur, i / FUSED_GROUP, i % FUSED_GROUP, sh, n_tiles, tail_stamp);
            return;
        }
        if (i >= n_tiles * G) return;
        if (i % G == 0) proj_tile<XT, G, true>(d, hot, cur, i / G, 0, sh, dec_rows != 0);
        else proj_tile<XT, G, false>(d, hot, cur, i / G, i % G, sh, dec_rows != 0);
    } else {
        // without pre-sums: the same workgroups per tile, wherever they land (n_tiles * G <= 96 workgroups)
        const int i = blockIdx.x;
        if (i % G == 0) proj_tile<XT, G, true>(d, hot, cur, i / G, 0, sh);
        else proj_tile<XT, G, false>(d, hot, cur, i / G, i % G, sh);
    }
}

// element (row, k) of a matrix stored in MFMA A-fragment order with NK fragments per row tile
template <typename XT>
__device__ __forceinline__ float frag_elem(const void* base, int NK, int row, int k)
{
    return to_float(reinterpret_cast<const XT*>(base)[xoff<XT>(NK, row, k)]);
}

// p = Pre(m_last) of one slot into both activation buffers (after a state overwrite; not on the step path)
template <typename XT>
__global__ __launch_bounds__(256) void k_prenet_slot(DevPtrs d, int slot)
{
    constexpr int KB = Frag<XT>::KB;
    __shared__ float s_mel[N_MEL];
    __shared__ float s_hid[PRENET];
    const int o = threadIdx.x;
    if (o < N_MEL) s_mel[o] = d.m_last[(size_t)slot * N_MEL + o];
    __syncthreads();
    float acc = 0.f;
    for (int k = 0; k < N_MEL; ++k) acc += frag_elem<XT>(d.Wp1, PrenetK1<XT>::value / KB, o, k) * to_float(from_float<XT>(s_mel[k]));
    s_hid[o] = fmaxf(acc, 0.f);
    __syncthreads();
    acc = 0.f;
    for (int k = 0; k < PRENET; ++k) acc += frag_elem<XT>(d.Wp2, PRENET / KB, o, k) * to_float(from_float<XT>(s_hid[k]));
    const XT p = from_float<XT>(fmaxf(acc, 0.f));
    for (int b = 0; b < 2; ++b) reinterpret_cast<XT*>(d.xatt[b])[xoff<XT>(K_ATT / KB, slot, XA_P + o)] = p;
}

// ---------------------------------------------------------------------------
// Pool bookkeeping on the device
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(MAX_POOL) void k_set_live(LiveArgs a, int* live)
{
    const int tid = threadIdx.x;
    live[tid] = (a.bits[tid >> 5] >> (tid & 31)) & 1u;
}

// a joining request starts from all-zero state (one workgroup of 256 threads)
template <typename XT>
__device__ __forceinline__ void slot_init(const DevPtrs& d, int slot, int L, int n_steps, int tid)
{
    constexpr int KB = Frag<XT>::KB;
    const XT z = from_float<XT>(0.f);
    for (int b = 0; b < 2; ++b) {
        XT* xa = reinterpret_cast<XT*>(d.xatt[b]);
        XT* xd = reinterpret_cast<XT*>(d.xdec[b]);
        for (int k = tid; k < K_ATT; k += 256) xa[xoff<XT>(K_ATT / KB, slot, k)] = z;
        for (int k = tid; k < K_DEC; k += 256) xd[xoff<XT>(K_DEC / KB, slot, k)] = z;
        for (int i = tid; i < d.max_enc_len; i += 256) {
            d.w_last[b][(size_t)slot * d.max_enc_len + i] = 0.f;
            d.w_acc[b][(size_t)slot * d.max_enc_len + i] = 0.f;
        }
    }
    for (int i = tid; i < HID; i += 256) {
        d.c_att[(size_t)slot * HID + i] = 0.f;
        d.c_dec[(size_t)slot * HID + i] = 0.f;
    }
    if (tid < N_MEL) d.m_last[(size_t)slot * N_MEL + tid] = 0.f;
    // gate pre-sums of a zero state: this slot's column of every row tile (thread = row tile)
    if (d.pre_att) {
        static_assert(HID / 4 == 256, "one thread per row tile");
        const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
        floatx4* pa = reinterpret_cast<floatx4*>(d.pre_att) + ((size_t)(slot >> 4) * (HID / 4) + tid) * 64 + (slot & 15);
        floatx4* pd = reinterpret_cast<floatx4*>(d.pre_dec) + ((size_t)(slot >> 4) * (HID / 4) + tid) * 64 + (slot & 15);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            pa[16 * g] = z4;
            if (d.pre_dec) pd[16 * g] = z4;
        }
    }
    if (tid == 0) {
        d.L[slot] = L;
        d.t[slot] = 0;
        d.n_steps[slot] = n_steps;
        d.done[slot] = 0;
        d.failed[slot] = 0;
    }
}

// n 16-byte (or 4-byte) pieces from src to dst, four strided pieces per thread in flight
template <typename V>
__device__ __forceinline__ void copy_strided(V* __restrict__ dst, const V* __restrict__ src, int n, int tid, int nth)
{
    for (int i0 = tid; i0 < n; i0 += 4 * nth) {
        V v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = src[min(i0 + u * nth, n - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u * nth < n) dst[i0 + u * nth] = v[u];
    }
}

// Running requests move from their slots to free ones (the host packs the pool into fewer slots when that shrinks
// what the step kernels must span): everything the step carries per slot.  blockIdx.y = which move; no slot is both
// a source and a destination within one launch.  The step's results do not depend on the slot a request sits in.
// A thread first requests all its pieces of the small arrays, then stores them (a copy loop per array would be one
// round trip to memory after the other).
template <typename XT, typename MT>
__global__ __launch_bounds__(256) void k_move_slots(DevPtrs d, MoveArgs mv)
{
    constexpr int KB = Frag<XT>::KB;
    const int from = mv.from[blockIdx.y], to = mv.to[blockIdx.y], L = mv.L[blockIdx.y], t = mv.t[blockIdx.y];
    const int tid = blockIdx.x * 256 + threadIdx.x, nth = MOVE_WGS * 256;
    static_assert(MOVE_WGS * 256 >= K_DEC && MOVE_WGS * 256 >= MAX_ENC_LEN && MOVE_WGS * 256 >= HID,
                  "one piece of each small array per thread");
    const size_t ML = d.max_enc_len;
    // ---- small arrays: loads (clamped, unconditional) ...
    XT xa[2], xd[2];
    float wl[2], wa[2];
    const int ka = min(tid, K_ATT - 1), kd = min(tid, K_DEC - 1), il = min(tid, L - 1);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        xa[b] = reinterpret_cast<const XT*>(d.xatt[b])[xoff<XT>(K_ATT / KB, from, ka)];
        xd[b] = reinterpret_cast<const XT*>(d.xdec[b])[xoff<XT>(K_DEC / KB, from, kd)];
        wl[b] = d.w_last[b][from * ML + il];
        wa[b] = d.w_acc[b][from * ML + il];
    }
    const int ih = min(tid, HID - 1), im = min(tid, N_MEL - 1);
    const float ca = d.c_att[(size_t)from * HID + ih], cd = d.c_dec[(size_t)from * HID + ih];
    const float ml = d.m_last[(size_t)from * N_MEL + im];
    // this slot's column of the gate pre-sums (thread = row tile)
    const bool pre = d.pre_att && tid < HID / 4, pre_d = pre && d.pre_dec;
    const size_t o_from = ((size_t)(from >> 4) * (HID / 4) + min(tid, HID / 4 - 1)) * 64 + (from & 15);
    const size_t o_to = ((size_t)(to >> 4) * (HID / 4) + min(tid, HID / 4 - 1)) * 64 + (to & 15);
    floatx4* pa = reinterpret_cast<floatx4*>(d.pre_att);
    floatx4* pdc = reinterpret_cast<floatx4*>(d.pre_dec);
    floatx4 va[4], vd[4];
    if (pre) {
#pragma unroll
        for (int g = 0; g < 4; ++g) va[g] = pa[o_from + 16 * g];
    }
    if (pre_d) {
#pragma unroll
        for (int g = 0; g < 4; ++g) vd[g] = pdc[o_from + 16 * g];
    }
    const int sL = d.L[from], st = d.t[from], sn = d.n_steps[from], sd = d.done[from], sf = d.failed[from];
    // ---- ... then stores
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        if (tid < K_ATT) reinterpret_cast<XT*>(d.xatt[b])[xoff<XT>(K_ATT / KB, to, tid)] = xa[b];
        if (tid < K_DEC) reinterpret_cast<XT*>(d.xdec[b])[xoff<XT>(K_DEC / KB, to, tid)] = xd[b];
        if (tid < L) {
            d.w_last[b][to * ML + tid] = wl[b];
            d.w_acc[b][to * ML + tid] = wa[b];
        }
    }
    if (tid < HID) {
        d.c_att[(size_t)to * HID + tid] = ca;
        d.c_dec[(size_t)to * HID + tid] = cd;
    }
    if (tid < N_MEL) d.m_last[(size_t)to * N_MEL + tid] = ml;
    if (pre) {
#pragma unroll
        for (int g = 0; g < 4; ++g) pa[o_to + 16 * g] = va[g];
    }
    if (pre_d) {
#pragma unroll
        for (int g = 0; g < 4; ++g) pdc[o_to + 16 * g] = vd[g];
    }
    if (tid == 0) {
        d.L[to] = sL;
        d.t[to] = st;
        d.n_steps[to] = sn;
        d.done[to] = sd;
        d.failed[to] = sf;
        d.failed[from] = 0;
    }
    // ---- encoder memory and processed memory, 16 bytes at a time (rows are whole multiples of that), and the
    // frames produced so far (some may not have been handed out yet)
    copy_strided(reinterpret_cast<uint4*>(reinterpret_cast<MT*>(d.Fmem) + (size_t)to * ML * ENC),
                 reinterpret_cast<const uint4*>(reinterpret_cast<const MT*>(d.Fmem) + (size_t)from * ML * ENC),
                 L * ENC * (int)sizeof(MT) / 16, tid, nth);
    copy_strided(reinterpret_cast<uint4*>(reinterpret_cast<MT*>(d.PM) + (size_t)to * ML * ATT),
                 reinterpret_cast<const uint4*>(reinterpret_cast<const MT*>(d.PM) + (size_t)from * ML * ATT),
                 L * ATT * (int)sizeof(MT) / 16, tid, nth);
    if (t > 0) {
        copy_strided(reinterpret_cast<float4*>(d.mel_ring + (size_t)to * d.max_steps * N_MEL),
                     reinterpret_cast<const float4*>(d.mel_ring + (size_t)from * d.max_steps * N_MEL), t * (N_MEL / 4), tid, nth);
        copy_strided(d.stop_ring + (size_t)to * d.max_steps, d.stop_ring + (size_t)from * d.max_steps, t, tid, nth);
    }
}

// Requests join (blockIdx.y = which): workgroup 0 of a request zeroes its state, workgroup 1 + b takes encoder
// positions 8 b .. 8 b + 7: stores the rows in the memory's type and forms PM[j] = W_mem F[j] in fp32.  A thread
// takes four attention dimensions and one eighth of K for all eight positions (a 16-byte piece of W_mem^T per k,
// pulled once for eight positions); the eight partial sums of an entry are added in the order of K.
template <typename XT, typename MT>
__global__ __launch_bounds__(256) void k_join(DevPtrs d, JoinArgs ja)
{
    const int r = blockIdx.y, tid = threadIdx.x;
    const int slot = ja.slot[r], L = ja.L[r];
    if (blockIdx.x == 0) {
        slot_init<XT>(d, slot, L, ja.n_steps[r], tid);
        return;
    }
    const int j0 = (blockIdx.x - 1) * JOIN_POS;
    if (j0 >= L) return;
    const int np = min(JOIN_POS, L - j0);
    const float* __restrict__ F = ja.F[r] + (size_t)j0 * ENC;
    constexpr int KG = 8, KPG = ENC / KG;         // K groups, k per group
    static_assert(256 == KG * (ATT / 4), "a thread = (K group, four attention dimensions)");
    __shared__ float s_f[JOIN_POS][ENC];
    __shared__ float4 s_p[KG][JOIN_POS][ATT / 4];
    MT* Fm = reinterpret_cast<MT*>(d.Fmem) + ((size_t)slot * d.max_enc_len + j0) * ENC;
    // all of a thread's loads are requested before the first is used (clamped, not branched around)
    constexpr int FPT = JOIN_POS * ENC / 256;
    float fx[FPT];
#pragma unroll
    for (int u = 0; u < FPT; ++u) fx[u] = F[min(tid + u * 256, np * ENC - 1)];
#pragma unroll
    for (int u = 0; u < FPT; ++u) {
        const int i = tid + u * 256;
        const bool in = i < np * ENC;
        s_f[i / ENC][i % ENC] = in ? fx[u] : 0.f;
        if (in) Fm[i] = from_float<MT>(fx[u]);
    }
    __syncthreads();
    const int a4 = tid & (ATT / 4 - 1), kg = tid / (ATT / 4);
    const float4* __restrict__ W4 = reinterpret_cast<const float4*>(d.WmemT) + (size_t)kg * KPG * (ATT / 4) + a4;
    float4 acc[JOIN_POS];
#pragma unroll
    for (int q = 0; q < JOIN_POS; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
    for (int k = 0; k < KPG; ++k) {
        const float4 w = W4[(size_t)k * (ATT / 4)];
#pragma unroll
        for (int q = 0; q < JOIN_POS; ++q) {
            const float f = s_f[q][kg * KPG + k];
            acc[q].x += w.x * f;
            acc[q].y += w.y * f;
            acc[q].z += w.z * f;
            acc[q].w += w.w * f;
        }
    }
#pragma unroll
    for (int q = 0; q < JOIN_POS; ++q) s_p[kg][q][a4] = acc[q];
    __syncthreads();
    // thread = (position q, attention dimensions 4 a4 .. 4 a4 + 3)
    const int q = tid / (ATT / 4);
    float4 t = s_p[0][q][a4];
#pragma unroll
    for (int g = 1; g < KG; ++g) {
        const float4 u = s_p[g][q][a4];
        t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    if (q < np) {
        MT* pm = reinterpret_cast<MT*>(d.PM) + ((size_t)slot * d.max_enc_len + j0 + q) * ATT + 4 * a4;
        pm[0] = from_float<MT>(t.x);
        pm[1] = from_float<MT>(t.y);
        pm[2] = from_float<MT>(t.z);
        pm[3] = from_float<MT>(t.w);
    }
}

// gather / scatter of one slot's piece of a slot-tiled activation array (state access, not on the step path)
template <typename XT>
__global__ __launch_bounds__(256) void k_x_get(const XT* X, int NK, int slot, int off, int n, float* out)
{
    for (int k = threadIdx.x; k < n; k += 256) out[k] = to_float(X[xoff<XT>(NK, slot, off + k)]);
}
template <typename XT>
__global__ __launch_bounds__(256) void k_x_set(XT* X, int NK, int slot, int off, int n, const float* in)
{
    for (int k = threadIdx.x; k < n; k += 256) X[xoff<XT>(NK, slot, off + k)] = from_float<XT>(in[k]);
}

// ---------------------------------------------------------------------------
// launch wrappers
// ---------------------------------------------------------------------------
// PM: 0 = no gate pre-sums, 1 = the attention LSTM's only (pools of more than four tiles), 2 = both LSTMs'
template <typename XT, typename MT, int PM>
static hipError_t step_typed(const DevPtrs& d, int n_req, int n_tiles, int lsa_split, int rows, int proj_group, int att_lead, int att_tail, int cur,
                             hipStream_t s, hipEvent_t* ev)
{
    constexpr int KB = Frag<XT>::KB;
    auto mark = [&](int i) { if (ev) (void)hipEventRecord(ev[i], s); };
    const uint4* xatt_cur = reinterpret_cast<const uint4*>(d.xatt[cur]);
    XT* xatt_nxt = reinterpret_cast<XT*>(d.xatt[cur ^ 1]);
    XT* xdec_cur = reinterpret_cast<XT*>(d.xdec[cur]);
    XT* xdec_nxt = reinterpret_cast<XT*>(d.xdec[cur ^ 1]);
    mark(0);
    constexpr bool PRE = PM != 0, PRE_DEC = PM == 2;
    constexpr bool HAS_WIDE = sizeof(XT) == 2;     // the fp32 fragments of several row tiles do not fit the register file
    if (!HAS_WIDE) rows = 1;
    // pre-sums beyond four tiles need the several-row-tile kernels (bf16)
    if (PRE && !HAS_WIDE && n_tiles > PRESUM_SMALL_TILES) return hipErrorInvalidValue;
    if (PRE && n_tiles * proj_group > 32) return hipErrorInvalidValue;   // the projection's workgroups must fit XCD 0
    if (PRE_DEC && rows > 2) return hipErrorInvalidValue;                // both pre-sums: at most four tiles
    const dim3 lg(HID / 4), lb(LSTM_WAVES * 64);
    // H_att(t): consumed by this step's decoder LSTM / attention and by the next step's attention LSTM.
    // With pre-sums: the tall kernel, which also hands the query over as partial products.  Without (fp32 pools of
    // more than four tiles): one row tile per workgroup, all of K.
    constexpr bool CO = PRE_DEC && sizeof(XT) == 2 && sizeof(MT) == 2;   // (the attention kernel for fp32 memory needs more than 128 registers)
    // only the fused last kernel can form the next step's attention LSTM, and only for a step that then runs without its own
    if ((att_tail || !att_lead) && !(CO && d.p_x && d.pre_x && d.wg_seq)) return hipErrorInvalidValue;
    if (!att_lead) {
        // formed by the step before, inside its last launch
    } else if constexpr (PRE) {
        if (n_tiles > 8)
            hipLaunchKernelGGL((k_lstm_att_tall<XT, 2>), dim3(QP_TALL * ((n_tiles + 1) / 2)), lb, 0, s, d.Wa, xatt_cur, d.ba, d.c_att, d.live, d.done,
                               reinterpret_cast<const floatx4*>(d.pre_att), d.Wq_epi, xdec_cur, K_DEC / KB, XD_HA, xatt_nxt, K_ATT / KB, XA_H, d.qpart, n_tiles);
        else
            hipLaunchKernelGGL((k_lstm_att_tall<XT, 1>), dim3(QP_TALL * n_tiles), lb, 0, s, d.Wa, xatt_cur, d.ba, d.c_att, d.live, d.done,
                               reinterpret_cast<const floatx4*>(d.pre_att), d.Wq_epi, xdec_cur, K_DEC / KB, XD_HA, xatt_nxt, K_ATT / KB, XA_H, d.qpart, n_tiles);
    } else {
        hipLaunchKernelGGL((k_lstm<XT, K_ATT, false>), lg, lb, 0, s, d.Wa, xatt_cur, d.ba, d.c_att, d.live, d.done, (const floatx4*)nullptr,
                           (const floatx4*)nullptr, xdec_cur, K_DEC / KB, XD_HA, xatt_nxt, K_ATT / KB, XA_H, n_tiles);
    }
    mark(1);
    const int n_pad = (n_req + 7) / 8 * 8;      // slots are dealt to the XCDs in eights
#define LSA_ARGS d.L, d.live, d.done, d.step_seq, d.qpart, d.w_last[cur], d.w_acc[cur], d.PM, d, cur, n_req
    // two-byte pools with both pre-sums: the decoder LSTM's sums over H_att ride in this launch
    if (CO != (d.pre_dec_b != nullptr) || (CO && !d.hdec_x)) return hipErrorInvalidValue;
    const int n_co = CO ? DEC_HATT_WGS * (n_tiles > 1 ? 2 : 1) : 0;
    if (lsa_split == 4) hipLaunchKernelGGL((k_lsa<XT, MT, 4, PRE, CO>), dim3(n_pad * 4 + n_co), dim3(LSA_THREADS), 0, s, LSA_ARGS);
    else if (CO) return hipErrorInvalidValue;     // such pools span at most 64 slots: four workgroups per slot
    else if (lsa_split == 2) hipLaunchKernelGGL((k_lsa<XT, MT, 2, PRE>), dim3(n_pad * 2), dim3(LSA_THREADS), 0, s, LSA_ARGS);
    else hipLaunchKernelGGL((k_lsa<XT, MT, 1, PRE>), dim3(n_pad), dim3(LSA_THREADS), 0, s, LSA_ARGS);
#undef LSA_ARGS
    mark(2);
    // H_dec(t): consumed by this step's projection and the next step's decoder LSTM (same buffer)
    const uint4* xdec_in = reinterpret_cast<const uint4*>(d.xdec[cur]);
    const floatx4* pre_dec = reinterpret_cast<const floatx4*>(d.pre_dec);
    const floatx4* pre_dec_b = reinterpret_cast<const floatx4*>(d.pre_dec_b);
    // pools of more than 64 slots with two-byte weights: the decoder LSTM's stream tiles are the first part of the last launch
    const int dec_rows = (PM == 1 && HAS_WIDE && d.hdec_x && (rows == 4 || rows == 2)) ? rows : 0;
    if (dec_rows == 2 && n_tiles > 8) return hipErrorInvalidValue;          // two groups of at most four pool tiles
    if constexpr (CO) {
        // the decoder LSTM is part of the last kernel's launch (below)
        if (proj_group != 6) return hipErrorInvalidValue;
    } else if (dec_rows) {
        // (below)
    } else if (rows == 4) {
        if constexpr (HAS_WIDE && !PRE_DEC)
            hipLaunchKernelGGL((k_lstm_stream<XT, K_DEC, 4, 4>), lg, lb, 0, s, d.Wd, xdec_in, d.bd, d.c_dec, d.live, d.done,
                               xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD, n_tiles);
    } else if (rows == 2) {
        if constexpr (HAS_WIDE && !PRE_DEC) {
            if (n_tiles > 8) return hipErrorInvalidValue;         // two groups of at most four pool tiles
            hipLaunchKernelGGL((k_lstm_stream<XT, K_DEC, 2, 4>), lg, lb, 0, s, d.Wd, xdec_in, d.bd, d.c_dec, d.live, d.done,
                               xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD, n_tiles);
        } else if constexpr (HAS_WIDE)
            hipLaunchKernelGGL((k_lstm_rc<XT, K_DEC, 2, PRE_DEC, CO>), lg, lb, 0, s, d.Wd, xdec_in, d.bd, d.c_dec, d.live, d.done, pre_dec, pre_dec_b,
                               xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD, n_tiles);
    } else
        hipLaunchKernelGGL((k_lstm<XT, K_DEC, PRE_DEC, CO>), lg, lb, 0, s, d.Wd, xdec_in, d.bd, d.c_dec, d.live, d.done, pre_dec, pre_dec_b,
                           xdec_nxt, K_DEC / KB, XD_HD, xdec_nxt, K_DEC / KB, XD_HD, n_tiles);
    mark(3);
    // with pre-sums the projection's launch fills the chip: XCD 0 runs the projection, the rest form the pre-sums
    const dim3 pg(PRE ? 256 : n_tiles * proj_group), pb(PROJ_THREADS);
#define PROJ_ARGS d.Wa, d.Wd, (const void*)d.xatt[cur ^ 1], (const void*)d.xdec[cur ^ 1], (const void*)d.xdec[cur], d.Wmel, (const int*)d.live, d.proj_seq, d, cur, n_tiles, att_tail, dec_rows
    if (proj_group == 6) hipLaunchKernelGGL((k_proj<XT, PRE, 6, CO>), pg, pb, 0, s, PROJ_ARGS);
    else if (proj_group == 3) hipLaunchKernelGGL((k_proj<XT, PRE, 3>), pg, pb, 0, s, PROJ_ARGS);
    else if (proj_group == 2) hipLaunchKernelGGL((k_proj<XT, PRE, 2>), pg, pb, 0, s, PROJ_ARGS);
#undef PROJ_ARGS
    else return hipErrorInvalidValue;
    mark(4);
    return hipGetLastError();
}

hipError_t launch_step(const DevPtrs& d, const StepLaunch& cfg, int cur, hipStream_t s, hipEvent_t* ev)
{
    if (cfg.n_blocks < 1 || cfg.n_tiles < 1) return hipSuccess;
    if (cfg.pre_gates) {
        if (cfg.n_tiles > MAX_TILES || !d.pre_att || !d.qpart || (cfg.pre_gates == 2) != (d.pre_dec != nullptr)) return hipErrorInvalidValue;
        if (cfg.pre_gates == 1) {
            if (cfg.wdtype == 1 && cfg.mdtype == 1) return step_typed<h16_t, bf16_t, 1>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
            if (cfg.wdtype == 1 && cfg.mdtype == 0) return step_typed<h16_t, float, 1>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
            return hipErrorInvalidValue;
        }
        if (cfg.n_tiles > PRESUM_SMALL_TILES) return hipErrorInvalidValue;
        if (cfg.wdtype == 0 && cfg.mdtype == 0) return step_typed<float, float, 2>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
        if (cfg.wdtype == 1 && cfg.mdtype == 1) return step_typed<h16_t, bf16_t, 2>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
        if (cfg.wdtype == 1 && cfg.mdtype == 0) return step_typed<h16_t, float, 2>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
        return hipErrorInvalidValue;
    }
    // without pre-sums: fp32 pools of more than four tiles (the fp32 mode is the parity vehicle)
    if (cfg.wdtype == 0 && cfg.mdtype == 0) return step_typed<float, float, 0>(d, cfg.n_blocks, cfg.n_tiles, cfg.lsa_split, cfg.lstm_rows, cfg.proj_group, cfg.att_lead, cfg.att_tail, cur, s, ev);
    return hipErrorInvalidValue;
}

hipError_t launch_set_live(const DevPtrs& d, const LiveArgs& args, hipStream_t s)
{
    hipLaunchKernelGGL(k_set_live, dim3(1), dim3(MAX_POOL), 0, s, args, d.live);
    return hipGetLastError();
}

hipError_t launch_move_slots(const DevPtrs& d, int wdtype, int mdtype, const MoveArgs& mv, int n, hipStream_t s)
{
    if (n < 1 || n > MOVE_BATCH) return hipErrorInvalidValue;
    for (int i = 0; i < n; ++i)
        if (mv.from[i] == mv.to[i] || mv.L[i] < 1 || mv.L[i] > d.max_enc_len || mv.t[i] < 0 || mv.t[i] > d.max_steps)
            return hipErrorInvalidValue;
    const dim3 g(MOVE_WGS, n), b(256);
    static_assert(MOVE_WGS * 256 >= HID / 4, "one thread per row tile of the pre-sums");
    if (wdtype == 0 && mdtype == 0) hipLaunchKernelGGL((k_move_slots<float, float>), g, b, 0, s, d, mv);
    else if (wdtype == 1 && mdtype == 1) hipLaunchKernelGGL((k_move_slots<h16_t, bf16_t>), g, b, 0, s, d, mv);
    else if (wdtype == 1 && mdtype == 0) hipLaunchKernelGGL((k_move_slots<h16_t, float>), g, b, 0, s, d, mv);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_join(const DevPtrs& d, int wdtype, int mdtype, const JoinArgs& ja, int n, hipStream_t s)
{
    if (n < 1 || n > JOIN_BATCH) return hipErrorInvalidValue;
    int Lmax = 0;
    for (int i = 0; i < n; ++i) {
        if (!ja.F[i] || ja.L[i] < 1 || ja.L[i] > d.max_enc_len || ja.slot[i] < 0 || ja.slot[i] >= MAX_POOL) return hipErrorInvalidValue;
        Lmax = ja.L[i] > Lmax ? ja.L[i] : Lmax;
    }
    const dim3 g(1 + (Lmax + JOIN_POS - 1) / JOIN_POS, n), b(256);
    if (wdtype == 0 && mdtype == 0) hipLaunchKernelGGL((k_join<float, float>), g, b, 0, s, d, ja);
    else if (wdtype == 1 && mdtype == 1) hipLaunchKernelGGL((k_join<h16_t, bf16_t>), g, b, 0, s, d, ja);
    else if (wdtype == 1 && mdtype == 0) hipLaunchKernelGGL((k_join<h16_t, float>), g, b, 0, s, d, ja);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_presum_tile(const DevPtrs& d, int wdtype, int tile, int nxt, hipStream_t s)
{
    if (!d.pre_att || tile < 0 || tile >= MAX_TILES) return hipErrorInvalidValue;
    if (wdtype == 0) hipLaunchKernelGGL((k_presum_tile<float>), dim3(HID / 4), dim3(LSTM_WAVES * 64), 0, s, d, nxt, tile);
    else hipLaunchKernelGGL((k_presum_tile<h16_t>), dim3(HID / 4), dim3(LSTM_WAVES * 64), 0, s, d, nxt, tile);
    return hipGetLastError();
}

hipError_t launch_prenet_slot(const DevPtrs& d, int wdtype, int slot, hipStream_t s)
{
    if (wdtype == 0) hipLaunchKernelGGL((k_prenet_slot<float>), dim3(1), dim3(256), 0, s, d, slot);
    else hipLaunchKernelGGL((k_prenet_slot<h16_t>), dim3(1), dim3(256), 0, s, d, slot);
    return hipGetLastError();
}

hipError_t launch_x_get(int wdtype, const void* X, int K, int slot, int off, int n, float* out, hipStream_t s)
{
    if (wdtype == 0)
        hipLaunchKernelGGL((k_x_get<float>), dim3(1), dim3(256), 0, s, reinterpret_cast<const float*>(X), K / Frag<float>::KB, slot, off, n, out);
    else
        hipLaunchKernelGGL((k_x_get<h16_t>), dim3(1), dim3(256), 0, s, reinterpret_cast<const h16_t*>(X), K / Frag<h16_t>::KB, slot, off, n, out);
    return hipGetLastError();
}

hipError_t launch_x_set(int wdtype, void* X, int K, int slot, int off, int n, const float* in, hipStream_t s)
{
    if (wdtype == 0)
        hipLaunchKernelGGL((k_x_set<float>), dim3(1), dim3(256), 0, s, reinterpret_cast<float*>(X), K / Frag<float>::KB, slot, off, n, in);
    else
        hipLaunchKernelGGL((k_x_set<h16_t>), dim3(1), dim3(256), 0, s, reinterpret_cast<h16_t*>(X), K / Frag<h16_t>::KB, slot, off, n, in);
    return hipGetLastError();
}

}  // namespace tts
