// Device helpers shared by the step kernels and the PostNet kernels: bf16 / fp16 <-> fp32, fast sigmoid / tanh,
// the MFMA fragment geometry and the fragment-order activation layout.  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tts {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };
// IEEE half precision: the two-byte MFMA operand type.  Weights given as bfloat16 values (8 significant bits) are exact
// in it (11 significant bits) down to 2^-14, and activations rounded to it carry 2^-11 relative error where bfloat16
// would carry 2^-8; v_mfma_f32_16x16x32_f16 runs at the rate of its bf16 twin.
struct h16_t { uint16_t bits; };
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float to_float(h16_t x) { return (float)__builtin_bit_cast(_Float16, x.bits); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32, two values
// per instruction) instead of integer arithmetic on the bit pattern
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f2bf_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// two floats -> one 32-bit word of two T (round to nearest even), `lo` in the low half
template <typename T> __device__ __forceinline__ uint32_t pack2(float lo, float hi);
template <> __device__ __forceinline__ uint32_t pack2<bf16_t>(float lo, float hi) { return pack_bf16x2(lo, hi); }
template <> __device__ __forceinline__ uint32_t pack2<h16_t>(float lo, float hi)
{
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, halfx2));
}
template <typename T> __device__ __forceinline__ T from_float(float x);
template <> __device__ __forceinline__ float from_float<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float x) { bf16_t r; r.bits = f2bf_bits(x); return r; }
template <> __device__ __forceinline__ h16_t from_float<h16_t>(float x) { h16_t r; r.bits = __builtin_bit_cast(uint16_t, (_Float16)x); return r; }

__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
// 1 - 2/(1+e^{2x}) with the hardware reciprocal (1 ulp): absolute error ~1e-7, saturates cleanly at +-1
__device__ __forceinline__ float tanhf_(float x) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x)); }

// (1 - tanh(x)) / 2 = 1 / (1 + e^{2x})
__device__ __forceinline__ float half_one_minus_tanh(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * x));
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// 16 bytes of T -> floats (4 for fp32, 8 for bf16)
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void unpack(const uint4& u, float* f)
    {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};
template <> struct Vec16<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void unpack(const uint4& u, float* f)
    {
        f[0] = bf16_lo(u.x); f[1] = bf16_hi(u.x); f[2] = bf16_lo(u.y); f[3] = bf16_hi(u.y);
        f[4] = bf16_lo(u.z); f[5] = bf16_hi(u.z); f[6] = bf16_lo(u.w); f[7] = bf16_hi(u.w);
    }
};

template <> struct Vec16<h16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void unpack(const uint4& u, float* f)
    {
        const halfx8 h = __builtin_bit_cast(halfx8, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
    }
};

// 16 bytes through a raw buffer descriptor (byte offset `off` from its base): a load that starts at or past the
// descriptor's size returns zeros and touches no memory (the hardware's range check), so ragged ends need neither
// clamped addresses nor branches.  BUFFER_RSRC_RAW is the descriptor's last word for untyped 32-bit data on gfx9.
constexpr int BUFFER_RSRC_RAW = 0x00020000;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, int off)
{
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Wait until at most N of this wave's vector-memory operations are still in flight.  Placed after each load of a long
// run of loads it keeps a short rolling window in flight instead of the whole run: a workgroup that asks for everything
// it needs at once gets 35-60 GB/s out of its compute unit's load path, one that keeps two to sixteen loads per wave in
// flight 85-125 GB/s (measured on MI355X: one workgroup pulling 224 KB from HBM in 5.0 us against 1.8 us).
template <int N> __device__ __forceinline__ void vm_in_flight_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a six-bit counter");
    // gfx9 s_waitcnt operand: vmcnt in bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] left at "do not wait"
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
    asm volatile("" ::: "memory");
}

// Fragment geometry for element type T: a fragment is 64 bytes of k per row / column.
template <typename T> struct Frag {
    static constexpr int KB = 64 / (int)sizeof(T);    // k elements per fragment
    static constexpr int EPL = 16 / (int)sizeof(T);   // k elements per lane
};

// element offset of (slot, k) in a slot-tiled activation array with NK fragments per tile
template <typename T>
__device__ __forceinline__ size_t xoff(int NK, int slot, int k)
{
    constexpr int KB = Frag<T>::KB, EPL = Frag<T>::EPL;
    return ((((size_t)(slot >> 4) * NK + k / KB) * 64) + (slot & 15) + 16 * ((k % KB) / EPL)) * EPL + (k % EPL);
}
// uint4 index of fragment `frag` of tile `tile`, lane `lane`
__device__ __forceinline__ size_t xfrag(int NK, int tile, int frag, int lane)
{
    return ((size_t)tile * NK + frag) * 64 + lane;
}

// D(16x16) += A(16 x 64B of k) * B(64B of k x 16): one fragment each.
// Lane l of A holds row l%16, bytes [16*(l/16), +16) of that row's 64-byte k chunk;
// lane l of B the same for column l%16.  A and B use the same k <-> (lane group,
// element) map, so the contraction is over the whole chunk whatever order the
// instruction walks it in.  D: lane l holds column l%16, rows 4*(l/16)..+3.
template <typename T> __device__ __forceinline__ floatx4 mfma_frag(const uint4& a, const uint4& b, floatx4 acc);
template <> __device__ __forceinline__ floatx4 mfma_frag<bf16_t>(const uint4& a, const uint4& b, floatx4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mfma_frag<h16_t>(const uint4& a, const uint4& b, floatx4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), acc, 0, 0, 0);
}
template <> __device__ __forceinline__ floatx4 mfma_frag<float>(const uint4& a, const uint4& b, floatx4 acc)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    return acc;
}

}  // namespace tts
