// Host-side helpers shared by the C-ABI translation units: error text, HIP call checking, arena
// carve-up, fp32 <-> bf16, uploads in the weight dtype and the MFMA A-fragment re-layout.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <vector>

#include "../../include/tts_pool.h"

namespace tts {

// records the text tts_last_error() returns (thread-local) and hands `code` back
int fail(int code, const char* fmt, ...);

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return tts::fail(TTS_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// hands out 256-byte aligned offsets into the caller's arena
struct Carver {
    size_t off = 0;
    size_t take(size_t bytes)
    {
        size_t o = off;
        off += (bytes + 255) & ~size_t(255);
        return o;
    }
};

inline uint16_t host_f2bf(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
inline float host_bf2f(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
// fp32 -> IEEE half, round to nearest even, subnormals kept, overflow to infinity
inline uint16_t host_f2h(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) return (uint16_t)(sign | 0x7C00u | (a > 0x7F800000u ? 0x200u : 0u));   // inf / nan
    if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);                                       // rounds to >= 65520: infinity
    if (a < 0x38800000u) {
        // below 2^-14: a multiple of 2^-24 (the add aligns the value to that grid with the FPU's round to nearest even)
        float v;
        memcpy(&v, &a, 4);
        const float shifted = v + 0.5f;          // 0.5f has the exponent whose last mantissa bit is 2^-24
        uint32_t s;
        memcpy(&s, &shifted, 4);
        return (uint16_t)(sign | (s & 0x7FFu));
    }
    const uint32_t r = a - 0x38000000u;          // rebias the exponent from 127 to 15
    return (uint16_t)(sign | (uint16_t)((r + 0xFFFu + ((r >> 13) & 1u)) >> 13));
}
// fp32 host values -> device array of the weight dtype.  The two-byte weight dtype is "bfloat16 values": each value
// is rounded to bfloat16 first (a no-op for weights that are bfloat16 values already) and then stored as the IEEE
// half of the same value, the operand type of the two-byte MFMA kernels (exact for magnitudes from 2^-14 up, within
// 2^-25 absolute below).
inline int upload(void* dst, const std::vector<float>& src, bool bf16)
{
    if (!bf16) {
        HIP_TRY(hipMemcpy(dst, src.data(), src.size() * 4, hipMemcpyHostToDevice));
    } else {
        std::vector<uint16_t> h(src.size());
        for (size_t i = 0; i < src.size(); ++i) h[i] = host_f2h(host_bf2f(host_f2bf(src[i])));
        HIP_TRY(hipMemcpy(dst, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    }
    return TTS_OK;
}

// A [rows][K] matrix given by an element accessor -> MFMA A-operand fragment
// order: tiles of 16 rows x (64 bytes of k); within a tile lane l holds row
// l%16, 16 bytes at byte offset 16*(l/16).
template <typename Get>
std::vector<float> pack_fragments(int rows, int K, bool bf16, Get get)
{
    const int KB = bf16 ? 32 : 16;   // k elements per 64-byte fragment row
    const int EPL = KB / 4;          // elements per lane
    const int NK = K / KB;
    std::vector<float> out((size_t)rows * K);
    for (int rt = 0; rt < rows / 16; ++rt)
        for (int ks = 0; ks < NK; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int i = 0; i < EPL; ++i)
                    out[(((size_t)rt * NK + ks) * 64 + lane) * EPL + i] =
                        get(rt * 16 + (lane & 15), ks * KB + (lane >> 4) * EPL + i);
    return out;
}

}  // namespace tts
