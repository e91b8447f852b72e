// Three machine costs that decide the shape of the decoder step on gfx950, measured with
// throw-away kernels (no part of the library):
//   1. what a kernel boundary costs inside a hipGraph, and what a kernel's first dependent
//      memory round trips cost after such a boundary;
//   2. what an all-to-all synchronisation between the workgroups of ONE persistent kernel costs
//      (flag array in global memory, data handed over through coherent stores and loads or
//      through release / acquire fences): the alternative to kernel boundaries;
//   3. how fast one workgroup (one CU) and the whole chip can stream from memory.
// Every wait in here is bounded: a flag that never arrives ends the kernel with an error flag.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("ERR %s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)

// ---- 1. a chain of `hops` dependent loads per thread (each address comes out of the previous load)
__global__ __launch_bounds__(256) void k_chain(const int* __restrict__ next, int mask, int hops, int* out)
{
    int i = (blockIdx.x * 256 + threadIdx.x) & mask;
    for (int h = 0; h < hops; ++h) i = next[(i + threadIdx.x) & mask];
    if (i == -12345) *out = i;
}

// ---- 2. rounds of "write, signal, wait for everybody, read somebody else's"
// MODE 0: flags only.  MODE 1: data + release / acquire fences (agent scope).
// MODE 2: data through agent-scope atomic stores / loads (they bypass the per-XCD L2).
template <int MODE>
__global__ __launch_bounds__(512) void k_rounds(unsigned* flags, float* buf, int per, int iters, unsigned* fail, float* out)
{
    const int tid = threadIdx.x, wg = blockIdx.x, G = gridDim.x;
    __shared__ int s_ok;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        float* mine = buf + ((size_t)(it & 1) * G + wg) * per;
        if (MODE == 1) for (int i = tid; i < per; i += 512) mine[i] = (float)(it + wg + i);
        if (MODE == 2) for (int i = tid; i < per; i += 512) __hip_atomic_store(&mine[i], (float)(it + wg + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (tid == 0) {
            if (MODE == 1) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __hip_atomic_store(&flags[wg], (unsigned)(it + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid < 64) {
            int ok = 0;
            for (int spin = 0; spin < (1 << 18); ++spin) {          // bounded
                bool all = true;
                for (int j = tid; j < G; j += 64)
                    all = all && (__hip_atomic_load(&flags[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)(it + 1));
                if (__all(all)) { ok = 1; break; }
            }
            if (tid == 0) { s_ok = ok; if (!ok) *fail = 1; }
            if (MODE == 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
        if (!s_ok) return;
        const float* other = buf + ((size_t)(it & 1) * G + (wg + 37) % G) * per;
        if (MODE == 1) for (int i = tid; i < per; i += 512) acc += other[i] - (float)(it + (wg + 37) % G + i);
        if (MODE == 2) for (int i = tid; i < per; i += 512) acc += __hip_atomic_load(&other[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - (float)(it + (wg + 37) % G + i);
    }
    if (acc != 0.f) out[0] = acc;      // stays 0 when every value read was the fresh one
}

// ---- 3. every workgroup streams NL * 8 KiB with all of its loads in flight at once
template <int NL>
__global__ __launch_bounds__(512) void k_stream(const uint4* __restrict__ a, unsigned* out)
{
    const uint4* p = a + (size_t)blockIdx.x * NL * 512 + threadIdx.x;
    uint4 v[NL];
#pragma unroll
    for (int k = 0; k < NL; ++k) v[k] = p[(size_t)k * 512];
    unsigned acc = 0;
#pragma unroll
    for (int k = 0; k < NL; ++k) acc ^= v[k].x ^ v[k].w;
    if (acc == 0x12345678u) *out = acc;
}

// ---- 3b. the same, PASSES times over the same NL * 8 KiB inside one kernel: passes after the first find the data in L2
template <int NL, int PASSES>
__global__ __launch_bounds__(512) void k_restream(const uint4* __restrict__ a, unsigned* out)
{
    const uint4* p = a + (size_t)blockIdx.x * NL * 512 + threadIdx.x;
    unsigned acc = 0;
    for (int pass = 0; pass < PASSES; ++pass) {
        uint4 v[NL];
#pragma unroll
        for (int k = 0; k < NL; ++k) v[k] = p[(size_t)k * 512];
#pragma unroll
        for (int k = 0; k < NL; ++k) acc ^= v[k].x ^ v[k].w;
        p += (acc == 0x9abcdef0u);              // unknown to the compiler: the next pass cannot reuse this one's registers
    }
    if (acc == 0x12345678u) *out = acc;
}

template <int NL, int PASSES> static int restream(hipStream_t s, const uint4* big, unsigned* out_u, double* t_prev)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float ms;
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL((k_restream<NL, PASSES>), dim3(1), dim3(512), 0, s, big, out_u);
    CK(hipEventRecord(e0, s));
    for (int i = 0; i < 50; ++i) hipLaunchKernelGGL((k_restream<NL, PASSES>), dim3(1), dim3(512), 0, s, big, out_u);
    CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    const double t = ms * 1e3 / 50;
    printf("    1 workgroup, %d pass(es) over the same %3d KiB: %6.2f us per launch", PASSES, NL * 8, t);
    if (*t_prev > 0) printf("   (each further pass: %.2f us = %.0f GB/s)", (t - *t_prev), NL * 8192.0 / ((t - *t_prev) * 1e-6) / 1e9);
    printf("\n");
    *t_prev = t;
    return 0;
}

// ---- 3c. one workgroup of T threads streams BYTES with all loads in flight: does the rate follow the number of waves?
template <int T, int BYTES>
__global__ __launch_bounds__(T) void k_stream_threads(const uint4* __restrict__ a, unsigned* out)
{
    constexpr int NL = BYTES / 16 / T;
    const uint4* p = a + threadIdx.x;
    uint4 v[NL];
#pragma unroll
    for (int k = 0; k < NL; ++k) v[k] = p[(size_t)k * T];
    unsigned acc = 0;
#pragma unroll
    for (int k = 0; k < NL; ++k) acc ^= v[k].x ^ v[k].w;
    if (acc == 0x12345678u) *out = acc;
}

template <int T, int BYTES> static int stream_threads(hipStream_t s, const uint4* big, unsigned* out_u)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float ms;
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL((k_stream_threads<T, BYTES>), dim3(1), dim3(T), 0, s, big, out_u);
    CK(hipEventRecord(e0, s));
    for (int i = 0; i < 50; ++i) hipLaunchKernelGGL((k_stream_threads<T, BYTES>), dim3(1), dim3(T), 0, s, big, out_u);
    CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    printf("    1 workgroup of %4d threads x %3d KiB: %6.2f us per launch\n", T, BYTES / 1024, ms * 1e3 / 50);
    return 0;
}

template <int NL> static int stream(hipStream_t s, const uint4* big, unsigned* out_u, int grid, double* t_prev, double* b_prev)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float ms;
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(k_stream<NL>, dim3(grid), dim3(512), 0, s, big, out_u);
    CK(hipEventRecord(e0, s));
    for (int i = 0; i < 50; ++i) hipLaunchKernelGGL(k_stream<NL>, dim3(grid), dim3(512), 0, s, big, out_u);
    CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    const double t = ms * 1e3 / 50, b = (double)NL * 8192 * grid;
    printf("  %3d workgroup(s) x %3d KiB: %6.2f us per launch", grid, NL * 8, t);
    if (*b_prev > 0) printf("   (slope against the previous size: %.0f GB/s)", (b - *b_prev) / ((t - *t_prev) * 1e-6) / 1e9);
    printf("\n");
    *t_prev = t; *b_prev = b;
    return 0;
}

// ---- 2b. the same exchange inside independent groups of `GS` neighbouring workgroups (each waits for its own
// group only): data through agent-scope stores, the flag stored with release / loaded with acquire semantics
template <int GS>
__global__ __launch_bounds__(512) void k_group_rounds(unsigned* flags, float* buf, int per, int iters, unsigned* fail, float* out)
{
    const int tid = threadIdx.x, wg = blockIdx.x, G = gridDim.x;
    const int g0 = wg / GS * GS;
    __shared__ int s_ok;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        float* mine = buf + ((size_t)(it & 1) * G + wg) * per;
        for (int i = tid; i < per; i += 512) __hip_atomic_store(&mine[i], (float)(it + wg + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (tid == 0) __hip_atomic_store(&flags[wg], (unsigned)(it + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        if (tid < 64) {
            int ok = 0;
            for (int spin = 0; spin < (1 << 18); ++spin) {          // bounded
                bool all = true;
                if (tid < GS) all = __hip_atomic_load(&flags[g0 + tid], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)(it + 1);
                if (__all(all)) { ok = 1; break; }
            }
            if (tid == 0) { s_ok = ok; if (!ok) *fail = 1; }
        }
        __syncthreads();
        if (!s_ok) return;
        const int peer = g0 + (wg - g0 + 1) % GS;
        const float* other = buf + ((size_t)(it & 1) * G + peer) * per;
        for (int i = tid; i < per; i += 512) acc += __hip_atomic_load(&other[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - (float)(it + peer + i);
    }
    if (acc != 0.f) out[0] = acc;
}

template <int GS> static int group_rounds(hipStream_t s, unsigned* flags, float* buf, unsigned* fail, float* out, int grid, int per)
{
    const int iters = 2000;
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    CK(hipMemsetAsync(flags, 0, 4096, s)); CK(hipMemsetAsync(fail, 0, 4, s)); CK(hipMemsetAsync(out, 0, 4, s));
    CK(hipEventRecord(e0, s));
    hipLaunchKernelGGL(k_group_rounds<GS>, dim3(grid), dim3(512), 0, s, flags, buf, per, iters, fail, out);
    CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    unsigned hf; float ho; CK(hipMemcpy(&hf, fail, 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(&ho, out, 4, hipMemcpyDeviceToHost));
    printf("  groups of %d among %3d workgroups, %5d B each, release/acquire flags: %6.2f us per round%s%s\n", GS, grid, per * 4,
           ms * 1e3 / iters, hf ? "  TIMED OUT" : "", ho != 0.f ? "  STALE DATA READ" : "");
    fflush(stdout);
    return hf ? 1 : 0;
}

template <int MODE> static int rounds(hipStream_t s, unsigned* flags, float* buf, unsigned* fail, float* out, int grid, int per, const char* name)
{
    const int iters = 2000;
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    CK(hipMemsetAsync(flags, 0, 4096, s)); CK(hipMemsetAsync(fail, 0, 4, s)); CK(hipMemsetAsync(out, 0, 4, s));
    CK(hipEventRecord(e0, s));
    hipLaunchKernelGGL(k_rounds<MODE>, dim3(grid), dim3(512), 0, s, flags, buf, per, iters, fail, out);
    CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    unsigned hf; float ho; CK(hipMemcpy(&hf, fail, 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(&ho, out, 4, hipMemcpyDeviceToHost));
    printf("  %-40s %3d workgroups, %5d B each: %6.2f us per round%s%s\n", name, grid, per * 4, ms * 1e3 / iters,
           hf ? "  TIMED OUT" : "", ho != 0.f ? "  STALE DATA READ" : "");
    fflush(stdout);
    return hf ? 1 : 0;
}

int main()
{
    hipStream_t s; CK(hipStreamCreate(&s));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float ms;
    int* chain; int* out_i;
    const int NBIG = 1 << 24;                       // 64 MiB of links: not L2-resident
    CK(hipMalloc(&chain, (size_t)NBIG * 4)); CK(hipMalloc(&out_i, 64));
    {
        int* h = (int*)malloc((size_t)NBIG * 4);
        unsigned x = 12345u;
        for (int i = 0; i < NBIG; ++i) { x = x * 1664525u + 1013904223u; h[i] = (int)(x >> 8) & (NBIG - 1); }
        CK(hipMemcpy(chain, h, (size_t)NBIG * 4, hipMemcpyHostToDevice));
        free(h);
    }

    printf("1. kernel boundaries and dependent loads (graphs of 32 kernels of 256 workgroups x 256 threads)\n");
    for (int mask : {4095, NBIG - 1})
        for (int hops : {0, 1, 2, 4}) {
            hipGraph_t g; hipGraphExec_t ge;
            CK(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
            for (int i = 0; i < 32; ++i) hipLaunchKernelGGL(k_chain, dim3(256), dim3(256), 0, s, chain, mask, hops, out_i);
            CK(hipStreamEndCapture(s, &g)); CK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
            for (int i = 0; i < 10; ++i) CK(hipGraphLaunch(ge, s));
            CK(hipStreamSynchronize(s));
            CK(hipEventRecord(e0, s));
            for (int i = 0; i < 200; ++i) CK(hipGraphLaunch(ge, s));
            CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
            printf("  kernel with %d dependent loads over a %s table: %.2f us per kernel\n", hops,
                   mask == 4095 ? "16 KiB" : "64 MiB", ms * 1e3 / 200 / 32);
        }

    // A step of two dependent kernels A -> B; a third kernel P that B also needs, either in line (A -> P -> B) or on a
    // side branch of the graph next to A (P and A both follow the previous B, B waits for both).
    printf("1b. a side branch in a graph (16 steps per graph; every kernel 256 workgroups with 2 dependent loads over the 64 MiB table)\n");
    {
        hipStream_t s1; CK(hipStreamCreate(&s1));
        hipEvent_t ef, ej; CK(hipEventCreateWithFlags(&ef, hipEventDisableTiming)); CK(hipEventCreateWithFlags(&ej, hipEventDisableTiming));
        int* out_p; CK(hipMalloc(&out_p, 64));
        for (int mode = 0; mode < 3; ++mode) {
            hipGraph_t g; hipGraphExec_t ge;
            CK(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
            for (int i = 0; i < 16; ++i) {
                if (mode == 2) {
                    CK(hipEventRecord(ef, s));
                    CK(hipStreamWaitEvent(s1, ef, 0));
                    hipLaunchKernelGGL(k_chain, dim3(256), dim3(256), 0, s1, chain, NBIG - 1, 2, out_p);     // P beside A
                    CK(hipEventRecord(ej, s1));
                }
                hipLaunchKernelGGL(k_chain, dim3(256), dim3(256), 0, s, chain, NBIG - 1, 2, out_i);          // A
                if (mode == 1) hipLaunchKernelGGL(k_chain, dim3(256), dim3(256), 0, s, chain, NBIG - 1, 2, out_p);   // P in line
                if (mode == 2) CK(hipStreamWaitEvent(s, ej, 0));
                hipLaunchKernelGGL(k_chain, dim3(256), dim3(256), 0, s, chain, NBIG - 1, 2, out_i);          // B
            }
            CK(hipStreamEndCapture(s, &g)); CK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
            for (int i = 0; i < 10; ++i) CK(hipGraphLaunch(ge, s));
            CK(hipStreamSynchronize(s));
            CK(hipEventRecord(e0, s));
            for (int i = 0; i < 200; ++i) CK(hipGraphLaunch(ge, s));
            CK(hipEventRecord(e1, s)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
            printf("  %-34s %.2f us per step\n", mode == 0 ? "A -> B:" : (mode == 1 ? "A -> P -> B:" : "A and P side by side -> B:"), ms * 1e3 / 200 / 16);
            CK(hipGraphExecDestroy(ge)); CK(hipGraphDestroy(g));
        }
    }

    printf("2. all-to-all synchronisation inside one persistent kernel\n");
    unsigned *flags, *fail; float *buf, *out;
    CK(hipMalloc(&flags, 4096)); CK(hipMalloc(&fail, 4)); CK(hipMalloc(&out, 4)); CK(hipMalloc(&buf, 64 << 20));
    for (int grid : {64, 128, 256}) {
        if (rounds<0>(s, flags, buf, fail, out, grid, 0, "flags only")) return 2;
        if (rounds<1>(s, flags, buf, fail, out, grid, 512, "data, release/acquire fences")) return 2;
        if (rounds<2>(s, flags, buf, fail, out, grid, 512, "data through coherent stores/loads")) return 2;
    }

    for (int grid : {4, 64, 256}) {
        if (group_rounds<4>(s, flags, buf, fail, out, grid, 300)) return 2;
        if (group_rounds<2>(s, flags, buf, fail, out, grid, 300)) return 2;
    }

    printf("3. streaming reads, all loads of a workgroup in flight at once (time includes the launch; slope = sustained rate)\n");
    uint4* big; unsigned* out_u; const size_t BYTES = (size_t)256 << 20;
    CK(hipMalloc(&big, BYTES)); CK(hipMalloc(&out_u, 64)); CK(hipMemset(big, 1, BYTES));
    for (int grid : {1, 256}) {
        double t_prev = 0, b_prev = 0;
        if (stream<4>(s, big, out_u, grid, &t_prev, &b_prev)) return 1;
        if (stream<8>(s, big, out_u, grid, &t_prev, &b_prev)) return 1;
        if (stream<16>(s, big, out_u, grid, &t_prev, &b_prev)) return 1;
        if (stream<32>(s, big, out_u, grid, &t_prev, &b_prev)) return 1;
        if (stream<48>(s, big, out_u, grid, &t_prev, &b_prev)) return 1;
    }
    printf("3b. one workgroup re-reading what it has just read (later passes are L2 hits)\n");
    {
        double tp = 0;
        if (restream<32, 1>(s, big, out_u, &tp)) return 1;
        if (restream<32, 2>(s, big, out_u, &tp)) return 1;
        tp = 0;
        if (restream<48, 1>(s, big, out_u, &tp)) return 1;
        if (restream<48, 2>(s, big, out_u, &tp)) return 1;
        if (restream<48, 3>(s, big, out_u, &tp)) return 1;
    }
    printf("3c. one workgroup, the same bytes with more or fewer waves\n");
    if (stream_threads<256, 128 << 10>(s, big, out_u)) return 1;
    if (stream_threads<512, 128 << 10>(s, big, out_u)) return 1;
    if (stream_threads<1024, 128 << 10>(s, big, out_u)) return 1;
    if (stream_threads<256, 256 << 10>(s, big, out_u)) return 1;
    if (stream_threads<512, 256 << 10>(s, big, out_u)) return 1;
    if (stream_threads<1024, 256 << 10>(s, big, out_u)) return 1;
    return 0;
}
