// Peak probes for the measurement section: what this GPU actually delivers for the two rooflines the
// kernels are priced against.  A register-only MFMA loop (no memory traffic: every wavefront keeps
// re-issuing the same instruction on its own accumulators) and a plain streaming copy.  Not part of
// the hot path; called by `bench.py --peak-probe` only.
#include "internal.h"
#include "../../include/anakin.h"

namespace ank {

typedef float pf16v __attribute__((ext_vector_type(16)));
typedef __bf16 pbf8 __attribute__((ext_vector_type(8)));
typedef float pf4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(WG) void probe_mfma_f32(float* out, int iters, float a0)
{
    pf16v acc[4];
    for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    const float a = a0 + (float)threadIdx.x, b = a0 * 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * WG + threadIdx.x] = s;
}

__global__ __launch_bounds__(WG) void probe_mfma_bf16(float* out, int iters, float a0)
{
    pf16v acc[4];
    for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    pbf8 a, b;
    for (int q = 0; q < 8; ++q) { a[q] = (__bf16)(a0 + (float)((threadIdx.x + q) & 7)); b[q] = (__bf16)(a0 * (float)q); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * WG + threadIdx.x] = s;
}

__global__ __launch_bounds__(WG) void probe_copy(const pf4v* __restrict__ src, pf4v* __restrict__ dst, size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n4; i += (size_t)gridDim.x * WG) dst[i] = src[i];
}

// read-only stream: every thread adds up what it reads; one word per thread leaves (so the loads cannot be dropped)
__global__ __launch_bounds__(WG) void probe_read(const pf4v* __restrict__ src, float* __restrict__ out, size_t n4)
{
    pf4v acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n4; i += (size_t)gridDim.x * WG) acc += src[i];
    out[(size_t)blockIdx.x * WG + threadIdx.x] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// L2 read stream in the bf16 acting kernel's pattern: every workgroup of 512 threads walks the same 1 MiB (two layers
// of 512 KiB in operand tiles: wavefront w reads tiles 2w and 2w + 1, 32 steps of 1 KiB each, four steps ahead) `reps`
// times; the buffer stays in every L2, so this is what the L2-to-CU path delivers when all units ask at once
typedef uint32_t pu4v __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void probe_l2_tiles(const pu4v* __restrict__ src, uint32_t* __restrict__ out, int reps)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t acc = 0;
    for (int r = 0; r < reps; ++r) {
        for (int layer = 0; layer < 2; ++layer) {
            const pu4v* base = src + (size_t)layer * (512 * 1024 / 16);
#pragma unroll 1
            for (int s = 0; s < 32; s += 4) {
                pu4v v[4][2];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int t = 0; t < 2; ++t) v[u][t] = base[((size_t)(wave * 2 + t) * 32 + (s + u)) * 64 + lane];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc += v[u][t][0] ^ v[u][t][1] ^ v[u][t][2] ^ v[u][t][3];
            }
        }
        asm volatile("" : "+v"(acc));                            // the passes are not merged
    }
    out[(size_t)blockIdx.x * 512 + tid] = acc;
}

}  // namespace ank

extern "C" int32_t anakin_peak_probe(int32_t kind, int32_t variant, void* scratch, size_t scratch_bytes, void* hip_stream,
                                     double* amount, double* milliseconds)
{
    using namespace ank;
    if (!scratch || !amount || !milliseconds || kind < 0 || kind > 5 || variant < 0 || variant > 65536) return ANAKIN_E_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return ANAKIN_E_HIP;
    const int iters = 4000;
    hipError_t err = hipSuccess;
    if (kind == ANAKIN_PROBE_COPY) {
        const size_t half = (scratch_bytes / 2) & ~(size_t)255;
        if (half < 256) return ANAKIN_E_INVALID_ARG;
        const size_t n4 = half / 16;
        auto* src = static_cast<pf4v*>(scratch);
        auto* dst = reinterpret_cast<pf4v*>(static_cast<char*>(scratch) + half);
        const int blocks = variant > 0 ? variant : 4096;
        hipLaunchKernelGGL(probe_copy, dim3(blocks), dim3(WG), 0, s, src, dst, n4);   // warm-up
        (void)hipEventRecord(e0, s);
        for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(probe_copy, dim3(blocks), dim3(WG), 0, s, src, dst, n4);
        (void)hipEventRecord(e1, s);
        *amount = 10.0 * 2.0 * (double)half;                 // bytes read + written
    } else if (kind == ANAKIN_PROBE_L2_TILES) {
        const int blocks = variant > 0 ? variant : 256;
        const size_t src_bytes = (size_t)1 << 20, out_bytes = (size_t)blocks * 512 * 4;
        if (scratch_bytes < src_bytes + out_bytes) return ANAKIN_E_INVALID_ARG;
        auto* src = static_cast<const pu4v*>(scratch);
        uint32_t* out = reinterpret_cast<uint32_t*>(static_cast<char*>(scratch) + src_bytes);
        const int reps = 200;
        hipLaunchKernelGGL(probe_l2_tiles, dim3(blocks), dim3(512), 0, s, src, out, 2);      // warm-up
        (void)hipEventRecord(e0, s);
        hipLaunchKernelGGL(probe_l2_tiles, dim3(blocks), dim3(512), 0, s, src, out, reps);
        (void)hipEventRecord(e1, s);
        *amount = (double)reps * (double)src_bytes * blocks;     // bytes delivered to the compute units
    } else if (kind == ANAKIN_PROBE_READ) {
        const int blocks = variant > 0 ? variant : 4096;
        const size_t tail = ((size_t)blocks * WG * 4 + 255) & ~(size_t)255;   // the sums go behind the range that is read
        if (scratch_bytes < tail + 256) return ANAKIN_E_INVALID_ARG;
        const size_t n4 = ((scratch_bytes - tail) & ~(size_t)255) / 16;
        auto* src = static_cast<pf4v*>(scratch);
        float* out = reinterpret_cast<float*>(static_cast<char*>(scratch) + n4 * 16);
        hipLaunchKernelGGL(probe_read, dim3(blocks), dim3(WG), 0, s, src, out, n4);    // warm-up
        (void)hipEventRecord(e0, s);
        for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(probe_read, dim3(blocks), dim3(WG), 0, s, src, out, n4);
        (void)hipEventRecord(e1, s);
        *amount = 10.0 * 16.0 * (double)n4;                  // bytes read
    } else if (kind == ANAKIN_PROBE_ADAM) {
        // theta | grad | m | v | one partial, P floats each; zeroed so that no value overflows over the repetitions
        size_t P = scratch_bytes / 20;
        if (P > ((size_t)1 << 26)) P = (size_t)1 << 26;
        P &= ~(size_t)63;
        if (P < 64) return ANAKIN_E_INVALID_ARG;
        float* base = static_cast<float*>(scratch);
        if (hipMemsetAsync(base, 0, P * 20, s) != hipSuccess) return ANAKIN_E_HIP;
        err = launch_adam_probe(base, (int)P, s);            // warm-up
        (void)hipEventRecord(e0, s);
        for (int r = 0; r < 5 && err == hipSuccess; ++r) err = launch_adam_probe(base, (int)P, s);
        (void)hipEventRecord(e1, s);
        if (err != hipSuccess) return ANAKIN_E_HIP;
        *amount = 5.0 * 32.0 * (double)P;                    // 28 B of Adam state per parameter + 4 B of the partial
    } else {
        const int blocks = variant > 0 ? variant : 768;
        if (scratch_bytes < (size_t)blocks * WG * 4) return ANAKIN_E_INVALID_ARG;
        float* out = static_cast<float*>(scratch);
        auto launch = [&](int n) {
            if (kind == ANAKIN_PROBE_MFMA_F32) hipLaunchKernelGGL(probe_mfma_f32, dim3(blocks), dim3(WG), 0, s, out, n, 1.0f);
            else hipLaunchKernelGGL(probe_mfma_bf16, dim3(blocks), dim3(WG), 0, s, out, n, 1.0f);
        };
        launch(10);
        (void)hipEventRecord(e0, s);
        launch(iters);
        (void)hipEventRecord(e1, s);
        const double flop_per_mfma = kind == ANAKIN_PROBE_MFMA_F32 ? 4096.0 : 32768.0;
        *amount = (double)blocks * 4.0 * iters * 8.0 * 4.0 * flop_per_mfma;
    }
    err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (err != hipSuccess || hipGetLastError() != hipSuccess) return ANAKIN_E_HIP;
    *milliseconds = (double)ms;
    return ANAKIN_OK;
}
