// Measurement aid: what the matrix cores of this machine sustain when a kernel does nothing but MFMAs.
// The compression kernels are priced against the published MFMA peaks; this probe gives the figure a real kernel could
// reach at best on the box it runs on, which for random bf16 operands is well below the published one (the chip lowers
// its clock under a full-rate MFMA stream whose operands change).  Declared in include/exat.h (exat_probe_mfma).
#include "../../include/exat.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t probe_hash(uint32_t x)
{
    x ^= x >> 16; x *= 0x9e3779b1u; x ^= x >> 15; x *= 0x85ebca77u; x ^= x >> 13;
    return x;
}
// a value in [-1, 1) with 10 random bits, or the constant 0.5
__device__ __forceinline__ float probe_value(uint32_t key, int random_operands)
{
    return random_operands ? (float)(probe_hash(key) & 1023u) / 512.0f - 1.0f : 0.5f;
}

// KIND 0: v_mfma_f32_32x32x16_bf16, KIND 1: v_mfma_f32_32x32x2_f32.  Eight waves per workgroup (two per SIMD, as in the
// compression kernels), each with four independent accumulators and eight operand registers per side that rotate, so
// that consecutive MFMAs never share an operand; 64 MFMAs per iteration.  out[0] receives a checksum (keeps the
// accumulators alive); workgroup 0 writes the elapsed core-clock and 100 MHz wall-clock ticks to ticks[0], ticks[1].
template <int KIND>
__global__ __launch_bounds__(512) void k_probe_mfma(float *out, uint64_t *ticks, int iters, int random_operands)
{
    f32x16 c[4];
#pragma unroll
    for (int t = 0; t < 4; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) c[t][e] = 0.0f;
    const uint32_t lane_key = (blockIdx.x * 512u + threadIdx.x) * 64u;
    const uint64_t t0 = clock64(), w0 = wall_clock64();
    if constexpr (KIND == 0) {
        bf16x8 a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int e = 0; e < 8; e++) {
                a[i][e] = (__bf16)probe_value(lane_key + i * 8 + e, random_operands);
                b[i][e] = (__bf16)probe_value(lane_key + 0x40000000u + i * 8 + e, random_operands);
            }
        for (int it = 0; it < iters; it++) {
#pragma unroll
            for (int t = 0; t < 64; t++) c[t & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t & 7], b[(t >> 3) & 7], c[t & 3], 0, 0, 0);
        }
    } else {
        float a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            a[i] = probe_value(lane_key + i, random_operands);
            b[i] = probe_value(lane_key + 0x40000000u + i, random_operands);
        }
        for (int it = 0; it < iters; it++) {
#pragma unroll
            for (int t = 0; t < 64; t++) c[t & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t & 7], b[(t >> 3) & 7], c[t & 3], 0, 0, 0);
        }
    }
    const uint64_t t1 = clock64(), w1 = wall_clock64();
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 4; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) s += c[t][e];
    if (s == 123456.789f) out[0] = s;   // never true in practice; the compiler cannot know
    if (blockIdx.x == 0 && threadIdx.x == 0) { ticks[0] = t1 - t0; ticks[1] = w1 - w0; }
}

}  // namespace

extern "C" int exat_probe_mfma(int32_t kind, int32_t random_operands, int32_t iters, int32_t workgroups, double *tflops, double *core_ghz)
{
    if (!tflops || !core_ghz) return EXAT_ERR_NULL;
    if (kind < 0 || kind > 1 || iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20)) return EXAT_ERR_SHAPE;
    float *out = nullptr;
    uint64_t *ticks = nullptr, host_ticks[2] = {0, 0};
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = EXAT_OK;
    if (hipMalloc((void **)&out, 256) != hipSuccess || hipMalloc((void **)&ticks, 256) != hipSuccess) rc = EXAT_ERR_ALLOC;
    if (rc == EXAT_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) rc = EXAT_ERR_HIP;
    float ms = 0.0f;
    if (rc == EXAT_OK) {
        auto launch = [&]() {
            if (kind == 0) hipLaunchKernelGGL(k_probe_mfma<0>, dim3((unsigned)workgroups), dim3(512), 0, nullptr, out, ticks, iters, random_operands);
            else hipLaunchKernelGGL(k_probe_mfma<1>, dim3((unsigned)workgroups), dim3(512), 0, nullptr, out, ticks, iters, random_operands);
        };
        launch();   // warm-up: the clock settles under load
        if (hipEventRecord(e0, nullptr) != hipSuccess) rc = EXAT_ERR_HIP;
        launch();
        if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipMemcpy(host_ticks, ticks, sizeof(host_ticks), hipMemcpyDeviceToHost) != hipSuccess)
            rc = EXAT_ERR_HIP;
    }
    if (rc == EXAT_OK) {
        const double flop_per_mfma = kind == 0 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
        *tflops = (double)workgroups * 8.0 * (double)iters * 64.0 * flop_per_mfma / ((double)ms * 1e-3) / 1e12;
        *core_ghz = host_ticks[1] ? (double)host_ticks[0] / (double)host_ticks[1] * 0.1 : 0.0;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out); (void)hipFree(ticks);
    return rc;
}
