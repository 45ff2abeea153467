// Measured ceilings of the device the library runs on, for judging the roofline fractions of its
// kernels against what this very chip sustains: a streaming read, a device copy and a loop of
// nothing but bf16 MFMAs (cascade_measure_ceilings of include/cascade_kv.h).  Diagnostics: the
// kernels here are not part of the hot path.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <string>

#include "../../include/cascade_kv.h"
#include "structure.h"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 cbf16x8_t;
typedef __attribute__((ext_vector_type(16))) float cf32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t cu32x4_t;

// every thread reads 16 bytes per step, consecutive threads consecutive addresses, grid-stride
__global__ __launch_bounds__(256) void ceiling_read_kernel(const cu32x4_t* __restrict__ src, size_t n16, uint32_t* __restrict__ sink)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const cu32x4_t v = __builtin_nontemporal_load(src + i);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9E3779B9u) *sink = acc;   // (practically never: keeps the loads alive)
}

// Every workgroup streams a contiguous region of its own, sixteen 4 KB loads in flight (the access
// pattern of the decode kernels, one region per split).  STORES: after every 64 KB read the workgroup
// writes 4 KB elsewhere, the ratio of logits written to keys read in the decode step's first pass.
template <bool STORES>
__global__ __launch_bounds__(256) void ceiling_regions_kernel(const cu32x4_t* __restrict__ src, size_t per_wg16, cu32x4_t* __restrict__ dst,
                                                              uint32_t* __restrict__ sink)
{
    constexpr int U = 16;
    uint32_t acc = 0;
    const cu32x4_t* p = src + (size_t)blockIdx.x * per_wg16;
    cu32x4_t* o = dst + (size_t)blockIdx.x * (per_wg16 / U);
    for (size_t i = threadIdx.x; i + (U - 1) * 256 < per_wg16; i += U * 256) {
        cu32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
        cu32x4_t x = v[0];
#pragma unroll
        for (int u = 1; u < U; ++u) x ^= v[u];
        if (STORES) o[(i / (U * 256)) * 256 + threadIdx.x] = x;     // 256 * iteration + thread: below per_wg16 / U
        else acc ^= x[0] ^ x[1] ^ x[2] ^ x[3];
    }
    if (!STORES && acc == 0x9E3779B9u) *sink = acc;
}

__global__ __launch_bounds__(256) void ceiling_copy_kernel(const cu32x4_t* __restrict__ src, cu32x4_t* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// four independent accumulator chains per wave, operands in registers: the matrix pipe alone
__global__ __launch_bounds__(512) void ceiling_mfma_kernel(int iters, float* __restrict__ sink)
{
    cf32x16_t acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[a][j] = 0.f;
    union { cbf16x8_t v; cu32x4_t u; } x, y;
    // operands of magnitude 1..2 with lane-dependent signs and mantissas (the power a matrix pipe draws
    // depends on the bits it multiplies; all-zero operands would flatter the figure)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t h = (threadIdx.x * 4u + i + 1u) * 2654435761u;
        x.u[i] = 0x3F803F80u | (h & 0x807F807Fu);
        y.u[i] = 0x3F803F80u | ((h >> 7) & 0x807F807Fu);
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int a = 0; a < 4; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, y.v, acc[a], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[a][j];
    if (s == -1.f) *sink = s;              // (practically never)
}

}  // namespace ckv

using namespace ckv;

static int ceil_fail(int code, const std::string& msg)
{
    set_init_error(msg);
    return code;
}

template <typename F> static int best_of(int reps, hipStream_t s, F launch, double* best_ms)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return CASCADE_E_HIP;
    *best_ms = 1e30;
    int rc = CASCADE_OK;
    for (int r = 0; r < reps + 1 && rc == CASCADE_OK; ++r) {       // the first repetition warms up
        (void)hipEventRecord(a, s);
        launch();
        (void)hipEventRecord(b, s);
        if (hipEventSynchronize(b) != hipSuccess || hipGetLastError() != hipSuccess) { rc = CASCADE_E_HIP; break; }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, a, b);
        if (r > 0) *best_ms = std::min(*best_ms, (double)ms);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

extern "C" int cascade_measure_ceilings(void* dev_buffer, size_t bytes, void* stream, cascade_ceilings* out)
{
    if (!dev_buffer || !out) return ceil_fail(CASCADE_E_NULL_ARG, "cascade_measure_ceilings: NULL argument");
    if (bytes < ((size_t)1 << 30) || ((uintptr_t)dev_buffer & 15)) return ceil_fail(CASCADE_E_BAD_ARG, "cascade_measure_ceilings: needs a 16-byte aligned buffer of at least 1 GiB");
    memset(out, 0, sizeof(*out));
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
        return ceil_fail(CASCADE_E_HIP, "cascade_measure_ceilings: device properties");
    out->compute_units = prop.multiProcessorCount;
    out->core_clock_mhz = prop.clockRate / 1000.0;
    out->memory_clock_mhz = prop.memoryClockRate / 1000.0;
    out->memory_bus_bits = prop.memoryBusWidth;
    hipStream_t s = (hipStream_t)stream;
    // Every single-launch figure is taken on the FIRST HALF of the buffer (the copy: its first quarter onto its
    // second), the pairs of launches on both halves: sized for the workload at hand, half the buffer is the
    // array one pass streams.
    const size_t full = bytes;
    bytes = (full / 2) & ~(size_t)4095;
    const size_t half = (bytes / 2) & ~(size_t)4095;
    const size_t n_read = (bytes & ~(size_t)4095) / 16, n_copy = half / 16;
    uint32_t* sink = (uint32_t*)dev_buffer;    // written only if a checksum takes one particular value
    const int blocks = prop.multiProcessorCount * 16;
    double ms = 0.0;
    int rc = best_of(5, s, [&] {
        hipLaunchKernelGGL(ceiling_read_kernel, dim3(blocks), dim3(256), 0, s, (const cu32x4_t*)dev_buffer, n_read, sink);
    }, &ms);
    if (rc) return ceil_fail(rc, "cascade_measure_ceilings: streaming read");
    out->read_gb_s = (double)n_read * 16 / (ms * 1e-3) / 1e9;
    {
        // regions: the first 15/16 of the buffer is read by 8 workgroups per compute unit, the rest takes the stores
        const int wgs_r = prop.multiProcessorCount * 8;
        const size_t per_wg16 = (((bytes / 16) * 15 / 16) / wgs_r) & ~(size_t)4095;     // whole iterations of 16 x 256 loads
        if (per_wg16 == 0) return ceil_fail(CASCADE_E_BAD_ARG, "cascade_measure_ceilings: buffer too small for this device");
        cu32x4_t* dst = (cu32x4_t*)dev_buffer + per_wg16 * wgs_r;                         // per_wg16 / 16 stores per workgroup fit behind
        rc = best_of(5, s, [&] {
            hipLaunchKernelGGL(ceiling_regions_kernel<false>, dim3(wgs_r), dim3(256), 0, s, (const cu32x4_t*)dev_buffer, per_wg16, dst, sink);
        }, &ms);
        if (rc) return ceil_fail(rc, "cascade_measure_ceilings: streaming read of regions");
        out->read_regions_gb_s = (double)per_wg16 * wgs_r * 16 / (ms * 1e-3) / 1e9;
        rc = best_of(5, s, [&] {
            hipLaunchKernelGGL(ceiling_regions_kernel<true>, dim3(wgs_r), dim3(256), 0, s, (const cu32x4_t*)dev_buffer, per_wg16, dst, sink);
        }, &ms);
        if (rc) return ceil_fail(rc, "cascade_measure_ceilings: streaming read with stores");
        out->read_with_stores_gb_s = (double)per_wg16 * wgs_r * 16 / (ms * 1e-3) / 1e9;   // bytes read only
        // The two passes of a decode step one after the other, as traffic alone: a read with stores (the keys,
        // the logits written) on one half of the buffer, then a plain read (the values) on the other half,
        // eight such pairs back to back (what the first launch wrote may still be on its way to memory while the
        // second reads).
        const size_t half16 = ((full / 2) / 16) & ~(size_t)255;
        const size_t per_a16 = ((half16 * 15 / 16) / wgs_r) & ~(size_t)4095;
        const size_t per_b16 = (half16 / wgs_r) & ~(size_t)4095;
        if (per_a16 == 0 || per_b16 == 0) return ceil_fail(CASCADE_E_BAD_ARG, "cascade_measure_ceilings: buffer too small for this device");
        const cu32x4_t* src_b = (const cu32x4_t*)dev_buffer + half16;
        cu32x4_t* dst_a = (cu32x4_t*)dev_buffer + per_a16 * wgs_r;          // behind the part of the first half that is read
        const int pairs = 8;
        rc = best_of(2, s, [&] {
            for (int i = 0; i < pairs; ++i) {
                hipLaunchKernelGGL(ceiling_regions_kernel<true>, dim3(wgs_r), dim3(256), 0, s, (const cu32x4_t*)dev_buffer, per_a16, dst_a, sink);
                hipLaunchKernelGGL(ceiling_regions_kernel<false>, dim3(wgs_r), dim3(256), 0, s, src_b, per_b16, dst_a, sink);
            }
        }, &ms);
        if (rc) return ceil_fail(rc, "cascade_measure_ceilings: pairs of launches");
        out->two_pass_read_gb_s = (double)(per_a16 + per_b16) * wgs_r * 16 * pairs / (ms * 1e-3) / 1e9;   // bytes read by both
    }
    rc = best_of(5, s, [&] {
        hipLaunchKernelGGL(ceiling_copy_kernel, dim3(blocks), dim3(256), 0, s, (const cu32x4_t*)dev_buffer,
                           (cu32x4_t*)((char*)dev_buffer + half), n_copy);
    }, &ms);
    if (rc) return ceil_fail(rc, "cascade_measure_ceilings: copy");
    out->copy_gb_s = 2.0 * (double)n_copy * 16 / (ms * 1e-3) / 1e9;       // bytes read plus bytes written
    const int iters = 20000, wgs = prop.multiProcessorCount;              // one workgroup of 8 waves per CU: 2 waves per SIMD
    rc = best_of(3, s, [&] { hipLaunchKernelGGL(ceiling_mfma_kernel, dim3(wgs), dim3(512), 0, s, iters, (float*)sink); }, &ms);
    if (rc) return ceil_fail(rc, "cascade_measure_ceilings: MFMA loop");
    out->mfma_bf16_tflops = (double)wgs * 8 * iters * 4 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    return CASCADE_OK;
}
