// Calibration kernels for benchmarks (not part of the method): what this GPU reaches on a plain streaming copy and on
// a loop of nothing but bf16 MFMAs, so that a kernel's distance from the published peaks (8 TB/s, 2.5 PFLOP/s) can be
// split into what the machine withholds and what the kernel loses.
#include "common.h"

namespace pa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Four 16-byte loads in flight per thread, streaming (non-temporal) in both directions.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void calib_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, int64_t n_vec) {
    const int64_t stride = gridDim.x * 256ll;
    int64_t x = blockIdx.x * 256ll + threadIdx.x;
    for (; x + 3 * stride < n_vec; x += 4 * stride) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(src + x + k * stride);
#pragma unroll
        for (int k = 0; k < 4; ++k) __builtin_nontemporal_store(v[k], dst + x + k * stride);
    }
    for (; x < n_vec; x += stride) dst[x] = src[x];
}

// Every wave runs iters rounds of kChains independent 32x32x16 bf16 MFMAs (each chain waits only for itself, so the
// matrix pipe always has an independent instruction to take).  out[0], out[1] (64-bit): shader cycles and ticks of the
// 100 MHz constant counter that wave 0 of workgroup 0 spent in its loop; behind them every lane leaves one float so
// that the arithmetic cannot be dropped.
constexpr int kChains = 4;
__global__ __launch_bounds__(256, 2) void calib_mfma_kernel(float* __restrict__ out, int iters) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {  // operands with busy bit patterns, in [-1, 1): what toggles costs power
        const unsigned ha = (static_cast<unsigned>(threadIdx.x * 8 + i) + 1u) * 2654435761u;
        const unsigned hb = (static_cast<unsigned>(threadIdx.x * 8 + i) + 77u) * 2246822519u;
        a[i] = static_cast<__bf16>(static_cast<float>(ha >> 16) * (1.f / 32768.f) - 1.f);
        b[i] = static_cast<__bf16>(static_cast<float>(hb >> 16) * (1.f / 32768.f) - 1.f);
    }
    f32x16 acc[kChains];
    for (int c = 0; c < kChains; ++c)
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float sum = 0.f;
    for (int c = 0; c < kChains; ++c)
        for (int i = 0; i < 16; ++i) sum += acc[c][i];
    const long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        reinterpret_cast<unsigned long long*>(out)[0] = static_cast<unsigned long long>(c1 - c0);
        reinterpret_cast<unsigned long long*>(out)[1] = static_cast<unsigned long long>(w1 - w0);
    }
    out[4 + (blockIdx.x * 256ll + threadIdx.x) % 4096] = sum;
}

constexpr int kCalibBlocks = 256 * 2;  // two workgroups of four waves on each of the 256 compute units

}  // namespace pa

extern "C" int pa_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
    PA_REQUIRE(dst && src, "pa_calib_copy: NULL pointer");
    PA_REQUIRE(pa::aligned16(dst) && pa::aligned16(src) && bytes % 16 == 0 && bytes > 0,
               "pa_calib_copy: buffers and size must be multiples of 16 bytes");
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        pa::ProfScope prof(pa::kProfCalibCopy, s);
        hipLaunchKernelGGL(pa::calib_copy_kernel, dim3(256 * 32), dim3(256), 0, s, static_cast<pa::u32x4*>(dst),
                           static_cast<const pa::u32x4*>(src), static_cast<int64_t>(bytes / 16));
    }
    PA_HIP(hipGetLastError());
    return PA_OK;
}

extern "C" int pa_calib_mfma(void* out, size_t out_bytes, int iters, int64_t* flops, void* stream) {
    PA_REQUIRE(out && flops, "pa_calib_mfma: NULL pointer");
    PA_REQUIRE(out_bytes >= (4 + 4096) * sizeof(float) && pa::aligned16(out), "pa_calib_mfma: out needs %zu bytes, 16-byte aligned",
               (4 + 4096) * sizeof(float));
    PA_REQUIRE(iters > 0 && iters <= (1 << 24), "pa_calib_mfma: iters out of range");
    hipStream_t s = static_cast<hipStream_t>(stream);
    *flops = static_cast<int64_t>(pa::kCalibBlocks) * 4 * iters * pa::kChains * (2ll * 32 * 32 * 16);
    {
        pa::ProfScope prof(pa::kProfCalibMfma, s);
        hipLaunchKernelGGL(pa::calib_mfma_kernel, dim3(pa::kCalibBlocks), dim3(256), 0, s, static_cast<float*>(out), iters);
    }
    PA_HIP(hipGetLastError());
    return PA_OK;
}
