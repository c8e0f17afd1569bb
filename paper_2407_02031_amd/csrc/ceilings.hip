// Measured ceilings for the roofline figures, run on the same device as the kernels they
// are compared with: a register-resident bf16 MFMA loop (no memory traffic at all), the issue
// rates of the vector ALU, and a streaming fp32 copy (one read and one write per element).  Vendor peaks assume the boost
// clock and ideal DRAM efficiency; these two say what this part sustains.
#include "common.hpp"

namespace sd {

// 4 independent 32x32x16 accumulators per wavefront, operands with pseudo-random bit patterns
// (all-equal operands toggle fewer wires and clock higher than real data does)
__global__ __launch_bounds__(256) void ceiling_mfma_kernel(float* __restrict__ out, int iters) {
    bf16x8 a, b;
    uint32_t s = 0x9e3779b9u * (threadIdx.x + 1u) + blockIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        s = s * 1664525u + 1013904223u;
        a[i] = (__bf16)(((int)(s >> 20) - 2048) * (1.0f / 4096.0f));
        s = s * 1664525u + 1013904223u;
        b[i] = (__bf16)(((int)(s >> 20) - 2048) * (1.0f / 4096.0f));
    }
    f32x16 c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) r += c[j][0] + c[j][15];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

// Issue rates of the vector ALU, out of registers: MODE 0 a chain of v_exp_f32 per accumulator,
// MODE 1 a chain of v_fma_f32, MODE 2 one exponential and four FMAs per accumulator and trip, MODE 3
// two exponentials per accumulator and trip dealt between the four MFMAs of the matrix-core loop
// above (same operands, same trip).  Eight independent accumulators per lane, so latency is covered
// and the issue port is what is timed.  Attention's key loop leans on this port as much as on the
// matrix cores: what an exponential costs in FMA slots and whether the two overlap decides whether a
// polynomial on the FMA pipe could take exponentials off it; whether exponentials issue under
// running MFMAs decides how much of them the key loop can hide at all.
template <int MODE>
__global__ __launch_bounds__(256) void ceiling_valu_kernel(float* __restrict__ out, int iters) {
    float a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = 0.25f + 1e-4f * (float)threadIdx.x + (float)i;
        b[i] = 0.5f + (float)i;
    }
    if (MODE == 3) {
        bf16x8 pa, pb;
        uint32_t s = 0x9e3779b9u * (threadIdx.x + 1u) + blockIdx.x;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s = s * 1664525u + 1013904223u;
            pa[i] = (__bf16)(((int)(s >> 20) - 2048) * (1.0f / 4096.0f));
            s = s * 1664525u + 1013904223u;
            pb[i] = (__bf16)(((int)(s >> 20) - 2048) * (1.0f / 4096.0f));
        }
        f32x16 c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
#pragma unroll 1
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa, pb, c[j], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) a[(j & 1) * 4 + i] = __builtin_amdgcn_exp2f(-__builtin_fabsf(a[(j & 1) * 4 + i]));
            }
        }
        float r = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) r += c[j][0] + c[j][15];
#pragma unroll
        for (int i = 0; i < 8; ++i) r += a[i];
        out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
        return;
    }
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // 2^-|a| stays in (0, 1]: a pure chain of exponentials (sign and magnitude are operand modifiers)
            if (MODE == 0 || MODE == 2) a[i] = __builtin_amdgcn_exp2f(-__builtin_fabsf(a[i]));
            if (MODE == 1 || MODE == 2) {
#pragma unroll
                for (int j = 0; j < 4; ++j) b[i] = __builtin_fmaf(b[i], 0.999f, 0.001f);
            }
        }
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) r += a[i] + b[i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

constexpr int COPY_THREADS = 128;
__global__ __launch_bounds__(COPY_THREADS) void ceiling_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n4) {
    size_t i = (size_t)blockIdx.x * COPY_THREADS + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * COPY_THREADS;
    for (; i < n4; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// the patch pass's traffic mix as a plain stream: every element read once and written twice
__global__ __launch_bounds__(COPY_THREADS) void ceiling_copy_1r2w_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst0,
                                                                        f32x4* __restrict__ dst1, size_t n4) {
    size_t i = (size_t)blockIdx.x * COPY_THREADS + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * COPY_THREADS;
    for (; i < n4; i += stride) {
        const f32x4 v = __builtin_nontemporal_load(src + i);
        __builtin_nontemporal_store(v, dst0 + i);
        __builtin_nontemporal_store(v, dst1 + i);
    }
}

}  // namespace sd

using namespace sd;

extern "C" int sd_ceiling_mfma_bf16(float* out, int32_t workgroups, int32_t iters, double* flops, void* stream) {
    SD_REQUIRE(out && workgroups > 0 && iters > 0, SD_EINVAL, "ceiling_mfma: out=%p workgroups=%d iters=%d", (void*)out, workgroups, iters);
    hipLaunchKernelGGL(ceiling_mfma_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
    SD_HIP_CHECK(hipGetLastError());
    if (flops) *flops = (double)workgroups * 4.0 /*waves*/ * iters * 4.0 /*MFMAs*/ * (2.0 * 32 * 32 * 16);
    return SD_OK;
}

extern "C" int sd_ceiling_valu(float* out, int32_t workgroups, int32_t iters, int32_t mode, double* exps, double* fmas, void* stream) {
    SD_REQUIRE(out && workgroups > 0 && iters > 0 && mode >= 0 && mode <= 3, SD_EINVAL, "ceiling_valu: out=%p workgroups=%d iters=%d mode=%d",
               (void*)out, workgroups, iters, mode);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == 0) hipLaunchKernelGGL(ceiling_valu_kernel<0>, dim3((unsigned)workgroups), dim3(256), 0, s, out, iters);
    else if (mode == 1) hipLaunchKernelGGL(ceiling_valu_kernel<1>, dim3((unsigned)workgroups), dim3(256), 0, s, out, iters);
    else if (mode == 2) hipLaunchKernelGGL(ceiling_valu_kernel<2>, dim3((unsigned)workgroups), dim3(256), 0, s, out, iters);
    else hipLaunchKernelGGL(ceiling_valu_kernel<3>, dim3((unsigned)workgroups), dim3(256), 0, s, out, iters);
    SD_HIP_CHECK(hipGetLastError());
    const double groups = (double)workgroups * 4.0 /*waves*/ * iters * 8.0;   // wavefront-wide instructions: per accumulator and trip
    if (exps) *exps = mode == 1 ? 0.0 : (mode == 3 ? 2.0 * groups : groups);
    if (fmas) *fmas = (mode == 0 || mode == 3) ? 0.0 : 4.0 * groups;
    return SD_OK;
}

extern "C" int sd_ceiling_copy_f32(const float* src, float* dst, size_t n, void* stream) {
    SD_REQUIRE(src && dst && aligned16(src) && aligned16(dst), SD_EINVAL, "ceiling_copy: pointers must be non-null and 16-byte aligned");
    SD_REQUIRE(n % 4 == 0, SD_EINVAL, "ceiling_copy: n must be a multiple of 4");
    if (n == 0) return SD_OK;
    const size_t n4 = n / 4;
    size_t wgs = (n4 + COPY_THREADS - 1) / COPY_THREADS;
    if (wgs > 131072) wgs = 131072;
    // 20 KB of dynamic LDS nobody touches: eight 128-thread workgroups per CU.  With every wave
    // slot filled the same copy is 10-15 % slower at footprints past the last-level cache (too many
    // streams in flight for HBM), and this is meant to be the best plain copy the machine does:
    // of 256 threads x 32/40/48 KB and 128 threads x 16/20/24 KB this shape measured fastest
    // (6.4 TB/s at 1 GiB, 6.15 TB/s at 3.1 GiB on one machine, 3-4 % above the others).
    hipLaunchKernelGGL(ceiling_copy_kernel, dim3((unsigned)wgs), dim3(COPY_THREADS), 20 * 1024, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const f32x4*>(src), reinterpret_cast<f32x4*>(dst), n4);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_ceiling_copy_1r2w_f32(const float* src, float* dst0, float* dst1, size_t n, void* stream) {
    SD_REQUIRE(src && dst0 && dst1 && aligned16(src) && aligned16(dst0) && aligned16(dst1), SD_EINVAL,
               "ceiling_copy_1r2w: pointers must be non-null and 16-byte aligned");
    SD_REQUIRE(n % 4 == 0, SD_EINVAL, "ceiling_copy_1r2w: n must be a multiple of 4");
    if (n == 0) return SD_OK;
    const size_t n4 = n / 4;
    size_t wgs = (n4 + COPY_THREADS - 1) / COPY_THREADS;
    if (wgs > 131072) wgs = 131072;
    // same launch shape as the plain copy (it measured best for this one too: 16 / 20 / 24 / 32 KB caps gave
    // 5.50 / 5.59 / 5.50 / 5.04 TB/s at 3.1 GiB per buffer)
    hipLaunchKernelGGL(ceiling_copy_1r2w_kernel, dim3((unsigned)wgs), dim3(COPY_THREADS), 20 * 1024, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const f32x4*>(src), reinterpret_cast<f32x4*>(dst0), reinterpret_cast<f32x4*>(dst1), n4);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}
