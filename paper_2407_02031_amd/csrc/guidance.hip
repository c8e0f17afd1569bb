// Classifier-free-guidance weighted sum of the two denoised latents of a step (Section 2,
// "Diffusion model inference"): out = eps_u + g * (eps_c - eps_u).  Elementwise and tiny (an
// SDXL latent is 128 KiB); one 16-byte load per input per lane, explicit single roundings so
// the result matches the fp32 chain fl32(eps_u + fl32(g * fl32(eps_c - eps_u))) exactly.
#include "common.hpp"

namespace sd {

__global__ __launch_bounds__(256) void cfg_combine_kernel(const uint16_t* __restrict__ eu, const uint16_t* __restrict__ ec, float g,
                                                          uint16_t* __restrict__ out, size_t n, int vec) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= n) return;
    if (vec && i + 8 <= n) {
        const u32x4 a = *reinterpret_cast<const u32x4*>(eu + i);
        const u32x4 b = *reinterpret_cast<const u32x4*>(ec + i);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float u0 = bf16lo_to_f32(a[e]), u1 = bf16hi_to_f32(a[e]);
            const float c0 = bf16lo_to_f32(b[e]), c1 = bf16hi_to_f32(b[e]);
            const float r0 = __fadd_rn(u0, __fmul_rn(g, __fsub_rn(c0, u0)));
            const float r1 = __fadd_rn(u1, __fmul_rn(g, __fsub_rn(c1, u1)));
            o[e] = pack_bf16x2(r0, r1);
        }
        *reinterpret_cast<u32x4*>(out + i) = o;
    } else {
        for (size_t j = i; j < n && j < i + 8; ++j) {
            const float u = bf16_to_f32(eu[j]), c = bf16_to_f32(ec[j]);
            out[j] = (uint16_t)f32_to_bf16_bits(__fadd_rn(u, __fmul_rn(g, __fsub_rn(c, u))));
        }
    }
}

}  // namespace sd

using namespace sd;

extern "C" int sd_cfg_combine(const uint16_t* eps_uncond, const uint16_t* eps_cond, float guidance, uint16_t* out, size_t n, void* stream) {
    if (n == 0) return SD_OK;
    SD_REQUIRE(eps_uncond && eps_cond && out, SD_EINVAL, "cfg_combine: null pointer");
    const int vec = aligned16(eps_uncond) && aligned16(eps_cond) && aligned16(out);
    const size_t wgs = (n + 2047) / 2048;
    SD_REQUIRE(wgs < 0x7fffffffu, SD_EUNSUPPORTED, "cfg_combine: n too large");
    hipLaunchKernelGGL(cfg_combine_kernel, dim3((unsigned)wgs), dim3(256), 0, static_cast<hipStream_t>(stream), eps_uncond, eps_cond, guidance, out, n, vec);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}
