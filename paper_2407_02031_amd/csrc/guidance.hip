// Classifier-free-guidance weighted sum of the two denoised latents of a step (Section 2,
// "Diffusion model inference"): out = eps_u + g * (eps_c - eps_u).  Elementwise and tiny (an
// SDXL latent is 128 KiB); one 16-byte load per input per lane, explicit single roundings so
// the result matches the fp32 chain fl32(eps_u + fl32(g * fl32(eps_c - eps_u))) exactly.
// Also here: the sum of ControlNet outputs added to a backbone tensor (further down).
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

// Sum of the ControlNets' outputs for one injection point, added to the backbone tensor
// (Section 2, "ControlNet"): out = h + (r_1 + ... + r_n), the sum first, left to right, one
// fp32 rounding per addition.  Streaming: n + 1 reads and one write of 2 bytes per element.
struct ResidualPtrs { const uint16_t* r[SD_CONTROLNET_MAX]; };

template <int NR>
__device__ __forceinline__ float residual_sum(const float (&v)[SD_CONTROLNET_MAX]) {
    float s = v[0];
#pragma unroll
    for (int i = 1; i < NR; ++i) s = __fadd_rn(s, v[i]);
    return s;
}

template <int NR>
__global__ __launch_bounds__(256) void controlnet_residual_add_kernel(const uint16_t* __restrict__ h, const ResidualPtrs rp,
                                                                       uint16_t* __restrict__ out, size_t n, int vec) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= n) return;
    if (vec && i + 8 <= n) {
        u32x4 r[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) r[k] = *reinterpret_cast<const u32x4*>(rp.r[k] + i);
        const u32x4 a = *reinterpret_cast<const u32x4*>(h + i);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float lo[SD_CONTROLNET_MAX], hi[SD_CONTROLNET_MAX];
#pragma unroll
            for (int k = 0; k < NR; ++k) { lo[k] = bf16lo_to_f32(r[k][e]); hi[k] = bf16hi_to_f32(r[k][e]); }
            o[e] = pack_bf16x2(__fadd_rn(bf16lo_to_f32(a[e]), residual_sum<NR>(lo)), __fadd_rn(bf16hi_to_f32(a[e]), residual_sum<NR>(hi)));
        }
        *reinterpret_cast<u32x4*>(out + i) = o;
    } else {
        for (size_t j = i; j < n && j < i + 8; ++j) {
            float v[SD_CONTROLNET_MAX];
#pragma unroll
            for (int k = 0; k < NR; ++k) v[k] = bf16_to_f32(rp.r[k][j]);
            out[j] = (uint16_t)f32_to_bf16_bits(__fadd_rn(bf16_to_f32(h[j]), residual_sum<NR>(v)));
        }
    }
}

template <int NR>
static void launch_residual_add(const uint16_t* h, const ResidualPtrs& rp, uint16_t* out, size_t n, int vec, unsigned wgs, hipStream_t stream) {
    hipLaunchKernelGGL((controlnet_residual_add_kernel<NR>), dim3(wgs), dim3(256), 0, stream, h, rp, out, n, vec);
}

}  // namespace sd

using namespace sd;

extern "C" int sd_controlnet_residual_add(const uint16_t* h, const uint16_t* const* residuals, int32_t n_res, uint16_t* out, size_t n, void* stream) {
    SD_REQUIRE(n_res >= 0 && n_res <= SD_CONTROLNET_MAX, SD_EINVAL, "controlnet_residual_add: %d residuals (0..%d)", n_res, SD_CONTROLNET_MAX);
    if (n == 0) return SD_OK;
    SD_REQUIRE(h && out && (n_res == 0 || residuals), SD_EINVAL, "controlnet_residual_add: null pointer");
    ResidualPtrs rp = {};
    int vec = aligned16(h) && aligned16(out);
    for (int i = 0; i < n_res; ++i) {
        SD_REQUIRE(residuals[i], SD_EINVAL, "controlnet_residual_add: residual %d is null", i);
        rp.r[i] = residuals[i];
        vec = vec && aligned16(residuals[i]);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_res == 0) {   // nothing to add: out = h
        if (out != h) SD_HIP_CHECK(hipMemcpyAsync(out, h, n * sizeof(uint16_t), hipMemcpyDeviceToDevice, st));
        return SD_OK;
    }
    const size_t wgs = (n + 2047) / 2048;
    SD_REQUIRE(wgs < 0x7fffffffu, SD_EUNSUPPORTED, "controlnet_residual_add: n too large");
    switch (n_res) {
        case 1: launch_residual_add<1>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 2: launch_residual_add<2>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 3: launch_residual_add<3>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 4: launch_residual_add<4>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 5: launch_residual_add<5>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 6: launch_residual_add<6>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        case 7: launch_residual_add<7>(h, rp, out, n, vec, (unsigned)wgs, st); break;
        default: launch_residual_add<8>(h, rp, out, n, vec, (unsigned)wgs, st); break;
    }
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

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
