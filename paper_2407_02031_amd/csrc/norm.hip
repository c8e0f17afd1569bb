// LayerNorm (per token) and token-major GroupNorm(32) for gfx950, plus the dtype
// converters at the stack boundary.  All statistics in fp32, biased variance, two passes
// over register-resident (LayerNorm) or shift-centred (GroupNorm) data.  HBM-bound.
#include "common.hpp"

namespace sd {

// ---------------------------------------------------------------------------------------
// LayerNorm: one wavefront per row, the row lives in registers (C <= 2048, C % 4 == 0).
// ---------------------------------------------------------------------------------------
constexpr int LN_MAXJ = 8;   // float4 chunks per lane: 64 lanes * 4 * 8 = 2048 channels

// JN: chunks per lane the row needs (C <= 256 * JN); R: rows per wavefront, all of whose loads
// are issued before the first is used (the kernel is a stream: bytes in flight are what counts).
// zero_ptr/zero_n: flags that a later launch of the same call expects to find cleared.
template <bool XF32, int JN, int R>
__global__ __launch_bounds__(256) void layernorm_kernel(const void* __restrict__ xv, const uint16_t* __restrict__ gamma,
                                                        const uint16_t* __restrict__ beta, float eps,
                                                        uint16_t* __restrict__ y, int M, int C, int32_t* zero_ptr, int zero_n) {
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < zero_n; i += 256) zero_ptr[i] = 0;
    const int lane = threadIdx.x & 63;
    const int row0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * R;
    if (row0 >= M) return;
    const int nch = C >> 2;   // 4-element chunks per row
    float v[R][JN][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = min(row0 + r, M - 1);   // rows past the end repeat the last one and are not stored
#pragma unroll
        for (int j = 0; j < JN; ++j) {
            const int ch = lane + j * 64;
            if (ch < nch) {
                if (XF32) {
                    const float4 t = reinterpret_cast<const float4*>(static_cast<const float*>(xv) + (size_t)row * C)[ch];
                    v[r][j][0] = t.x; v[r][j][1] = t.y; v[r][j][2] = t.z; v[r][j][3] = t.w;
                } else {
                    const uint2 t = reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(xv) + (size_t)row * C)[ch];
                    v[r][j][0] = bf16lo_to_f32(t.x); v[r][j][1] = bf16hi_to_f32(t.x);
                    v[r][j][2] = bf16lo_to_f32(t.y); v[r][j][3] = bf16hi_to_f32(t.y);
                }
            } else {
                v[r][j][0] = v[r][j][1] = v[r][j][2] = v[r][j][3] = 0.f;
            }
        }
    }
    uint2 gg[JN], bb[JN];
#pragma unroll
    for (int j = 0; j < JN; ++j) {
        const int ch = lane + j * 64;
        gg[j] = ch < nch ? reinterpret_cast<const uint2*>(gamma)[ch] : make_uint2(0, 0);
        bb[j] = ch < nch ? reinterpret_cast<const uint2*>(beta)[ch] : make_uint2(0, 0);
    }
    const float inv_c = 1.0f / (float)C;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // One pass over the registers for both moments, taken about the row's first element (a
        // sample of the row, so the variance below loses no digits to a large common offset),
        // and one reduction for the pair.
        const float shift = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v[r][0][0])));
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < JN; ++j) {
            const int ch = lane + j * 64;
            if (ch < nch) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[r][j][e] -= shift;
                    s1 += v[r][j][e];
                    s2 += v[r][j][e] * v[r][j][e];
                }
            }
        }
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        const float dmean = s1 * inv_c;                      // mean - shift
        const float var = fmaxf(s2 * inv_c - dmean * dmean, 0.f);
        const float rstd = rsqrtf(var + eps);
        if (row0 + r < M) {
#pragma unroll
            for (int j = 0; j < JN; ++j) {
                const int ch = lane + j * 64;
                if (ch < nch) {
                    const float o0 = (v[r][j][0] - dmean) * rstd * bf16lo_to_f32(gg[j].x) + bf16lo_to_f32(bb[j].x);
                    const float o1 = (v[r][j][1] - dmean) * rstd * bf16hi_to_f32(gg[j].x) + bf16hi_to_f32(bb[j].x);
                    const float o2 = (v[r][j][2] - dmean) * rstd * bf16lo_to_f32(gg[j].y) + bf16lo_to_f32(bb[j].y);
                    const float o3 = (v[r][j][3] - dmean) * rstd * bf16hi_to_f32(gg[j].y) + bf16hi_to_f32(bb[j].y);
                    uint2 o;
                    o.x = pack_bf16x2(o0, o1);
                    o.y = pack_bf16x2(o2, o3);
                    reinterpret_cast<uint2*>(y + (size_t)(row0 + r) * C)[ch] = o;
                }
            }
        }
    }
}

// rows per wavefront: whole-step timings favour one (more, smaller workgroups) over two or four
constexpr int LN_ROWS = 1;
template <bool XF32, int JN, int R>
static void launch_ln(const void* x, const uint16_t* gamma, const uint16_t* beta, float eps, uint16_t* y, int M, int C,
                      int32_t* zero_ptr, int zero_n, hipStream_t stream) {
    hipLaunchKernelGGL((layernorm_kernel<XF32, JN, R>), dim3((M + 4 * R - 1) / (4 * R)), dim3(256), 0, stream, x, gamma, beta, eps, y, M, C,
                       zero_ptr, zero_n);
}

int launch_layernorm(const void* x, int x_f32, const uint16_t* gamma, const uint16_t* beta, float eps,
                     uint16_t* y, int M, int C, hipStream_t stream, int32_t* zero_ptr, int zero_n) {
    SD_REQUIRE(C % 4 == 0 && C > 0 && C <= 64 * 4 * LN_MAXJ, SD_EUNSUPPORTED, "layernorm: C=%d (need C %% 4 == 0, C <= %d)", C,
               64 * 4 * LN_MAXJ);
    if (M <= 0) return zero_n > 0 ? launch_clear_flags(zero_ptr, zero_n, stream) : SD_OK;
    if (C <= 768) {          // SDXL's 320 and 640 channels: three chunks per lane
        if (x_f32) launch_ln<true, 3, LN_ROWS>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
        else launch_ln<false, 3, LN_ROWS>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
    } else if (C <= 1280) {
        if (x_f32) launch_ln<true, 5, 1>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
        else launch_ln<false, 5, 1>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
    } else {
        if (x_f32) launch_ln<true, LN_MAXJ, 1>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
        else launch_ln<false, LN_MAXJ, 1>(x, gamma, beta, eps, y, M, C, zero_ptr, zero_n, stream);
    }
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

// ---------------------------------------------------------------------------------------
// dtype converters (n % 4 == 0 handled by the tail loop)
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cvt_bf16_f32_kernel(const uint16_t* __restrict__ x, float* __restrict__ y, size_t n) {
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i + 3 < n) {
        const uint2 t = *reinterpret_cast<const uint2*>(x + i);
        float4 o = {bf16lo_to_f32(t.x), bf16hi_to_f32(t.x), bf16lo_to_f32(t.y), bf16hi_to_f32(t.y)};
        *reinterpret_cast<float4*>(y + i) = o;
    } else {
        for (; i < n; ++i) y[i] = bf16_to_f32(x[i]);
    }
}
__global__ __launch_bounds__(256) void cvt_f32_bf16_kernel(const float* __restrict__ x, uint16_t* __restrict__ y, size_t n) {
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i + 3 < n) {
        const float4 t = *reinterpret_cast<const float4*>(x + i);
        uint2 o;
        o.x = pack_bf16x2(t.x, t.y);
        o.y = pack_bf16x2(t.z, t.w);
        *reinterpret_cast<uint2*>(y + i) = o;
    } else {
        for (; i < n; ++i) y[i] = (uint16_t)f32_to_bf16_bits(x[i]);
    }
}
int launch_cvt_bf16_to_f32(const uint16_t* x, float* y, size_t n, hipStream_t stream) {
    if (!n) return SD_OK;
    hipLaunchKernelGGL(cvt_bf16_f32_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, stream, x, y, n);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}
int launch_cvt_f32_to_bf16(const float* x, uint16_t* y, size_t n, hipStream_t stream) {
    if (!n) return SD_OK;
    hipLaunchKernelGGL(cvt_f32_bf16_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, stream, x, y, n);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

// ---------------------------------------------------------------------------------------
// GroupNorm, token-major [Bn, T, C].  Pass 1: per (sample, chunk of 64 tokens, group) sums of
// (x - shift) and (x - shift)^2 with shift = the group's first element in the sample
// (shifted-data variance: no catastrophic cancellation for data with a large mean).
// Pass 2: every workgroup combines the chunk partials of its sample in a fixed order (a few
// KB through LDS, so there is no finalize launch in between) and normalises its tokens.
// Thread t of a block owns channel pair (2t, 2t+1); groups hold an even number of channels.
// ---------------------------------------------------------------------------------------
constexpr int GN_TCHUNK = 8;    // tokens per apply block and per inner step of the partial pass: every load of a thread in flight at once
constexpr int GN_PCHUNK_MIN = 32;    // tokens per partial-sum block ...
constexpr int GN_MAX_PCHUNKS = 128;  // ... more for long samples, so that a sample never has more blocks than this

__global__ void groupnorm_partial_kernel(const uint16_t* __restrict__ x, float* __restrict__ partials,
                                         int T, int C, int groups, int nchunks, int pchunk) {
    extern __shared__ float sh[];   // [C/2][2]
    const int b = blockIdx.y, chunk = blockIdx.x;
    const int cp = threadIdx.x;
    const int cpg = C / groups;
    const int npairs = C >> 1;
    const uint16_t* xb = x + (size_t)b * T * C;
    const int t0 = chunk * pchunk;
    const int t1 = min(T, t0 + pchunk);
    float s1 = 0.f, s2 = 0.f;
    if (cp < npairs) {
        const int g = (2 * cp) / cpg;
        const float shift = bf16_to_f32(xb[g * cpg]);
        int t = t0;
        for (; t + GN_TCHUNK <= t1; t += GN_TCHUNK) {
            uint32_t pr[GN_TCHUNK];
#pragma unroll
            for (int i = 0; i < GN_TCHUNK; ++i) pr[i] = reinterpret_cast<const uint32_t*>(xb + (size_t)(t + i) * C)[cp];
#pragma unroll
            for (int i = 0; i < GN_TCHUNK; ++i) {
                const float a = bf16lo_to_f32(pr[i]) - shift, c = bf16hi_to_f32(pr[i]) - shift;
                s1 += a + c;
                s2 += a * a + c * c;
            }
        }
        for (; t < t1; ++t) {
            const uint32_t pr = reinterpret_cast<const uint32_t*>(xb + (size_t)t * C)[cp];
            const float a = bf16lo_to_f32(pr) - shift, c = bf16hi_to_f32(pr) - shift;
            s1 += a + c;
            s2 += a * a + c * c;
        }
        sh[2 * cp] = s1;
        sh[2 * cp + 1] = s2;
    }
    __syncthreads();
    if (cp < groups) {
        const int ppg = cpg >> 1;
        float a1 = 0.f, a2 = 0.f;
        for (int i = 0; i < ppg; ++i) { a1 += sh[2 * (cp * ppg + i)]; a2 += sh[2 * (cp * ppg + i) + 1]; }
        float* o = partials + (((size_t)b * nchunks + chunk) * groups + cp) * 2;
        o[0] = a1;
        o[1] = a2;
    }
}

// SILU: y = n * sigmoid(n) on the normalised value, the GroupNorm + SiLU pair of the base model's
// ResNet blocks as one operator (Section 4.3, "Kernel-level optimizations")
template <bool SILU>
__global__ void groupnorm_apply_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ y,
                                       const uint16_t* __restrict__ gamma, const uint16_t* __restrict__ beta,
                                       const float* __restrict__ partials, int T, int C, int groups, int nchunks, float eps) {
    extern __shared__ float sh[];   // [nchunks * groups][2] partials of this sample + [8 * groups][2] run sums, then [groups][2] (mean, rstd)
    const int b = blockIdx.y, chunk = blockIdx.x;
    const int cp = threadIdx.x;
    const int cpg = C / groups;
    const int npairs = C >> 1;
    const uint16_t* xb = x + (size_t)b * T * C;
    uint16_t* yb = y + (size_t)b * T * C;
    // this thread's inputs first: they are in flight while the statistics are put together
    const int t0 = chunk * GN_TCHUNK;
    const int t1 = min(T, t0 + GN_TCHUNK);
    uint32_t pr[GN_TCHUNK];
#pragma unroll
    for (int i = 0; i < GN_TCHUNK; ++i)
        pr[i] = (cp < npairs && t0 + i < t1) ? reinterpret_cast<const uint32_t*>(xb + (size_t)(t0 + i) * C)[cp] : 0u;
    // ---- statistics of the sample's groups: chunk partials summed in chunk order
    {
        const int np = nchunks * groups;
        const float2* src = reinterpret_cast<const float2*>(partials) + (size_t)b * np;
        float2* dst = reinterpret_cast<float2*>(sh);
        for (int i = cp; i < np; i += blockDim.x) dst[i] = src[i];
        __syncthreads();
        // group g's chunks are summed in `split` contiguous runs by `split` threads, and the runs
        // then in run order: a fixed order for a given shape, and no long serial chain
        const int split = min(8, (int)blockDim.x / groups);
        const int run = (nchunks + split - 1) / split;
        float2* sub = dst + np;   // [split][groups]
        if (cp < split * groups) {
            const int g = cp % groups, part = cp / groups;
            float a1 = 0.f, a2 = 0.f;
            for (int c = part * run; c < min(nchunks, (part + 1) * run); ++c) { a1 += dst[c * groups + g].x; a2 += dst[c * groups + g].y; }
            sub[part * groups + g] = make_float2(a1, a2);
        }
        __syncthreads();
        float mean = 0.f, rstd = 0.f;
        if (cp < groups) {
            float a1 = 0.f, a2 = 0.f;
            for (int p = 0; p < split; ++p) { a1 += sub[p * groups + cp].x; a2 += sub[p * groups + cp].y; }
            const float n = (float)T * (float)cpg;
            const float m1 = a1 / n;
            const float var = fmaxf(a2 / n - m1 * m1, 0.f);
            mean = bf16_to_f32(xb[cp * cpg]) + m1;
            rstd = rsqrtf(var + eps);
        }
        __syncthreads();
        if (cp < groups) { sh[2 * cp] = mean; sh[2 * cp + 1] = rstd; }
        __syncthreads();
    }
    if (cp >= npairs) return;
    const int g = (2 * cp) / cpg;
    const float mean = sh[2 * g], rstd = sh[2 * g + 1];
    const uint32_t gg = reinterpret_cast<const uint32_t*>(gamma)[cp];
    const uint32_t bb = reinterpret_cast<const uint32_t*>(beta)[cp];
    const float g0 = bf16lo_to_f32(gg) * rstd, g1 = bf16hi_to_f32(gg) * rstd;
    const float b0 = bf16lo_to_f32(bb), b1 = bf16hi_to_f32(bb);
#pragma unroll
    for (int i = 0; i < GN_TCHUNK; ++i) {
        if (t0 + i >= t1) break;
        float o0 = (bf16lo_to_f32(pr[i]) - mean) * g0 + b0;
        float o1 = (bf16hi_to_f32(pr[i]) - mean) * g1 + b1;
        if (SILU) {
            o0 = o0 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * o0));
            o1 = o1 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * o1));
        }
        reinterpret_cast<uint32_t*>(yb + (size_t)(t0 + i) * C)[cp] = pack_bf16x2(o0, o1);
    }
}

// tokens per partial-sum block for samples of T tokens
static int groupnorm_pchunk(int T) {
    int p = (T + GN_MAX_PCHUNKS - 1) / GN_MAX_PCHUNKS;
    p = (p + GN_TCHUNK - 1) / GN_TCHUNK * GN_TCHUNK;
    return p < GN_PCHUNK_MIN ? GN_PCHUNK_MIN : p;
}

size_t groupnorm_partials_bytes(int Bn, int T, int groups) {
    (void)T;
    return round_up((size_t)Bn * GN_MAX_PCHUNKS * groups * 2 * sizeof(float), 256);
}

int launch_groupnorm(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta,
                     int Bn, int T, int C, int groups, float eps, float* partials, hipStream_t stream, bool silu) {
    SD_REQUIRE(groups > 0 && C % groups == 0 && (C / groups) % 2 == 0, SD_EUNSUPPORTED,
               "groupnorm: C=%d groups=%d (need an even number of channels per group)", C, groups);
    SD_REQUIRE(C <= 2048, SD_EUNSUPPORTED, "groupnorm: C=%d > 2048", C);
    if (Bn <= 0 || T <= 0) return SD_OK;
    const int pchunk = groupnorm_pchunk(T);
    const int nchunks = (T + pchunk - 1) / pchunk;
    // the apply pass keeps one sample's chunk partials in LDS
    const size_t stats_lds = ((size_t)nchunks * groups + 8 * groups) * 2 * sizeof(float);
    SD_REQUIRE(nchunks <= GN_MAX_PCHUNKS && stats_lds <= 64 * 1024, SD_EUNSUPPORTED, "groupnorm: T=%d groups=%d exceed the statistics buffer (%zu bytes of LDS)", T,
               groups, stats_lds);
    int threads = ((C / 2 + 63) / 64) * 64;
    if (threads < 64) threads = 64;
    if (threads < groups) threads = ((groups + 63) / 64) * 64;
    hipLaunchKernelGGL(groupnorm_partial_kernel, dim3(nchunks, Bn), dim3(threads), (size_t)C * sizeof(float), stream, x, partials, T, C, groups, nchunks, pchunk);
    SD_HIP_CHECK(hipGetLastError());
    const dim3 grid((T + GN_TCHUNK - 1) / GN_TCHUNK, Bn);
    if (silu) hipLaunchKernelGGL(groupnorm_apply_kernel<true>, grid, dim3(threads), stats_lds, stream, x, y, gamma, beta, partials, T, C, groups, nchunks, eps);
    else hipLaunchKernelGGL(groupnorm_apply_kernel<false>, grid, dim3(threads), stats_lds, stream, x, y, gamma, beta, partials, T, C, groups, nchunks, eps);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

}  // namespace sd
