// Grouped bf16 MFMA GEMM for gfx950 with the rank-r LoRA update fused into the main loop.
//
// Every projection of the transformer block is y = x W^T (+ bias) with an optional LoRA
// term scale * (x A^T) B^T (Section 2, "Low-Rank Adaptation").  The down-projection
// t = scale * x A^T is a first, small GEMM; the up-projection then rides in the base
// GEMM's K loop: [x | t] [W | B]^T, i.e. a second K segment of length r.  Epilogues:
// bias, exact-erf GEGLU (Section 4.3's fused GEGLU), residual add, bf16 or fp32 store.
//
// Tiling: BM x BN output tile per workgroup, BK = 64, WGM x WGN wavefronts, each owning
// (BM/WGM) x (BN/WGN) as 32x32x16 bf16 MFMA tiles with fp32 accumulators.  Operand tiles
// go global -> registers -> LDS (16-byte chunks, XOR-swizzled so that the 32 rows one
// MFMA operand read touches fall in distinct banks) and are double-buffered: the global
// loads of tile t+1 are in flight while tile t is multiplied.
#include "common.hpp"

namespace sd {

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, int WGM, int WGN, bool GEGLU>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(const GemmGroup g) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int CHA = BM * 8 / NT, CHB = BN * 8 / NT;
    constexpr int RSTEP = NT / 8;   // rows between two chunks of one thread
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");
    static_assert(!GEGLU || (NI % 2 == 0), "GEGLU needs value/gate column-block pairs per wave");

    __shared__ u32x4 lds[2][(BM + BN) * 8];

    // ---- which problem, which tile ----
    const int tile = blockIdx.x;
    int pi = 0;
#pragma unroll 1
    for (int i = 1; i < g.n; ++i)
        if (tile >= g.p[i].tile_begin) pi = i;
    const GemmProblem& P = g.p[pi];
    const int local = tile - P.tile_begin;
    const int tn = local % P.tiles_n, tm = local / P.tiles_n;
    constexpr int BN_OUT = GEGLU ? BN / 2 : BN;
    const int m0 = tm * BM, n0 = tn * BN_OUT;
    const int Mp = P.Mp, N = P.N, K0 = P.K0, K1 = P.K1;
    const int nk0 = (K0 + 63) >> 6, nk1 = (K1 + 63) >> 6, nkt = nk0 + nk1;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
    const int lrow = tid >> 3, lc = tid & 7;

    // Q-operand (weight) row of tile row j.  GEGLU: 32-row blocks alternate value / gate
    // rows of the same 32 output columns, so one lane ends up holding both halves.
    auto qrow = [&](int j) -> int {
        if (GEGLU) {
            int blk = j >> 5;
            int col = n0 + (blk >> 1) * 32 + (j & 31);
            col = col < N ? col : N - 1;
            return col + ((blk & 1) ? P.geglu_F : 0);
        } else {
            int col = n0 + j;
            return col < N ? col : N - 1;
        }
    };

    const uint16_t* pa[CHA];
    const uint16_t* pb[CHB];
    auto setup = [&](int seg) {
        const uint16_t* pbase = seg ? P.p1 : P.p0;
        const uint16_t* qbase = seg ? P.q1 : P.q0;
        const int64_t ldp = seg ? P.ldp1 : P.ldp0, ldq = seg ? P.ldq1 : P.ldq0;
#pragma unroll
        for (int i = 0; i < CHA; ++i) {
            int r = m0 + lrow + i * RSTEP;
            r = r < Mp ? r : Mp - 1;
            pa[i] = pbase + (int64_t)r * ldp + lc * 8;
        }
#pragma unroll
        for (int i = 0; i < CHB; ++i) pb[i] = qbase + (int64_t)qrow(lrow + i * RSTEP) * ldq + lc * 8;
    };

    u32x4 ra[CHA], rb[CHB];
    auto load_tile = [&](int t) {
        if (t == nk0) setup(1);
        const int kt = t < nk0 ? t : t - nk0;
        const int Kseg = t < nk0 ? K0 : K1;
        const int kb = kt * 64;
        const bool kval = kb + lc * 8 < Kseg;   // K segments are multiples of 8
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < CHA; ++i) ra[i] = kval ? *reinterpret_cast<const u32x4*>(pa[i] + kb) : zero;
#pragma unroll
        for (int i = 0; i < CHB; ++i) rb[i] = kval ? *reinterpret_cast<const u32x4*>(pb[i] + kb) : zero;
    };
    auto store_lds = [&](int buf) {
        u32x4* la = lds[buf];
        u32x4* lb = lds[buf] + BM * 8;
#pragma unroll
        for (int i = 0; i < CHA; ++i) { int r = lrow + i * RSTEP; la[r * 8 + swz(r, lc)] = ra[i]; }
#pragma unroll
        for (int i = 0; i < CHB; ++i) { int r = lrow + i * RSTEP; lb[r * 8 + swz(r, lc)] = rb[i]; }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    setup(0);
    load_tile(0);
    store_lds(0);
    __syncthreads();

#pragma unroll 1
    for (int t = 0; t < nkt; ++t) {
        const bool more = t + 1 < nkt;
        if (more) load_tile(t + 1);
        const u32x4* la = lds[t & 1];
        const u32x4* lb = lds[t & 1] + BM * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                int r = wm + mi * 32 + l32;
                af[mi] = __builtin_bit_cast(bf16x8, la[r * 8 + swz(r, kk * 2 + hi)]);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                int r = wn + ni * 32 + l32;
                bfr[ni] = __builtin_bit_cast(bf16x8, lb[r * 8 + swz(r, kk * 2 + hi)]);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) store_lds((t + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue.  Accumulator layout of the 32x32 MFMA: lane holds column l32 and rows
    // 8*(v/4) + 4*hi + (v%4), v = 0..15. ----
    const float alpha = P.alpha;
    const uint16_t* bias = P.bias;
    auto emit = [&](int p, int q, float val) {
        if (p >= Mp || q >= N) return;
        if (bias) val += bf16_to_f32(bias[P.bias_on_rows ? p : q]);
        const int64_t oi = (int64_t)p * P.ldy + q;
        if (P.y_f32) {
            if (P.res) val += static_cast<const float*>(P.res)[(int64_t)p * P.ldr + q];
            static_cast<float*>(P.y)[oi] = val;
        } else {
            if (P.res) val += bf16_to_f32(static_cast<const uint16_t*>(P.res)[(int64_t)p * P.ldr + q]);
            static_cast<uint16_t*>(P.y)[oi] = (uint16_t)f32_to_bf16_bits(val);
        }
    };
    if constexpr (GEGLU) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < NI / 2; ++nj) {
                const int q = n0 + (wn >> 1) + nj * 32 + l32;
                float bv = 0.f, bg = 0.f;
                if (bias && q < N) { bv = bf16_to_f32(bias[q]); bg = bf16_to_f32(bias[q + P.geglu_F]); }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int p = m0 + wm + mi * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                    if (p < Mp && q < N) {
                        float val = alpha * acc[mi][2 * nj][v] + bv;
                        float gate = alpha * acc[mi][2 * nj + 1][v] + bg;
                        float ge = 0.5f * gate * (1.0f + erff(gate * 0.70710678118654752440f));
                        float o = val * ge;
                        const int64_t oi = (int64_t)p * P.ldy + q;
                        if (P.y_f32) static_cast<float*>(P.y)[oi] = o;
                        else static_cast<uint16_t*>(P.y)[oi] = (uint16_t)f32_to_bf16_bits(o);
                    }
                }
            }
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int p = m0 + wm + mi * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
                    const int q = n0 + wn + ni * 32 + l32;
                    emit(p, q, alpha * acc[mi][ni][v]);
                }
    }
}

template <int BM, int BN, int WGM, int WGN, bool GEGLU>
static int launch_cfg(GemmGroup& g, hipStream_t stream) {
    constexpr int BN_OUT = GEGLU ? BN / 2 : BN;
    int total = 0;
    for (int i = 0; i < g.n; ++i) {
        GemmProblem& P = g.p[i];
        P.tiles_m = (P.Mp + BM - 1) / BM;
        P.tiles_n = (P.N + BN_OUT - 1) / BN_OUT;
        P.tile_begin = total;
        total += P.tiles_m * P.tiles_n;
    }
    g.total_tiles = total;
    if (total == 0) return SD_OK;
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, GEGLU>), dim3(total), dim3(64 * WGM * WGN), 0, stream, g);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

int launch_gemm_group(GemmGroup& g, hipStream_t stream) {
    SD_REQUIRE(g.n >= 1 && g.n <= GEMM_MAX_PROBLEMS, SD_EINVAL, "gemm group: %d problems", g.n);
    bool geglu = g.p[0].geglu_F > 0;
    long tiles128 = 0, tiles256 = 0;
    int maxN = 0;
    for (int i = 0; i < g.n; ++i) {
        const GemmProblem& P = g.p[i];
        SD_REQUIRE((P.geglu_F > 0) == geglu, SD_EINVAL, "gemm group mixes GEGLU and plain problems");
        SD_REQUIRE(P.Mp >= 0 && P.N >= 0 && P.K0 > 0 && P.K0 % 8 == 0 && P.K1 >= 0 && P.K1 % 8 == 0, SD_EINVAL,
                   "gemm problem %d: bad sizes M=%d N=%d K0=%d K1=%d", i, P.Mp, P.N, P.K0, P.K1);
        SD_REQUIRE(P.p0 && P.q0 && P.y && (P.K1 == 0 || (P.p1 && P.q1)), SD_EINVAL, "gemm problem %d: null operand", i);
        SD_REQUIRE(P.ldp0 % 8 == 0 && P.ldq0 % 8 == 0 && (P.K1 == 0 || (P.ldp1 % 8 == 0 && P.ldq1 % 8 == 0)), SD_EINVAL,
                   "gemm problem %d: leading dimensions must be multiples of 8", i);
        if (P.Mp == 0 || P.N == 0) continue;
        int bo = geglu ? 64 : 128;
        tiles128 += (long)((P.Mp + 127) / 128) * ((P.N + bo - 1) / bo);
        tiles256 += (long)((P.Mp + 255) / 256) * ((P.N + bo - 1) / bo);
        if (P.N > maxN) maxN = P.N;
    }
    // drop empty problems
    int w = 0;
    for (int i = 0; i < g.n; ++i)
        if (g.p[i].Mp > 0 && g.p[i].N > 0) { if (w != i) g.p[w] = g.p[i]; ++w; }
    g.n = w;
    if (w == 0) return SD_OK;
    if (geglu) {
        if (tiles256 >= 512) return launch_cfg<256, 128, 2, 2, true>(g, stream);
        return launch_cfg<128, 128, 2, 2, true>(g, stream);
    }
    if (maxN <= 64) return launch_cfg<64, 64, 2, 2, false>(g, stream);
    if (tiles256 >= 512) return launch_cfg<256, 128, 2, 2, false>(g, stream);
    return launch_cfg<128, 128, 2, 2, false>(g, stream);
}

}  // namespace sd
