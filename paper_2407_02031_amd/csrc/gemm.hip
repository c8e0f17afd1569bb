// Grouped bf16 MFMA GEMM for gfx950 with the rank-r LoRA update fused into the main loop.
//
// Every projection of the transformer block is y = x W^T (+ bias) with an optional LoRA
// term scale * (x A^T) B^T (Section 2, "Low-Rank Adaptation").  The down-projection
// t = scale * x A^T is a small GEMM of its own; the up-projection then rides in the base
// GEMM's K loop: [x | t] [W | B]^T, i.e. a second K segment of length r.  Both run in one
// launch: the down-projection's tiles come first in the grid and raise a flag per row block,
// and a base-GEMM tile looks at its flag only when it reaches the second K segment.
// Epilogues: bias, exact-erf GEGLU (Section 4.3's fused GEGLU), residual add, bf16 or fp32
// store.
//
// Tiling: BM x BN output tile per workgroup, BK = 64, WGM x WGN wavefronts, each owning
// (BM/WGM) x (BN/WGN) as 32x32x16 bf16 MFMA tiles with fp32 accumulators.
// Pipeline: operand tiles go global -> LDS directly (wave-wide 1 KB loads of 16-byte
// chunks, XOR-swizzled so the 32 rows one MFMA operand read touches fall in distinct
// banks) into a ring of STAGES tiles, STAGES-1 of them in flight ahead of the one being
// multiplied; inside a tile the operand fragments of k-step kk+1 are read from LDS while
// the MFMAs of k-step kk run.  The epilogue stages 32-row x 64-column pieces of a wave's
// accumulators through LDS so that global stores (and residual loads) are 16-byte rows.
#include "common.hpp"

namespace sd {

// XOR swizzle of the 16-byte chunk index inside an LDS row of CPR chunks (8: 128-byte rows,
// 4: 64-byte rows): any 16 consecutive rows put the same logical chunk in 16 distinct
// 16-byte slots of a 256-byte bank window.
template <int CPR>
__device__ __forceinline__ int swz(int row, int chunk) {
    return CPR == 8 ? (chunk ^ ((row >> 1) & 7)) : (chunk ^ ((row >> 2) & 3));
}

// GELU, exact (erf) form, with erf by Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7, far below
// bf16 resolution): erf(|x|) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p |x|).
// With x = z / sqrt(2) and h = z / 2:  gelu(z) = h (1 + erf(x)) = h + |h| erf(|x|), because erf is
// odd and h has the sign of x: no sign transfer, and sqrt(1/2) folds into the constants.
__device__ __forceinline__ float gelu_erf(float z) {
    const float az = fabsf(z);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, az, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f((-0.5f * 1.44269504088896340736f * z) * z);
    const float r = fmaf(-p, e, 1.0f);          // erf(|x|) in [0, 1]
    const float h = 0.5f * z;
    return fmaf(fabsf(h), r, h);
}

constexpr int EPI_STRIDE = 72;   // floats per staged row: 4 rows apart differ by 128 B mod 256 (no bank overlap)

// 256 bytes of zeros: where the lanes of a direct-to-LDS load point when their chunk lies
// past the end of a K segment (the load itself cannot zero-fill)
__device__ __attribute__((aligned(256))) uint32_t g_gemm_zeros[64];

// One direct global -> LDS load: every lane fetches 16 bytes from its own global address and
// the wavefront's 64 pieces land contiguously at LDS byte address `lds_base` (wave-uniform).
// Written as inline assembly so that the compiler does not serialise the LDS reads of the
// tile being multiplied behind loads that target another ring stage; completion is tracked
// by hand with vmcnt (loads retire in order) and a workgroup barrier.
// DEV: the load is of device scope (it must observe data that a workgroup on another XCD, with
// its own L2, wrote during this launch with device-scope stores).
template <bool DEV = false>
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
    if (DEV)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off sc1" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(gptr) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(gptr) : "memory", "m0");
}
// Same with a wave-uniform 64-bit base and a 32-bit unsigned byte offset per lane, which
// keeps the per-step address arithmetic on the scalar unit.
template <bool DEV = false>
__device__ __forceinline__ void dma16_so(const void* sbase, uint32_t voff, uint32_t lds_base) {
    if (DEV)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 sc1" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(voff), "s"(uniform_ptr(sbase)) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(voff), "s"(uniform_ptr(sbase)) : "memory", "m0");
}
// Tiles that gave up waiting for a producer's flag (never, unless the dependency protocol is
// broken): the wait is bounded so that every wavefront exits whatever happens.
__device__ unsigned long long g_gemm_dep_timeouts = 0;
constexpr int DEP_SPIN_LIMIT = 1 << 19;
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Tiles of signalling problems (down-projections, N = rank) run a body of their own inside the
// same kernel: BN = 64 instead of the launch's BN, which frees LDS for a deeper ring.  Other
// tiles of the launch wait for these, and what a down-projection tile spends is latency per
// k-step, so tiles in flight are what shortens it.
constexpr int DOWN_BN = 64;
template <int BM, int BN, int BK, int STAGES>
constexpr int down_stages() {
    if (BN <= DOWN_BN) return STAGES;
    const int fit = STAGES * (BM + BN) / (BM + DOWN_BN);   // stages of the narrower tile in the same bytes
    return fit > 5 ? 5 : (fit < 3 ? 3 : fit);
}
template <int BM, int BN, int BK, int WGM, int WGN, int STAGES>
constexpr int gemm_lds_chunks() {
    constexpr int ring = STAGES * (BM + BN) * (BK / 8);
    constexpr int dring = down_stages<BM, BN, BK, STAGES>() * (BM + (BN < DOWN_BN ? BN : DOWN_BN)) * (BK / 8);
    constexpr int epi = WGM * WGN * 32 * EPI_STRIDE / 4;
    constexpr int m = ring > dring ? ring : dring;
    return m > epi ? m : epi;
}

// GUARD: K segments that are not multiples of 64 (tail chunks read zeros).
// Two workgroups per CU whenever the ring leaves room for it (LDS <= 80 KB): the register
// budget is then 256 per lane (accumulators in AGPRs, the rest in VGPRs).
template <int BM, int BN, int BK, int WGM, int WGN, int STAGES>
constexpr int gemm_min_waves() {
    return gemm_lds_chunks<BM, BN, BK, WGM, WGN, STAGES>() * 16 <= 80 * 1024 ? 2 : 1;
}

template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, bool GEGLU, bool GUARD, bool RES32>
__device__ __forceinline__ void gemm_tile(const GemmProblem& P, const int tile, u32x4* const lds) {
    constexpr int NW = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MI = WM / 32, NI = WN / 32;
    constexpr int CPR = BK / 8;                // 16-byte chunks per LDS row
    constexpr int RPB = 64 / CPR;              // tile rows per 1 KB block (one wave-wide load)
    constexpr int KK = BK / 16;                // MFMA k-steps per tile
    constexpr int NBLK = (BM + BN) / RPB;      // 1 KB blocks per stage
    constexpr int LPT = NBLK / NW;             // direct-to-LDS loads per wave (= per lane) per tile
    constexpr int STAGE = (BM + BN) * CPR;     // 16-byte chunks per stage
    static_assert(BK == 64 || BK == 32, "BK");
    constexpr int DIST = STAGES - 1;           // tiles in flight ahead of the one being multiplied
    static_assert(NBLK % NW == 0, "tile/waves mismatch");
    static_assert(!GEGLU || (NI % 2 == 0), "GEGLU needs value/gate column-block pairs per wave");
    static_assert(DIST >= 1 && DIST <= 4, "ring depth");

    // ---- which tile of the problem ----
    const int local = tile - P.tile_begin;
    const int band_tiles = 8 * P.tiles_n;
    const int band = local / band_tiles, rem = local - band * band_tiles;
    const int band_rows = min(8, P.tiles_m - band * 8);
    const int tn = rem / band_rows, tm = band * 8 + rem % band_rows;
    constexpr int BN_OUT = GEGLU ? BN / 2 : BN;
    const int m0 = tm * BM, n0 = tn * BN_OUT;
    const int Mp = P.Mp, N = P.N, K0 = P.K0, K1 = P.K1;
    const int nk0 = (K0 + BK - 1) / BK, nk1 = (K1 + BK - 1) / BK, nkt = nk0 + nk1;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

    // ---- dependency on a producer problem of this launch.  The flags are read once now (the
    // answer arrives with the first operand tile); tiles that start after the producer has
    // finished, the usual case, never look again.  Device-scope loads: the producer's tile may
    // have run on another XCD.
    const int32_t* const wflag = K1 ? P.wait : nullptr;
    const int32_t* fptr = nullptr;
    int f_early = 0;
    if (wflag) {
        const int lo = P.wait_cols ? n0 : m0;
        const int hi = P.wait_cols ? min(n0 + BN_OUT, N) : min(m0 + BM, Mp);
        const int f0 = lo / BM, f1 = (hi - 1) / BM;
        fptr = wflag + f0 + min(lane, f1 - f0);
        f_early = __hip_atomic_load(fptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

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

    // ---- loader.  Load j of wave w fills 1 KB block (j*NW + w) of a stage: RPB tile rows
    // (P rows first, then Q rows) of CPR chunks; lane l lands at chunk position l % CPR of row
    // l / CPR, so it must fetch the logical chunk that the XOR swizzle places there.  The
    // first JP loads of a lane are P rows, the rest Q rows; a lane's source is a wave-uniform
    // base (operand start + k offset of the step, scalar arithmetic) plus a constant 32-bit
    // byte offset (row, chunk).
    constexpr int JP = (BM / RPB) / NW;
    static_assert((BM / RPB) % NW == 0, "P/Q split must fall on a load index");
    uint32_t off0[LPT];          // byte offset of this lane's chunk from the operand start, K segment 0
    uint32_t off1[LPT];          // ... K segment 1 (LoRA); equals off0 when there is none
    int kcol[GUARD ? LPT : 1];   // first k of that chunk within a tile (only partial tiles need it)
    const uint16_t* const pb0 = P.p0 + (int64_t)m0 * P.ldp0;
    const uint16_t* const pb1 = K1 ? P.p1 + (int64_t)m0 * P.ldp1 : pb0;
    const uint16_t* const qb0 = P.q0 + (int64_t)n0 * P.ldq0;
    const uint16_t* const qb1 = K1 ? P.q1 + (int64_t)n0 * P.ldq1 : qb0;
    {
        const int64_t ldp0 = P.ldp0, ldq0 = P.ldq0;
        const int64_t ldp1 = K1 ? P.ldp1 : P.ldp0, ldq1 = K1 ? P.ldq1 : P.ldq0;
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int row = (j * NW + wave) * RPB + lane / CPR;    // row within the stage
            const int c = swz<CPR>(row, lane % CPR);               // logical chunk fetched by this lane
            if (GUARD) kcol[j] = c * 8;
            if (j < JP) {
                int r = m0 + row;
                r = (r < Mp ? r : Mp - 1) - m0;
                off0[j] = (uint32_t)((r * ldp0 + c * 8) * 2);
                off1[j] = (uint32_t)((r * ldp1 + c * 8) * 2);
            } else {
                const int qr = qrow(row - BM) - n0;
                off0[j] = (uint32_t)((qr * ldq0 + c * 8) * 2);
                off1[j] = (uint32_t)((qr * ldq1 + c * 8) * 2);
            }
        }
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
    const uint32_t wave_base = lds_base + (uint32_t)wave * 1024;
    // issue the loads of k-step t into ring stage `stg`.  A partial last tile of a segment
    // (GUARD only) takes per-lane 64-bit addresses so that chunks past the segment's end can
    // point at the zero page.
    bool dep_ready = wflag == nullptr;
    bool timed_out = false;      // this wavefront gave up waiting: its output is poisoned below
    auto issue_tile = [&](int t, int stg) {
        const bool s1 = t >= nk0;
        const int kb = (s1 ? t - nk0 : t) * BK;
        const int Kseg = s1 ? K1 : K0;
        const uint32_t sbase = wave_base + (uint32_t)stg * (STAGE * 16);
        const uint16_t* pb = (s1 ? pb1 : pb0) + kb;
        const uint16_t* qb = (s1 ? qb1 : qb0) + kb;
        const bool dev = s1 && wflag;   // segment 1 was written during this launch
        if (dev && !dep_ready) {
            // the producer's tiles were dispatched before this one and wait for nothing, so
            // this ends; the bound is there so that it ends even if that reasoning is wrong
            for (int spins = 0;; ++spins) {
                const int v = __hip_atomic_load(fptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__all(v >= P.wait_need)) break;
                if (spins >= DEP_SPIN_LIMIT) {
                    if (tid == 0) atomicAdd(&g_gemm_dep_timeouts, 1ull);
                    timed_out = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            dep_ready = true;
        }
        if (GUARD && kb + BK > Kseg) {
#pragma unroll
            for (int j = 0; j < LPT; ++j) {
                const char* src = reinterpret_cast<const char*>(j < JP ? pb : qb) + (s1 ? off1[j] : off0[j]);
                src = (kb + kcol[GUARD ? j : 0] < Kseg) ? src : reinterpret_cast<const char*>(g_gemm_zeros);
                if (dev) dma16<true>(src, sbase + (uint32_t)j * (NW * 1024));
                else dma16<false>(src, sbase + (uint32_t)j * (NW * 1024));
            }
        } else if (dev) {
#pragma unroll
            for (int j = 0; j < LPT; ++j)
                dma16_so<true>(j < JP ? pb : qb, off1[j], sbase + (uint32_t)j * (NW * 1024));
        } else {
#pragma unroll
            for (int j = 0; j < LPT; ++j)
                dma16_so<false>(j < JP ? pb : qb, s1 ? off1[j] : off0[j], sbase + (uint32_t)j * (NW * 1024));
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    // one BK-deep tile out of ring stage `st`; fragments of k-step kk+1 are fetched while
    // the MFMAs of k-step kk execute
    auto compute = [&](int st) {
        const u32x4* la = lds + st * STAGE;
        const u32x4* lb = la + BM * CPR;
        bf16x8 af[2][MI], bfr[2][NI];
        auto fetch = [&](int kk, int fs) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int r = wm + mi * 32 + l32;
                af[fs][mi] = __builtin_bit_cast(bf16x8, la[r * CPR + swz<CPR>(r, kk * 2 + hi)]);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int r = wn + ni * 32 + l32;
                bfr[fs][ni] = __builtin_bit_cast(bf16x8, lb[r * CPR + swz<CPR>(r, kk * 2 + hi)]);
            }
        };
        fetch(0, 0);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk + 1 < KK) fetch(kk + 1, (kk + 1) & 1);
            // keep the reads of k-step kk+1 ahead of the MFMAs of k-step kk: left alone, the
            // scheduler sinks them to just before their use and exposes the LDS latency
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][mi], bfr[kk & 1][ni], acc[mi][ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: the first DIST tiles in flight
#pragma unroll
    for (int d = 0; d < DIST; ++d)
        if (d < nkt) issue_tile(d, d);
    if (!dep_ready) dep_ready = __all(f_early >= P.wait_need);

    // ---- main loop.  Step t: wait until this wave's loads of tile t have landed (loads of
    // newer tiles may stay in flight), barrier (every wave's part of tile t is in LDS and
    // every wave is done reading the stage of tile t-1), refill that stage with tile t+DIST,
    // multiply tile t.  The steady-state loop has no conditionals; the last DIST steps run
    // in a second loop with the shrinking wait counts.
    int st = 0;                         // stage of tile t
    int sf = DIST;                      // stage to refill (= stage of tile t-1)
    int t = 0;
#pragma unroll 1
    for (; t + DIST < nkt; ++t) {
        wait_vmcnt<(DIST - 1) * LPT>();
        __syncthreads();
        issue_tile(t + DIST, sf);
        compute(st);
        sf = st;
        st = st + 1 == STAGES ? 0 : st + 1;
    }
#pragma unroll 1
    for (; t + 1 < nkt; ++t) {
        const int newer = nkt - 1 - t;  // tiles issued after tile t
        if (DIST >= 4 && newer >= 3) wait_vmcnt<3 * LPT>();
        else if (DIST >= 3 && newer >= 2) wait_vmcnt<2 * LPT>();
        else wait_vmcnt<LPT>();
        __syncthreads();
        compute(st);
        st = st + 1 == STAGES ? 0 : st + 1;
    }
    wait_vmcnt<0>();
    __syncthreads();

    // ---- epilogue geometry.  Accumulator layout of the 32x32 MFMA: lane holds column l32 and
    // rows 8*(v/4) + 4*hi + (v%4), v = 0..15.  Each wave stages a 32-row x CCOLS-column piece at
    // a time in its own LDS region (fp32, padded rows) and writes it out as 16-byte row pieces:
    // lane handles 4 consecutive columns (lcol) of row lr, lr + RPP, ... of the piece.
    constexpr int NOUT = GEGLU ? NI / 2 : NI;   // 32-column output blocks per wave
    constexpr int CB = (NOUT % 2 == 0) ? 2 : 1; // 32-column blocks staged per pass (<= 64 columns)
    constexpr int CCOLS = CB * 32;              // staged columns
    constexpr int LPR = CCOLS / 4;              // lanes per staged row (4 columns each)
    constexpr int RPP = 64 / LPR;               // rows per pass
    constexpr int NPASS = 32 / RPP;
    static_assert(NOUT % CB == 0, "column chunking");
    const int wn_out = GEGLU ? (wn >> 1) : wn;
    const bool y_f32 = P.y_f32 != 0;
    const int lr = lane / LPR, lcol = (lane % LPR) * 4;
    const bool ld_ok = ((P.ldy & 3) == 0) && (!P.res || (P.ldr & 3) == 0);

    // fp32 residual: fetch this lane's pieces of the whole wave tile now, so that the loads
    // fly during the last tile's MFMAs and the epilogue never waits piece by piece
    f32x4 rpre[RES32 ? MI : 1][RES32 ? NOUT / CB : 1][RES32 ? NPASS : 1];
    const bool res_pre = RES32 && P.res && P.res_f32 && ld_ok;
    if (RES32 && res_pre) {
        const float* rp = static_cast<const float*>(P.res);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int cc = 0; cc < NOUT / CB; ++cc) {
                const int q4 = n0 + wn_out + cc * CCOLS + lcol;
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass) {
                    const int p = m0 + wm + mi * 32 + pass * RPP + lr;
                    f32x4 r = {0.f, 0.f, 0.f, 0.f};
                    if (p < Mp && q4 + 4 <= N) r = *reinterpret_cast<const f32x4*>(rp + (int64_t)p * P.ldr + q4);
                    rpre[RES32 ? mi : 0][RES32 ? cc : 0][RES32 ? pass : 0] = r;
                }
            }
    }
    // per-column bias of this lane's output columns: fetched now as well (raw bits, widened after
    // the last MFMAs; a column past N reads the last valid one and is never stored)
    const uint16_t* bias = P.bias;
    uint32_t bv_raw[NOUT], bg_raw[NOUT];
#pragma unroll
    for (int nj = 0; nj < NOUT; ++nj) bv_raw[nj] = bg_raw[nj] = 0u;
    if (bias && !P.bias_on_rows) {
#pragma unroll
        for (int nj = 0; nj < NOUT; ++nj) {
            const int q = min(n0 + wn_out + nj * 32 + l32, N - 1);
            bv_raw[nj] = bias[q];
            if (GEGLU) bg_raw[nj] = bias[q + P.geglu_F];
        }
    }
    compute(st);
    __syncthreads();   // ring reads done before the epilogue reuses LDS

    // ---- epilogue
    float* stage = reinterpret_cast<float*>(lds) + wave * 32 * EPI_STRIDE;
    // a wavefront that read its second K segment without the producer's flag stores NaN: what it
    // computed from a stale or half-written down-projection must not look like a result
    const float alpha = timed_out ? __builtin_nanf("") : P.alpha;
    int32_t* const sig = P.signal;
    // a tile that lies inside the output with 16-byte-aligned rows takes straight-line code: all
    // staged pieces read, then all residual pieces, then all stores (no per-lane bounds)
    const bool full = ld_ok && m0 + BM <= Mp && n0 + BN_OUT <= N;
    float bv[NOUT], bg[NOUT];
#pragma unroll
    for (int nj = 0; nj < NOUT; ++nj) {
        // (opaque to the optimiser, which would otherwise widen right after the loads and wait for them there)
        asm volatile("" : "+v"(bv_raw[nj]), "+v"(bg_raw[nj]));
        bv[nj] = __uint_as_float(bv_raw[nj] << 16);
        bg[nj] = __uint_as_float(bg_raw[nj] << 16);
    }

#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int cc = 0; cc < NOUT / CB; ++cc) {
            // 1) registers -> staging (value after alpha, bias, GEGLU)
#pragma unroll
            for (int cj = 0; cj < CB; ++cj) {
                const int nj = cc * CB + cj;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rr = 8 * (v >> 2) + 4 * hi + (v & 3);
                    float val;
                    if (GEGLU) {
                        const float a = alpha * acc[mi][2 * nj][v] + bv[nj];
                        const float gt = alpha * acc[mi][2 * nj + 1][v] + bg[nj];
                        val = a * gelu_erf(gt);
                    } else {
                        val = alpha * acc[mi][nj][v] + bv[nj];
                    }
                    stage[rr * EPI_STRIDE + cj * 32 + l32] = val;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // 2) staging -> global: lane handles 4 consecutive columns of one row per pass
            const int q4 = n0 + wn_out + cc * CCOLS + lcol;
            if (full) {
                f32x4 val[NPASS];
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass)
                    val[pass] = *reinterpret_cast<const f32x4*>(stage + (pass * RPP + lr) * EPI_STRIDE + lcol);
                const int p0 = m0 + wm + mi * 32 + lr;          // row of pass 0; pass k is RPP * k rows further
                if (bias && P.bias_on_rows) {
                    float br[NPASS];
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) br[pass] = bf16_to_f32(bias[p0 + pass * RPP]);
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) val[pass] += br[pass];
                }
                if (P.res) {
                    if (RES32 && res_pre) {
#pragma unroll
                        for (int pass = 0; pass < NPASS; ++pass) val[pass] += rpre[RES32 ? mi : 0][RES32 ? cc : 0][RES32 ? pass : 0];
                    } else if (P.res_f32) {
                        const float* rf = static_cast<const float*>(P.res) + (int64_t)p0 * P.ldr + q4;
                        f32x4 r[NPASS];
#pragma unroll
                        for (int pass = 0; pass < NPASS; ++pass) r[pass] = *reinterpret_cast<const f32x4*>(rf + (int64_t)(pass * RPP) * P.ldr);
#pragma unroll
                        for (int pass = 0; pass < NPASS; ++pass) val[pass] += r[pass];
                    } else {
                        const uint16_t* rb = static_cast<const uint16_t*>(P.res) + (int64_t)p0 * P.ldr + q4;
                        u32x2 r[NPASS];
#pragma unroll
                        for (int pass = 0; pass < NPASS; ++pass) r[pass] = *reinterpret_cast<const u32x2*>(rb + (int64_t)(pass * RPP) * P.ldr);
#pragma unroll
                        for (int pass = 0; pass < NPASS; ++pass) {
                            val[pass][0] += bf16lo_to_f32(r[pass][0]); val[pass][1] += bf16hi_to_f32(r[pass][0]);
                            val[pass][2] += bf16lo_to_f32(r[pass][1]); val[pass][3] += bf16hi_to_f32(r[pass][1]);
                        }
                    }
                }
                if (y_f32) {
                    float* yp = static_cast<float*>(P.y) + (int64_t)p0 * P.ldy + q4;
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) *reinterpret_cast<f32x4*>(yp + (int64_t)(pass * RPP) * P.ldy) = val[pass];
                } else {
                    uint16_t* yp = static_cast<uint16_t*>(P.y) + (int64_t)p0 * P.ldy + q4;
#pragma unroll
                    for (int pass = 0; pass < NPASS; ++pass) {
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (__bf16)val[pass][e];
                        uint16_t* const yq = yp + (int64_t)(pass * RPP) * P.ldy;
                        if (sig)   // device-scope store: read by tiles of this launch on other XCDs
                            __hip_atomic_store(reinterpret_cast<uint64_t*>(yq), __builtin_bit_cast(uint64_t, o), __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                        else
                            *reinterpret_cast<bf16x4*>(yq) = o;
                    }
                }
            } else {
                const bool vec_ok = ld_ok && (q4 + 4 <= N);   // 16-byte path: whole piece inside N, aligned rows
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass) {
                    const int rr = pass * RPP + lr;
                    const int p = m0 + wm + mi * 32 + rr;
                    if (p < Mp && q4 < N) {
                        f32x4 val = *reinterpret_cast<const f32x4*>(stage + rr * EPI_STRIDE + lcol);
                        if (bias && P.bias_on_rows) val += bf16_to_f32(bias[p]);
                        const int64_t oi = (int64_t)p * P.ldy + q4;
                        const int64_t ri = (int64_t)p * P.ldr + q4;
                        if (y_f32) {
                            float* yp = static_cast<float*>(P.y) + oi;
                            const float* rp = static_cast<const float*>(P.res);
                            if (vec_ok) {
                                if (RES32 && res_pre) val += rpre[RES32 ? mi : 0][RES32 ? cc : 0][RES32 ? pass : 0];
                                else if (rp) val += *reinterpret_cast<const f32x4*>(rp + ri);
                                *reinterpret_cast<f32x4*>(yp) = val;
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (q4 + e < N) yp[e] = val[e] + (rp ? rp[ri + e] : 0.f);
                            }
                        } else {
                            uint16_t* yp = static_cast<uint16_t*>(P.y) + oi;
                            const uint16_t* rp = static_cast<const uint16_t*>(P.res);
                            if (P.res_f32 && rp) {      // fp32 residual stream into a bf16 output
                                const float* rf = static_cast<const float*>(P.res);
                                if (RES32 && res_pre) val += rpre[RES32 ? mi : 0][RES32 ? cc : 0][RES32 ? pass : 0];
                                else if (vec_ok) val += *reinterpret_cast<const f32x4*>(rf + ri);
                                else
#pragma unroll
                                    for (int e = 0; e < 4; ++e)
                                        if (q4 + e < N) val[e] += rf[ri + e];
                                rp = nullptr;
                            }
                            if (vec_ok) {
                                if (rp) {
                                    const u32x2 rv = *reinterpret_cast<const u32x2*>(rp + ri);
                                    val[0] += bf16lo_to_f32(rv[0]); val[1] += bf16hi_to_f32(rv[0]);
                                    val[2] += bf16lo_to_f32(rv[1]); val[3] += bf16hi_to_f32(rv[1]);
                                }
                                bf16x4 o;
#pragma unroll
                                for (int e = 0; e < 4; ++e) o[e] = (__bf16)val[e];
                                if (sig)   // device-scope store: read by tiles of this launch on other XCDs
                                    __hip_atomic_store(reinterpret_cast<uint64_t*>(yp), __builtin_bit_cast(uint64_t, o), __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                                else
                                    *reinterpret_cast<bf16x4*>(yp) = o;
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (q4 + e < N) {
                                        const float f = val[e] + (rp ? bf16_to_f32(rp[ri + e]) : 0.f);
                                        yp[e] = __builtin_bit_cast(uint16_t, (__bf16)f);
                                    }
                            }
                        }
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
    // ---- tell the tiles that wait for this one: every wave's stores have completed at device
    // scope (vmcnt counts a device-scope store until it is visible there), then one flag add
    if (sig) {
        wait_vmcnt<0>();
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(sig + tm, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The group's header (everything before p[]) and one problem record are fetched as a few wide
// scalar loads (dword-aligned vector types)
typedef uint32_t u32x16u __attribute__((ext_vector_type(16), aligned(4)));
typedef uint32_t u32x8u __attribute__((ext_vector_type(8), aligned(4)));
typedef uint32_t u32x4u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2u __attribute__((ext_vector_type(2), aligned(4)));
struct alignas(8) ProblemWords { uint32_t w[44]; };
static_assert(offsetof(GemmGroup, p) == 88 && offsetof(GemmGroup, first_tile) == 24 && offsetof(GemmGroup, zero_ptr) == 16 &&
              offsetof(GemmGroup, n_lead) == 8 && offsetof(GemmGroup, zero_n) == 12, "header layout");
static_assert(sizeof(GemmProblem) == sizeof(ProblemWords), "problem record size");

template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, bool GEGLU, bool GUARD, bool RES32>
__global__ __launch_bounds__(64 * WGM * WGN, (gemm_min_waves<BM, BN, BK, WGM, WGN, STAGES>())) void gemm_kernel(const GemmGroup g) {
    constexpr int NW = WGM * WGN;
    __shared__ u32x4 lds[gemm_lds_chunks<BM, BN, BK, WGM, WGN, STAGES>()];
    // ---- which problem, which tile ----
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD a
    // contiguous range of tiles, and order tiles inside a problem in bands of 8 row-tiles
    // (row-tile index fastest), so that the workgroups resident on one XCD share a small set
    // of activation rows and weight rows.
    // The tiles of signalling problems (down-projections that tiles of this same launch wait
    // for) come first and are dealt round-robin: they are the first workgroups dispatched on
    // every XCD, so all of them are running, or done, before any tile can wait for them.
    // Kernel arguments arrive through scalar loads of ~0.25 us each, and the compiler issues a
    // load next to its first use: left alone, a workgroup pays six or seven such rounds one after
    // the other before its first operand load.  Two rounds are forced instead: the header in one
    // batch (made opaque right away, so no load can sink below), then the whole problem record.
    const uint32_t* const hw = reinterpret_cast<const uint32_t*>(&g);
    u32x16u ha = *reinterpret_cast<const u32x16u*>(hw);
    u32x4u hb = *reinterpret_cast<const u32x4u*>(hw + 16);
    u32x2u hc = *reinterpret_cast<const u32x2u*>(hw + 20);
    uint32_t grid = gridDim.x;     // one more kernel argument (the launch geometry): same batch
    asm volatile("" : "+s"(ha), "+s"(hb), "+s"(hc), "+s"(grid));
    const int lead = (int)ha[2], zero_n = (int)ha[3], np = (int)ha[0];
    int32_t* const zero_ptr = reinterpret_cast<int32_t*>(((uint64_t)ha[5] << 32) | ha[4]);
    int tile = blockIdx.x;
    {
        const int rest = (int)grid - lead;
        if (tile >= lead && (rest & 7) == 0) {
            const int r = tile - lead;
            tile = lead + (r & 7) * (rest >> 3) + (r >> 3);
        }
    }
    int pi = 0;
#pragma unroll
    for (int i = 1; i < GEMM_MAX_PROBLEMS; ++i) {
        const int ft = (int)(i < 10 ? ha[6 + i] : i < 14 ? hb[i - 10] : hc[i - 14]);
        if (i < np && tile >= ft) pi = i;
    }
    const uint32_t* const pw = reinterpret_cast<const uint32_t*>(&g.p[pi]);
    u32x16u ra = *reinterpret_cast<const u32x16u*>(pw);
    u32x16u rb = *reinterpret_cast<const u32x16u*>(pw + 16);
    u32x8u rc = *reinterpret_cast<const u32x8u*>(pw + 32);
    u32x4u rd = *reinterpret_cast<const u32x4u*>(pw + 40);
    asm volatile("" : "+s"(ra), "+s"(rb), "+s"(rc), "+s"(rd));
    ProblemWords words;
#pragma unroll
    for (int i = 0; i < 16; ++i) { words.w[i] = ra[i]; words.w[16 + i] = rb[i]; }
#pragma unroll
    for (int i = 0; i < 8; ++i) words.w[32 + i] = rc[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) words.w[40 + i] = rd[i];
    const GemmProblem P = __builtin_bit_cast(GemmProblem, words);
    // flags of the next dependent launch, a few words per workgroup: nothing reads them before this kernel ends
    for (int i = blockIdx.x * (64 * NW) + threadIdx.x; i < zero_n; i += (int)grid * (64 * NW)) zero_ptr[i] = 0;
    if constexpr (BN > DOWN_BN) {
        if (P.signal) {
            gemm_tile<BM, DOWN_BN, BK, WGM, WGN, down_stages<BM, BN, BK, STAGES>(), false, GUARD, false>(P, tile, lds);
            return;
        }
    }
    gemm_tile<BM, BN, BK, WGM, WGN, STAGES, GEGLU, GUARD, RES32>(P, tile, lds);
}

template <int BM, int BN, int BK, int WGM, int WGN, int STAGES, bool GEGLU, bool RES32>
static int launch_cfg(GemmGroup& g, bool guard, hipStream_t stream) {
    constexpr int BN_OUT = GEGLU ? BN / 2 : BN;
    int total = 0;
    g.n_lead = 0;
    for (int i = 0; i < g.n; ++i) {
        GemmProblem& P = g.p[i];
        P.tiles_m = (P.Mp + BM - 1) / BM;
        P.tiles_n = P.signal ? (P.N + (BN < DOWN_BN ? BN : DOWN_BN) - 1) / (BN < DOWN_BN ? BN : DOWN_BN) : (P.N + BN_OUT - 1) / BN_OUT;
        P.tile_begin = total;
        g.first_tile[i] = total;
        total += P.tiles_m * P.tiles_n;
        if (P.signal) g.n_lead = total;
        P.wait_need = (P.K1 + (BN < DOWN_BN ? BN : DOWN_BN) - 1) / (BN < DOWN_BN ? BN : DOWN_BN);   // column tiles of the producer, whose N is this problem's K1
    }
    g.total_tiles = total;
    if (total == 0) return SD_OK;
    if (guard)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WGM, WGN, STAGES, GEGLU, true, RES32>), dim3(total), dim3(64 * WGM * WGN), 0, stream, g);
    else
        hipLaunchKernelGGL((gemm_kernel<BM, BN, BK, WGM, WGN, STAGES, GEGLU, false, RES32>), dim3(total), dim3(64 * WGM * WGN), 0, stream, g);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

int launch_gemm_group(GemmGroup& g, hipStream_t stream) {
    SD_REQUIRE(g.n >= 1 && g.n <= GEMM_MAX_PROBLEMS, SD_EINVAL, "gemm group: %d problems", g.n);
    bool geglu = false;   // a GEGLU group: GEGLU problems plus, possibly, the plain down-projections they wait for
    for (int i = 0; i < g.n; ++i) geglu = geglu || g.p[i].geglu_F > 0;
    bool guard = false;
    int maxN = 0, maxK = 0;
    long t128 = 0;        // workgroup tiles at 128x128
    long t256 = 0;        // workgroup tiles of 256 rows x 128 output columns
    long t64 = 0;         // workgroup tiles of 64 rows x 128 columns, down-projections aside
    bool res32 = false;   // some problem adds an fp32 residual: take the kernel that prefetches it
    int n_main = 0;       // problems that are not down-projections
    for (int i = 0; i < g.n; ++i) {
        const GemmProblem& P = g.p[i];
        if (!P.signal && P.Mp > 0 && P.N > 0) ++n_main;
        if (P.res && P.res_f32 && P.Mp > 0 && P.N > 0) res32 = true;
        SD_REQUIRE((P.geglu_F > 0) == geglu || P.signal, SD_EINVAL, "gemm group mixes GEGLU and plain problems");
        SD_REQUIRE(P.Mp >= 0 && P.N >= 0 && P.K0 > 0 && P.K0 % 8 == 0 && P.K1 >= 0 && P.K1 % 8 == 0, SD_EINVAL,
                   "gemm problem %d: bad sizes M=%d N=%d K0=%d K1=%d", i, P.Mp, P.N, P.K0, P.K1);
        SD_REQUIRE(P.p0 && P.q0 && P.y && (P.K1 == 0 || (P.p1 && P.q1)), SD_EINVAL, "gemm problem %d: null operand", i);
        SD_REQUIRE(P.ldp0 % 8 == 0 && P.ldq0 % 8 == 0 && (P.K1 == 0 || (P.ldp1 % 8 == 0 && P.ldq1 % 8 == 0)), SD_EINVAL,
                   "gemm problem %d: leading dimensions must be multiples of 8", i);
        // lane offsets inside a tile are 32-bit byte offsets
        const int64_t span = 256 + (P.geglu_F > 0 ? P.geglu_F : 0);
        SD_REQUIRE(P.ldp0 > 0 && P.ldq0 > 0 && P.ldp0 * 256 < (1ll << 31) && P.ldq0 * span < (1ll << 31) &&
                       (P.K1 == 0 || (P.ldp1 > 0 && P.ldq1 > 0 && P.ldp1 * 256 < (1ll << 31) && P.ldq1 * span < (1ll << 31))),
                   SD_EINVAL, "gemm problem %d: leading dimension out of range", i);
        if (P.signal) {
            SD_REQUIRE(i == 0 || g.p[i - 1].signal, SD_EINVAL, "gemm group: signalling problem %d after a plain one", i);
            SD_REQUIRE(!P.y_f32 && !P.res && !P.wait && P.N % 4 == 0 && P.ldy % 4 == 0 && P.geglu_F == 0, SD_EINVAL,
                       "gemm problem %d: a signalling problem stores plain bf16 rows", i);
        }
        SD_REQUIRE(!P.wait || (P.K1 > 0 && g.p[0].signal), SD_EINVAL, "gemm problem %d waits but the group has no producer", i);
        if (P.Mp == 0 || P.N == 0) continue;
        if ((P.K0 & 63) || (P.K1 & 63)) guard = true;
        if (P.N > maxN) maxN = P.N;
        if (P.K0 > maxK) maxK = P.K0;
        t128 += (long)((P.Mp + 127) / 128) * ((P.N + 127) / 128);
        if (!P.signal) t256 += (long)((P.Mp + 255) / 256) * ((P.N + 127) / 128);
        if (!P.signal) t64 += (long)((P.Mp + 63) / 64) * ((P.N + 127) / 128);
    }
    // drop empty problems
    int w = 0;
    for (int i = 0; i < g.n; ++i)
        if (g.p[i].Mp > 0 && g.p[i].N > 0) { if (w != i) g.p[w] = g.p[i]; ++w; }
    g.n = w;
    if (w == 0) return SD_OK;
    // Tile choice, from timing whole transformer-block steps with each variant on one machine.
    // What pays is wavefronts in flight per CU, not operand reuse: these GEMMs wait on the
    // L2 -> LDS operand stream and on their own prologues and epilogues, and 256x128, 128x160
    // (one exact round) and 3-stage variants all lost.  Launches of fewer than 1024 tiles at
    // 128x128 (everything in the block except the feed-forward in-projection) run 64x128 tiles,
    // 4 waves, 48 KB of LDS, three workgroups per CU; larger ones run 128x128 tiles with 8 waves
    // of 32x64, two workgroups per CU.  Down-projections (N = rank <= 64): 64x64 tiles, 5-stage
    // ring.
    // (a GEGLU group never takes this one: its tiles need the value / gate pairing, which the
    // 64x128 body below provides for any F)
    if (maxN <= 64 && !geglu) return launch_cfg<64, 64, 64, 2, 2, 5, false, false>(g, guard, stream);
    // ... except long-K launches (the feed-forward out-projection, K = 4C) that still give every CU
    // a 128x128 tile: over 40 k-steps the operand bytes per FLOP decide, not the ramps
    if (t128 < 1024 && !(maxK >= 2048 && t128 >= 256)) {
        // at most two workgroups per CU anyway (2048 tokens): a third ring stage in the LDS the
        // third workgroup would have used, -3 to -10 % per launch
        if (t64 <= 512) {
            if (geglu) return launch_cfg<64, 128, 64, 2, 2, 3, true, false>(g, guard, stream);
            if (res32) return launch_cfg<64, 128, 64, 2, 2, 3, false, true>(g, guard, stream);
            return launch_cfg<64, 128, 64, 2, 2, 3, false, false>(g, guard, stream);
        }
        if (geglu) return launch_cfg<64, 128, 64, 2, 2, 2, true, false>(g, guard, stream);
        if (res32) return launch_cfg<64, 128, 64, 2, 2, 2, false, true>(g, guard, stream);
        return launch_cfg<64, 128, 64, 2, 2, 2, false, false>(g, guard, stream);
    }
    // The feed-forward in-projection at 8192 tokens: 256x256 tiles (128 output columns after GEGLU)
    // of eight 64x128 wavefronts, one workgroup per CU, when that still gives every CU two rounds
    // or more.  Half the operand bytes per FLOP from L2 and from LDS; measured 5 % faster per launch
    // than 128x128 in spite of the last, partly empty round (640 tiles on 256 CUs).
    if (geglu && t256 >= 512) return launch_cfg<256, 256, 64, 4, 2, 2, true, false>(g, guard, stream);
    // One large plain projection with a long K loop (no launch of the transformer block: the
    // 8192 x 4096 x 4096 yardstick runs at 1.18 PFLOP/s this way, 1.04 at 128x128).  Not for grouped
    // launches: the q/k/v group with its short text-context problems loses a third.
    if (!geglu && !res32 && n_main == 1 && t256 >= 512 && maxK >= 2048) return launch_cfg<256, 256, 64, 4, 2, 2, false, false>(g, guard, stream);
    if (geglu) return launch_cfg<128, 128, 64, 4, 2, 2, true, false>(g, guard, stream);
    if (res32) return launch_cfg<128, 128, 64, 4, 2, 2, false, true>(g, guard, stream);
    return launch_cfg<128, 128, 64, 4, 2, 2, false, false>(g, guard, stream);
}

__global__ void clear_flags_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
int launch_clear_flags(int32_t* p, int n, hipStream_t stream) {
    if (n <= 0) return SD_OK;
    hipLaunchKernelGGL(clear_flags_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}
int gemm_dep_timeouts(long long* count) {
    unsigned long long v = 0;
    SD_HIP_CHECK(hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_gemm_dep_timeouts), sizeof(v)));
    *count = (long long)v;
    return SD_OK;
}

}  // namespace sd
