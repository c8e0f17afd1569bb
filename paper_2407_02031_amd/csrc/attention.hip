// Flash-style attention for gfx950, head dim 64, no mask: softmax(q k^T / 8) v per
// (sample, head) without ever writing the scores (the transformer block's self-attention
// over the latent tokens and cross-attention to the text tokens).
//
// The kernel works on the TRANSPOSED score tile S^T = K Q^T: with the 32x32x16 bf16 MFMA
// the accumulator of lane l then holds one query (column l % 32) and 16 of the tile's keys
// (rows), so the softmax row maximum and row sum are in-register reductions plus a single
// exchange between the two half-wavefronts, the running rescale factor is a per-lane
// scalar, and the exponentials, packed to bf16, are already laid out as the B operand of
// the second MFMA, O^T += V^T P^T.  V is consumed transposed ([C, keys]), which is how the
// v-projection GEMM writes it, so both K and V^T tiles are staged with 16-byte rows.
//
// Workgroup: 4 wavefronts, each owning 32 queries; K / V^T tiles of 64 keys go from
// global memory straight into LDS rings (wave-wide 1 KB loads of XOR-swizzled 16-byte
// chunks), one tile ahead of the one being used.  K rows are placed in LDS with the keys
// of every 16-key group in the order [0-3, 8-11, 4-7, 12-15]: the score accumulator of a
// lane then holds 8 consecutive keys per 16-key group, and the matching V^T operand is a
// single 16-byte LDS read of the plain [C, keys] layout.
//
// Work split.  A (sample, head, 128-query tile) is a tile; a workgroup normally takes one.
// When the tile count lies between two and three per CU (640 tiles on 256 CUs leaves half
// the CUs with three tiles and half with two), the launch is padded to exactly three
// workgroups per CU by cutting the key range of the surplus tiles in half: every CU then
// holds two whole tiles and one half.  The two halves of a cut tile leave their unnormalised
// accumulator, reference maximum and row sum in a scratch buffer and count themselves in on a
// per-tile counter; the half that arrives second merges the two inside the launch (without
// counters, a second, small kernel merges them).
#include "common.hpp"

namespace sd {

__device__ __forceinline__ int aswz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

constexpr float RESCALE_LOG2 = 8.0f;

// where lanes of a direct-to-LDS load point when their V^T chunk lies past the padded keys
__device__ __attribute__((aligned(256))) uint32_t g_attn_zeros[64];

// one direct global -> LDS load: each lane fetches 16 bytes from its own address, the 64
// pieces land contiguously at LDS byte address `lds_base` (wave-uniform).  Completion is
// tracked by hand with vmcnt and a workgroup barrier.
__device__ __forceinline__ void attn_dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(gptr) : "memory", "m0");
}
// same with a wave-uniform 64-bit base and a 32-bit unsigned byte offset per lane: the
// per-tile address arithmetic stays on the scalar unit
__device__ __forceinline__ void attn_dma16_so(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(voff), "s"(uniform_ptr(sbase)) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void attn_wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int PART_FLOATS = 34 * 256;   // one half of a cut tile: 32 accumulator values, max, sum per thread

// normalise and store one 32-query block of a tile: lane holds query l32, d = db*32 + 8*(v/4) + 4*hi + v%4
__device__ __forceinline__ void store_queries(const f32x16 (&o)[2], float l, uint16_t* __restrict__ out, int64_t ldo,
                                              int b, int Tq, int row, int head, int hi) {
    float l_lo, l_hi;
    both_halves(l, l_lo, l_hi);   // the two half-wavefronts summed different keys of the same query
    const float inv = 1.0f / (l_lo + l_hi);
    if (row < Tq) {
        uint16_t* op = out + ((int64_t)b * Tq + row) * ldo + head * 64 + 4 * hi;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][4 * v4 + e] * inv);
                *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * v4) = w;
            }
    }
}

// PRE: the keys arrive multiplied by 1/8 * log2(e) (the K projection's epilogue does it before
// rounding to bf16), so a score is already the exponent of 2, and the running reference maximum
// is subtracted by the matrix core: a fifth, half-depth k-step multiplies a fragment of ones (K side) with
// (-m split into three bf16 terms, exact to fp32) on the query side, so the accumulator holds
// s - m and the vector ALU only exponentiates.  Without PRE one FMA per score does both.
// MEASURE: the maximum of every key tile is measured before its exponentials are formed and the
// reference moves whenever a tile's maximum exceeds it by 2^8.  PRE tries without first.  What
// the reference maximum is for is range, not accuracy: p = 2^(s - m) is formed, rounded and
// accumulated in floating point, whose relative precision does not depend on magnitude, so any m
// gives the same result as long as nothing overflows and the row sum does not vanish.  The first
// attempt therefore measures only a segment's first tile (m becomes a score that occurs: the row
// sum is >= 1 from then on) and its last (which may be masked); in between the exponentials are
// formed against that fixed reference with no maximum pass at all.  At the end every lane looks at
// its row sum and accumulator: if anything is not finite, some score lay 2^100 or more above the
// first tile's; a workgroup in which any wavefront saw that returns true without storing
// anything, and its caller runs the segment again in the measured form.
// nsplit == 0: workgroup i takes tile i.  Otherwise the grid holds nfull whole tiles and
// 2 * nsplit half tiles (both multiples of 8), dealt so that each XCD, and in dispatch order
// each CU, first receives its share of whole tiles and then its share of halves.
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) int32_t lds_i32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;

// ldsK: [2][64 keys (permuted within 16)][8 chunks of 8 d], 2-deep ring;  ldsV: [3][64 d][8 chunks of 8 keys], 3-deep ring
template <bool PRE, bool MEASURE>
__device__ __forceinline__ bool attention_body(const uint16_t* __restrict__ q, int64_t ldq,
                                               const uint16_t* __restrict__ k, int64_t ldk,
                                               const uint16_t* __restrict__ vt, int64_t ldvt,
                                               uint16_t* __restrict__ out, int64_t ldo,
                                               int Tq, int Tk, int Tkp, int heads, int qtiles, float c,
                                               int nfull, int nsplit, float* __restrict__ parts, int32_t* __restrict__ arrived,
                                               lds_u32x4* const ldsK, lds_u32x4* const ldsV, lds_i32* const wg_redo, const int tid, const int bid) {
    static_assert(PRE || MEASURE, "only prescaled keys have the unmeasured form");
    constexpr int QB = 1;             // 32-query blocks per wavefront
    constexpr int BQ = 4 * 32 * QB;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // (sample, head, query tile) so that one head's K and V stay in one XCD's L2.
    const int nt = (Tk + 63) >> 6;
    int tile, s0 = 0, s1 = nt, part = -1;   // steps [s0, s1) of the tile; part >= 0: a half tile
    if (nsplit == 0) {
        const int total = gridDim.x;
        tile = bid;
        if ((total & 7) == 0) tile = (tile & 7) * (total >> 3) + (tile >> 3);
    } else {
        const int xcd = bid & 7, j = bid >> 3;
        const int fpx = nfull >> 3, hpx = nsplit >> 2;   // whole tiles / halves per XCD
        if (j < fpx) {
            tile = xcd * fpx + j;
        } else {
            const int h = xcd * hpx + (j - fpx);
            tile = nfull + (h >> 1);
            part = h & 1;
            const int mid = (nt + 1) >> 1;
            s0 = part ? mid : 0;
            s1 = part ? nt : mid;
        }
    }
    const int qt = tile % qtiles;
    const int head = (tile / qtiles) % heads, b = tile / (qtiles * heads);
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int q0 = qt * BQ + wave * 32 * QB;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds q[row l32][d = kk*16 + hi*8 ..+8]
    bf16x8 qf[QB][4];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + l32;
        row = row < Tq ? row : Tq - 1;
        const uint16_t* qp = q + ((int64_t)b * Tq + row) * ldq + head * 64 + hi * 8;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qf[qb][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + kk * 16));
    }

    // ---- tile loaders.  A tile is 8 blocks of 1 KB (8 rows x 8 chunks); load j of wave w
    // fills block j*4 + w: lane l lands at chunk position l % 8 of row l / 8 and fetches the
    // logical chunk the XOR swizzle places there.  K row r holds key (r with bits 2 and 3
    // exchanged); keys past Tk re-read the last key (masked later), V^T chunks past the
    // padded key count read zeros.
    const uint32_t ldsK_base = (uint32_t)(uintptr_t)ldsK;
    const uint32_t ldsV_base = (uint32_t)(uintptr_t)ldsV;
    const uint16_t* kbase = k + (int64_t)b * Tk * ldk + head * 64;
    // rows of the two loads of a lane are 32 apart: same swizzled chunk for both
    const int r0 = wave * 8 + (lane >> 3);
    const int kc8 = aswz(r0, lane & 7) * 8;
    const int kkey0 = (r0 & ~12) | ((r0 & 4) << 1) | ((r0 & 8) >> 1);
    // full tiles: byte offset of this lane's first K row and first V^T row from the tile's base; the
    // second row of each lies 32 rows further, a wave-uniform distance that goes into the scalar base
    const uint32_t koff = (uint32_t)(((int64_t)kkey0 * ldk + kc8) * 2);
    const uint32_t voff = (uint32_t)(((int64_t)r0 * ldvt + kc8) * 2);
    const int64_t krow32 = 64 * ldk, vrow32 = 64 * ldvt;     // bytes
    const char* vbase = reinterpret_cast<const char*>(vt + (int64_t)(head * 64) * ldvt + (int64_t)b * Tkp);
    const bool ragged = (Tk & 63) != 0;
    auto issue_kv = [&](int t, int kslot, int vslot) {
        const int key0 = t * 64;
        const uint32_t kdst = ldsK_base + (uint32_t)(kslot * 8192 + wave * 1024);
        const uint32_t vdst = ldsV_base + (uint32_t)(vslot * 8192 + wave * 1024);
        if (ragged && t == nt - 1) {
            // (the lane's row and chunk are derived afresh from a laundered lane index, so that
            // nothing of this rare path is kept in registers through the key loop)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int rr = wave * 8 + (ln >> 3);
            const int cc8 = aswz(rr, ln & 7) * 8;
            const int kk0 = (rr & ~12) | ((rr & 4) << 1) | ((rr & 8) >> 1);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int key = key0 + kk0 + j * 32;
                key = key < Tk ? key : Tk - 1;
                attn_dma16(kbase + (int64_t)key * ldk + cc8, kdst + j * 4096);
            }
            const bool inside = key0 + cc8 < Tkp;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const void* src = inside ? (const void*)(vbase + key0 * 2 + ((int64_t)(rr + j * 32) * ldvt + cc8) * 2) : (const void*)g_attn_zeros;
                attn_dma16(src, vdst + j * 4096);
            }
        } else {
            const char* kb = reinterpret_cast<const char*>(kbase) + (int64_t)key0 * ldk * 2;
            const char* vb = vbase + key0 * 2;
#pragma unroll
            for (int j = 0; j < 2; ++j) attn_dma16_so(kb + j * krow32, koff, kdst + j * 4096);
#pragma unroll
            for (int j = 0; j < 2; ++j) attn_dma16_so(vb + j * vrow32, voff, vdst + j * 4096);
        }
    };
    // padding keys [Tk, Tkp) of the last tile hold whatever the caller's buffer held: zero
    // them in LDS so that 0 * garbage stays 0 (thread: row tid / 4, keys Tk + tid % 4 (+ 4))
    auto zero_pad_keys = [&](int t, int vslot) {
        lds_u16* lv = reinterpret_cast<lds_u16*>(ldsV + vslot * 512);
        const int d = tid >> 2;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int key = Tk + (tid & 3) + 4 * i;
            const int kl = key - t * 64;
            if (key < Tkp && kl < 64) lv[(d * 8 + aswz(d, kl >> 3)) * 8 + (kl & 7)] = 0;
        }
    };

    f32x16 o[QB][2];
    float m[QB], l[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = PRE ? 0.f : -INFINITY;
        l[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][db][v] = 0.f;
    }

    // S^T tile of key tile t: 64 keys x (32*QB) queries.  The K fragments of the first two
    // k-steps are fetched by the caller ahead of time (their LDS latency hides behind the
    // running-maximum update), the other two are read here.
    auto load_kfrags = [&](int t, int kk0, bf16x8 (&kf)[2][2]) {
        const lds_u32x4* lk = ldsK + (t & 1) * 512;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int r = kb * 32 + l32;
                kf[kk][kb] = __builtin_bit_cast(bf16x8, lk[r * 8 + aswz(r, (kk0 + kk) * 2 + hi)]);
            }
    };
    // PRE: operands of the extra k-step, a 32x32x8 MFMA (half the cost of a 16-deep one; a lane
    // supplies k-slots 4*hi .. 4*hi+3).  K side: 1.0 in k-slots 0..2 of every key row; query side:
    // -m as three bf16 terms in those slots; the upper half-wavefront supplies zeros.
    const u32x2 ones_bits = {hi ? 0u : 0x3F803F80u, hi ? 0u : 0x00003F80u};
    const bf16x4 ones_frag = __builtin_bit_cast(bf16x4, ones_bits);
    bf16x4 mfrag[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) mfrag[qb] = __builtin_bit_cast(bf16x4, u32x2{0u, 0u});
    auto set_mfrag = [&](int qb) {
        const float x = -m[qb];
        const __bf16 h = (__bf16)x;
        const float r1 = x - (float)h;
        const __bf16 md = (__bf16)r1;
        const __bf16 lo = (__bf16)(r1 - (float)md);
        const uint32_t w0 = (uint32_t)__builtin_bit_cast(uint16_t, h) | ((uint32_t)__builtin_bit_cast(uint16_t, md) << 16);
        const uint32_t w1 = (uint32_t)__builtin_bit_cast(uint16_t, lo);
        mfrag[qb] = __builtin_bit_cast(bf16x4, u32x2{hi ? 0u : w0, hi ? 0u : w1});
    };
    auto compute_s = [&](int t, f32x16 (&s)[QB][2], bf16x8 (&kf0)[2][2]) {
        bf16x8 kf1[2][2];
        load_kfrags(t, 2, kf1);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[qb][kb][v] = 0.f;
        if (PRE) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ones_frag, mfrag[qb], s[qb][kb], 0, 0, 0);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 a = kk < 2 ? kf0[kk][kb] : kf1[kk - 2][kb];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][kk], s[qb][kb], 0, 0, 0);
            }
    };
    // keys past Tk (last tile only) get a score of -inf
    auto mask_tail = [&](int t, f32x16 (&s)[QB][2]) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = t * 64 + kb * 32 + 16 * (v >> 3) + 8 * hi + (v & 7);
                if (key >= Tk) {
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) s[qb][kb][v] = -INFINITY;
                }
            }
    };
    // running-maximum bookkeeping of one tile: the reference maximum m only moves when the
    // tile maximum exceeds it by more than RESCALE_LOG2 in the exponent (p <= 2^RESCALE_LOG2
    // stays far inside fp32 / bf16 range), so the O and l rescale runs on the first tiles and
    // almost never afterwards.  This lane's query is column l32, its keys are its registers.
    // PRE: the scores arrive already shifted by m, so the tile maximum is the excess over it; the
    // segment's first tile always re-references (m starts at 0, not at the scores' level).
    auto update_max = [&](f32x16 (&s)[QB][2], bool first) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = fmaxf(s[qb][0][0], s[qb][1][0]);
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, s[qb][0][v]), s[qb][1][v]);
            // the other half-wavefront holds the other 32 keys of this query: exchange the
            // two halves with a lane swap (a vector-ALU operation, no LDS round trip)
            float mx_lo, mx_hi;
            both_halves(mx, mx_lo, mx_hi);
            mx = fmaxf(mx_lo, mx_hi);
            if (PRE) {
                const bool need = first || mx > RESCALE_LOG2;
                if (__builtin_amdgcn_ballot_w64(need) != 0ull) {
                    const float delta = need ? mx : 0.f;
                    const float alpha = __builtin_amdgcn_exp2f(-delta);
                    m[qb] += delta;
                    l[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < 2; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[qb][db][v] *= alpha;
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) s[qb][kb][v] -= delta;
                    set_mfrag(qb);
                }
                continue;
            }
            const bool need = (mx - m[qb]) * c > RESCALE_LOG2;
            if (__builtin_amdgcn_ballot_w64(need) != 0ull) {
                const float mnew = need ? mx : m[qb];
                const float alpha = __builtin_amdgcn_exp2f((m[qb] - mnew) * c);
                m[qb] = mnew;
                l[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[qb][db][v] *= alpha;
            }
        }
    };
    // p = exp2((s - m) * c) packed to bf16 in MFMA operand order; the row sum adds up the
    // packed (rounded) values with a bf16 dot-product against ones, two per instruction, so
    // the normaliser matches exactly what the second MFMA multiplies
    auto exponentials = [&](f32x16 (&s)[QB][2], bf16x8 (&pf)[QB][2][2]) {
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float mc = m[qb] * c;
            float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g2 = 0; g2 < 2; ++g2) {
                    bf16x8 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p0 = __builtin_amdgcn_exp2f(PRE ? s[qb][kb][g2 * 8 + 2 * e] : s[qb][kb][g2 * 8 + 2 * e] * c - mc);
                        const float p1 = __builtin_amdgcn_exp2f(PRE ? s[qb][kb][g2 * 8 + 2 * e + 1] : s[qb][kb][g2 * 8 + 2 * e + 1] * c - mc);
                        const bf16x2 pp = {(__bf16)p0, (__bf16)p1};
                        pk[2 * e] = pp[0];
                        pk[2 * e + 1] = pp[1];
                        if (e & 1) ls1 = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, ls1, false);
                        else ls0 = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, ls0, false);
                    }
                    pf[qb][kb][g2] = pk;
                }
            l[qb] += ls0 + ls1;
        }
    };
    // O^T += V^T P^T.  With the K row order above, accumulator register v of block kb is key
    // kb*32 + 16*(v/8) + 8*hi + v%8: sub-step (kb, g2) multiplies keys kb*32 + 16*g2 + 8*hi ..+8,
    // the 16-byte chunk kb*4 + g2*2 + hi of a V^T row
    auto accumulate_o = [&](int vslot, bf16x8 (&pf)[QB][2][2]) {
        const lds_u32x4* lv = ldsV + vslot * 512;
        // (row index laundered: the four swizzled chunk addresses are formed here, a few vector
        // operations per tile, instead of living in registers through the whole key loop)
        int lrow = l32;
        asm volatile("" : "+v"(lrow));
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    const int r = db * 32 + lrow;
                    const bf16x8 a = __builtin_bit_cast(bf16x8, lv[r * 8 + aswz(r, kb * 4 + g2 * 2 + hi)]);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qb][kb][g2], o[qb][db], 0, 0, 0);
                }
    };

    // ---- prologue: the first two key tiles in flight, S of the first
    issue_kv(s0, s0 & 1, 0);
    if (s0 + 1 < s1) {
        issue_kv(s0 + 1, (s0 + 1) & 1, 1);
        attn_wait_vmcnt<4>();
    } else {
        attn_wait_vmcnt<0>();
    }
    __syncthreads();
    f32x16 sa[QB][2], sb[QB][2];
    {
        bf16x8 kf0[2][2];
        load_kfrags(s0, 0, kf0);
        compute_s(s0, sa, kf0);
    }
    // unmeasured form: the segment's first tile sets the reference (a one-tile segment masks its tail first, below)
    if (!MEASURE && s1 - s0 > 1) update_max(sa, true);

    // ---- main loop, software-pipelined: the score MFMAs of tile t+1 are independent of the
    // exponentials of tile t and sit in the same basic block, so the matrix pipe and the
    // vector ALU overlap inside one wavefront.  Two tiles per trip (the score buffers swap
    // roles), the last tile is peeled: nothing to prefetch, and only it may need masking.
    int vslot = 0;
    bf16x8 pf[QB][2][2];
    // One pipelined step: finish tile t (scores in `cur`), start tile t+1 (scores into `nxt`).
    // On entry tile t+1 is the only load in flight: wait for this wave's part, barrier (all
    // of tile t+1 is in LDS, every wave is done with step t-1), then refill the slots step
    // t-1 read last (K slot t%2 held K(t), V slot (t+2)%3 held V(t-1)) with tile t+2.
    auto step = [&](int t, f32x16 (&cur)[QB][2], f32x16 (&nxt)[QB][2]) {
        attn_wait_vmcnt<0>();
        __syncthreads();
        const int vnext2 = vslot == 0 ? 2 : vslot - 1;   // (vslot + 2) % 3
        if (t + 2 < s1) issue_kv(t + 2, t & 1, vnext2);
        bf16x8 kf0[2][2];
        load_kfrags(t + 1, 0, kf0);
        __builtin_amdgcn_sched_barrier(0);
        if (MEASURE) update_max(cur, t == s0);
        compute_s(t + 1, nxt, kf0);
        exponentials(cur, pf);
        accumulate_o(vslot, pf);
        vslot = vslot == 2 ? 0 : vslot + 1;
    };
    const bool mask_last = ragged && s1 == nt;
    int t = s0;
#pragma unroll 1
    for (; t + 2 < s1; t += 2) {
        step(t, sa, sb);
        step(t + 1, sb, sa);
    }
    if (t + 1 < s1) {            // one more pipelined step, last tile's scores end up in sb
        step(t, sa, sb);
        if (mask_last) mask_tail(nt - 1, sb);
        update_max(sb, s1 - s0 == 1);
        exponentials(sb, pf);
    } else {                     // last tile's scores are in sa
        if (mask_last) mask_tail(nt - 1, sa);
        update_max(sa, s1 - s0 == 1);
        exponentials(sa, pf);
    }
    // the last tile's V^T landed before the barrier of the step before (or of the prologue)
    if ((Tk & 7) && s1 == nt) {
        zero_pad_keys(nt - 1, vslot);
        __syncthreads();
    }
    accumulate_o(vslot, pf);

    if (!MEASURE) {
        // did the attempt stay in range?  (a row sum of +inf, or NaN anywhere, says no)
        float mag = l[0];
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) mag += fabsf(o[0][db][v]);
        const bool bad = __builtin_amdgcn_ballot_w64(!(mag <= 3.0e38f)) != 0ull;
        if (bad && lane == 0) *wg_redo = 1;
        __syncthreads();             // (which also ends every wavefront's LDS reads of this attempt)
        if (__builtin_expect(*wg_redo != 0, 0)) return true;
    }

    // ---- a whole tile is normalised and stored; half of a cut tile leaves its state behind
    if (part < 0) {
        store_queries(o[0], l[0], out, ldo, b, Tq, q0 + l32, head, hi);
    } else if (!arrived) {
        float* pp = parts + ((size_t)(tile - nfull) * 2 + part) * PART_FLOATS + tid;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) pp[(db * 16 + v) * 256] = o[0][db][v];
        pp[32 * 256] = m[0];
        pp[33 * 256] = l[0];
    } else {
        // Merge inside the launch: both halves leave their state (device-scope stores: the other
        // half may run on another XCD), then count themselves in; the one that arrives second
        // reads the first one's state and finishes the tile.  Nobody waits.  The counter is
        // zero before the launch and the second arrival puts it back.
        const int cut = tile - nfull;
        float* pp = parts + ((size_t)cut * 2 + part) * PART_FLOATS + tid;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) __hip_atomic_store(pp + (db * 16 + v) * 256, o[0][db][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pp + 32 * 256, m[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pp + 33 * 256, l[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a device-scope store counts until it is visible at that scope
        __syncthreads();                                    // ... for every wave of this half; LDS is free from here on
        lds_i32* const first = reinterpret_cast<lds_i32*>(ldsK);
        if (tid == 0) *first = __hip_atomic_fetch_add(arrived + cut, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*first == 1) {
            if (tid == 0) __hip_atomic_store(arrived + cut, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float* po = parts + ((size_t)cut * 2 + (1 - part)) * PART_FLOATS + tid;
            const float mo = __hip_atomic_load(po + 32 * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float lo = __hip_atomic_load(po + 33 * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // the halves' maxima are in score units, or already in exponent units when the keys were prescaled
            const float cm = PRE ? 1.0f : c;
            const float mm = fmaxf(m[0], mo);
            const float fs = __builtin_amdgcn_exp2f((m[0] - mm) * cm), fo = __builtin_amdgcn_exp2f((mo - mm) * cm);
            // same expression, operand for operand, whichever half arrives second: first half's term, then second's
            const float f0 = part == 0 ? fs : fo, f1 = part == 0 ? fo : fs;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float ov = __hip_atomic_load(po + (db * 16 + v) * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const float a0 = part == 0 ? o[0][db][v] : ov, a1 = part == 0 ? ov : o[0][db][v];
                    o[0][db][v] = a0 * f0 + a1 * f1;
                }
            const float lsum = (part == 0 ? l[0] : lo) * f0 + (part == 0 ? lo : l[0]) * f1;
            store_queries(o[0], lsum, out, ldo, b, Tq, q0 + l32, head, hi);
        }
    }
    return false;
}

template <bool PRE>
__global__ __launch_bounds__(256, 3) void attention_kernel(const uint16_t* __restrict__ q, int64_t ldq,
                                                        const uint16_t* __restrict__ k, int64_t ldk,
                                                        const uint16_t* __restrict__ vt, int64_t ldvt,
                                                        uint16_t* __restrict__ out, int64_t ldo,
                                                        int Tq, int Tk, int Tkp, int heads, int qtiles, float c,
                                                        int nfull, int nsplit, float* __restrict__ parts, int32_t* __restrict__ arrived) {
    __shared__ u32x4 ldsK[2 * 64 * 8];
    __shared__ u32x4 ldsV[3 * 64 * 8];
    __shared__ int32_t wg_redo;         // PRE: some wavefront's unmeasured attempt overflowed
    lds_u32x4* const lk = (lds_u32x4*)ldsK;
    lds_u32x4* const lv = (lds_u32x4*)ldsV;
    lds_i32* const redo = (lds_i32*)&wg_redo;
    if constexpr (PRE) {
        if (threadIdx.x == 0) *redo = 0;    // (ordered before its first use by the key loop's barriers)
        if (attention_body<true, false>(q, ldq, k, ldk, vt, ldvt, out, ldo, Tq, Tk, Tkp, heads, qtiles, c, nfull, nsplit, parts, arrived, lk, lv, redo,
                                        (int)threadIdx.x, (int)blockIdx.x)) {
            // Second attempt, in the measured form, for inputs whose scores climb by more than 2^100
            // over a key range.  Its inputs pass through empty assembly statements so that it shares
            // no value with the first attempt: nothing of it may stay in registers through the first
            // attempt's key loop and tail.
            int tid2 = threadIdx.x, bid2 = blockIdx.x;
            const uint16_t *q2 = q, *k2 = k, *vt2 = vt;
            uint16_t* out2 = out;
            lds_u32x4 *lk2 = lk, *lv2 = lv;
            asm volatile("" : "+v"(tid2), "+s"(bid2), "+s"(q2), "+s"(k2), "+s"(vt2), "+s"(out2), "+s"(lk2), "+s"(lv2));
            (void)attention_body<true, true>(q2, ldq, k2, ldk, vt2, ldvt, out2, ldo, Tq, Tk, Tkp, heads, qtiles, c, nfull, nsplit, parts, arrived, lk2, lv2,
                                             redo, tid2, bid2);
        }
    } else {
        (void)attention_body<false, true>(q, ldq, k, ldk, vt, ldvt, out, ldo, Tq, Tk, Tkp, heads, qtiles, c, nfull, nsplit, parts, arrived, lk, lv, redo,
                                          (int)threadIdx.x, (int)blockIdx.x);
    }
}

// One workgroup per cut tile: combine the two halves about their common maximum.
__global__ __launch_bounds__(256) void attention_merge_kernel(const float* __restrict__ parts, uint16_t* __restrict__ out, int64_t ldo,
                                                              int Tq, int heads, int qtiles, int nfull, float c) {
    const int tile = nfull + blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const float* pa = parts + ((size_t)blockIdx.x * 2) * PART_FLOATS + tid;
    const float* pb = pa + PART_FLOATS;
    const float ma = pa[32 * 256], mb = pb[32 * 256];
    const float mm = fmaxf(ma, mb);
    const float fa = __builtin_amdgcn_exp2f((ma - mm) * c), fb = __builtin_amdgcn_exp2f((mb - mm) * c);
    f32x16 o[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = pa[(db * 16 + v) * 256] * fa + pb[(db * 16 + v) * 256] * fb;
    const float l = pa[33 * 256] * fa + pb[33 * 256] * fb;
    const int qt = tile % qtiles;
    const int head = (tile / qtiles) % heads, b = tile / (qtiles * heads);
    store_queries(o, l, out, ldo, b, Tq, qt * 128 + wave * 32 + l32, head, hi);
}

// CUs of the current device (cached; the query allocates nothing)
static int device_cus() {
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

// number of tiles to cut in half (0: one workgroup per tile)
static int attention_nsplit(int Bn, int Tq, int Tk, int heads) {
    const long tiles = (long)((Tq + 127) / 128) * heads * Bn;
    const int nt = (Tk + 63) / 64;
    const long cus = device_cus();
    if (nt < 8 || tiles <= 2 * cus || tiles >= 3 * cus) return 0;
    const long nsplit = 3 * cus - tiles, nfull = tiles - nsplit;
    if (nfull <= 0 || (nfull & 7) || (nsplit & 3)) return 0;
    return (int)nsplit;
}

size_t attention_scratch_bytes(int Bn, int Tq, int Tk, int heads) {
    if (Bn <= 0 || Tq <= 0 || Tk <= 0 || heads <= 0) return 0;
    return (size_t)attention_nsplit(Bn, Tq, Tk, heads) * 2 * PART_FLOATS * sizeof(float);
}

int launch_attention(const uint16_t* q, int64_t ldq, const uint16_t* k, int64_t ldk,
                     const uint16_t* vt, int64_t ldvt, uint16_t* out, int64_t ldo,
                     int Bn, int Tq, int Tk, int Tkp, int heads, bool k_prescaled, void* scratch, size_t scratch_bytes, int* cut_tiles,
                     hipStream_t stream, int32_t* arrived, int arrived_n) {
    SD_REQUIRE(q && k && vt && out, SD_EINVAL, "attention: null pointer");
    SD_REQUIRE(Tk >= 1 && Tkp >= Tk && Tkp % 8 == 0, SD_EINVAL, "attention: Tk=%d Tkp=%d", Tk, Tkp);
    SD_REQUIRE(ldq % 8 == 0 && ldk % 8 == 0 && ldvt % 8 == 0 && ldo % 4 == 0, SD_EINVAL, "attention: leading dimensions");
    SD_REQUIRE(ldk > 0 && ldvt > 0 && ldk < (1 << 23) && ldvt < (1 << 23), SD_EINVAL, "attention: leading dimensions out of range");
    *cut_tiles = 0;
    if (Bn <= 0 || Tq <= 0 || heads <= 0) return SD_OK;
    const float c = 0.125f * 1.44269504088896340736f;   // 1/sqrt(64) * log2(e)
    const int qtiles = (Tq + 127) / 128;
    const long tiles = (long)qtiles * heads * Bn;
    SD_REQUIRE(tiles < (1l << 30), SD_EINVAL, "attention: problem too large");
    int nsplit = attention_nsplit(Bn, Tq, Tk, heads);
    const size_t need = (size_t)nsplit * 2 * PART_FLOATS * sizeof(float);
    if (nsplit > 0 && !(scratch && scratch_bytes >= need && (reinterpret_cast<uintptr_t>(scratch) & 15) == 0)) nsplit = 0;
    const int nfull = (int)tiles - nsplit;
    if (nsplit > arrived_n) arrived = nullptr;   // not enough counters: the halves are merged by the second kernel
    if (k_prescaled)
        hipLaunchKernelGGL((attention_kernel<true>), dim3((unsigned)(nfull + 2 * nsplit)), dim3(256), 0, stream, q, ldq, k, ldk, vt, ldvt, out,
                           ldo, Tq, Tk, Tkp, heads, qtiles, c, nfull, nsplit, static_cast<float*>(scratch), arrived);
    else
        hipLaunchKernelGGL((attention_kernel<false>), dim3((unsigned)(nfull + 2 * nsplit)), dim3(256), 0, stream, q, ldq, k, ldk, vt, ldvt, out,
                           ldo, Tq, Tk, Tkp, heads, qtiles, c, nfull, nsplit, static_cast<float*>(scratch), arrived);
    SD_HIP_CHECK(hipGetLastError());
    *cut_tiles = arrived ? 0 : nsplit;
    return SD_OK;
}

int launch_attention_merge(const void* scratch, uint16_t* out, int64_t ldo, int Bn, int Tq, int heads, bool k_prescaled, int cut_tiles,
                           hipStream_t stream) {
    if (cut_tiles <= 0) return SD_OK;
    // the halves' maxima are in score units, or already in exponent units when the keys were prescaled
    const float c = k_prescaled ? 1.0f : 0.125f * 1.44269504088896340736f;
    const int qtiles = (Tq + 127) / 128;
    const int nfull = qtiles * heads * Bn - cut_tiles;
    hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned)cut_tiles), dim3(256), 0, stream, static_cast<const float*>(scratch), out, ldo,
                       Tq, heads, qtiles, nfull, c);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

}  // namespace sd
