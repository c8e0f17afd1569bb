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
// Workgroup: 4 wavefronts, each owning 32*QB queries; K / V^T tiles of 64 keys are staged
// in LDS (XOR-swizzled 16-byte chunks), double-buffered against the global loads.
#include "common.hpp"

namespace sd {

__device__ __forceinline__ int aswz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

constexpr float RESCALE_LOG2 = 8.0f;

template <int QB>
__global__ __launch_bounds__(256) void attention_kernel(const uint16_t* __restrict__ q, int64_t ldq,
                                                        const uint16_t* __restrict__ k, int64_t ldk,
                                                        const uint16_t* __restrict__ vt, int64_t ldvt,
                                                        uint16_t* __restrict__ out, int64_t ldo,
                                                        int Tq, int Tk, int Tkp, int heads, int qtiles, float c) {
    constexpr int BQ = 4 * 32 * QB;
    __shared__ u32x4 ldsK[2][64 * 8];   // [key][8 chunks of 8 d], 2-deep ring
    __shared__ u32x4 ldsV[3][64 * 8];   // [d][8 chunks of 8 keys, key order permuted], 3-deep ring

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // (sample, head, query tile) so that one head's K and V stay in one XCD's L2.
    const int total = gridDim.x;
    int wi = blockIdx.x;
    if ((total & 7) == 0) wi = (wi & 7) * (total >> 3) + (wi >> 3);
    const int qt = wi % qtiles;
    const int head = (wi / qtiles) % heads, b = wi / (qtiles * heads);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // ---- tile loaders: thread owns chunks (row lrow, lrow + 32; chunk lc) of both tiles
    const int lrow = tid >> 3, lc = tid & 7;
    const uint16_t* kbase = k + (int64_t)b * Tk * ldk + head * 64 + lc * 8;
    const uint16_t* vbase = vt + (int64_t)(head * 64) * ldvt + (int64_t)b * Tkp + lc * 8;
    u32x4 rk[2], rv[2];
    auto load_kv = [&](int t) {
        const int key0 = t * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = lrow + i * 32;
            int key = key0 + r;
            key = key < Tk ? key : Tk - 1;
            rk[i] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)key * ldk);
            const int kc = key0 + lc * 8;   // first key of this V^T chunk
            u32x4 v = {0u, 0u, 0u, 0u};
            if (kc < Tkp) {
                v = *reinterpret_cast<const u32x4*>(vbase + (int64_t)r * ldvt + key0);
                if (kc + 8 > Tk) {   // zero the padding keys: 0 * garbage must stay 0
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uint32_t w = v[e];
                        if (kc + 2 * e >= Tk) w &= 0xffff0000u;
                        if (kc + 2 * e + 1 >= Tk) w &= 0x0000ffffu;
                        v[e] = w;
                    }
                }
            }
            rv[i] = v;
        }
    };
    // K rows go in as they are.  V^T rows are stored with the keys of every 16-key group
    // permuted to [0-3, 8-11, 4-7, 12-15], the order in which the score accumulator of one
    // half-wavefront holds them, so the MFMA operand is a single 16-byte read.
    auto store_kv = [&](int kslot, int vslot) {
        u32x2* lv2 = reinterpret_cast<u32x2*>(ldsV[vslot]);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = lrow + i * 32;
            ldsK[kslot][r * 8 + aswz(r, lc)] = rk[i];
            const int c0 = aswz(r, lc & ~1);           // physical chunk of the group's first half
            const int c1 = c0 ^ 1;
            const u32x2 lo = {rv[i][0], rv[i][1]}, hh = {rv[i][2], rv[i][3]};
            lv2[(r * 8 + c0) * 2 + (lc & 1)] = lo;
            lv2[(r * 8 + c1) * 2 + (lc & 1)] = hh;
        }
    };

    f32x16 o[QB][2];
    float m[QB], l[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = -INFINITY;
        l[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][db][v] = 0.f;
    }

    // S^T tile of key tile t: 64 keys x (32*QB) queries
    auto compute_s = [&](int t, f32x16 (&s)[QB][2]) {
        const u32x4* lk = ldsK[t & 1];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[qb][kb][v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int r = kb * 32 + l32;
                const bf16x8 a = __builtin_bit_cast(bf16x8, lk[r * 8 + aswz(r, kk * 2 + hi)]);
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
                const int key = t * 64 + kb * 32 + 8 * (v >> 2) + 4 * hi + (v & 3);
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
    auto update_max = [&](f32x16 (&s)[QB][2]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = fmaxf(s[qb][0][0], s[qb][1][0]);
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, s[qb][0][v]), s[qb][1][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
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
                        const float p0 = __builtin_amdgcn_exp2f(s[qb][kb][g2 * 8 + 2 * e] * c - mc);
                        const float p1 = __builtin_amdgcn_exp2f(s[qb][kb][g2 * 8 + 2 * e + 1] * c - mc);
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
    // O^T += V^T P^T.  k-slot j of sub-step (kb, g2) is key kb*32 + 16*g2 + 8*(j/4) + 4*hi + j%4,
    // which is the 16-byte piece (2*(kb*2+g2) + hi) of the permuted V^T row
    auto accumulate_o = [&](int vslot, bf16x8 (&pf)[QB][2][2]) {
        const u32x4* lv = ldsV[vslot];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    const int r = db * 32 + l32;
                    const bf16x8 a = __builtin_bit_cast(bf16x8, lv[r * 8 + aswz(r, kb * 4 + g2 * 2 + hi)]);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qb][kb][g2], o[qb][db], 0, 0, 0);
                }
    };

    // ---- prologue: tiles 0 and 1 into LDS, S of tile 0
    const int nt = (Tk + 63) >> 6;
    load_kv(0);
    store_kv(0, 0);
    if (nt > 1) {
        load_kv(1);
        store_kv(1, 1);
    }
    __syncthreads();
    f32x16 sa[QB][2], sb[QB][2];
    compute_s(0, sa);

    // ---- main loop, software-pipelined: the score MFMAs of tile t+1 are independent of the
    // exponentials of tile t and sit in the same basic block, so the matrix pipe and the
    // vector ALU overlap inside one wavefront.  Two tiles per trip (the score buffers swap
    // roles), the last tile is peeled: nothing to prefetch, and only it may need masking.
    int vslot = 0;
    bf16x8 pf[QB][2][2];
    // one pipelined step: finish tile t (scores in `cur`), start tile t+1 (scores into `nxt`)
    auto step = [&](int t, f32x16 (&cur)[QB][2], f32x16 (&nxt)[QB][2]) {
        const bool pre = t + 2 < nt;
        if (pre) load_kv(t + 2);
        update_max(cur);
        compute_s(t + 1, nxt);
        exponentials(cur, pf);
        accumulate_o(vslot, pf);
        // tile t+2: K slot t%2 was last read for S(t) one step ago, V slot (t+2)%3 for
        // tile t-1: both free since the previous barrier
        const int vnext2 = vslot == 0 ? 2 : vslot - 1;   // (vslot + 2) % 3
        if (pre) store_kv(t & 1, vnext2);
        vslot = vslot == 2 ? 0 : vslot + 1;
        __syncthreads();
    };
    int t = 0;
#pragma unroll 1
    for (; t + 2 < nt; t += 2) {
        step(t, sa, sb);
        step(t + 1, sb, sa);
    }
    if (t + 1 < nt) {            // one more pipelined step, last tile's scores end up in sb
        step(t, sa, sb);
        if ((nt - 1) * 64 + 64 > Tk) mask_tail(nt - 1, sb);
        update_max(sb);
        exponentials(sb, pf);
        accumulate_o(vslot, pf);
    } else {                     // last tile's scores are in sa
        if ((nt - 1) * 64 + 64 > Tk) mask_tail(nt - 1, sa);
        update_max(sa);
        exponentials(sa, pf);
        accumulate_o(vslot, pf);
    }

    // ---- normalise and store: lane holds query l32, d = db*32 + 8*(v/4) + 4*hi + v%4
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float lt = l[qb] + __shfl_xor(l[qb], 32, 64);
        const float inv = 1.0f / lt;
        const int row = q0 + qb * 32 + l32;
        if (row < Tq) {
            uint16_t* op = out + ((int64_t)b * Tq + row) * ldo + head * 64 + 4 * hi;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[qb][db][4 * v4 + e] * inv);
                    *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * v4) = w;
                }
        }
    }
}

int launch_attention(const uint16_t* q, int64_t ldq, const uint16_t* k, int64_t ldk,
                     const uint16_t* vt, int64_t ldvt, uint16_t* out, int64_t ldo,
                     int Bn, int Tq, int Tk, int Tkp, int heads, hipStream_t stream) {
    SD_REQUIRE(q && k && vt && out, SD_EINVAL, "attention: null pointer");
    SD_REQUIRE(Tk >= 1 && Tkp >= Tk && Tkp % 8 == 0, SD_EINVAL, "attention: Tk=%d Tkp=%d", Tk, Tkp);
    SD_REQUIRE(ldq % 8 == 0 && ldk % 8 == 0 && ldvt % 8 == 0 && ldo % 4 == 0, SD_EINVAL, "attention: leading dimensions");
    if (Bn <= 0 || Tq <= 0 || heads <= 0) return SD_OK;
    const float c = 0.125f * 1.44269504088896340736f;   // 1/sqrt(64) * log2(e)
    const int qtiles = (Tq + 127) / 128;
    dim3 grid((unsigned)(qtiles * heads * Bn));
    hipLaunchKernelGGL(attention_kernel<1>, grid, dim3(256), 0, stream, q, ldq, k, ldk, vt, ldvt, out, ldo, Tq, Tk, Tkp, heads, qtiles, c);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

}  // namespace sd
