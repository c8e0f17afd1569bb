// In-place LoRA patching for gfx950: W <- W + scale * (B A) over a list of fp32 matrices in
// one grouped launch, with W's old bits saved to an undo record in the same pass, and the
// inverse pass that copies them back (Section 4.2, "Efficient LoRA patching": merge into the
// base parameters in place; take the adapter off after the request).
//
// HBM-bound: 4 B read + 4 B write (+ 4 B undo) per element against 2r FLOP, so the rank-r
// product must not become the limit: it runs on the fp32 matrix cores (32x32x2 MFMA) while
// the W loads of the same tile are in flight.  One wavefront owns 32 rows x 128 columns;
// lane l holds columns c0 + 4*(l%32) + {0..3} of 16 rows, i.e. four MFMA column blocks
// interleaved so that every W access is a 16-byte float4 and a wavefront load covers two
// 512-byte row segments.
#include "common.hpp"

namespace sd {

// streaming accesses: W, W' and the undo record are touched exactly once per pass
typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float* p) {
    nt_f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(p));
    return float4{t[0], t[1], t[2], t[3]};
}
__device__ __forceinline__ void nt_store4(float* p, float4 v) {
    nt_f32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<nt_f32x4*>(p));
}
#define NT_LOAD4(p) nt_load4(p)
#define NT_STORE4(p, v) nt_store4(p, v)

// These kernels stream: what limits them is how well HBM copes with the mix of requests in
// flight, and past a point more wavefronts per CU make that worse (more streams interleaved per
// channel).  The copies back therefore ask for dynamic LDS that no kernel touches, only to cap
// the workgroups per CU (160 KB of LDS per CU) at six: +5 % on the 310-matrix sweep.  The patch
// pass is capped by its registers at four workgroups per CU, which is where it runs best (a cap
// of three cost 4 % once the undo record went out first; two cost 15 %).
constexpr int UNPATCH_THROTTLE_LDS = 24 * 1024;

struct PatchPlanEntry {
    sd_patch_desc d;       // 48 bytes
    int64_t tile_begin;    // first workgroup tile of this matrix
    int32_t tiles_c;       // column tiles (128 wide)
    int32_t ntiles;        // workgroup tiles of this matrix
};
static_assert(sizeof(sd_patch_desc) == 48, "descriptor layout");
static_assert(sizeof(PatchPlanEntry) == 64, "plan entry layout");

// workgroup tile: PT_WAVES wavefronts side by side, 32 rows x 128 columns each (two waves
// per workgroup measured ~4 % faster than four or one on the 310-matrix sweep)
struct PatchMultiEntry {
    sd_patch_multi_desc d;
    int64_t tile_begin;
    int32_t tiles_c;
    int32_t ntiles;
};
static_assert(sizeof(PatchMultiEntry) % 8 == 0, "plan entry layout");

constexpr int PT_WAVES = 2;
constexpr int PT_ROWS = 32, PT_COLS = 128 * PT_WAVES;
constexpr int PT_THREADS = 64 * PT_WAVES;

__device__ __forceinline__ int find_entry(const PatchPlanEntry* __restrict__ plan, int n, int64_t tile) {
    int lo = 0, hi = n - 1;   // last entry with tile_begin <= tile
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (plan[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// k pairs per batch of fragment loads in the rank-32 path.  Measured on the 310-matrix sweep:
// 8 beats 16 (all fragments up front) by 1 % with one adapter and by 10 % with two, and beats 4
// and 2; requesting a batch while the batch before it multiplies (double registers) lost.
constexpr int FRAG_KP = 8;
// acc[j][v] += sum_k B[row(v)][k] * A[k][col + j] for one adapter on a full tile (all 32 rows
// and 128 columns inside the matrix, in % 4 == 0): lane l32 supplies B row r0 + l32 and the
// four A columns col..col+3, k pair (2 kp + hi) per MFMA.
__device__ __forceinline__ void delta_full(const float* __restrict__ A, const float* __restrict__ B, int r, int in, int r0,
                                           int col, int l32, int hi, f32x16 (&acc)[4]) {
    const float* bp = B + (size_t)(r0 + l32) * r + hi;
    const float* ap = A + (size_t)hi * in + col;
    const int kp_n = r >> 1;
    if (r == 32) {
        // the common rank: the A and B fragments (they come out of L2) are requested in two
        // batches of FRAG_KP k pairs, 32 MFMAs behind each
#pragma unroll 1
        for (int k0 = 0; k0 < 16; k0 += FRAG_KP) {
            float bv[FRAG_KP];
            float4 av[FRAG_KP];
#pragma unroll
            for (int kp = 0; kp < FRAG_KP; ++kp) bv[kp] = bp[2 * (k0 + kp)];
#pragma unroll
            for (int kp = 0; kp < FRAG_KP; ++kp) av[kp] = *reinterpret_cast<const float4*>(ap + (size_t)(2 * (k0 + kp)) * in);
#pragma unroll
            for (int kp = 0; kp < FRAG_KP; ++kp) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[kp], av[kp].x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[kp], av[kp].y, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[kp], av[kp].z, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[kp], av[kp].w, acc[3], 0, 0, 0);
            }
        }
    } else {
#pragma unroll 4
        for (int kp = 0; kp < kp_n; ++kp) {
            const float bv = bp[2 * kp];
            const float4 av = *reinterpret_cast<const float4*>(ap + (size_t)(2 * kp) * in);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.x, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.y, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.z, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.w, acc[3], 0, 0, 0);
        }
    }
    if (r & 1) {   // odd rank: last k pairs with a zero
        const int kk = r - 1;
        const float bv = hi ? 0.f : B[(size_t)(r0 + l32) * r + kk];
        float4 av = {0.f, 0.f, 0.f, 0.f};
        if (!hi) av = *reinterpret_cast<const float4*>(A + (size_t)kk * in + col);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.x, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.y, acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.z, acc[2], 0, 0, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av.w, acc[3], 0, 0, 0);
    }
}

// the same product on a ragged tile: every access guarded and scalar
__device__ __forceinline__ void delta_ragged(const float* __restrict__ A, const float* __restrict__ B, int r, int out, int in,
                                             int r0, int col, int l32, int hi, f32x16 (&acc)[4]) {
    const int brow = r0 + l32;
    const int kp_n = (r + 1) >> 1;
#pragma unroll 1
    for (int kp = 0; kp < kp_n; ++kp) {
        const int kk = 2 * kp + hi;
        const bool kv = kk < r;
        const float bv = (kv && brow < out) ? B[(size_t)brow * r + kk] : 0.f;
        float av[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) av[j] = (kv && col + j < in) ? A[(size_t)kk * in + col + j] : 0.f;
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[0], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[1], acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[2], acc[2], 0, 0, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, av[3], acc[3], 0, 0, 0);
    }
}

__global__ __launch_bounds__(PT_THREADS, 2) void lora_patch_kernel(const PatchPlanEntry* __restrict__ plan, int n) {
    const int64_t tile = blockIdx.x;
    const PatchPlanEntry& E = plan[find_entry(plan, n, tile)];
    const int out = E.d.out, in = E.d.in, r = E.d.r;
    const float scale = E.d.scale;
    float* __restrict__ W = E.d.W;
    float* __restrict__ U = E.d.undo;
    const float* __restrict__ A = E.d.A;
    const float* __restrict__ B = E.d.B;
    const int local = (int)(tile - E.tile_begin);
    const int tc = local % E.tiles_c, tr = local / E.tiles_c;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int r0 = tr * PT_ROWS;
    const int c0 = tc * PT_COLS + wave * 128;
    if (c0 >= in) return;
    const int col = c0 + 4 * l32;
    const bool full = (r0 + 32 <= out) && (c0 + 128 <= in) && ((in & 3) == 0);

    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    if (full) {
        float4 w[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            w[v] = NT_LOAD4(W + (size_t)row * in + col);
        }
        // the undo record needs nothing but W: it goes out as one burst of stores before the
        // rank-r product, whose MFMAs then run under those stores (a little faster than with the
        // undo and result stores interleaved afterwards)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            NT_STORE4(U + (size_t)row * in + col, w[v]);
        }
        delta_full(A, B, r, in, r0, col, l32, hi, acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            const size_t idx = (size_t)row * in + col;
            float4 o;
            o.x = __fadd_rn(w[v].x, __fmul_rn(scale, acc[0][v]));
            o.y = __fadd_rn(w[v].y, __fmul_rn(scale, acc[1][v]));
            o.z = __fadd_rn(w[v].z, __fmul_rn(scale, acc[2][v]));
            o.w = __fadd_rn(w[v].w, __fmul_rn(scale, acc[3][v]));
            NT_STORE4(W + idx, o);
        }
    } else {
        // ragged tile: same arithmetic, every access guarded and scalar
        delta_ragged(A, B, r, out, in, r0, col, l32, hi, acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            if (row >= out) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (col + j >= in) continue;
                const size_t idx = (size_t)row * in + col + j;
                const float wv = W[idx];
                U[idx] = wv;
                W[idx] = __fadd_rn(wv, __fmul_rn(scale, acc[j][v]));
            }
        }
    }
}

__device__ __forceinline__ int find_entry_multi(const PatchMultiEntry* __restrict__ plan, int n, int64_t tile) {
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (plan[mid].tile_begin <= tile) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Several adapters on one matrix in one pass over W (one or two LoRAs per request is the norm,
// Section 3.1; each is merged as in Section 4.2): the tile's W values stay in registers while
// the adapters are applied one after the other, W_i = fl32(W_{i-1} + fl32(scale_i * (B_i A_i))),
// so the result equals successive single patches bit for bit at one third of their traffic for
// two adapters.  Optionally also writes the bf16 copy of W' that the bf16 GEMMs read.
//
// CB: 32-column MFMA blocks per wavefront, interleaved so that lane l holds CB adjacent columns
// (c0 + CB * (l % 32) + {0 .. CB-1}) of 16 rows.  A workgroup covers 32 rows x 256 columns with
// 8 / CB wavefronts.  The second adapter doubles the matrix-core time of a tile (64 fp32 MFMAs of
// 64 clocks per adapter and 32 x 128 elements) while its traffic stays the same, and a wavefront
// that multiplies has nothing in flight.  CB = 2 keeps a tile in half the registers (W 32,
// accumulators 32), so four wavefronts fit a SIMD instead of two: measured 15 % slower on the
// 310-matrix sweep (8-byte accesses, more streams per channel), so CB = 4 is what is launched; what
// did help is the pipelined path below.
template <int CB>
struct PatchVec;
template <>
struct PatchVec<4> { typedef float4 type; };
template <>
struct PatchVec<2> { typedef float2 type; };
template <int CB>
__device__ __forceinline__ float& pv_at(typename PatchVec<CB>::type& v, int j) { return reinterpret_cast<float*>(&v)[j]; }

template <int CB>
__device__ __forceinline__ typename PatchVec<CB>::type nt_loadv(const float* p) {
    typedef float nt_vec __attribute__((ext_vector_type(CB)));
    nt_vec t = __builtin_nontemporal_load(reinterpret_cast<const nt_vec*>(p));
    typename PatchVec<CB>::type r;
#pragma unroll
    for (int j = 0; j < CB; ++j) reinterpret_cast<float*>(&r)[j] = t[j];
    return r;
}
template <int CB>
__device__ __forceinline__ void nt_storev(float* p, const typename PatchVec<CB>::type& v) {
    typedef float nt_vec __attribute__((ext_vector_type(CB)));
    nt_vec t;
#pragma unroll
    for (int j = 0; j < CB; ++j) t[j] = reinterpret_cast<const float*>(&v)[j];
    __builtin_nontemporal_store(t, reinterpret_cast<nt_vec*>(p));
}

// delta_full for CB column blocks: acc[j][v] += sum_k B[row(v)][k] * A[k][col + j]
template <int CB>
__device__ __forceinline__ void delta_full_cb(const float* __restrict__ A, const float* __restrict__ B, int r, int in, int r0,
                                              int col, int l32, int hi, f32x16 (&acc)[CB]) {
    typedef typename PatchVec<CB>::type vec;
    const float* bp = B + (size_t)(r0 + l32) * r + hi;
    const float* ap = A + (size_t)hi * in + col;
    const int kp_n = r >> 1;
    int kp0 = 0;
    // batches of FRAG_KP k pairs: fragments requested together, their MFMAs behind them
#pragma unroll 1
    for (; kp0 + FRAG_KP <= kp_n; kp0 += FRAG_KP) {
        float bv[FRAG_KP];
        vec av[FRAG_KP];
#pragma unroll
        for (int kp = 0; kp < FRAG_KP; ++kp) bv[kp] = bp[2 * (kp0 + kp)];
#pragma unroll
        for (int kp = 0; kp < FRAG_KP; ++kp) av[kp] = *reinterpret_cast<const vec*>(ap + (size_t)(2 * (kp0 + kp)) * in);
#pragma unroll
        for (int kp = 0; kp < FRAG_KP; ++kp)
#pragma unroll
            for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[kp], pv_at<CB>(av[kp], j), acc[j], 0, 0, 0);
    }
#pragma unroll 1
    for (; kp0 < kp_n; ++kp0) {
        const float bv = bp[2 * kp0];
        vec av = *reinterpret_cast<const vec*>(ap + (size_t)(2 * kp0) * in);
#pragma unroll
        for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, pv_at<CB>(av, j), acc[j], 0, 0, 0);
    }
    if (r & 1) {   // odd rank: last k with a zero partner
        const int kk = r - 1;
        const float bv = hi ? 0.f : B[(size_t)(r0 + l32) * r + kk];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const float a = hi ? 0.f : A[(size_t)kk * in + col + j];
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, a, acc[j], 0, 0, 0);
        }
    }
}

template <int CB>
__device__ __forceinline__ void delta_ragged_cb(const float* __restrict__ A, const float* __restrict__ B, int r, int out, int in,
                                                int r0, int col, int l32, int hi, f32x16 (&acc)[CB]) {
    const int brow = r0 + l32;
    const int kp_n = (r + 1) >> 1;
#pragma unroll 1
    for (int kp = 0; kp < kp_n; ++kp) {
        const int kk = 2 * kp + hi;
        const bool kv = kk < r;
        const float bv = (kv && brow < out) ? B[(size_t)brow * r + kk] : 0.f;
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const float a = (kv && col + j < in) ? A[(size_t)kk * in + col + j] : 0.f;
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv, a, acc[j], 0, 0, 0);
        }
    }
}

// A full tile under NA adapters of rank 32, the common case, as one straight line.  What a
// wavefront spends per tile is a chain of round trips: with the fragments of a batch requested
// only after the MFMAs of the batch before have been issued (a wavefront issues its 32x32x2 fp32
// MFMAs one per 64 clocks, in order), every batch pays an L2 round trip on top of its matrix
// time, and a second adapter adds all of its own.  Here the k pairs form units of PIPE_KP, the
// fragments of unit u + PIPE_DEPTH are requested before the MFMAs of unit u, across adapter
// boundaries, and the first units are requested ahead of the W tile itself.  Same MFMAs in the
// same order on the same operands as the plain loop: same bits.
// (measured on the 310-matrix sweep with two adapters: 2.77 ms with the plain loop, 2.55 ms with
// units of 4 k pairs two units ahead; three units ahead spills and loses; where W's undo stores
// sit among the first units makes no difference)
constexpr int PIPE_KP = 4, PIPE_DEPTH = 2;
template <int NA>
__device__ __forceinline__ void patch_tile_rank32(const PatchMultiEntry& E, int in, int r0, int col, int l32, int hi) {
    constexpr int UPA = 16 / PIPE_KP;            // units per adapter
    constexpr int U = NA * UPA, SLOTS = PIPE_DEPTH + 1;
    float* __restrict__ W = E.d.W;
    float* __restrict__ Und = E.d.undo;
    uint16_t* __restrict__ S = E.d.serving;
    float bvb[SLOTS][PIPE_KP];
    float4 avb[SLOTS][PIPE_KP];
    // addresses as a wave-uniform base (adapter, k pair: scalar arithmetic) plus one 32-bit byte
    // offset per lane for all of B's fragments and one for all of A's
    const uint32_t boff = (uint32_t)(((r0 + l32) * 32 + hi) * 4);
    const uint32_t aoff = (uint32_t)(((size_t)hi * in + col) * 4);
    auto issue = [&](int u, int slot) {
        const int a = u / UPA, k0 = (u % UPA) * PIPE_KP;
        const char* bbase = reinterpret_cast<const char*>(E.d.B[a]);
        const char* abase = reinterpret_cast<const char*>(E.d.A[a]);
#pragma unroll
        for (int kp = 0; kp < PIPE_KP; ++kp) bvb[slot][kp] = *reinterpret_cast<const float*>(bbase + 8 * (k0 + kp) + boff);
#pragma unroll
        for (int kp = 0; kp < PIPE_KP; ++kp)
            avb[slot][kp] = *reinterpret_cast<const float4*>(abase + (size_t)(2 * (k0 + kp)) * in * 4 + aoff);
    };
#pragma unroll
    for (int u = 0; u < PIPE_DEPTH && u < U; ++u) issue(u, u);
    // W, undo and serving addresses likewise: the row of register v lies d(v) = 8 * (v / 4) + v % 4
    // rows below the lane's first, a wave-uniform distance; one 32-bit byte offset per lane serves
    // all three arrays (the caller checked that the matrix has fewer than 2^30 elements)
    const uint32_t woff = (uint32_t)(((size_t)(r0 + 4 * hi) * in + col) * 4);
    auto row_bytes = [&](int v) -> size_t { return (size_t)(8 * (v >> 2) + (v & 3)) * in * 4; };
    float4 w[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) w[v] = NT_LOAD4(reinterpret_cast<const float*>(reinterpret_cast<const char*>(W) + row_bytes(v) + woff));
    // W's old bits go out first, as one burst of stores, before any adapter's product
#pragma unroll
    for (int v = 0; v < 16; ++v) NT_STORE4(reinterpret_cast<float*>(reinterpret_cast<char*>(Und) + row_bytes(v) + woff), w[v]);
    f32x16 acc[4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u % UPA == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
        }
        // (the scheduler is kept from hoisting every unit's requests to the top, which would need
        // registers for all of them at once)
        __builtin_amdgcn_sched_barrier(0);
        if (u + PIPE_DEPTH < U) issue(u + PIPE_DEPTH, (u + PIPE_DEPTH) % SLOTS);
        __builtin_amdgcn_sched_barrier(0);
        const int slot = u % SLOTS;
#pragma unroll
        for (int kp = 0; kp < PIPE_KP; ++kp) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bvb[slot][kp], avb[slot][kp].x, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bvb[slot][kp], avb[slot][kp].y, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bvb[slot][kp], avb[slot][kp].z, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bvb[slot][kp], avb[slot][kp].w, acc[3], 0, 0, 0);
        }
        if (u % UPA == UPA - 1) {
            const float scale = E.d.scale[u / UPA];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                w[v].x = __fadd_rn(w[v].x, __fmul_rn(scale, acc[0][v]));
                w[v].y = __fadd_rn(w[v].y, __fmul_rn(scale, acc[1][v]));
                w[v].z = __fadd_rn(w[v].z, __fmul_rn(scale, acc[2][v]));
                w[v].w = __fadd_rn(w[v].w, __fmul_rn(scale, acc[3][v]));
            }
        }
    }
    // (the offset is laundered so that the sixteen row addresses are formed again here instead of
    // being carried, or spilled, through the adapters' products)
    uint32_t woff2 = woff;
    asm volatile("" : "+v"(woff2));
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        NT_STORE4(reinterpret_cast<float*>(reinterpret_cast<char*>(W) + row_bytes(v) + woff2), w[v]);
        if (S) {
            bf16x4 o = {(__bf16)w[v].x, (__bf16)w[v].y, (__bf16)w[v].z, (__bf16)w[v].w};
            *reinterpret_cast<bf16x4*>(reinterpret_cast<char*>(S) + row_bytes(v) / 2 + woff2 / 2) = o;
        }
    }
}

template <int CB>
__global__ __launch_bounds__(64 * 8 / CB, CB == 2 ? 4 : 2) void lora_patch_multi_kernel(const PatchMultiEntry* __restrict__ plan, int n) {
    typedef typename PatchVec<CB>::type vec;
    const int64_t tile = blockIdx.x;
    const PatchMultiEntry& E = plan[find_entry_multi(plan, n, tile)];
    const int out = E.d.out, in = E.d.in, na = E.d.n_adapters;
    float* __restrict__ W = E.d.W;
    float* __restrict__ U = E.d.undo;
    uint16_t* __restrict__ S = E.d.serving;
    const int local = (int)(tile - E.tile_begin);
    const int tc = local % E.tiles_c, tr = local / E.tiles_c;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int r0 = tr * PT_ROWS;
    const int c0 = tc * PT_COLS + wave * (32 * CB);
    if (c0 >= in) return;
    const int col = c0 + CB * l32;
    const bool full = (r0 + 32 <= out) && (c0 + 32 * CB <= in) && ((in & 3) == 0);
    if constexpr (CB == 4) {
        bool all32 = full && (int64_t)out * in < (int64_t(1) << 30);
#pragma unroll
        for (int a = 0; a < SD_PATCH_MAX_ADAPTERS; ++a) all32 = all32 && (a >= na || E.d.r[a] == 32);
        // (one or two adapters, the production norm; with three or four the straight line would
        // need more registers than two wavefronts per SIMD leave, and the plain loop below serves)
        if (all32 && na == 1) { patch_tile_rank32<1>(E, in, r0, col, l32, hi); return; }
        if (all32 && na == 2) { patch_tile_rank32<2>(E, in, r0, col, l32, hi); return; }
    }
    f32x16 acc[CB];
    if (full) {
        vec w[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            w[v] = nt_loadv<CB>(W + (size_t)row * in + col);
        }
        // W's old bits go out first, as one burst of stores, before any adapter's product
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            nt_storev<CB>(U + (size_t)row * in + col, w[v]);
        }
#pragma unroll 1
        for (int a = 0; a < na; ++a) {
#pragma unroll
            for (int j = 0; j < CB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
            delta_full_cb<CB>(E.d.A[a], E.d.B[a], E.d.r[a], in, r0, col, l32, hi, acc);
            const float scale = E.d.scale[a];
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int j = 0; j < CB; ++j) pv_at<CB>(w[v], j) = __fadd_rn(pv_at<CB>(w[v], j), __fmul_rn(scale, acc[j][v]));
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            const size_t idx = (size_t)row * in + col;
            nt_storev<CB>(W + idx, w[v]);
            if (S) {
                typedef __bf16 bvec __attribute__((ext_vector_type(CB)));
                bvec o;
#pragma unroll
                for (int j = 0; j < CB; ++j) o[j] = (__bf16)pv_at<CB>(w[v], j);
                *reinterpret_cast<bvec*>(S + idx) = o;
            }
        }
    } else {
        float wv[16][CB];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                const bool ok = row < out && col + j < in;
                wv[v][j] = ok ? W[(size_t)row * in + col + j] : 0.f;
                if (ok) U[(size_t)row * in + col + j] = wv[v][j];
            }
        }
#pragma unroll 1
        for (int a = 0; a < na; ++a) {
#pragma unroll
            for (int j = 0; j < CB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
            delta_ragged_cb<CB>(E.d.A[a], E.d.B[a], E.d.r[a], out, in, r0, col, l32, hi, acc);
            const float scale = E.d.scale[a];
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int j = 0; j < CB; ++j) wv[v][j] = __fadd_rn(wv[v][j], __fmul_rn(scale, acc[j][v]));
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = r0 + 8 * (v >> 2) + 4 * hi + (v & 3);
            if (row >= out) continue;
#pragma unroll
            for (int j = 0; j < CB; ++j) {
                if (col + j >= in) continue;
                const size_t idx = (size_t)row * in + col + j;
                W[idx] = wv[v][j];
                if (S) S[idx] = __builtin_bit_cast(uint16_t, (__bf16)wv[v][j]);
            }
        }
    }
}

// W <- undo (flat linear copy), and the serving copy follows it: bf16(undo)
__global__ __launch_bounds__(PT_THREADS) void lora_unpatch_multi_kernel(const PatchMultiEntry* __restrict__ plan, int n) {
    const int64_t tile = blockIdx.x;
    const PatchMultiEntry& E = plan[find_entry_multi(plan, n, tile)];
    float* __restrict__ W = E.d.W;
    const float* __restrict__ U = E.d.undo;
    uint16_t* __restrict__ S = E.d.serving;
    const int64_t elems = (int64_t)E.d.out * E.d.in;
    // the matrix's workgroups sweep it together, see lora_unpatch_kernel
    const int64_t stride = (int64_t)E.ntiles * PT_THREADS * 4;
    int64_t i = ((tile - E.tile_begin) * PT_THREADS + threadIdx.x) * 4;
#pragma unroll 4
    for (; i + 4 <= elems; i += stride) {
        const float4 v = NT_LOAD4(U + i);
        NT_STORE4(W + i, v);
        if (S) {
            bf16x4 o = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
            *reinterpret_cast<bf16x4*>(S + i) = o;
        }
    }
    if (i < elems)   // the matrix's last 1..3 elements
        for (int64_t j = i; j < elems; ++j) {
            W[j] = U[j];
            if (S) S[j] = __builtin_bit_cast(uint16_t, (__bf16)U[j]);
        }
}

// Unpatch: W <- undo, a pure copy.  The matrix's workgroups (as many as the patch pass used)
// sweep it together as one flat array: in every round workgroup w copies the w-th 2 KB, so all
// that is in flight at any moment is one narrow, contiguous window of the matrix.  HBM likes
// that best: 6.0 TB/s, against 5.6 when every workgroup copies a contiguous 32 KB of its own.
__global__ __launch_bounds__(PT_THREADS) void lora_unpatch_kernel(const PatchPlanEntry* __restrict__ plan, int n) {
    const int64_t tile = blockIdx.x;
    const PatchPlanEntry& E = plan[find_entry(plan, n, tile)];
    float* __restrict__ W = E.d.W;
    const float* __restrict__ U = E.d.undo;
    const int64_t elems = (int64_t)E.d.out * E.d.in;
    const int64_t stride = (int64_t)E.ntiles * PT_THREADS * 4;
    int64_t i = ((tile - E.tile_begin) * PT_THREADS + threadIdx.x) * 4;
#pragma unroll 4
    for (; i + 4 <= elems; i += stride) NT_STORE4(W + i, NT_LOAD4(U + i));
    if (i < elems)   // the matrix's last 1..3 elements
        for (int64_t j = i; j < elems; ++j) W[j] = U[j];
}

}  // namespace sd

using namespace sd;

extern "C" size_t sd_patch_plan_bytes(int32_t n) { return n > 0 ? (size_t)n * sizeof(PatchPlanEntry) : 0; }

extern "C" int sd_patch_plan_build(const sd_patch_desc* descs, int32_t n, void* plan_host, size_t plan_bytes,
                                   int64_t* total_tiles) {
    SD_REQUIRE(n >= 0, SD_EINVAL, "patch plan: n=%d", n);
    SD_REQUIRE(total_tiles, SD_EINVAL, "patch plan: total_tiles is null");
    *total_tiles = 0;
    if (n == 0) return SD_OK;
    SD_REQUIRE(descs && plan_host, SD_EINVAL, "patch plan: null pointer");
    SD_REQUIRE(plan_bytes >= sd_patch_plan_bytes(n), SD_EWORKSPACE, "patch plan: buffer of %zu bytes, need %zu", plan_bytes,
               sd_patch_plan_bytes(n));
    PatchPlanEntry* plan = static_cast<PatchPlanEntry*>(plan_host);
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        const sd_patch_desc& d = descs[i];
        SD_REQUIRE(d.W && d.A && d.B && d.undo, SD_EINVAL, "patch desc %d: null pointer (W, A, B and undo are required)", i);
        SD_REQUIRE(aligned16(d.W) && aligned16(d.A) && aligned16(d.B) && aligned16(d.undo), SD_EINVAL,
                   "patch desc %d: pointers must be 16-byte aligned", i);
        SD_REQUIRE(d.out > 0 && d.in > 0 && d.r > 0 && d.r <= 1024, SD_EINVAL, "patch desc %d: out=%d in=%d r=%d", i, d.out, d.in, d.r);
        SD_REQUIRE(d.undo != d.W, SD_EINVAL, "patch desc %d: undo aliases W", i);
        plan[i].d = d;
        plan[i].tile_begin = total;
        plan[i].tiles_c = (d.in + PT_COLS - 1) / PT_COLS;
        const int64_t nt = (int64_t)plan[i].tiles_c * ((d.out + PT_ROWS - 1) / PT_ROWS);
        SD_REQUIRE(nt < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch desc %d: too many tiles", i);
        plan[i].ntiles = (int32_t)nt;
        total += nt;
    }
    SD_REQUIRE(total < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch plan: %lld tiles exceed one grid", (long long)total);
    *total_tiles = total;
    return SD_OK;
}

static int patch_launch(bool undo, const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    SD_REQUIRE(n >= 0 && total_tiles >= 0, SD_EINVAL, "patch: n=%d tiles=%lld", n, (long long)total_tiles);
    if (n == 0 || total_tiles == 0) return SD_OK;
    SD_REQUIRE(plan_dev, SD_EINVAL, "patch: plan is null");
    SD_REQUIRE(total_tiles < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch: %lld tiles exceed one grid", (long long)total_tiles);
    const PatchPlanEntry* plan = static_cast<const PatchPlanEntry*>(plan_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (undo) hipLaunchKernelGGL(lora_unpatch_kernel, dim3((unsigned)total_tiles), dim3(PT_THREADS), UNPATCH_THROTTLE_LDS, s, plan, n);
    else hipLaunchKernelGGL(lora_patch_kernel, dim3((unsigned)total_tiles), dim3(PT_THREADS), 0, s, plan, n);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_lora_patch(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    return patch_launch(false, plan_dev, n, total_tiles, stream);
}
extern "C" int sd_lora_unpatch(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    return patch_launch(true, plan_dev, n, total_tiles, stream);
}

extern "C" size_t sd_patch_multi_plan_bytes(int32_t n) { return n > 0 ? (size_t)n * sizeof(PatchMultiEntry) : 0; }

extern "C" int sd_patch_multi_plan_build(const sd_patch_multi_desc* descs, int32_t n, void* plan_host, size_t plan_bytes,
                                         int64_t* total_tiles) {
    SD_REQUIRE(n >= 0, SD_EINVAL, "patch plan: n=%d", n);
    SD_REQUIRE(total_tiles, SD_EINVAL, "patch plan: total_tiles is null");
    *total_tiles = 0;
    if (n == 0) return SD_OK;
    SD_REQUIRE(descs && plan_host, SD_EINVAL, "patch plan: null pointer");
    SD_REQUIRE(plan_bytes >= sd_patch_multi_plan_bytes(n), SD_EWORKSPACE, "patch plan: buffer of %zu bytes, need %zu", plan_bytes,
               sd_patch_multi_plan_bytes(n));
    PatchMultiEntry* plan = static_cast<PatchMultiEntry*>(plan_host);
    int64_t total = 0;
    for (int i = 0; i < n; ++i) {
        const sd_patch_multi_desc& d = descs[i];
        SD_REQUIRE(d.W && d.undo && aligned16(d.W) && aligned16(d.undo), SD_EINVAL, "patch desc %d: W and undo must be non-null and 16-byte aligned", i);
        SD_REQUIRE(d.undo != d.W, SD_EINVAL, "patch desc %d: undo aliases W", i);
        SD_REQUIRE(!d.serving || (reinterpret_cast<uintptr_t>(d.serving) & 7) == 0, SD_EINVAL, "patch desc %d: serving copy must be 8-byte aligned", i);
        SD_REQUIRE(d.out > 0 && d.in > 0, SD_EINVAL, "patch desc %d: out=%d in=%d", i, d.out, d.in);
        SD_REQUIRE(d.n_adapters >= 1 && d.n_adapters <= SD_PATCH_MAX_ADAPTERS, SD_EINVAL, "patch desc %d: %d adapters (1..%d)", i, d.n_adapters,
                   SD_PATCH_MAX_ADAPTERS);
        for (int a = 0; a < d.n_adapters; ++a) {
            SD_REQUIRE(d.A[a] && d.B[a] && aligned16(d.A[a]) && aligned16(d.B[a]), SD_EINVAL,
                       "patch desc %d adapter %d: A and B must be non-null and 16-byte aligned", i, a);
            SD_REQUIRE(d.r[a] > 0 && d.r[a] <= 1024, SD_EINVAL, "patch desc %d adapter %d: r=%d", i, a, d.r[a]);
        }
        plan[i].d = d;
        plan[i].tile_begin = total;
        plan[i].tiles_c = (d.in + PT_COLS - 1) / PT_COLS;
        const int64_t nt = (int64_t)plan[i].tiles_c * ((d.out + PT_ROWS - 1) / PT_ROWS);
        SD_REQUIRE(nt < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch desc %d: too many tiles", i);
        plan[i].ntiles = (int32_t)nt;
        total += nt;
    }
    SD_REQUIRE(total < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch plan: %lld tiles exceed one grid", (long long)total);
    *total_tiles = total;
    return SD_OK;
}

static int patch_multi_launch(bool undo, const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    SD_REQUIRE(n >= 0 && total_tiles >= 0, SD_EINVAL, "patch: n=%d tiles=%lld", n, (long long)total_tiles);
    if (n == 0 || total_tiles == 0) return SD_OK;
    SD_REQUIRE(plan_dev, SD_EINVAL, "patch: plan is null");
    SD_REQUIRE(total_tiles < (int64_t)0x7fffffff, SD_EUNSUPPORTED, "patch: %lld tiles exceed one grid", (long long)total_tiles);
    const PatchMultiEntry* plan = static_cast<const PatchMultiEntry*>(plan_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // (the multi-adapter patch kernel is held to fewer waves by its registers already)
    if (undo) hipLaunchKernelGGL(lora_unpatch_multi_kernel, dim3((unsigned)total_tiles), dim3(PT_THREADS), UNPATCH_THROTTLE_LDS, s, plan, n);
    else hipLaunchKernelGGL((lora_patch_multi_kernel<4>), dim3((unsigned)total_tiles), dim3(PT_THREADS), 0, s, plan, n);
    SD_HIP_CHECK(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_lora_patch_multi(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    return patch_multi_launch(false, plan_dev, n, total_tiles, stream);
}
extern "C" int sd_lora_unpatch_multi(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream) {
    return patch_multi_launch(true, plan_dev, n, total_tiles, stream);
}
