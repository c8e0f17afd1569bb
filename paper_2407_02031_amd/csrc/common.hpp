// Shared device/host helpers of the gfx950 kernels: vector types, bf16 conversion,
// error reporting.  gfx950 only; wavefront = 64 lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdarg.h>
#include <stdio.h>
#include <type_traits>

#include "../../include/swiftdiff.h"

namespace sd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- bf16 <-> f32 (bit level; round-to-nearest-even) ----
// A pointer the program knows to be wave-uniform, pinned into scalar registers (inline
// assembly operands with an "s" constraint need this where the compiler cannot prove it).
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
    return reinterpret_cast<const void*>((static_cast<uint64_t>(hi) << 32) | lo);
}
// Both halves of a wavefront see both halves' values of x: on return lo holds the value of
// lane (l % 32) and hi that of lane (l % 32) + 32, in every lane.  Written as inline assembly
// with both registers as read-write operands: given the same value twice, the compiler's
// builtin for this instruction was seen to fold the two results into one.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}
// Sum over the 64 lanes of a wavefront, result in every lane, without LDS traffic: four
// DPP steps inside each row of 16 lanes (swap lane pairs, swap pairs, mirror the half rows,
// mirror the row: after each step the lanes that were combined hold equal values, so the
// mirrors act as exchanges), then the row-pair and half-wavefront swaps.
__device__ __forceinline__ float dpp_add(float v, const int which) {
    const int x = __builtin_bit_cast(int, v);
    int y;
    if (which == 0) y = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
    else if (which == 1) y = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
    else if (which == 2) y = __builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, false);  // row_half_mirror
    else y = __builtin_amdgcn_update_dpp(0, x, 0x140, 0xf, 0xf, false);                  // row_mirror
    return v + __builtin_bit_cast(float, y);
}
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add(v, 0);
    v = dpp_add(v, 1);
    v = dpp_add(v, 2);
    v = dpp_add(v, 3);
    float a = v, b = v;   // odd rows of a <-> even rows of b: a + b is the sum of each row pair
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    v = a + b;
    float lo, hi;
    both_halves(v, lo, hi);
    return lo + hi;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);   // finite inputs only on this path
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// ---- error text (per host thread) ----
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

#define SD_HIP_CHECK(expr)                                         \
    do {                                                           \
        hipError_t _e = (expr);                                    \
        if (_e != hipSuccess) return ::sd::hip_fail(_e, #expr);    \
    } while (0)

#define SD_REQUIRE(cond, code, ...)                                \
    do {                                                           \
        if (!(cond)) { ::sd::set_error(__VA_ARGS__); return (code); } \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Bump allocator over the caller's workspace (256-byte granules).
struct Workspace {
    char* base; size_t size; size_t used;
    Workspace(void* p, size_t n) : base(static_cast<char*>(p)), size(n), used(0) {}
    void* take(size_t bytes) {
        size_t b = round_up(bytes, 256);
        if (!base || used + b > size) { used = size + 1; return nullptr; }
        void* r = base + used; used += b; return r;
    }
    bool ok() const { return used <= size; }
};

// ---------------------------------------------------------------------------------------
// Grouped GEMM:  D[p][q] = alpha * sum_k P[p][k] Q[q][k]  over two K segments, then
// + bias, GEGLU, + residual, store.  Both operands are K-contiguous (row-major [rows, K]).
// ---------------------------------------------------------------------------------------
struct GemmProblem {
    const uint16_t* p0; const uint16_t* q0;   // segment 0: P [Mp, K0], Q [Nq, K0]
    const uint16_t* p1; const uint16_t* q1;   // segment 1 (LoRA: P = scaled x A^T, Q = B), or null
    const uint16_t* bias;                      // per output column (or per row if bias_on_rows)
    const void* res;                           // [Mp, N], or null
    void* y;
    int64_t ldp0, ldq0, ldp1, ldq1, ldr, ldy;
    int32_t Mp, N;                             // output rows, output columns
    int32_t K0, K1;
    int32_t geglu_F;                           // > 0: Q has 2F rows (value, gate); N == F
    int32_t y_f32;                             // output dtype: 1 fp32, 0 bf16
    int32_t res_f32;                           // residual dtype (an fp32 stream may be added into a bf16 output)
    int32_t bias_on_rows;
    float alpha;
    int32_t tile_begin, tiles_m, tiles_n;      // filled by the launcher
    // Dependencies inside one launch (a down-projection and the base GEMM that reads it as its
    // second K segment).  signal: every finished tile of this problem adds 1 to
    // signal[row-tile index]; its y is bf16 without residual.  wait: before loading K segment 1
    // a tile waits until wait[i] >= wait_need for every row-tile i of the producer that covers
    // its P rows (or its Q rows if wait_cols).  Flags are zero when the launch starts.
    int32_t* signal;
    const int32_t* wait;
    int32_t wait_need;                         // filled by the launcher
    int32_t wait_cols;
};

constexpr int GEMM_MAX_PROBLEMS = 16;
struct GemmGroup {
    int32_t n;
    int32_t total_tiles;
    int32_t n_lead;                          // tiles of the signalling problems (first in the group), filled by the launcher
    int32_t zero_n;                          // the launch also clears zero_ptr[0 .. zero_n): the flags of the next launch
    int32_t* zero_ptr;
    int32_t first_tile[GEMM_MAX_PROBLEMS];   // copy of p[i].tile_begin, read by every workgroup in one scalar load
    GemmProblem p[GEMM_MAX_PROBLEMS];
};

// Launch every problem of `g` in one grid.  Problems must all be GEGLU or all plain; signalling
// problems come first and every problem that waits on one is in the same group.
int launch_gemm_group(GemmGroup& g, hipStream_t stream);
// n zeros at p (the flags of the first dependent launch of a call)
int launch_clear_flags(int32_t* p, int n, hipStream_t stream);
// number of tiles, since the library was loaded, that gave up waiting for a flag (0 unless the
// in-launch dependency protocol is broken); synchronises the device
int gemm_dep_timeouts(long long* count);

// LayerNorm rows of x [M, C] (fp32 or bf16) -> bf16.
// zero_ptr[0 .. zero_n) is cleared by the same launch (dependency flags of a later launch)
int launch_layernorm(const void* x, int x_f32, const uint16_t* gamma, const uint16_t* beta, float eps,
                     uint16_t* y, int M, int C, hipStream_t stream, int32_t* zero_ptr = nullptr, int zero_n = 0);
// fp32 [n] -> bf16, bf16 -> fp32 converters for the stack boundary
int launch_cvt_bf16_to_f32(const uint16_t* x, float* y, size_t n, hipStream_t stream);
int launch_cvt_f32_to_bf16(const float* x, uint16_t* y, size_t n, hipStream_t stream);

int launch_groupnorm(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta,
                     int Bn, int T, int C, int groups, float eps, float* partials, hipStream_t stream, bool silu = false);
size_t groupnorm_partials_bytes(int Bn, int T, int groups);

// scratch: attention_scratch_bytes(...) bytes, 16-byte aligned, for the launches that cut
// some tiles' key range in half (without it every workgroup takes one whole tile).
// arrived: arrived_n counters, zero before the launch and zero again after it; with them the
// half that finishes second merges the two inside the launch and *cut_tiles comes back 0
int launch_attention(const uint16_t* q, int64_t ldq, const uint16_t* k, int64_t ldk,
                     const uint16_t* vt, int64_t ldvt, uint16_t* out, int64_t ldo,
                     int Bn, int Tq, int Tk, int Tkp, int heads, bool k_prescaled, void* scratch, size_t scratch_bytes, int* cut_tiles,
                     hipStream_t stream, int32_t* arrived = nullptr, int arrived_n = 0);
// second kernel of a launch that cut tiles (*cut_tiles > 0 above): merges the halves into `out`
int launch_attention_merge(const void* scratch, uint16_t* out, int64_t ldo, int Bn, int Tq, int heads, bool k_prescaled, int cut_tiles,
                           hipStream_t stream);
// softmax scale in exponent-of-2 units: k_prescaled means the keys were multiplied by this
constexpr float ATTN_KSCALE = 0.125f * 1.44269504088896340736f;
size_t attention_scratch_bytes(int Bn, int Tq, int Tk, int heads);

}  // namespace sd
