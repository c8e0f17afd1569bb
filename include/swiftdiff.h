/*
 * swiftdiff.h — C ABI of the MI355X (gfx950) kernels for the base-model denoising hot
 * path of SwiftDiffusion (arXiv 2407.02031): the LoRA-augmented SDXL spatial-transformer
 * block run on the classifier-free-guidance pair, and in-place LoRA patching.
 *
 * Conventions common to every call
 * --------------------------------
 *  - Return value: SD_OK (0) or a negative SD_E* code; sd_last_error() gives the text of
 *    the most recent failure on the calling thread.  Nothing is printed, nothing aborts.
 *  - "device" pointers are HIP device memory owned by the caller, 16-byte aligned, dense
 *    row-major.  "host" pointers are ordinary host memory read during the call only.
 *  - bf16 tensors are passed as uint16_t bit patterns.  Accumulation is always fp32.
 *  - Weights are stored [out, in]; y = x W^T.  A LoRA adapter is A [r, in] (down) and
 *    B [out, r] (up) with a scalar scale = alpha / r; r must be a multiple of 8.
 *  - The library never allocates, frees or synchronises.  Scratch memory comes from the
 *    caller's workspace `ws` (device, 256-byte aligned) of at least the size the matching
 *    *_workspace_bytes query returns; all work is enqueued on `stream` (a hipStream_t).
 *    Its contents on entry do not matter and are undefined afterwards.  A workspace belongs
 *    to one call at a time: the kernels of a call signal each other through flags in it, so
 *    two calls that may run concurrently (different streams, overlapping graph launches) need
 *    a workspace each.
 *  - Same inputs give bit-identical outputs run to run (atomics only count arrivals, they
 *    never carry data or decide an order of summation).
 */
#ifndef SWIFTDIFF_H
#define SWIFTDIFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SD_OK 0
#define SD_EINVAL (-1)       /* null / misaligned pointer, bad dimension or flag            */
#define SD_EUNSUPPORTED (-2) /* a shape the kernels do not cover (e.g. head dim != 64)      */
#define SD_EWORKSPACE (-3)   /* workspace missing or too small                              */
#define SD_EHIP (-4)         /* HIP runtime error; text in sd_last_error()                  */
#define SD_ETIMEOUT (-5)     /* bal: adapters still loading after the wait at the bound     */
#define SD_ELOAD (-6)        /* bal: a loader callback reported failure                      */

#define SD_BF16 0
#define SD_F32 1

#define SD_EPI_NONE 0
#define SD_EPI_GEGLU 1

/* One linear projection with an optional rank-r adapter (Section 2, "Low-Rank
 * Adaptation": the patched weight is the base weight plus a rank-r product).
 * All pointers are device memory; bias, A, B may be NULL (A and B together). */
typedef struct sd_proj {
    const uint16_t* W;    /* [N, K] bf16 (GEGLU: [2N, K], value rows first, gate rows second) */
    const uint16_t* bias; /* [N] bf16 (GEGLU: [2N]) or NULL                                   */
    const uint16_t* A;    /* [r, K] bf16 or NULL                                              */
    const uint16_t* B;    /* [N, r] bf16 (GEGLU: [2N, r]) or NULL                             */
    int32_t r;            /* adapter rank; 0 = none                                           */
    float scale;          /* alpha / r                                                        */
} sd_proj;

/* Parameters of one transformer block (all device pointers, bf16). */
typedef struct sd_block_params {
    const uint16_t *ln1_g, *ln1_b; sd_proj q1, k1, v1, o1;   /* self-attention             */
    const uint16_t *ln2_g, *ln2_b; sd_proj q2, k2, v2, o2;   /* cross-attention (k2,v2: [C, Dc]) */
    const uint16_t *ln3_g, *ln3_b; sd_proj ff1, ff2;         /* GEGLU feed-forward          */
} sd_block_params;

/* Parameters of a spatial-transformer stack.  `blocks` is a HOST array of `depth` entries. */
typedef struct sd_stack_params {
    const uint16_t *gn_g, *gn_b;      /* GroupNorm(32) affine, [C]            */
    sd_proj proj_in, proj_out;        /* Linear C -> C with bias, no adapter  */
    const sd_block_params* blocks;    /* host array                           */
    int32_t depth;
} sd_stack_params;

/* One weight matrix to patch (fp32, device pointers). */
typedef struct sd_patch_desc {
    float* W;         /* [out, in], patched in place                                    */
    const float* A;   /* [r, in]                                                        */
    const float* B;   /* [out, r]                                                       */
    float* undo;      /* [out, in] record of W's bits before the patch; required        */
    int32_t out, in, r;
    float scale;
} sd_patch_desc;

/* One weight matrix patched with several adapters in one pass (fp32, device pointers). */
#define SD_PATCH_MAX_ADAPTERS 4
typedef struct sd_patch_multi_desc {
    float* W;            /* [out, in], patched in place                                  */
    float* undo;         /* [out, in] record of W's bits before the patch; required      */
    uint16_t* serving;   /* [out, in] bf16 copy of the patched W, or NULL                */
    int32_t out, in;
    int32_t n_adapters;  /* 1 .. SD_PATCH_MAX_ADAPTERS                                   */
    int32_t pad_;
    const float* A[SD_PATCH_MAX_ADAPTERS];   /* A_i [r_i, in]                            */
    const float* B[SD_PATCH_MAX_ADAPTERS];   /* B_i [out, r_i]                           */
    int32_t r[SD_PATCH_MAX_ADAPTERS];
    float scale[SD_PATCH_MAX_ADAPTERS];
} sd_patch_multi_desc;

const char* sd_last_error(void);
int32_t sd_version(void);
/* Self-check of the projection launches.  Section 2's LoRA projection runs as one launch: the
 * tiles of the down-projection t = scale * x A^T come first in the grid, and a tile of the base
 * GEMM waits, behind a bounded spin, for the rows of t it reads.
 *   Forward progress rests on two things: (i) the down-projection tiles are the lowest-numbered
 *   workgroups of the launch and the hardware dispatches workgroups in index order on every XCD,
 *   so each of them is running or done before any tile can wait for it, and they wait for
 *   nothing; (ii) a workspace serves one call at a time (its flags are per call).  HIP does not
 *   promise (i) in writing; the spin is bounded (2^19 polls, about half a second) so that every wavefront
 *   exits even if it should not hold.
 *   A tile that runs out of spins writes NaN to its whole output tile, so the damage is visible in
 *   the data of that call and of everything computed from it; the forward call itself has long
 *   returned SD_OK by then (calls only enqueue).  *count receives how many tiles, since the library
 *   was loaded, ran out of spins: 0 unless the protocol is broken.
 *   count: host.  This call synchronises the device: a serving loop polls it once per request,
 *   after the request's last step, not per step. */
int sd_gemm_dep_timeouts(int64_t* count);
/* Diagnostic switch for the same: on = 0 makes every later call run a projection as two
 * launches (all down-projections, then all base GEMMs) instead of one, and merge the halves
 * of cut attention tiles in a kernel of their own instead of inside the attention launch;
 * on = 1 (the default) restores the single launches.  Both give the same bits.  Returns the
 * previous setting.  Process-wide, not thread-safe against concurrent forward calls. */
int32_t sd_set_projection_fusion(int32_t on);

/* ---- instrumentation (off by default) --------------------------------------------------
 * Measurement support for the roofline figures: when enabled, the sub-layer and stack calls
 * record a HIP event on their stream immediately before and after the launch of the kernels
 * tagged below, so a benchmark can read per-launch durations of the dominant kernels inside
 * a real step.  Not for use under HIP graph capture.  enable() creates the events (host
 * side), collect() waits for them and writes up to `capacity` durations in milliseconds to
 * the host array, disable() destroys them.  One process-wide instance, not thread-safe. */
#define SD_TIMING_SELF_ATTENTION 0   /* flash attention over the latent tokens            */
#define SD_TIMING_CROSS_ATTENTION 1  /* flash attention to the text tokens                */
#define SD_TIMING_QKV 2              /* grouped q, k, v^T base GEMMs of self-attention     */
#define SD_TIMING_ATTN_OUT 3         /* attention output projection + residual            */
#define SD_TIMING_FF1 4              /* feed-forward in-projection with GEGLU epilogue     */
#define SD_TIMING_FF2 5              /* feed-forward out-projection + residual             */
#define SD_TIMING_CROSS_Q 6          /* cross-attention query projection                   */
#define SD_TIMING_PROJ_IO 7          /* the stack's proj_in and proj_out                   */
#define SD_TIMING_LAYERNORM 8        /* every LayerNorm launch                             */
#define SD_TIMING_GROUPNORM 9        /* the stack's GroupNorm (partial sums + apply)       */
#define SD_TIMING_TAGS 10
int sd_timing_enable(int32_t records_per_tag);
int sd_timing_collect(int32_t tag, float* ms_host, int32_t capacity, int32_t* count);
int sd_timing_disable(void);

/* ---- measured ceilings (measurement support, not part of the method) --------------------
 * What this device sustains, to set beside the vendor peaks in a roofline figure.
 * ceiling_mfma_bf16: `workgroups` x 4 wavefronts each run `iters` x 4 independent
 *   32x32x16 bf16 MFMAs out of registers; out: device, workgroups * 256 floats (written so
 *   the loop is not optimised away); *flops (host, may be NULL) receives the FLOP count of
 *   the launch.  Time it with events on `stream`.
 * ceiling_copy_f32: dst[i] = src[i] for n floats (n % 4 == 0, 16-byte aligned device
 *   pointers, no overlap): 8 bytes of traffic per element. */
int sd_ceiling_mfma_bf16(float* out, int32_t workgroups, int32_t iters, double* flops, void* stream);
int sd_ceiling_copy_f32(const float* src, float* dst, size_t n, void* stream);
/* ceiling_valu: `workgroups` x 4 wavefronts run `iters` trips over 8 independent register chains:
 *   mode 0 one v_exp_f32 per chain and trip, mode 1 four v_fma_f32, mode 2 both, mode 3 two
 *   exponentials per chain and trip dealt between the four MFMAs of ceiling_mfma_bf16's trip.  out as
 *   for ceiling_mfma_bf16; *exps and *fmas (host, may be NULL) receive the wavefront-wide instruction
 *   counts of the launch.  From the durations: what an exponential costs in FMA issue slots, whether
 *   the two overlap, and how much of the exponentials runs under the MFMAs (mode 3 against
 *   ceiling_mfma_bf16 with the same workgroups and iters): the vector-ALU side of the attention
 *   kernel's bound. */
int sd_ceiling_valu(float* out, int32_t workgroups, int32_t iters, int32_t mode, double* exps, double* fmas, void* stream);
/* the same with two destinations (dst0 = dst1 = src afterwards): one read and two writes per element, the
 * traffic mix of the patch pass (W read, undo record and W' written) */
int sd_ceiling_copy_1r2w_f32(const float* src, float* dst0, float* dst1, size_t n, void* stream);

/* ---- lora_linear_fwd ------------------------------------------------------------------
 * y = epi( LN?(x) W^T + bias + scale * (LN?(x) A^T) B^T ) + residual
 * The unmerged form of Section 2's W' = W + A B applied to an input; the rank-r update
 * runs inside the base GEMM's main loop (K extended by r).  With p->r == 0 it is the
 * plain linear layer a patched (merged) weight needs.
 *   x        device [M, K]; bf16, or fp32 when a LayerNorm is given (x_dtype = SD_F32)
 *   ln_gamma, ln_beta  device [K] bf16 or both NULL (no LayerNorm); biased variance
 *   residual device [M, N] of y_dtype or NULL; may alias y
 *   y        device [M, N], y_dtype bf16 or fp32
 *   epilogue SD_EPI_GEGLU: W, bias, B have 2N rows and y = value * gelu(gate) (exact erf
 *            GELU; Section 4.3's fused GEGLU); residual must then be NULL
 * K and p->r must be multiples of 8.  Errors: SD_EINVAL, SD_EWORKSPACE, SD_EHIP. */
size_t sd_lora_linear_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t r, int32_t has_ln);
int sd_lora_linear_fwd(const void* x, int32_t x_dtype, const sd_proj* p,
                       const uint16_t* ln_gamma, const uint16_t* ln_beta, float ln_eps,
                       const void* residual, void* y, int32_t y_dtype, int32_t epilogue,
                       int32_t M, int32_t N, int32_t K,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- lora_linear_fwd_static --------------------------------------------------------------
 * sd_lora_linear_fwd for callers that cannot allocate device memory or carry a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, semantics and bits as sd_lora_linear_fwd without `ws`: the scratch memory (LayerNorm
 * output, down-projection, dependency flags) is a device array of SD_STATIC_SCRATCH_BYTES built
 * into the library, which every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing.
 *   - SD_EWORKSPACE if sd_lora_linear_workspace_bytes(M, N, K, p->r, has_ln) exceeds
 *     SD_STATIC_SCRATCH_BYTES (text names both sizes); use sd_lora_linear_fwd then.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents (each
 *     call clears the flags it needs itself).  Calls that may overlap on one GPU - different
 *     streams, concurrent graph launches - race on it: serialise them, or use sd_lora_linear_fwd
 *     with a workspace each.
 *   - The first call on a device looks up the array's address on that device (host-side, no
 *     allocation); make that first call outside graph capture. */
#define SD_STATIC_SCRATCH_BYTES (16u << 20)
int sd_lora_linear_fwd_static(const void* x, int32_t x_dtype, const sd_proj* p,
                              const uint16_t* ln_gamma, const uint16_t* ln_beta, float ln_eps,
                              const void* residual, void* y, int32_t y_dtype, int32_t epilogue,
                              int32_t M, int32_t N, int32_t K, void* stream);

/* ---- attn_block_fwd -------------------------------------------------------------------
 * y = x + out( attention( q(LN x), k(src), v(src) ) ),  src = LN x (ctx NULL: latent
 * self-attention) or ctx (cross-attention to the text tokens that guide every denoising
 * step, Section 2).  Attention is softmax(q k^T / 8) v per (sample, head), head dim 64,
 * no mask; scores are never written to memory.
 *   x, y     device [Bn, T, C] of io_dtype (bf16 or fp32); y may alias x
 *   ctx      device [Bn, Tc, Dc] bf16 or NULL
 *   q,k,v,o  host structs; q,o: [C, C]; k,v: [C, C] (self) or [C, Dc] (cross)
 * Requires C == 64 * heads, C and Dc multiples of 8. */
size_t sd_attn_block_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t Tc, int32_t Dc, int32_t r_max);
int sd_attn_block_fwd(const void* x, void* y, int32_t io_dtype,
                      const uint16_t* ctx, int32_t Tc, int32_t Dc,
                      const uint16_t* ln_gamma, const uint16_t* ln_beta, float ln_eps,
                      const sd_proj* q, const sd_proj* k, const sd_proj* v, const sd_proj* o,
                      int32_t Bn, int32_t T, int32_t C, int32_t heads,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- attention_fwd (helper) -----------------------------------------------------------
 * The attention operator of the base model's transformer blocks (Section 4.3, "Kernel-level
 * optimizations" names it among the operators worth a kernel of their own), on its own:
 * out[b, t, h*64 + d] = softmax_k(q[b,t,h,:] . k[b,k,h,:] / 8) v[b,k,h,d]
 *   q   device [Bn, Tq, C] bf16;  k device [Bn, Tk, C] bf16
 *   vt  device [C, Bn * Tkp] bf16: V transposed, sample b's keys at columns
 *       [b*Tkp, b*Tkp + Tk), Tkp = Tk rounded up to a multiple of 8
 *   out device [Bn, Tq, C] bf16
 *   ws  device scratch of sd_attention_workspace_bytes(...) bytes, 256-byte aligned: for
 *       shapes whose (sample, head, 128-query) tiles would load the CUs unevenly, some
 *       tiles' key range is halved between two workgroups and their partial results meet
 *       there.  SD_EWORKSPACE if it is too small. */
size_t sd_attention_workspace_bytes(int32_t Bn, int32_t Tq, int32_t Tk, int32_t heads);
int sd_attention_fwd(const uint16_t* q, const uint16_t* k, const uint16_t* vt, uint16_t* out,
                     int32_t Bn, int32_t Tq, int32_t Tk, int32_t C, int32_t heads,
                     void* ws, size_t ws_bytes, void* stream);

/* ---- ff_block_fwd (helper) ------------------------------------------------------------
 * The block's feed-forward sub-layer with the GEGLU of Section 4.3 ("Kernel-level optimizations":
 * GELU and the matrix multiplication as one operator) in the first projection's epilogue:
 * y = x + ff2( geglu( ff1( LN x ) ) );  ff1: [2F, C] with bias, ff2: [C, F] with bias. */
size_t sd_ff_block_workspace_bytes(int32_t M, int32_t C, int32_t F, int32_t r_max);
int sd_ff_block_fwd(const void* x, void* y, int32_t io_dtype,
                    const uint16_t* ln_gamma, const uint16_t* ln_beta, float ln_eps,
                    const sd_proj* ff1, const sd_proj* ff2, int32_t M, int32_t C, int32_t F,
                    void* ws, size_t ws_bytes, void* stream);

/* ---- groupnorm_fwd (helper) -----------------------------------------------------------
 * The GroupNorm that precedes the transformer blocks (Section 4.3, "Kernel-level optimizations"
 * lists GroupNorm among the base model's operators), token-major: x, y device [Bn, T, C] bf16; statistics per (sample, group of
 * C/groups adjacent channels) over all tokens, biased variance, per-channel affine. */
size_t sd_groupnorm_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t groups);
int sd_groupnorm_fwd(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta,
                     int32_t Bn, int32_t T, int32_t C, int32_t groups, float eps,
                     void* ws, size_t ws_bytes, void* stream);
/* The same followed by SiLU, y = n * sigmoid(n): the GroupNorm + SiLU pair of the base model's
 * ResNet blocks as one operator (Section 4.3, "Kernel-level optimizations").  Same arguments
 * and workspace. */
int sd_groupnorm_silu_fwd(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta,
                          int32_t Bn, int32_t T, int32_t C, int32_t groups, float eps,
                          void* ws, size_t ws_bytes, void* stream);

/* ---- spatial_transformer_fwd ----------------------------------------------------------
 * The whole hot path on the guidance pair (Section 3.3: both latents in one batch):
 * y = proj_out( blocks( proj_in( GroupNorm32(x) ) ) ) + x, each block = self-attention,
 * cross-attention, GEGLU feed-forward, each behind a LayerNorm and with a residual.
 * The residual stream is kept in fp32 inside the call.
 *   x, y device [Bn, T, C] bf16;  ctx device [Bn, Tc, Dc] bf16;  p host struct. */
size_t sd_spatial_transformer_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t Tc, int32_t Dc, int32_t r_max);
int sd_spatial_transformer_fwd(const uint16_t* x, const uint16_t* ctx, const sd_stack_params* p,
                               uint16_t* y, int32_t Bn, int32_t T, int32_t C, int32_t heads,
                               int32_t Tc, int32_t Dc, void* ws, size_t ws_bytes, void* stream);

/* ---- multi_lora_linear_fwd ------------------------------------------------------------
 * Several requests' rows stacked in one matrix, each row segment with its own adapter
 * (the batched multi-LoRA operators of Section 7 applied per request):
 *   y[rows of segment i] = x W^T + bias + scales[a] * (x A_a^T) B_a^T,  a = seg_adapter[i]
 * (a = -1: no adapter).  Segments are contiguous, ordered, and cover [0, M).
 *   A_ptrs, B_ptrs  host arrays of `nadapters` device pointers (A_a [ranks[a], K],
 *                   B_a [N, ranks[a]], bf16);  ranks, scales host arrays
 *   seg_offsets     host [nseg + 1], seg_adapter host [nseg] */
size_t sd_multi_lora_linear_workspace_bytes(int32_t M, int32_t r_max);
int sd_multi_lora_linear_fwd(const uint16_t* x, const uint16_t* W, const uint16_t* bias,
                             const uint16_t* const* A_ptrs, const uint16_t* const* B_ptrs,
                             const int32_t* ranks, const float* scales,
                             const int32_t* seg_offsets, const int32_t* seg_adapter,
                             int32_t nseg, int32_t nadapters, uint16_t* y,
                             int32_t M, int32_t N, int32_t K,
                             void* ws, size_t ws_bytes, void* stream);

/* ---- lora_patch / lora_unpatch --------------------------------------------------------
 * Section 4.2, "Efficient LoRA patching": the adapter is merged into the base parameters
 * in place, W <- fl32(W + fl32(scale * fl32(B A))), and taken off after the request.
 * Taking it off must give back W's exact bits, which subtraction cannot do, so the patch
 * pass also writes W's old bits to `undo` and unpatch copies them back.
 *
 * A plan is built once on the host from the descriptor list (validates it, splits every
 * matrix into tiles), uploaded by the caller, and reused by patch and unpatch:
 *   sd_patch_plan_bytes(n)            size of the plan for n matrices
 *   sd_patch_plan_build(descs, n, plan_host, bytes, &tiles)   descs, plan_host: host
 *   sd_lora_patch(plan_dev, n, tiles, stream)     one grouped launch over all matrices
 *   sd_lora_unpatch(plan_dev, n, tiles, stream)   W <- undo, bit-exact
 * Calling unpatch without a preceding patch on the same undo buffers copies whatever the
 * buffers hold; the library cannot detect that.  Nor can it detect a second patch without an
 * unpatch in between: that one overwrites `undo` with already-patched bits and the base weights
 * are lost (stack two adapters with sd_lora_patch_multi instead, or give the second patch its
 * own undo buffers and unpatch in reverse order).  Ordering against kernels that read W on
 * other streams is the caller's job (events). */
size_t sd_patch_plan_bytes(int32_t n);
int sd_patch_plan_build(const sd_patch_desc* descs, int32_t n, void* plan_host, size_t plan_bytes,
                        int64_t* total_tiles);
int sd_lora_patch(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream);
int sd_lora_unpatch(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream);

/* ---- lora_patch_multi / lora_unpatch_multi ----------------------------------------------
 * A request carries one or two LoRAs (Section 3.1, add-on usage table), loaded in parallel
 * and each merged into the base weights (Section 4.2).  This pass applies up to
 * SD_PATCH_MAX_ADAPTERS adapters to a matrix while its tile is in registers, in order:
 *   W_0 = W,  W_i = fl32(W_{i-1} + fl32(scale_i * fl32(B_i A_i))),  W' = W_n,
 * bit for bit what n successive sd_lora_patch calls give, at the memory traffic of one.
 * `undo` receives W_0; `serving` (optional) receives bf16(W'), round to nearest even, the
 * copy the bf16 GEMMs of the forward path read.  unpatch_multi restores W <- undo exactly
 * and rewrites serving <- bf16(undo).  Plans as for sd_lora_patch (host build, caller uploads). */
size_t sd_patch_multi_plan_bytes(int32_t n);
int sd_patch_multi_plan_build(const sd_patch_multi_desc* descs, int32_t n, void* plan_host, size_t plan_bytes,
                              int64_t* total_tiles);
int sd_lora_patch_multi(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream);
int sd_lora_unpatch_multi(const void* plan_dev, int32_t n, int64_t total_tiles, void* stream);

/* ---- cfg_combine --------------------------------------------------------------------------
 * The classifier-free-guidance weighted sum of the two denoised latents of a step
 * (Section 2, "Diffusion model inference"): out = eps_u + g * (eps_c - eps_u), formed in fp32 as
 * fl32(eps_u + fl32(g * fl32(eps_c - eps_u))) and rounded to bf16 (nearest even).
 *   eps_uncond, eps_cond, out   device bf16 [n]; out may alias either input; n elements */
int sd_cfg_combine(const uint16_t* eps_uncond, const uint16_t* eps_cond, float guidance, uint16_t* out, size_t n, void* stream);

/* ---- controlnet_residual_add -------------------------------------------------------------
 * Where ControlNet outputs enter the backbone (Section 2, "ControlNet": the outputs go into the
 * skip connections and the middle block; those of several ControlNets are summed first):
 *   out = h + (r_1 + r_2 + ... + r_n),
 * the sum formed left to right with one fp32 rounding per addition, then one more for "+ h",
 * then bf16 (nearest even).  No ControlNet is part of this library: the residuals are inputs.
 *   h, out       device bf16 [n]; out may alias h or any residual
 *   residuals    HOST array of n_res device pointers, each bf16 [n]; read during the call only
 *   n_res        0 .. SD_CONTROLNET_MAX (0: out = h); outside that range SD_EINVAL
 * Hipmemcpy-free except for n_res == 0 with out != h (one device-to-device copy). */
#define SD_CONTROLNET_MAX 8
int sd_controlnet_residual_add(const uint16_t* h, const uint16_t* const* residuals, int32_t n_res, uint16_t* out, size_t n, void* stream);

/* ---- bal: bounded asynchronous LoRA loading, host side ------------------------------------
 * Section 4.2, "Bounded asynchronous LoRA loading (BAL)": when a request arrives its adapters
 * load in the background, in parallel, while the base model early-starts denoising unpatched;
 * once they are in, they are patched at the next step boundary; at step k (the bound, found by
 * profiling where the with/without-LoRA latents start to diverge) the base model is held until
 * loading completes; after the request the adapters are patched off.  Host logic only: `load`
 * fills whatever buffers the caller patches from (it runs on a thread of this library, one per
 * adapter), and the caller issues the copies and sd_lora_patch* calls when told to.
 *   sd_bal_create(n, load, user)     handle, or NULL (n < 0, or n > 0 without a callback)
 *   sd_bal_start(b)                  request arrival: starts the n loader threads
 *   sd_bal_before_step(b, step, k, timeout_s, &patch_now)
 *        at the boundary before denoising step `step` (from 1).  *patch_now = 1 exactly once,
 *        at the first boundary where every adapter is loaded: patch, then run the step.  If
 *        step >= k and loading is not complete, blocks until it is; SD_ETIMEOUT after
 *        timeout_s seconds, SD_ELOAD if a loader returned non-zero.
 *   sd_bal_loaded(b)                 1 when every loader has returned
 *   sd_bal_stats(b, &patched_at_step, &stall_s, &load_s)   any pointer may be NULL; step 0 =
 *        never patched; load_s < 0 while loading
 *   sd_bal_finish(b, &unpatch_due)   joins the loaders; *unpatch_due = 1 if a patch was ordered
 *   sd_bal_destroy(b)
 * One handle per request; calls on one handle come from one thread. */
typedef struct sd_bal sd_bal;
typedef int32_t (*sd_bal_load_fn)(void* user, int32_t adapter);
sd_bal* sd_bal_create(int32_t n_adapters, sd_bal_load_fn load, void* user);
int sd_bal_start(sd_bal* b);
int sd_bal_loaded(sd_bal* b);
int sd_bal_before_step(sd_bal* b, int32_t step, int32_t k, double timeout_s, int32_t* patch_now);
int sd_bal_stats(sd_bal* b, int32_t* patched_at_step, double* stall_seconds, double* load_seconds);
int sd_bal_finish(sd_bal* b, int32_t* unpatch_due);
void sd_bal_destroy(sd_bal* b);

#ifdef __cplusplus
}
#endif
#endif /* SWIFTDIFF_H */
