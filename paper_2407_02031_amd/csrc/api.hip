// C-ABI entry points: argument checks, workspace carving, and the composition of the
// kernels into projections, attention sub-layers, the feed-forward sub-layer and the whole
// spatial-transformer stack.  Host code only; every arithmetic step runs in the kernels.
#include "common.hpp"

#include <string.h>
#include <mutex>
#include <vector>

namespace sd {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
int hip_fail(hipError_t e, const char* what) {
    set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return SD_EHIP;
}

// ---------------------------------------------------------------------------------------
// optional instrumentation: HIP events around selected kernel launches (off by default)
// ---------------------------------------------------------------------------------------
struct TimingState {
    bool on = false;
    int cap = 0;
    std::vector<hipEvent_t> ev[SD_TIMING_TAGS][2];
    int count[SD_TIMING_TAGS] = {0};
};
static TimingState g_timing;

static void timing_mark(int tag, int which, hipStream_t stream) {
    if (!g_timing.on || tag < 0) return;
    int& n = g_timing.count[tag];
    if (n >= g_timing.cap) return;
    (void)hipEventRecord(g_timing.ev[tag][which][n], stream);
    if (which == 1) ++n;
}

// ---------------------------------------------------------------------------------------
// projection -> GEMM problems
// ---------------------------------------------------------------------------------------
struct ProjOut {
    void* y; int64_t ldy; int y_f32;
    const void* res; int64_t ldr;
    bool transposed;    // store y^T: y[n * ldy + m]
    int geglu_F;        // > 0: GEGLU epilogue, N == F
    float alpha;        // output scale applied to the accumulator before bias (0 means 1)
    int res_f32;        // residual is fp32 although y is bf16 (with an fp32 y the residual always is)
};

static int check_proj(const sd_proj* p, const char* name, int K) {
    SD_REQUIRE(p && p->W, SD_EINVAL, "%s: projection or its W is null", name);
    SD_REQUIRE(aligned16(p->W), SD_EINVAL, "%s: W not 16-byte aligned", name);
    SD_REQUIRE(p->r >= 0 && p->r % 8 == 0, SD_EUNSUPPORTED, "%s: rank %d is not a multiple of 8", name, p->r);
    if (p->r > 0) {
        SD_REQUIRE(p->A && p->B, SD_EINVAL, "%s: rank %d but A or B is null", name, p->r);
        SD_REQUIRE(aligned16(p->A) && aligned16(p->B), SD_EINVAL, "%s: A/B not 16-byte aligned", name);
    }
    SD_REQUIRE(K > 0 && K % 8 == 0, SD_EUNSUPPORTED, "%s: K=%d is not a positive multiple of 8", name, K);
    return SD_OK;
}

static int push(GemmGroup& g, const GemmProblem& P, hipStream_t stream) {
    if (g.n == GEMM_MAX_PROBLEMS) {   // group full: flush it, order within a stream is kept
        int rc = launch_gemm_group(g, stream);
        if (rc) return rc;
        g.n = 0;
    }
    g.p[g.n++] = P;
    return SD_OK;
}

// One projection y = x W^T (+ bias) (+ scale (x A^T) B^T) as GEMM problems: the
// down-projection t = scale * x A^T (bf16 [M, r]) and the K-extended base GEMM.
struct ProjCall {
    const uint16_t* x; int64_t ldx; int M, K, N;
    const sd_proj* p; uint16_t* tbuf; ProjOut o;
};

static int push_down(GemmGroup& g, hipStream_t stream, const ProjCall& c, int32_t* signal = nullptr) {
    const sd_proj& p = *c.p;
    if (p.r <= 0) return SD_OK;
    GemmProblem D;
    memset(&D, 0, sizeof(D));
    D.p0 = c.x; D.ldp0 = c.ldx; D.q0 = p.A; D.ldq0 = c.K;
    D.y = c.tbuf; D.ldy = p.r; D.Mp = c.M; D.N = p.r; D.K0 = c.K; D.K1 = 0; D.alpha = p.scale;
    D.signal = signal;
    return push(g, D, stream);
}

static int push_main(GemmGroup& g, hipStream_t stream, const ProjCall& c, const int32_t* wait = nullptr) {
    const sd_proj& p = *c.p;
    const ProjOut& o = c.o;
    const int r = p.r;
    GemmProblem G;
    memset(&G, 0, sizeof(G));
    G.alpha = o.alpha != 0.f ? o.alpha : 1.0f;
    G.bias = p.bias;
    G.res = o.res; G.ldr = o.ldr;
    G.y = o.y; G.ldy = o.ldy; G.y_f32 = o.y_f32; G.res_f32 = o.y_f32 || o.res_f32;
    G.geglu_F = o.geglu_F;
    G.K0 = c.K; G.K1 = r;
    if (!o.transposed) {
        G.p0 = c.x; G.ldp0 = c.ldx; G.q0 = p.W; G.ldq0 = c.K;
        G.p1 = r ? c.tbuf : nullptr; G.ldp1 = r; G.q1 = r ? p.B : nullptr; G.ldq1 = r;
        G.Mp = c.M; G.N = c.N;
    } else {
        G.p0 = p.W; G.ldp0 = c.K; G.q0 = c.x; G.ldq0 = c.ldx;
        G.p1 = r ? p.B : nullptr; G.ldp1 = r; G.q1 = r ? c.tbuf : nullptr; G.ldq1 = r;
        G.Mp = c.N; G.N = c.M;
        G.bias_on_rows = 1;
    }
    if (r) { G.wait = wait; G.wait_cols = o.transposed; }
    return push(g, G, stream);
}

static int flush(GemmGroup& g, hipStream_t stream) {
    if (g.n == 0) return SD_OK;
    int rc = launch_gemm_group(g, stream);
    memset(&g, 0, sizeof(g));
    return rc;
}

// Flags for launches whose base GEMMs wait, tile by tile, for down-projections of the same
// launch: two arrays of `cap` flags in the caller's workspace.  A launch signals in one array
// and clears the other for the next launch; the first launch of a call follows clear().
struct DepFlags {
    int32_t* f[2] = {nullptr, nullptr};
    int cap = 0;
    int turn = 0;
    bool pending = false;   // f[0] still has to be cleared: by the next LayerNorm launch, or by a launch of its own
    // Behind the first array: counters of the attention launches that cut tiles in half (who
    // arrived first), cleared with it; every launch leaves them at zero again.
    static constexpr int ARRIVED = 1024;
    int32_t* arrived = nullptr;
    static int cap_for(size_t rows) { return (int)(4 * ((rows + 63) / 64) + 64); }
    static size_t half_bytes(size_t rows) { return round_up((size_t)(cap_for(rows) + ARRIVED) * 4, 256); }
    static size_t bytes_for(size_t rows) { return half_bytes(rows) * 2; }
    bool carve(Workspace& ws, size_t rows) {
        cap = cap_for(rows);
        char* b = (char*)ws.take(bytes_for(rows));
        f[0] = (int32_t*)b;
        f[1] = b ? (int32_t*)(b + half_bytes(rows)) : nullptr;
        arrived = b ? f[0] + cap : nullptr;
        turn = 0;
        return b != nullptr;
    }
    void reset() { turn = 0; pending = f[0] != nullptr; }
    int clear_words() const { return cap + ARRIVED; }
    int clear_now(hipStream_t stream) {
        if (!pending) return SD_OK;
        pending = false;
        return launch_clear_flags(f[0], clear_words(), stream);
    }
};

// LayerNorm that also clears the first flag array of the call if that is still due
static int layernorm(const void* x, int x_f32, const uint16_t* g, const uint16_t* b, float eps, uint16_t* y, int M, int C,
                     hipStream_t stream, DepFlags* dep) {
    timing_mark(SD_TIMING_LAYERNORM, 0, stream);
    int rc;
    if (dep && dep->pending && M > 0) {
        dep->pending = false;
        rc = launch_layernorm(x, x_f32, g, b, eps, y, M, C, stream, dep->f[0], dep->clear_words());
    } else {
        rc = launch_layernorm(x, x_f32, g, b, eps, y, M, C, stream);
    }
    timing_mark(SD_TIMING_LAYERNORM, 1, stream);
    return rc;
}

// Run independent projections.  With flags, as one launch: down-projection tiles first, and a
// base GEMM tile waits for the down-projection rows it reads just before its second K segment
// (by then they are long done, except in the first round of workgroups).  Without, or when the
// projections do not fit one group, as two rounds of launches: every down-projection, then
// every base GEMM.
static bool g_fuse_projections = true;   // diagnostic switch, see sd_set_projection_fusion
static bool g_fuse_attention_merge = true;

static int run_projections(const ProjCall* calls, int n, hipStream_t stream, int tag = -1, DepFlags* dep = nullptr) {
    GemmGroup g;
    memset(&g, 0, sizeof(g));
    int rc;
    auto problems_of = [](const ProjCall& c) { return c.M <= 0 ? 0 : (c.p->r > 0 ? 2 : 1); };
    auto flags_of = [](const ProjCall& c) { return (c.M > 0 && c.p->r > 0) ? ((size_t)c.M + 63) / 64 : (size_t)0; };
    bool fuse = g_fuse_projections && dep && dep->f[0];
    if (fuse) {
        bool any_down = false;
        for (int i = 0; i < n; ++i) {
            if (flags_of(calls[i]) > (size_t)dep->cap) fuse = false;   // one projection alone overflows the flags
            if (flags_of(calls[i])) any_down = true;
        }
        fuse = fuse && any_down;
    }
    if (fuse) {
        // as many projections per launch as fit a group and the flags (projections are independent
        // of each other, so any split is valid)
        timing_mark(tag, 0, stream);
        int i0 = 0;
        while (i0 < n) {
            int i1 = i0, problems = 0;
            size_t flags = 0;
            while (i1 < n && problems + problems_of(calls[i1]) <= GEMM_MAX_PROBLEMS && flags + flags_of(calls[i1]) <= (size_t)dep->cap) {
                problems += problems_of(calls[i1]);
                flags += flags_of(calls[i1]);
                ++i1;
            }
            if (flags > 0 && (rc = dep->clear_now(stream))) return rc;
            int32_t* const base = dep->f[dep->turn];
            // (no heap for the usual handful of projections: the single-projection entry points allocate nothing)
            int32_t* slot_small[32] = {nullptr};
            std::vector<int32_t*> slot_big;
            if (n > 32) slot_big.assign(n, nullptr);
            int32_t** const slot = n > 32 ? slot_big.data() : slot_small;
            size_t used = 0;
            for (int i = i0; i < i1; ++i) {
                if (!flags_of(calls[i])) continue;
                slot[i] = base + used;
                used += flags_of(calls[i]);
                if ((rc = push_down(g, stream, calls[i], slot[i]))) return rc;
            }
            for (int i = i0; i < i1; ++i)
                if (calls[i].M > 0 && (rc = push_main(g, stream, calls[i], slot[i]))) return rc;
            if (flags > 0) {
                dep->turn ^= 1;
                g.zero_ptr = dep->f[dep->turn];
                g.zero_n = dep->cap;
            }
            if ((rc = flush(g, stream))) return rc;
            i0 = i1;
        }
        timing_mark(tag, 1, stream);
        return SD_OK;
    }
    for (int i = 0; i < n; ++i)
        if (calls[i].M > 0 && (rc = push_down(g, stream, calls[i]))) return rc;
    if ((rc = flush(g, stream))) return rc;
    for (int i = 0; i < n; ++i)
        if (calls[i].M > 0 && (rc = push_main(g, stream, calls[i]))) return rc;
    timing_mark(tag, 0, stream);
    rc = flush(g, stream);
    timing_mark(tag, 1, stream);
    return rc;
}

static inline int pad8(int v) { return (v + 7) & ~7; }

// ---------------------------------------------------------------------------------------
// sub-layers (shared by the single-call entry points and the stack driver)
// ---------------------------------------------------------------------------------------
struct AttnWs {
    uint16_t *n, *q, *k, *vt, *a, *tq, *tk, *tv, *to;
    uint16_t *k2, *vt2, *tk2, *tv2;   // text-context keys / values computed ahead of the cross-attention sub-layer (stack driver)
    void* scratch; size_t scratch_bytes;
};

static bool carve_attn(Workspace& ws, AttnWs& w, int Bn, int T, int C, int Tk, int rmax, int heads, int Tc_ahead = 0) {
    const size_t M = (size_t)Bn * T, Mk = (size_t)Bn * Tk;
    const size_t r = rmax > 0 ? rmax : 8;
    w.n = (uint16_t*)ws.take(M * C * 2);
    w.q = (uint16_t*)ws.take(M * C * 2);
    w.k = (uint16_t*)ws.take(Mk * C * 2);
    w.vt = (uint16_t*)ws.take((size_t)C * Bn * pad8(Tk) * 2);
    w.a = (uint16_t*)ws.take(M * C * 2);
    w.tq = (uint16_t*)ws.take(M * r * 2);
    w.tk = (uint16_t*)ws.take(Mk * r * 2);
    w.tv = (uint16_t*)ws.take(Mk * r * 2);
    w.to = (uint16_t*)ws.take(M * r * 2);
    const size_t Mc = (size_t)Bn * Tc_ahead;
    w.k2 = (uint16_t*)ws.take(Mc * C * 2);
    w.vt2 = (uint16_t*)ws.take((size_t)C * Bn * pad8(Tc_ahead) * 2);
    w.tk2 = (uint16_t*)ws.take(Mc * r * 2);
    w.tv2 = (uint16_t*)ws.take(Mc * r * 2);
    // sized for the larger of the two key counts the sub-layer is used with (Tk here, T for self-attention)
    w.scratch_bytes = std::max(attention_scratch_bytes(Bn, T, Tk, heads), attention_scratch_bytes(Bn, T, T, heads));
    w.scratch = ws.take(w.scratch_bytes);
    return ws.ok();
}

// k and v^T projections of `src` ([Bn * Tk, Kkv]) into kbuf ([Bn * Tk, C]) and vtbuf ([C, Bn * Tkp]:
// one problem per sample, operands exchanged, so that each sample's keys start at a multiple
// of 8).  The keys leave their projection multiplied by the softmax scale (in exponent-of-2
// units), applied to the fp32 accumulator before the one rounding to bf16; a k bias would have
// to be scaled too, so with one the attention kernel scales the scores itself.
static bool push_kv_calls(std::vector<ProjCall>& calls, const uint16_t* src, int Kkv, int Tk, const sd_proj& pk, const sd_proj& pv,
                          uint16_t* kbuf, uint16_t* vtbuf, uint16_t* tkbuf, uint16_t* tvbuf, int Bn, int C) {
    const int Tkp = pad8(Tk);
    const bool k_prescaled = pk.bias == nullptr;
    calls.push_back({src, Kkv, Bn * Tk, Kkv, C, &pk, tkbuf, {kbuf, C, 0, nullptr, 0, false, 0, k_prescaled ? ATTN_KSCALE : 0.f}});
    for (int s = 0; s < Bn; ++s)
        calls.push_back({src + (size_t)s * Tk * Kkv, Kkv, Tk, Kkv, C, &pv, tvbuf + (size_t)s * Tk * (pv.r > 0 ? pv.r : 0),
                         {vtbuf + (size_t)s * Tkp, (int64_t)Bn * Tkp, 0, nullptr, 0, true, 0}});
    return k_prescaled;
}

// ahead:    projections that do not depend on x, launched in this sub-layer's grouped GEMMs (the
//           stack driver puts the next cross-attention's text keys / values here: on their own
//           their long K loops set the duration of a launch, inside the much larger self-attention
//           q/k/v launch they are hidden)
// kv_ready: the context's keys / values are already in w.k2 / w.vt2
static int attn_sublayer(const void* x, void* y, int io_f32, const uint16_t* ctx, int Tc, int Dc,
                         const uint16_t* g, const uint16_t* b, float eps, const sd_proj& pq, const sd_proj& pk,
                         const sd_proj& pv, const sd_proj& po, int Bn, int T, int C, int heads, const AttnWs& w,
                         hipStream_t stream, const std::vector<ProjCall>* ahead = nullptr, bool kv_ready = false, DepFlags* dep = nullptr) {
    const int M = Bn * T;
    const int Tk = ctx ? Tc : T;
    const int Kkv = ctx ? Dc : C;
    const int Tkp = pad8(Tk);
    int rc = layernorm(x, io_f32, g, b, eps, w.n, M, C, stream, dep);
    if (rc) return rc;
    const uint16_t* src = ctx ? ctx : w.n;
    std::vector<ProjCall> calls;
    // first in the group = first in the tile order: the long-K problems start in the first round
    if (ahead) calls.insert(calls.end(), ahead->begin(), ahead->end());
    calls.push_back({w.n, C, M, C, C, &pq, w.tq, {w.q, C, 0, nullptr, 0, false, 0}});
    bool k_prescaled = pk.bias == nullptr;
    const uint16_t* kbuf = w.k;
    const uint16_t* vtbuf = w.vt;
    if (kv_ready) {
        kbuf = w.k2;
        vtbuf = w.vt2;
    } else {
        k_prescaled = push_kv_calls(calls, src, Kkv, Tk, pk, pv, w.k, w.vt, w.tk, w.tv, Bn, C);
    }
    if ((rc = run_projections(calls.data(), (int)calls.size(), stream, ctx ? SD_TIMING_CROSS_Q : SD_TIMING_QKV, dep))) return rc;
    const int atag = ctx ? SD_TIMING_CROSS_ATTENTION : SD_TIMING_SELF_ATTENTION;
    timing_mark(atag, 0, stream);
    int cut = 0;
    // the counters were cleared by this call's first LayerNorm launch, at the latest by the one above
    int32_t* const arrived = (dep && dep->arrived && !dep->pending && g_fuse_attention_merge) ? dep->arrived : nullptr;
    rc = launch_attention(w.q, C, kbuf, C, vtbuf, (int64_t)Bn * Tkp, w.a, C, Bn, T, Tk, Tkp, heads, k_prescaled, w.scratch, w.scratch_bytes, &cut, stream,
                          arrived, DepFlags::ARRIVED);
    timing_mark(atag, 1, stream);
    if (rc) return rc;
    if ((rc = launch_attention_merge(w.scratch, w.a, C, Bn, T, heads, k_prescaled, cut, stream))) return rc;
    ProjCall oc = {w.a, C, M, C, C, &po, w.to, {y, C, io_f32, x, C, false, 0}};
    return run_projections(&oc, 1, stream, SD_TIMING_ATTN_OUT, dep);
}

struct FfWs { uint16_t *n, *g, *t1, *t2; };

static bool carve_ff(Workspace& ws, FfWs& w, int M, int C, int F, int rmax) {
    const size_t r = rmax > 0 ? rmax : 8;
    w.n = (uint16_t*)ws.take((size_t)M * C * 2);
    w.g = (uint16_t*)ws.take((size_t)M * F * 2);
    w.t1 = (uint16_t*)ws.take((size_t)M * r * 2);
    w.t2 = (uint16_t*)ws.take((size_t)M * r * 2);
    return ws.ok();
}

static int ff_sublayer(const void* x, void* y, int io_f32, const uint16_t* g, const uint16_t* b, float eps,
                       const sd_proj& p1, const sd_proj& p2, int M, int C, int F, const FfWs& w, hipStream_t stream, DepFlags* dep = nullptr,
                       uint16_t* y_bf16 = nullptr) {
    int rc = layernorm(x, io_f32, g, b, eps, w.n, M, C, stream, dep);
    if (rc) return rc;
    ProjCall c1 = {w.n, C, M, C, F, &p1, w.t1, {w.g, F, 0, nullptr, 0, false, F}};
    if ((rc = run_projections(&c1, 1, stream, SD_TIMING_FF1, dep))) return rc;
    // y_bf16: the sub-layer's output goes there, rounded once from the fp32 sum, instead of to y
    // (the stack's last block: what follows reads bf16, and the fp32 stream is not needed again)
    ProjCall c2 = {w.g, F, M, F, C, &p2, w.t2, {y, C, io_f32, x, C, false, 0}};
    if (y_bf16) c2.o = {y_bf16, C, 0, x, C, false, 0, 0.f, io_f32};
    return run_projections(&c2, 1, stream, SD_TIMING_FF2, dep);
}

static int rmax_of(const sd_proj* const* ps, int n) {
    int r = 0;
    for (int i = 0; i < n; ++i)
        if (ps[i] && ps[i]->r > r) r = ps[i]->r;
    return r;
}

}  // namespace sd

using namespace sd;

extern "C" const char* sd_last_error(void) { return g_err; }
extern "C" int32_t sd_version(void) { return 1; }
extern "C" int32_t sd_set_projection_fusion(int32_t on) {
    const int32_t was = g_fuse_projections ? 1 : 0;
    g_fuse_projections = on != 0;
    g_fuse_attention_merge = on != 0;
    return was;
}
extern "C" int sd_gemm_dep_timeouts(int64_t* count) {
    SD_REQUIRE(count, SD_EINVAL, "gemm_dep_timeouts: null count");
    long long v = 0;
    int rc = gemm_dep_timeouts(&v);
    *count = v;
    return rc;
}

extern "C" int sd_timing_enable(int32_t records_per_tag) {
    SD_REQUIRE(records_per_tag > 0 && records_per_tag <= 65536, SD_EINVAL, "timing: records_per_tag=%d", records_per_tag);
    SD_REQUIRE(!g_timing.on, SD_EINVAL, "timing: already enabled");
    for (int t = 0; t < SD_TIMING_TAGS; ++t) {
        g_timing.count[t] = 0;
        for (int w = 0; w < 2; ++w) {
            g_timing.ev[t][w].resize(records_per_tag);
            for (int i = 0; i < records_per_tag; ++i) SD_HIP_CHECK(hipEventCreate(&g_timing.ev[t][w][i]));
        }
    }
    g_timing.cap = records_per_tag;
    g_timing.on = true;
    return SD_OK;
}

extern "C" int sd_timing_collect(int32_t tag, float* ms_host, int32_t capacity, int32_t* count) {
    SD_REQUIRE(g_timing.on, SD_EINVAL, "timing: not enabled");
    SD_REQUIRE(tag >= 0 && tag < SD_TIMING_TAGS && ms_host && count && capacity >= 0, SD_EINVAL, "timing: bad arguments");
    const int n = g_timing.count[tag] < capacity ? g_timing.count[tag] : capacity;
    for (int i = 0; i < n; ++i) {
        SD_HIP_CHECK(hipEventSynchronize(g_timing.ev[tag][1][i]));
        SD_HIP_CHECK(hipEventElapsedTime(&ms_host[i], g_timing.ev[tag][0][i], g_timing.ev[tag][1][i]));
    }
    *count = n;
    return SD_OK;
}

extern "C" int sd_timing_disable(void) {
    if (!g_timing.on) return SD_OK;
    g_timing.on = false;
    for (int t = 0; t < SD_TIMING_TAGS; ++t)
        for (int w = 0; w < 2; ++w) {
            for (hipEvent_t e : g_timing.ev[t][w]) (void)hipEventDestroy(e);
            g_timing.ev[t][w].clear();
        }
    g_timing.cap = 0;
    return SD_OK;
}

// ---------------------------------------------------------------------------------------
// lora_linear_fwd
// ---------------------------------------------------------------------------------------
extern "C" size_t sd_lora_linear_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t r, int32_t has_ln) {
    (void)N;
    if (M <= 0 || K <= 0) return 256;
    Workspace ws(nullptr, 0);
    size_t total = 0;
    if (has_ln) total += round_up((size_t)M * K * 2, 256);
    total += round_up((size_t)M * (r > 0 ? r : 8) * 2, 256);
    if (r > 0) total += DepFlags::bytes_for(M);
    (void)ws;
    return total;
}

static int lora_linear_impl(const char* who, const void* x, int32_t x_dtype, const sd_proj* p, const uint16_t* ln_gamma,
                            const uint16_t* ln_beta, float ln_eps, const void* residual, void* y, int32_t y_dtype,
                            int32_t epilogue, int32_t M, int32_t N, int32_t K, void* ws, size_t ws_bytes, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool has_ln = ln_gamma || ln_beta;
    Workspace w(ws, ws_bytes);
    const uint16_t* xin = static_cast<const uint16_t*>(x);
    uint16_t* n = has_ln ? (uint16_t*)w.take((size_t)M * K * 2) : nullptr;
    uint16_t* t = (uint16_t*)w.take((size_t)M * (p->r > 0 ? p->r : 8) * 2);
    DepFlags dep;
    if (p->r > 0) dep.carve(w, M);
    SD_REQUIRE(w.ok(), SD_EWORKSPACE, "%s: workspace too small", who);
    dep.reset();
    int rc;
    if (has_ln) {
        if ((rc = layernorm(x, x_dtype == SD_F32, ln_gamma, ln_beta, ln_eps, n, M, K, s, &dep))) return rc;
        xin = n;
    }
    ProjCall c = {xin, K, M, K, N, p, t, {y, N, y_dtype == SD_F32, residual, N, false, epilogue == SD_EPI_GEGLU ? N : 0}};
    return run_projections(&c, 1, s, -1, &dep);
}

// argument checks shared by the two entry points; *empty: nothing to do
static int lora_linear_check(const char* who, const void* x, int32_t x_dtype, const sd_proj* p, const uint16_t* ln_gamma,
                             const uint16_t* ln_beta, const void* residual, void* y, int32_t y_dtype, int32_t epilogue, int32_t M,
                             int32_t N, int32_t K, bool* empty) {
    *empty = false;
    SD_REQUIRE(M >= 0 && N >= 0, SD_EINVAL, "%s: M=%d N=%d", who, M, N);
    int rc = check_proj(p, who, K);
    if (rc) return rc;
    SD_REQUIRE(x_dtype == SD_BF16 || x_dtype == SD_F32, SD_EINVAL, "%s: x_dtype=%d", who, x_dtype);
    SD_REQUIRE(y_dtype == SD_BF16 || y_dtype == SD_F32, SD_EINVAL, "%s: y_dtype=%d", who, y_dtype);
    SD_REQUIRE(epilogue == SD_EPI_NONE || epilogue == SD_EPI_GEGLU, SD_EINVAL, "%s: epilogue=%d", who, epilogue);
    const bool has_ln = ln_gamma || ln_beta;
    SD_REQUIRE(!has_ln || (ln_gamma && ln_beta), SD_EINVAL, "%s: LayerNorm needs both gamma and beta", who);
    SD_REQUIRE(has_ln || x_dtype == SD_BF16, SD_EINVAL, "%s: fp32 x is only accepted together with a LayerNorm", who);
    SD_REQUIRE(!(epilogue == SD_EPI_GEGLU && residual), SD_EINVAL, "%s: GEGLU epilogue takes no residual", who);
    if (M == 0 || N == 0) { *empty = true; return SD_OK; }
    SD_REQUIRE(x && y, SD_EINVAL, "%s: x or y is null", who);
    SD_REQUIRE(aligned16(x) && aligned16(y) && aligned16(residual) && aligned16(p->bias), SD_EINVAL,
               "%s: pointers must be 16-byte aligned", who);
    return SD_OK;
}

extern "C" int sd_lora_linear_fwd(const void* x, int32_t x_dtype, const sd_proj* p, const uint16_t* ln_gamma,
                                  const uint16_t* ln_beta, float ln_eps, const void* residual, void* y, int32_t y_dtype,
                                  int32_t epilogue, int32_t M, int32_t N, int32_t K, void* ws, size_t ws_bytes, void* stream) {
    bool empty;
    int rc = lora_linear_check("lora_linear", x, x_dtype, p, ln_gamma, ln_beta, residual, y, y_dtype, epilogue, M, N, K, &empty);
    if (rc || empty) return rc;
    const bool has_ln = ln_gamma || ln_beta;
    SD_REQUIRE(ws_bytes >= sd_lora_linear_workspace_bytes(M, N, K, p->r, has_ln) && ws, SD_EWORKSPACE,
               "lora_linear: workspace of %zu bytes, need %zu", ws_bytes, sd_lora_linear_workspace_bytes(M, N, K, p->r, has_ln));
    return lora_linear_impl("lora_linear", x, x_dtype, p, ln_gamma, ln_beta, ln_eps, residual, y, y_dtype, epilogue, M, N, K, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------
// lora_linear_fwd_static: the same call for callers that cannot allocate a workspace
// ---------------------------------------------------------------------------------------
// The scratch memory of sd_lora_linear_fwd (LayerNorm output, down-projection, dependency
// flags) in a device array of the library itself.  Every GPU the library runs on holds its
// own copy, at its own address, until the process ends.  The name below is a host-side
// stand-in: only the address hipGetSymbolAddress returns may be handed to kernels.
namespace sd {
static __device__ __align__(256) unsigned char scratch[SD_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device, looked up once per device
static int static_scratch(void** out) {
    int dev = -1;
    SD_HIP_CHECK(hipGetDevice(&dev));
    SD_REQUIRE(dev >= 0 && dev < MAX_DEVICES, SD_EUNSUPPORTED, "lora_linear_static: device %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        SD_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        SD_REQUIRE(ptr && (reinterpret_cast<uintptr_t>(ptr) & 255u) == 0, SD_EHIP, "lora_linear_static: scratch array at %p", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SD_OK;
}
}  // namespace sd

extern "C" int sd_lora_linear_fwd_static(const void* x, int32_t x_dtype, const sd_proj* p, const uint16_t* ln_gamma,
                                         const uint16_t* ln_beta, float ln_eps, const void* residual, void* y, int32_t y_dtype,
                                         int32_t epilogue, int32_t M, int32_t N, int32_t K, void* stream) {
    bool empty;
    int rc = lora_linear_check("lora_linear_static", x, x_dtype, p, ln_gamma, ln_beta, residual, y, y_dtype, epilogue, M, N, K, &empty);
    if (rc || empty) return rc;
    const bool has_ln = ln_gamma || ln_beta;
    const size_t need = sd_lora_linear_workspace_bytes(M, N, K, p->r, has_ln);
    SD_REQUIRE(need <= (size_t)SD_STATIC_SCRATCH_BYTES, SD_EWORKSPACE,
               "lora_linear_static: M=%d K=%d r=%d%s needs %zu bytes of scratch, the built-in array holds %zu: use sd_lora_linear_fwd with a workspace",
               M, K, p->r, has_ln ? " with LayerNorm" : "", need, (size_t)SD_STATIC_SCRATCH_BYTES);
    void* ptr = nullptr;
    if ((rc = static_scratch(&ptr))) return rc;
    return lora_linear_impl("lora_linear_static", x, x_dtype, p, ln_gamma, ln_beta, ln_eps, residual, y, y_dtype, epilogue, M, N, K, ptr,
                            SD_STATIC_SCRATCH_BYTES, stream);
}

// ---------------------------------------------------------------------------------------
// attention_fwd / attn_block_fwd
// ---------------------------------------------------------------------------------------
extern "C" size_t sd_attention_workspace_bytes(int32_t Bn, int32_t Tq, int32_t Tk, int32_t heads) {
    return attention_scratch_bytes(Bn, Tq, Tk, heads) + 256;
}

extern "C" int sd_attention_fwd(const uint16_t* q, const uint16_t* k, const uint16_t* vt, uint16_t* out, int32_t Bn,
                                int32_t Tq, int32_t Tk, int32_t C, int32_t heads, void* ws, size_t ws_bytes, void* stream) {
    SD_REQUIRE(Bn >= 0 && Tq >= 0 && Tk >= 0 && heads > 0, SD_EINVAL, "attention: Bn=%d Tq=%d Tk=%d heads=%d", Bn, Tq, Tk, heads);
    SD_REQUIRE(C == heads * 64, SD_EUNSUPPORTED, "attention: C=%d heads=%d (head dim must be 64)", C, heads);
    if (Bn == 0 || Tq == 0) return SD_OK;
    SD_REQUIRE(Tk >= 1, SD_EINVAL, "attention: no keys");
    SD_REQUIRE(aligned16(q) && aligned16(k) && aligned16(vt) && aligned16(out), SD_EINVAL, "attention: pointers must be 16-byte aligned");
    const int Tkp = pad8(Tk);
    const size_t need = attention_scratch_bytes(Bn, Tq, Tk, heads);
    Workspace w(ws, ws_bytes);
    void* scratch = need ? w.take(need) : nullptr;
    SD_REQUIRE(need == 0 || (ws && w.ok()), SD_EWORKSPACE, "attention: workspace of %zu bytes, need %zu", ws_bytes,
               sd_attention_workspace_bytes(Bn, Tq, Tk, heads));
    int cut = 0;
    const int rc = launch_attention(q, C, k, C, vt, (int64_t)Bn * Tkp, out, C, Bn, Tq, Tk, Tkp, heads, false, scratch, need, &cut,
                                    static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_attention_merge(scratch, out, C, Bn, Tq, heads, false, cut, static_cast<hipStream_t>(stream));
}

extern "C" size_t sd_attn_block_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t Tc, int32_t Dc, int32_t r_max) {
    (void)Dc;
    if (Bn <= 0 || T <= 0 || C <= 0) return 256;
    Workspace ws((void*)256, (size_t)-1 / 2);
    AttnWs w;
    carve_attn(ws, w, Bn, T, C, Tc > 0 ? (Tc > T ? Tc : T) : T, r_max, C / 64);
    return ws.used + DepFlags::bytes_for((size_t)Bn * (Tc > T ? Tc : T));
}

extern "C" int sd_attn_block_fwd(const void* x, void* y, int32_t io_dtype, const uint16_t* ctx, int32_t Tc, int32_t Dc,
                                 const uint16_t* ln_gamma, const uint16_t* ln_beta, float ln_eps, const sd_proj* q,
                                 const sd_proj* k, const sd_proj* v, const sd_proj* o, int32_t Bn, int32_t T, int32_t C,
                                 int32_t heads, void* ws, size_t ws_bytes, void* stream) {
    SD_REQUIRE(Bn >= 0 && T >= 0 && C > 0 && heads > 0, SD_EINVAL, "attn_block: Bn=%d T=%d C=%d heads=%d", Bn, T, C, heads);
    SD_REQUIRE(C == heads * 64, SD_EUNSUPPORTED, "attn_block: C=%d heads=%d (head dim must be 64)", C, heads);
    SD_REQUIRE(io_dtype == SD_BF16 || io_dtype == SD_F32, SD_EINVAL, "attn_block: io_dtype=%d", io_dtype);
    SD_REQUIRE(ln_gamma && ln_beta, SD_EINVAL, "attn_block: LayerNorm gamma/beta are null");
    const int Kkv = ctx ? Dc : C;
    if (ctx) SD_REQUIRE(Tc >= 1 && Dc > 0, SD_EINVAL, "attn_block: Tc=%d Dc=%d", Tc, Dc);
    int rc;
    if ((rc = check_proj(q, "attn_block q", C)) || (rc = check_proj(k, "attn_block k", Kkv)) ||
        (rc = check_proj(v, "attn_block v", Kkv)) || (rc = check_proj(o, "attn_block o", C)))
        return rc;
    if (Bn == 0 || T == 0) return SD_OK;
    SD_REQUIRE(x && y && aligned16(x) && aligned16(y) && aligned16(ctx), SD_EINVAL, "attn_block: x/y/ctx null or misaligned");
    const sd_proj* ps[4] = {q, k, v, o};
    const int rmax = rmax_of(ps, 4);
    const int Tk = ctx ? Tc : T;
    Workspace w(ws, ws_bytes);
    AttnWs aw;
    DepFlags dep;
    SD_REQUIRE(ws && carve_attn(w, aw, Bn, T, C, Tk, rmax, heads) && dep.carve(w, (size_t)Bn * (Tk > T ? Tk : T)), SD_EWORKSPACE,
               "attn_block: workspace of %zu bytes is too small", ws_bytes);
    dep.reset();
    return attn_sublayer(x, y, io_dtype == SD_F32, ctx, Tc, Dc, ln_gamma, ln_beta, ln_eps, *q, *k, *v, *o, Bn, T, C, heads, aw,
                         static_cast<hipStream_t>(stream), nullptr, false, &dep);
}

// ---------------------------------------------------------------------------------------
// ff_block_fwd
// ---------------------------------------------------------------------------------------
extern "C" size_t sd_ff_block_workspace_bytes(int32_t M, int32_t C, int32_t F, int32_t r_max) {
    if (M <= 0 || C <= 0 || F <= 0) return 256;
    Workspace ws((void*)256, (size_t)-1 / 2);
    FfWs w;
    carve_ff(ws, w, M, C, F, r_max);
    return ws.used + DepFlags::bytes_for(M);
}

extern "C" int sd_ff_block_fwd(const void* x, void* y, int32_t io_dtype, const uint16_t* ln_gamma, const uint16_t* ln_beta,
                               float ln_eps, const sd_proj* ff1, const sd_proj* ff2, int32_t M, int32_t C, int32_t F, void* ws,
                               size_t ws_bytes, void* stream) {
    SD_REQUIRE(M >= 0 && C > 0 && F > 0, SD_EINVAL, "ff_block: M=%d C=%d F=%d", M, C, F);
    SD_REQUIRE(io_dtype == SD_BF16 || io_dtype == SD_F32, SD_EINVAL, "ff_block: io_dtype=%d", io_dtype);
    SD_REQUIRE(ln_gamma && ln_beta, SD_EINVAL, "ff_block: LayerNorm gamma/beta are null");
    int rc;
    if ((rc = check_proj(ff1, "ff_block ff1", C)) || (rc = check_proj(ff2, "ff_block ff2", F))) return rc;
    if (M == 0) return SD_OK;
    SD_REQUIRE(x && y && aligned16(x) && aligned16(y), SD_EINVAL, "ff_block: x/y null or misaligned");
    const sd_proj* ps[2] = {ff1, ff2};
    Workspace w(ws, ws_bytes);
    FfWs fw;
    DepFlags dep;
    SD_REQUIRE(ws && carve_ff(w, fw, M, C, F, rmax_of(ps, 2)) && dep.carve(w, M), SD_EWORKSPACE, "ff_block: workspace of %zu bytes is too small", ws_bytes);
    dep.reset();
    return ff_sublayer(x, y, io_dtype == SD_F32, ln_gamma, ln_beta, ln_eps, *ff1, *ff2, M, C, F, fw, static_cast<hipStream_t>(stream), &dep);
}

// ---------------------------------------------------------------------------------------
// groupnorm_fwd
// ---------------------------------------------------------------------------------------
extern "C" size_t sd_groupnorm_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t groups) {
    (void)C;
    if (Bn <= 0 || T <= 0 || groups <= 0) return 256;
    return round_up(groupnorm_partials_bytes(Bn, T, groups), 256);
}

static int groupnorm_entry(bool silu, const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta, int32_t Bn,
                                int32_t T, int32_t C, int32_t groups, float eps, void* ws, size_t ws_bytes, void* stream) {
    SD_REQUIRE(Bn >= 0 && T >= 0 && C > 0 && groups > 0, SD_EINVAL, "groupnorm: Bn=%d T=%d C=%d groups=%d", Bn, T, C, groups);
    if (Bn == 0 || T == 0) return SD_OK;
    SD_REQUIRE(x && y && gamma && beta, SD_EINVAL, "groupnorm: null pointer");
    SD_REQUIRE(aligned16(x) && aligned16(y) && aligned16(gamma) && aligned16(beta), SD_EINVAL, "groupnorm: misaligned pointer");
    SD_REQUIRE(ws && ws_bytes >= sd_groupnorm_workspace_bytes(Bn, T, C, groups), SD_EWORKSPACE, "groupnorm: workspace of %zu bytes, need %zu",
               ws_bytes, sd_groupnorm_workspace_bytes(Bn, T, C, groups));
    return launch_groupnorm(x, y, gamma, beta, Bn, T, C, groups, eps, static_cast<float*>(ws), static_cast<hipStream_t>(stream), silu);
}

extern "C" int sd_groupnorm_fwd(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta, int32_t Bn,
                                int32_t T, int32_t C, int32_t groups, float eps, void* ws, size_t ws_bytes, void* stream) {
    return groupnorm_entry(false, x, y, gamma, beta, Bn, T, C, groups, eps, ws, ws_bytes, stream);
}

extern "C" int sd_groupnorm_silu_fwd(const uint16_t* x, uint16_t* y, const uint16_t* gamma, const uint16_t* beta, int32_t Bn,
                                     int32_t T, int32_t C, int32_t groups, float eps, void* ws, size_t ws_bytes, void* stream) {
    return groupnorm_entry(true, x, y, gamma, beta, Bn, T, C, groups, eps, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------
// spatial_transformer_fwd
// ---------------------------------------------------------------------------------------
namespace sd {
struct StackWs { float* h; uint16_t* g; float* gn; AttnWs a; FfWs f; DepFlags dep; };
static bool carve_stack(Workspace& ws, StackWs& w, int Bn, int T, int C, int Tc, int rmax) {
    const size_t M = (size_t)Bn * T;
    w.h = (float*)ws.take(M * C * 4);
    w.g = (uint16_t*)ws.take(M * C * 2);
    w.gn = (float*)ws.take(groupnorm_partials_bytes(Bn, T, 32));
    carve_attn(ws, w.a, Bn, T, C, Tc > T ? Tc : T, rmax, C / 64, Tc);
    carve_ff(ws, w.f, (int)M, C, 4 * C, rmax);
    w.dep.carve(ws, std::max(M, (size_t)Bn * Tc));
    return ws.ok();
}
}  // namespace sd

extern "C" size_t sd_spatial_transformer_workspace_bytes(int32_t Bn, int32_t T, int32_t C, int32_t Tc, int32_t Dc, int32_t r_max) {
    (void)Dc;
    if (Bn <= 0 || T <= 0 || C <= 0) return 256;
    Workspace ws((void*)256, (size_t)-1 / 2);
    StackWs w;
    carve_stack(ws, w, Bn, T, C, Tc, r_max);
    return ws.used;
}

extern "C" int sd_spatial_transformer_fwd(const uint16_t* x, const uint16_t* ctx, const sd_stack_params* p, uint16_t* y,
                                          int32_t Bn, int32_t T, int32_t C, int32_t heads, int32_t Tc, int32_t Dc, void* ws,
                                          size_t ws_bytes, void* stream) {
    SD_REQUIRE(Bn >= 0 && T >= 0 && C > 0 && heads > 0 && Tc >= 1 && Dc > 0, SD_EINVAL,
               "spatial_transformer: Bn=%d T=%d C=%d heads=%d Tc=%d Dc=%d", Bn, T, C, heads, Tc, Dc);
    SD_REQUIRE(C == heads * 64, SD_EUNSUPPORTED, "spatial_transformer: C=%d heads=%d (head dim must be 64)", C, heads);
    SD_REQUIRE(C % 32 == 0 && (C / 32) % 2 == 0, SD_EUNSUPPORTED, "spatial_transformer: C=%d does not split into 32 even groups", C);
    SD_REQUIRE(p && p->depth >= 0 && (p->depth == 0 || p->blocks), SD_EINVAL, "spatial_transformer: params null or depth < 0");
    SD_REQUIRE(p->gn_g && p->gn_b, SD_EINVAL, "spatial_transformer: GroupNorm affine is null");
    int rc;
    if ((rc = check_proj(&p->proj_in, "proj_in", C)) || (rc = check_proj(&p->proj_out, "proj_out", C))) return rc;
    int rmax = 0;
    for (int i = 0; i < p->depth; ++i) {
        const sd_block_params& b = p->blocks[i];
        SD_REQUIRE(b.ln1_g && b.ln1_b && b.ln2_g && b.ln2_b && b.ln3_g && b.ln3_b, SD_EINVAL, "block %d: LayerNorm affine is null", i);
        if ((rc = check_proj(&b.q1, "q1", C)) || (rc = check_proj(&b.k1, "k1", C)) || (rc = check_proj(&b.v1, "v1", C)) ||
            (rc = check_proj(&b.o1, "o1", C)) || (rc = check_proj(&b.q2, "q2", C)) || (rc = check_proj(&b.k2, "k2", Dc)) ||
            (rc = check_proj(&b.v2, "v2", Dc)) || (rc = check_proj(&b.o2, "o2", C)) || (rc = check_proj(&b.ff1, "ff1", C)) ||
            (rc = check_proj(&b.ff2, "ff2", 4 * C)))
            return rc;
        const sd_proj* ps[10] = {&b.q1, &b.k1, &b.v1, &b.o1, &b.q2, &b.k2, &b.v2, &b.o2, &b.ff1, &b.ff2};
        const int r = rmax_of(ps, 10);
        if (r > rmax) rmax = r;
    }
    if (Bn == 0 || T == 0) return SD_OK;
    SD_REQUIRE(x && y && ctx && aligned16(x) && aligned16(y) && aligned16(ctx), SD_EINVAL, "spatial_transformer: x/y/ctx null or misaligned");
    Workspace w(ws, ws_bytes);
    StackWs sw;
    SD_REQUIRE(ws && carve_stack(w, sw, Bn, T, C, Tc, rmax), SD_EWORKSPACE, "spatial_transformer: workspace of %zu bytes, need %zu", ws_bytes,
               sd_spatial_transformer_workspace_bytes(Bn, T, C, Tc, Dc, rmax));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int M = Bn * T;
    // GroupNorm -> proj_in -> fp32 residual stream h
    timing_mark(SD_TIMING_GROUPNORM, 0, s);
    rc = launch_groupnorm(x, sw.g, p->gn_g, p->gn_b, Bn, T, C, 32, 1e-6f, sw.gn, s);
    timing_mark(SD_TIMING_GROUPNORM, 1, s);
    if (rc) return rc;
    ProjCall cin = {sw.g, C, M, C, C, &p->proj_in, sw.f.t1, {sw.h, C, 1, nullptr, 0, false, 0}};
    sw.dep.reset();
    if ((rc = run_projections(&cin, 1, s, SD_TIMING_PROJ_IO, &sw.dep))) return rc;
    for (int i = 0; i < p->depth; ++i) {
        const sd_block_params& b = p->blocks[i];
        // the text keys / values of this block's cross-attention ride in the self-attention launches
        std::vector<ProjCall> ahead;
        push_kv_calls(ahead, ctx, Dc, Tc, b.k2, b.v2, sw.a.k2, sw.a.vt2, sw.a.tk2, sw.a.tv2, Bn, C);
        if ((rc = attn_sublayer(sw.h, sw.h, 1, nullptr, 0, 0, b.ln1_g, b.ln1_b, 1e-5f, b.q1, b.k1, b.v1, b.o1, Bn, T, C, heads, sw.a, s, &ahead, false, &sw.dep)))
            return rc;
        if ((rc = attn_sublayer(sw.h, sw.h, 1, ctx, Tc, Dc, b.ln2_g, b.ln2_b, 1e-5f, b.q2, b.k2, b.v2, b.o2, Bn, T, C, heads, sw.a, s, nullptr, true, &sw.dep)))
            return rc;
        // the last block hands its output to proj_out as bf16 directly
        if ((rc = ff_sublayer(sw.h, sw.h, 1, b.ln3_g, b.ln3_b, 1e-5f, b.ff1, b.ff2, M, C, 4 * C, sw.f, s, &sw.dep,
                              i == p->depth - 1 ? sw.g : nullptr)))
            return rc;
    }
    // proj_out + input residual, bf16 out
    if (p->depth == 0 && (rc = launch_cvt_f32_to_bf16(sw.h, sw.g, (size_t)M * C, s))) return rc;
    ProjCall cout = {sw.g, C, M, C, C, &p->proj_out, sw.f.t1, {y, C, 0, x, C, false, 0}};
    return run_projections(&cout, 1, s, SD_TIMING_PROJ_IO, &sw.dep);
}

// ---------------------------------------------------------------------------------------
// multi_lora_linear_fwd
// ---------------------------------------------------------------------------------------
extern "C" size_t sd_multi_lora_linear_workspace_bytes(int32_t M, int32_t r_max) {
    if (M <= 0) return 256;
    return round_up((size_t)M * (r_max > 0 ? r_max : 8) * 2, 256) + (r_max > 0 ? DepFlags::bytes_for(M) : 0);
}

extern "C" int sd_multi_lora_linear_fwd(const uint16_t* x, const uint16_t* W, const uint16_t* bias, const uint16_t* const* A_ptrs,
                                        const uint16_t* const* B_ptrs, const int32_t* ranks, const float* scales,
                                        const int32_t* seg_offsets, const int32_t* seg_adapter, int32_t nseg, int32_t nadapters,
                                        uint16_t* y, int32_t M, int32_t N, int32_t K, void* ws, size_t ws_bytes, void* stream) {
    SD_REQUIRE(M >= 0 && N >= 0 && K > 0 && K % 8 == 0, SD_EINVAL, "multi_lora: M=%d N=%d K=%d", M, N, K);
    SD_REQUIRE(nseg >= 0 && nadapters >= 0, SD_EINVAL, "multi_lora: nseg=%d nadapters=%d", nseg, nadapters);
    if (M == 0 || N == 0) return SD_OK;
    SD_REQUIRE(x && W && y && aligned16(x) && aligned16(W) && aligned16(y) && aligned16(bias), SD_EINVAL, "multi_lora: x/W/y null or misaligned");
    SD_REQUIRE(seg_offsets && seg_adapter && nseg >= 1, SD_EINVAL, "multi_lora: segment table missing");
    SD_REQUIRE(nadapters == 0 || (A_ptrs && B_ptrs && ranks && scales), SD_EINVAL, "multi_lora: adapter tables missing");
    SD_REQUIRE(seg_offsets[0] == 0 && seg_offsets[nseg] == M, SD_EINVAL, "multi_lora: segments must cover [0, M)");
    int rmax = 0;
    for (int a = 0; a < nadapters; ++a) {
        SD_REQUIRE(ranks[a] > 0 && ranks[a] % 8 == 0, SD_EUNSUPPORTED, "multi_lora: adapter %d rank %d is not a positive multiple of 8", a, ranks[a]);
        SD_REQUIRE(A_ptrs[a] && B_ptrs[a] && aligned16(A_ptrs[a]) && aligned16(B_ptrs[a]), SD_EINVAL, "multi_lora: adapter %d A/B null or misaligned", a);
        if (ranks[a] > rmax) rmax = ranks[a];
    }
    for (int i = 0; i < nseg; ++i) {
        SD_REQUIRE(seg_offsets[i + 1] >= seg_offsets[i], SD_EINVAL, "multi_lora: segment %d has negative length", i);
        SD_REQUIRE(seg_adapter[i] >= -1 && seg_adapter[i] < nadapters, SD_EINVAL, "multi_lora: segment %d names adapter %d", i, seg_adapter[i]);
    }
    SD_REQUIRE(ws && ws_bytes >= sd_multi_lora_linear_workspace_bytes(M, rmax), SD_EWORKSPACE, "multi_lora: workspace of %zu bytes, need %zu",
               ws_bytes, sd_multi_lora_linear_workspace_bytes(M, rmax));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace wsp(ws, ws_bytes);
    uint16_t* t = (uint16_t*)wsp.take((size_t)M * (rmax > 0 ? rmax : 8) * 2);   // segment i's down-projection lives at t + offset_i * rmax
    DepFlags dep;
    if (rmax > 0) dep.carve(wsp, M);
    SD_REQUIRE(wsp.ok(), SD_EWORKSPACE, "multi_lora: workspace too small");
    dep.reset();
    std::vector<sd_proj> projs(nseg);
    std::vector<ProjCall> calls;
    for (int i = 0; i < nseg; ++i) {
        const int lo = seg_offsets[i], rows = seg_offsets[i + 1] - lo;
        if (rows == 0) continue;
        const int a = seg_adapter[i];
        sd_proj& pr = projs[i];
        pr.W = W; pr.bias = bias; pr.A = a >= 0 ? A_ptrs[a] : nullptr; pr.B = a >= 0 ? B_ptrs[a] : nullptr;
        pr.r = a >= 0 ? ranks[a] : 0; pr.scale = a >= 0 ? scales[a] : 0.f;
        calls.push_back({x + (size_t)lo * K, K, rows, K, N, &pr, t + (size_t)lo * rmax, {y + (size_t)lo * N, N, 0, nullptr, 0, false, 0}});
    }
    return run_projections(calls.data(), (int)calls.size(), s, -1, &dep);
}
