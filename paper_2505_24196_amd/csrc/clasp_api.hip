// Host side of the C ABI declared in include/clasp.h: argument checks, workspace carving and the kernel sequences
// of the three calls of the hot path (verify forward, DP layer selection, draft step). Everything is enqueued on the
// caller's stream; no call synchronises or allocates device memory.
#include "../../include/clasp.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <new>
#include <type_traits>
#include <vector>

#include "clasp_attn.h"
#include "clasp_sample.h"
#include "clasp_common.h"
#include "clasp_gemm.h"
#include "clasp_misc.h"
#include "clasp_prefill.h"

using namespace clasp;

// Working memory of clasp_prefill_static (the prompt pass for callers that cannot allocate and hold no workspace):
// one copy per GPU that loads the library, kept until the process ends. Host code never uses this name as an address:
// static_scratch_ptr() asks the runtime for the device address once per device and every launch takes that pointer.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (null on failure).
void* static_scratch_ptr() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

// Tuning constants (each can be overridden on the compiler command line for sweeps; the values are the measured best
// on MI355X at the LLaMA-3-8B and -70B shapes).
// --- several-row streaming GEMM: a workgroup has CW x KW wavefronts (CW column-tile groups that share their activation
//     fragments, KW slices of K reduced through LDS); NACC = column tiles per wavefront
#ifndef CLASP_QKV_CW
#define CLASP_QKV_CW 1
#endif
#ifndef CLASP_QKV_KW
#define CLASP_QKV_KW 4
#endif
#ifndef CLASP_QKV_NACC
#define CLASP_QKV_NACC 1
#endif
#ifndef CLASP_QKV_WIDE_NACC
#define CLASP_QKV_WIDE_NACC 4  // column tiles per wavefront when the projection has 2 x CUs tiles or more
#endif
#ifndef CLASP_OPROJ_CW
#define CLASP_OPROJ_CW 1
#endif
#ifndef CLASP_OPROJ_KW
#define CLASP_OPROJ_KW 8
#endif
#ifndef CLASP_OPROJ_NACC
#define CLASP_OPROJ_NACC 1
#endif
#ifndef CLASP_GATEUP_CW
#define CLASP_GATEUP_CW 4  // gate|up and lm_head only take this kernel when they have no more tiles than the GPU has CUs
#endif
#ifndef CLASP_GATEUP_KW
#define CLASP_GATEUP_KW 2
#endif
#ifndef CLASP_GATEUP_NACC
#define CLASP_GATEUP_NACC 4  // column tiles per wavefront when gate|up streams (K too long for the resident kernels: 70B shape)
#endif
#ifndef CLASP_DOWN_CW
#define CLASP_DOWN_CW 1
#endif
#ifndef CLASP_DOWN_KW
#define CLASP_DOWN_KW 8
#endif
#ifndef CLASP_DOWN_NACC
#define CLASP_DOWN_NACC 1
#endif
#ifndef CLASP_HEAD_CW
#define CLASP_HEAD_CW 4
#endif
#ifndef CLASP_HEAD_KW
#define CLASP_HEAD_KW 2
#endif
// the DP's down projection: K split over CLASP_DOWNP_KS workgroups per group of column tiles, slices added by the
// select kernel
#ifndef CLASP_DOWNP_CW
#define CLASP_DOWNP_CW 2
#endif
#ifndef CLASP_DOWNP_KW
#define CLASP_DOWNP_KW 4
#endif
#ifndef CLASP_DOWNP_KS
#define CLASP_DOWNP_KS 4
#endif
#ifndef CLASP_DOWNP_NACC
#define CLASP_DOWNP_NACC 2
#endif
// launches with two 16-row groups (17..32 rows): four activation loads per k-step, shared by this many column tiles
#ifndef CLASP_R2_NACC
#define CLASP_R2_NACC 4
#endif
#ifndef CLASP_R2_DEPTH
#define CLASP_R2_DEPTH 2  // k-steps per register stage of those launches
#endif
// ... per projection (tiles per wavefront, column-tile wavefronts, K-slice wavefronts of a two-group launch)
#ifndef CLASP_R2_OPROJ
#define CLASP_R2_OPROJ 2, 1, 8
#endif
#ifndef CLASP_R2_GATEUP
#define CLASP_R2_GATEUP CLASP_R2_NACC, CLASP_GATEUP_CW, CLASP_GATEUP_KW
#endif
#ifndef CLASP_R2_QKV
#define CLASP_R2_QKV 4, 1, 4
#endif
// k-steps per register stage (two stages in flight)
#ifndef CLASP_STREAM_DEPTH
#define CLASP_STREAM_DEPTH 8  // several-row streaming kernel, one row group
#endif
#ifndef CLASP_GEMM_DEPTH
#define CLASP_GEMM_DEPTH 4  // resident-activation kernel
#endif
#ifndef CLASP_ACT_SPLIT
#define CLASP_ACT_SPLIT 2  // 2: activations enter the MFMAs as bf16 hi + lo; 1: hi only
#endif
// --- single-row kernel (draft steps, plain decoding)
#ifndef CLASP_GEMV
#define CLASP_GEMV 1  // 0: single-row launches take the several-row kernel
#endif
#ifndef CLASP_GEMV_PERSISTENT
#define CLASP_GEMV_PERSISTENT 1  // one-row gate|up and lm_head take the persistent single-row kernel
#endif
#ifndef CLASP_FEW_ROWS
#define CLASP_FEW_ROWS 8  // launches of up to this many rows (<= kFewRows) take it
#endif
#ifndef CLASP_GEMVP_DEPTH
#define CLASP_GEMVP_DEPTH 4
#endif
#ifndef CLASP_GEMV_DEPTH
#define CLASP_GEMV_DEPTH 4  // more loads in flight than HBM latency x bandwidth needs only queue (16 is 5 % slower)
#endif
#ifndef CLASP_GEMV_KW_QKV
#define CLASP_GEMV_KW_QKV 8
#endif
#ifndef CLASP_GEMV_KW_RESID
#define CLASP_GEMV_KW_RESID 8
#endif
// --- attention
#ifndef CLASP_ATTN_DEFER
#define CLASP_ATTN_DEFER 1  // one-row launches: the output projection merges the attention's prefix splits
#endif
#ifndef CLASP_ATTN_SHORT_WAVES
#define CLASP_ATTN_SHORT_WAVES 8
#endif
#ifndef CLASP_ATTN_SHORT_BLOCKS
#define CLASP_ATTN_SHORT_BLOCKS 40  // prefixes of up to this many 32-key blocks take the latency-oriented launch
#endif
#ifndef CLASP_ATTN_BLOCKS_PER_SPLIT
#define CLASP_ATTN_BLOCKS_PER_SPLIT 32  // 32-key blocks per workgroup before the prefix is split further
#endif
#ifndef CLASP_ATTN_NT2_BLOCKS
#define CLASP_ATTN_NT2_BLOCKS 512  // head_dim 128: from this many blocks on a workgroup takes two query tiles
#endif
constexpr int kMaxSplit = 64;  // most workgroups that share one KV head's prefix

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Carver {
    char* base;
    size_t off = 0;
    template <class T>
    T* take(size_t bytes) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align256(bytes);
        return p;
    }
};

}  // namespace

struct clasp_ctx {
    clasp_config cfg;
    int qkv_dim, q_dim, kv_dim, group;
    size_t esz;  // bytes of a weight / cache element
    const void *embed, *lm_head;
    const float* final_norm;
    std::vector<const float*> attn_norm, mlp_norm;
    std::vector<const void*> wq, wk, wv, wo, w_gate_up, w_down;
    char *k_cache, *v_cache;
    size_t kv_layer_bytes;
    // workspace
    float2* rope;
    float* qkv;
    void *op_h, *op_attn, *op_a, *op_act;
    float *ss_h, *ss_a;
    float *a_buf, *h[2], *g[2], *G;
    float* logits;
    float* attn_partial;
    float* down_parts;  // [CLASP_DOWNP_KS][32][d] K-slices of the DP's down projection
    void* head_parts;   // [32][vocab/16] x 16 bytes: per-tile pieces of the greedy head
    void *q_frag, *k_self, *v_self;
    uint8_t* choice;
    int32_t* tok_tmp;
    // optional per-kernel timing (host-side event objects only; no device memory)
    std::vector<int> kept;  // host scratch of masked_layers (sized once at create: no allocation per call)
    int n_cu = 256;  // compute units of the device, queried at create (this value only if the query fails)
    int device = 0;  // the HIP device the context was created on
    void* static_scratch = nullptr;  // that device's copy of the library's static scratch array
    int timer_kind = -1, timer_every = 1;
    size_t timer_used = 0, timer_seen = 0;
    std::vector<hipEvent_t> timer_start, timer_stop;
};

namespace {

size_t carve(const clasp_config& c, char* base, clasp_ctx* ctx) {
    Carver w{base};
    const size_t d = c.d_model, qd = (size_t)c.n_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
    const size_t qkvd = qd + 2 * kvd, rows = kMaxRows;
    auto* rope = w.take<float2>((size_t)c.max_seq * (c.head_dim / 2) * sizeof(float2));
    auto* qkv = w.take<float>(rows * qkvd * 4);
    auto* op_h = w.take<void>(rows * d * 4);
    auto* op_attn = w.take<void>(rows * qd * 4);
    auto* op_a = w.take<void>(rows * d * 4);
    auto* op_act = w.take<void>(rows * (size_t)c.d_ffn * 4);
    auto* ss_h = w.take<float>((d / 16) * rows * 4);
    auto* ss_a = w.take<float>((d / 16) * rows * 4);
    auto* a_buf = w.take<float>(rows * d * 4);
    auto* h0 = w.take<float>(rows * d * 4);
    auto* h1 = w.take<float>(rows * d * 4);
    auto* g0 = w.take<float>((rows + 1) * d * 4);
    auto* g1 = w.take<float>((rows + 1) * d * 4);
    auto* G = w.take<float>(rows * d * 4);
    auto* logits = w.take<float>(rows * (size_t)c.vocab * 4);
    const size_t grp = c.n_heads / c.n_kv_heads;
    auto* part = w.take<float>((size_t)c.n_kv_heads * (2 * grp + 4) * 16 * kMaxSplit * (c.head_dim + 2) * 4);
    auto* head_parts = w.take<void>((size_t)(c.vocab / 16) * rows * 16);
    auto* down_parts = w.take<float>((size_t)CLASP_DOWNP_KS * rows * d * 4);
    auto* q_frag = w.take<void>(qd * 64 + 4 * (size_t)c.head_dim * 32);  // + 4 query tiles of slack for padded groups
    auto* k_self = w.take<void>(kvd * 64);
    auto* v_self = w.take<void>(kvd * 64);
    auto* choice = w.take<uint8_t>((size_t)(c.n_layers + 1) * (rows + 1));
    auto* tok = w.take<int32_t>(256);
    if (ctx) {
        ctx->rope = rope; ctx->qkv = qkv; ctx->op_h = op_h; ctx->op_attn = op_attn; ctx->op_a = op_a;
        ctx->op_act = op_act; ctx->ss_h = ss_h; ctx->ss_a = ss_a; ctx->a_buf = a_buf; ctx->h[0] = h0; ctx->h[1] = h1;
        ctx->g[0] = g0; ctx->g[1] = g1; ctx->G = G; ctx->logits = logits; ctx->attn_partial = part;
        ctx->choice = choice; ctx->tok_tmp = tok; 
        ctx->down_parts = down_parts; ctx->head_parts = head_parts; ctx->q_frag = q_frag; ctx->k_self = k_self; ctx->v_self = v_self;
    }
    return w.off;
}

int check_config(const clasp_config* c) {
    if (!c) return CLASP_E_INVALID_ARG;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 || c->d_ffn < 1 ||
        c->vocab < 1 || c->max_seq < 1 || c->max_rows < 1)
        return CLASP_E_INVALID_ARG;
    if (c->dtype != CLASP_F32 && c->dtype != CLASP_BF16) return CLASP_E_INVALID_ARG;
    if (c->max_rows > kMaxRows || c->max_seq % 32 || c->n_heads % c->n_kv_heads || c->vocab % 16)
        return CLASP_E_UNSUPPORTED;
    const int qd = c->n_heads * c->head_dim, kvd = c->n_kv_heads * c->head_dim;
    if (c->dtype == CLASP_BF16) {
        if (c->d_model % 32 || c->d_ffn % 32 || qd % 32 || kvd % 16) return CLASP_E_UNSUPPORTED;
        if (c->head_dim != 64 && c->head_dim != 128) return CLASP_E_UNSUPPORTED;
        if (c->n_heads / c->n_kv_heads > 16) return CLASP_E_UNSUPPORTED;
    } else {
        if (c->d_model % 16 || c->d_ffn % 16 || qd % 16 || kvd % 16 || c->head_dim % 2) return CLASP_E_UNSUPPORTED;
        if (c->max_seq > 8192 || c->head_dim > 256) return CLASP_E_UNSUPPORTED;  // attention keeps all scores in LDS
    }
    return CLASP_OK;
}

#define CLASP_LAUNCH_CHECK()                                 \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return CLASP_E_HIP; \
    } while (0)

// ---- per-kernel timer ----------------------------------------------------------------------------------------------
// Every `timer_every`-th launch of the chosen kernel kind gets an event pair. Where a scope holds exactly one launch
// the pair is attached to the launch itself (launch_timed: the events then carry the kernel's own begin and end time
// stamps, no extra packets on the stream); a scope with several launches is bracketed by two recorded events.
struct TimerScope {
    clasp_ctx* ctx;
    hipStream_t st;
    bool on, bracket;
    TimerScope(const clasp_ctx* c, int kind, hipStream_t s, bool bracket_launches)
        : ctx(const_cast<clasp_ctx*>(c)), st(s), bracket(bracket_launches) {
        on = ctx->timer_kind == kind && ctx->timer_used < ctx->timer_start.size() &&
             (ctx->timer_seen++ % ctx->timer_every) == 0;
        if (on && bracket) (void)hipEventRecord(start(), st);
    }
    hipEvent_t start() const { return ctx->timer_start[ctx->timer_used]; }
    hipEvent_t stop() const { return ctx->timer_stop[ctx->timer_used]; }
    ~TimerScope() {
        if (!on) return;
        if (bracket) (void)hipEventRecord(stop(), st);
        ++ctx->timer_used;
    }
};

template <class K, class... Args>
void launch_timed(const TimerScope& t, K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
    if (t.on && !t.bracket)
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, t.start(), t.stop(), 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
}

// ---- GEMM dispatch ---------------------------------------------------------------------------------------------
// Which projections may use the resident-activation kernel (bit = CLASP_KERNEL_* kind) when it applies (one row group
// and K <= 32 * kResidentKW * kResidentKSW).
#ifndef CLASP_RESIDENT_MASK
#define CLASP_RESIDENT_MASK ((1 << CLASP_KERNEL_GATE_UP) | (1 << CLASP_KERNEL_LM_HEAD))
#endif
constexpr int kResidentKW = 8, kResidentKSW = 16;

constexpr size_t kGemvMaxLds = 96 * 1024;

// LDS bytes the single-row kernel needs for this contraction length with KWV wavefronts, 0 if it cannot take it.
template <int KWV>
size_t gemv_lds_bytes(int K) {
    const int nks_max = (K / 32 + KWV - 1) / KWV;
    if (nks_max * CLASP_ACT_SPLIT * 4 > kGemvLoads * 64) return 0;
    const size_t lds = (size_t)KWV * nks_max * CLASP_ACT_SPLIT * 64;
    return lds <= kGemvMaxLds ? lds : 0;
}

template <int EPI, int KWV, int ASRC = 0>
int launch_gemv(const TimerScope& timer, const GemmArgs& g, size_t lds, hipStream_t st) {
    static bool opted_in = false;  // more than 64 KiB of LDS per workgroup has to be requested once per kernel
    auto kernel = gemv_bf16_kernel<KWV, EPI, CLASP_GEMV_DEPTH, CLASP_ACT_SPLIT, ASRC>;
    if (!opted_in) {
        if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemvMaxLds) !=
            hipSuccess)
            return CLASP_E_HIP;
        opted_in = true;
    }
    launch_timed(timer, kernel, dim3(g.N / 16), dim3(KWV * 64), lds, st, g, (g.K / 32 + KWV - 1) / KWV);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

template <int EPI, int CW, int KW, int NACC = 1, int R2NACC = CLASP_R2_NACC, int R2CW = CW, int R2KW = KW>
int launch_gemm(const clasp_ctx* ctx, const GemmArgs& g, hipStream_t st, int kind) {
    const int tiles = g.N / 16;
    TimerScope timer(ctx, kind, st, false);
    if (ctx->cfg.dtype == CLASP_BF16) {
        const bool resident = g.R == 1 && ((CLASP_RESIDENT_MASK >> kind) & 1) &&
                              (g.K / 32 + kResidentKW - 1) / kResidentKW <= kResidentKSW && tiles > ctx->n_cu;
        constexpr int KWV = EPI == kEpiQkv ? CLASP_GEMV_KW_QKV : (EPI == kEpiResid ? CLASP_GEMV_KW_RESID : 8);
        const size_t gemv_lds =
            (CLASP_GEMV && g.n_rows == 1 && g.R == 1 && EPI != kEpiPartial) ? gemv_lds_bytes<KWV>(g.K) : 0;
        if (resident && CLASP_GEMV_PERSISTENT && g.n_rows <= CLASP_FEW_ROWS) {
            // few rows: they sit in LDS, the registers hold a whole tile slice of weights per wavefront
            auto kernel = gemv_persistent_bf16_kernel<kResidentKSW, kResidentKW, EPI, CLASP_GEMVP_DEPTH, CLASP_ACT_SPLIT>;
            static bool opted_in = false;  // more than 64 KiB of LDS per workgroup has to be requested once per kernel
            if (!opted_in) {
                if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        kResidentKW * kResidentKSW * CLASP_ACT_SPLIT * 64 * kFewRows) != hipSuccess)
                    return CLASP_E_HIP;
                opted_in = true;
            }
            const int rounds = (tiles + ctx->n_cu - 1) / ctx->n_cu, grid = (tiles + rounds - 1) / rounds;
            launch_timed(timer, kernel, dim3(grid), dim3((kResidentKW + 1) * 64),
                         (size_t)kResidentKW * kResidentKSW * CLASP_ACT_SPLIT * 64 * g.n_rows, st, g);
        } else if (resident && !(gemv_lds && kind == CLASP_KERNEL_LM_HEAD)) {  // one-row lm_head: the single-row kernel is 3 % faster
            // every workgroup takes the same number of tiles (+-1): rounds = ceil(tiles / CUs), grid = ceil(tiles / rounds)
            const int rounds = (tiles + ctx->n_cu - 1) / ctx->n_cu, grid = (tiles + rounds - 1) / rounds;
            launch_timed(timer, gemm_bf16_resident_kernel<kResidentKSW, kResidentKW, EPI, CLASP_GEMM_DEPTH, CLASP_ACT_SPLIT>,
                         dim3(grid), dim3(kResidentKW * 64), 0, st, g);
        } else if (gemv_lds) {
            if constexpr (EPI == kEpiResid) {
                if (g.attn_partial) return launch_gemv<EPI, KWV, 1>(timer, g, gemv_lds, st);
            }
            return launch_gemv<EPI, KWV>(timer, g, gemv_lds, st);
        } else {
            if constexpr (EPI == kEpiQkv && NACC == 1 && CLASP_QKV_WIDE_NACC > 1) {
                // a projection with at least two column tiles per CU and wavefront-to-be (the 70B shape's q|k|v: 640
                // tiles) lets a wavefront carry several tiles, which share its activation loads, and still fills the chip
                if (g.R == 1 && tiles >= 2 * ctx->n_cu) {
                    constexpr int WN = CLASP_QKV_WIDE_NACC;
                    launch_timed(timer, gemm_bf16_kernel<1, CW, KW, EPI, CLASP_STREAM_DEPTH / WN, CLASP_ACT_SPLIT, WN>,
                                 dim3((tiles + CW * WN - 1) / (CW * WN)), dim3(CW * KW * 64), 0, st, g);
                    CLASP_LAUNCH_CHECK();
                    return CLASP_OK;
                }
            }
            if (g.R == 1) {  // NACC tiles per wavefront share the activation fragments; the stage depth shrinks to match
                const dim3 grid((tiles + CW * NACC - 1) / (CW * NACC));
                launch_timed(timer, gemm_bf16_kernel<1, CW, KW, EPI, CLASP_STREAM_DEPTH / NACC, CLASP_ACT_SPLIT, NACC>, grid,
                             dim3(CW * KW * 64), 0, st, g);
            } else {
                // two row groups: R2NACC column tiles per wavefront share the four activation loads of a k-step (weight
                // fragments per stage stay the same, so fewer tiles per wavefront mean more k-steps per stage)
                const dim3 grid((tiles + R2CW * R2NACC - 1) / (R2CW * R2NACC));
                launch_timed(timer, gemm_bf16_kernel<2, R2CW, R2KW, EPI, CLASP_R2_DEPTH * CLASP_R2_NACC / R2NACC, CLASP_ACT_SPLIT, R2NACC>,
                             grid, dim3(R2CW * R2KW * 64), 0, st, g);
            }
        }
    } else {
        if constexpr (EPI == kEpiQkv || EPI == kEpiHead || EPI == kEpiPartial) return CLASP_E_UNSUPPORTED;
        else launch_timed(timer, gemm_f32_kernel<EPI>, dim3(tiles), dim3(256), 0, st, g);
    }
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

template <int HD, int NT, int NW, bool STREAM>
int launch_attn_one(const AttnArgs& a, dim3 grid, hipStream_t st) {
    constexpr size_t lds = (size_t)NW * HD * 17 * sizeof(float);
    static bool opted_in = false;  // more than 64 KiB of LDS per workgroup has to be requested once per kernel
    if (!opted_in) {
        if (hipFuncSetAttribute((const void*)attn_bf16_kernel<HD, NT, NW, STREAM>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess)
            return CLASP_E_HIP;
        opted_in = true;
    }
    hipLaunchKernelGGL((attn_bf16_kernel<HD, NT, NW, STREAM>), grid, dim3(NW * 64), lds, st, a);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

// short = latency-oriented launch: one query tile per workgroup, keys and values through plain (cached) loads
template <int HD>
int launch_attn_bf16(const AttnArgs& a, bool short_prefix, int nt, dim3 grid, hipStream_t st) {
    if (short_prefix) return launch_attn_one<HD, 1, CLASP_ATTN_SHORT_WAVES, false>(a, grid, st);
    if (nt == 1) return launch_attn_one<HD, 1, 8, true>(a, grid, st);
    if (nt == 2) return launch_attn_one<HD, 2, 8, true>(a, grid, st);
    if constexpr (HD <= 64) {
        if (nt == 3) return launch_attn_one<HD, 3, 8, true>(a, grid, st);
        return launch_attn_one<HD, 4, 8, true>(a, grid, st);
    } else {
        // head_dim 128: three or four query tiles (33..64 queries of a KV group: 9..16 DP rows at 4 heads per group) need
        // more registers than two wavefronts per SIMD leave: four wavefronts, one per SIMD, each with the whole file
        if (nt == 3) return launch_attn_one<HD, 3, 4, true>(a, grid, st);
        return launch_attn_one<HD, 4, 4, true>(a, grid, st);
    }
}

// Prefix splits of a one-row launch whose merge the output projection takes over (0 = merge here as usual): the
// single-row projection kernel stages its input through LDS anyway and can merge up to kGemvMaxSplit pieces per
// query while doing so, which saves the combine launch of long prefixes and lets short prefixes use several
// workgroups per KV head (one workgroup cannot pull its 256 KiB at T = 512 faster than ~50 GB/s).
int attn_deferred_splits(const clasp_ctx* ctx, int n, int R, int mode, int pos0) {
    const clasp_config& c = ctx->cfg;
    if (!CLASP_GEMV || !CLASP_ATTN_DEFER || c.dtype != CLASP_BF16 || n != 1 || R != 1 || c.head_dim % 8) return 0;
    if (!gemv_lds_bytes<CLASP_GEMV_KW_RESID>(ctx->q_dim)) return 0;
    const int nblk = (pos0 + (mode ? n : 0) + 31) / 32;
    const int per = nblk <= CLASP_ATTN_SHORT_BLOCKS ? CLASP_ATTN_SHORT_WAVES : CLASP_ATTN_BLOCKS_PER_SPLIT;
    int split = (nblk + per - 1) / per;
    // a few thousand tokens: as many pieces as the merge takes, so that 64 rather than 16 workgroups pull the prefix
    if (nblk > CLASP_ATTN_SHORT_BLOCKS && split < kGemvMaxSplit) split = std::min(kGemvMaxSplit, (nblk + 7) / 8);
    return (split >= 2 && split <= kGemvMaxSplit) ? split : 0;
}

int launch_attention(const clasp_ctx* ctx, int layer, int n, int R, int mode, int pos0, hipStream_t st,
                     int deferred_splits = 0) {
    const clasp_config& c = ctx->cfg;
    AttnArgs a{};
    a.qkv = ctx->qkv; a.ld_qkv = ctx->qkv_dim;
    a.n_rows = n; a.n_heads = c.n_heads; a.n_kv_heads = c.n_kv_heads; a.head_dim = c.head_dim;
    a.pos0 = pos0; a.mode = mode; a.rope = ctx->rope;
    a.Kc = ctx->k_cache + (size_t)layer * ctx->kv_layer_bytes;
    a.Vt = ctx->v_cache + (size_t)layer * ctx->kv_layer_bytes;
    a.t_max = c.max_seq; a.out_op = ctx->op_attn; a.R = R;
    a.partial = ctx->attn_partial;
    a.scale = 1.0f / sqrtf((float)c.head_dim);
    a.q_frag = ctx->q_frag; a.k_self = ctx->k_self; a.v_self = ctx->v_self;
    a.n_split = 1;
    TimerScope timer(ctx, CLASP_KERNEL_ATTENTION, st, true);
    if (c.dtype == CLASP_F32) {
        const size_t lds = (size_t)(c.head_dim + pos0 + 32) * sizeof(float);
        hipLaunchKernelGGL(attn_f32_kernel, dim3(c.n_heads, n), dim3(256), lds, st, a);
        CLASP_LAUNCH_CHECK();
        return CLASP_OK;
    }
    // Short prefixes are latency-bound: one query tile per workgroup (more workgroups, each key block re-read from
    // L2 by the few workgroups of a KV head) and 16 wavefronts, so that a wavefront sees one or two key blocks.
    // Long prefixes are bandwidth-bound: up to 4 query tiles per workgroup (keys read once) and the prefix split
    // across workgroups.
    const int nQ = n * ctx->group, ntq = (nQ + 15) / 16;
    const int nblk = (pos0 + (mode ? n : 0) + 31) / 32;
    const bool short_prefix = nblk <= CLASP_ATTN_SHORT_BLOCKS;
    // query tiles per workgroup: what the register file holds without spilling (O^T alone is head_dim/4 registers
    // per tile); further tiles go to sibling workgroups, launched next to each other so that their key reads meet in L2
    // (head_dim 128: one tile below CLASP_ATTN_NT2_BLOCKS blocks; from there on as many as the queries fill, up to 4: one
    // pass over the prefix serves all of them, where sibling workgroups re-read 12 % of it from HBM and take 33 us
    // instead of 24 per layer at 32768 tokens)
    const int max_nt = c.head_dim > 64 ? (nblk >= CLASP_ATTN_NT2_BLOCKS ? 4 : 1) : 4;
    const int nt = short_prefix ? 1 : (ntq < max_nt ? ntq : max_nt), qgroups = (ntq + nt - 1) / nt;
    int split = short_prefix ? 1 : (nblk + CLASP_ATTN_BLOCKS_PER_SPLIT - 1) / CLASP_ATTN_BLOCKS_PER_SPLIT;
    {   // a CU holds one of these workgroups: a launch a little above a whole number of rounds would leave most CUs
        // idle for its last round, so the split count is trimmed to fill whole rounds
        const int per_split = c.n_kv_heads * qgroups, wgs = per_split * split;
        if (wgs > ctx->n_cu) {
            const int rounds = (wgs + ctx->n_cu / 2) / ctx->n_cu, trimmed = rounds * ctx->n_cu / per_split;
            if (trimmed >= 1 && trimmed < split) split = trimmed;
        }
    }
    if (!short_prefix) {
        // a few thousand tokens leave the launch well below one workgroup per CU at 32 blocks per split: split further, down
        // to 4 blocks per workgroup, until the CUs are covered (a workgroup pulls ~50 GB/s, the chip a hundred times that)
        const int per_split = c.n_kv_heads * qgroups, fill = ctx->n_cu / per_split, most = nblk / 4;
        if (split < fill) split = std::max(split, std::min(fill, most));
    }
    split = split < 1 ? 1 : (split > kMaxSplit ? kMaxSplit : split);
    if (deferred_splits) split = deferred_splits;
    a.n_split = split;
    const dim3 grid(c.n_kv_heads, qgroups, split);
    const int rc = c.head_dim == 64 ? launch_attn_bf16<64>(a, short_prefix, nt, grid, st)
                                    : launch_attn_bf16<128>(a, short_prefix, nt, grid, st);
    if (rc) return rc;
    if (split > 1 && !deferred_splits) {
        hipLaunchKernelGGL(attn_combine_kernel, dim3(c.n_kv_heads, nQ), dim3(kCombineWaves * 64), 0, st, a, nt, qgroups);
        CLASP_LAUNCH_CHECK();
    }
    return CLASP_OK;
}

// One decoder layer on n rows. The rows' fp32 values are at h_in ([n][d]); their GEMM operand (times the layer's
// attention-norm gains) and sums of squares must already sit in op_h / ss_h. Writes h_out ([n][d]) and, if asked,
// the operand / sums of squares of h_out for whatever consumes it next, and a copy for hidden-state capture.
// down_split > 1: the down projection only leaves its K-slices in ctx->down_parts (rows of a_buf are the residual);
// the caller's next kernel adds them up (the DP's select kernel does).
int run_layer(const clasp_ctx* ctx, int l, int n, int R, int mode, int pos0, const float* h_in, float* h_out,
              void* next_op, const float* next_gain, float* next_ss, float* capture, hipStream_t st,
              int down_split = 1) {
    const clasp_config& c = ctx->cfg;
    const int d = c.d_model, F = c.d_ffn;
    int rc;
    {
        GemmArgs g{};
        g.W[0] = ctx->wq[l]; g.W[1] = ctx->wk[l]; g.W[2] = ctx->wv[l];
        g.tile_end[0] = ctx->q_dim / 16; g.tile_end[1] = (ctx->q_dim + ctx->kv_dim) / 16; g.tile_end[2] = ctx->qkv_dim / 16;
        g.A = ctx->op_h; g.n_rows = n; g.N = ctx->qkv_dim; g.K = d; g.R = R;
        g.ss_parts = ctx->ss_h; g.n_parts = d / 16; g.inv_dim = 1.0f / d; g.eps = c.rms_eps;
        g.out = ctx->qkv; g.ldo = ctx->qkv_dim;
        if (c.dtype == CLASP_BF16) {
            QkvOut& o = g.qkv;
            o.n_heads = c.n_heads; o.n_kv_heads = c.n_kv_heads; o.head_dim = c.head_dim;
            o.pos0 = pos0; o.mode = mode; o.t_max = c.max_seq; o.rope = ctx->rope;
            o.q_scale = 1.4426950408889634f / sqrtf((float)c.head_dim);
            o.q_frag = ctx->q_frag;
            o.k_cache = ctx->k_cache + (size_t)l * ctx->kv_layer_bytes;
            o.v_cache = ctx->v_cache + (size_t)l * ctx->kv_layer_bytes;
            o.k_self = ctx->k_self; o.v_self = ctx->v_self;
            if ((rc = launch_gemm<kEpiQkv, CLASP_QKV_CW, CLASP_QKV_KW, CLASP_QKV_NACC, CLASP_R2_QKV>(ctx, g, st, CLASP_KERNEL_QKV))) return rc;
        } else {
            if ((rc = launch_gemm<kEpiScale, 1, 1>(ctx, g, st, CLASP_KERNEL_QKV))) return rc;
        }
    }
    const int deferred = attn_deferred_splits(ctx, n, R, mode, pos0);
    if ((rc = launch_attention(ctx, l, n, R, mode, pos0, st, deferred))) return rc;
    {
        GemmArgs g{};
        g.W[0] = ctx->wo[l]; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = d / 16;
        g.A = ctx->op_attn; g.n_rows = n; g.N = d; g.K = ctx->q_dim; g.R = R;
        if (deferred) {
            g.attn_partial = ctx->attn_partial; g.attn_split = deferred; g.attn_group = ctx->group; g.attn_hd = c.head_dim;
        }
        g.out = ctx->a_buf; g.ldo = d; g.resid = h_in; g.ldr = d;
        g.next_op = ctx->op_a; g.next_gain = ctx->mlp_norm[l]; g.next_ss = ctx->ss_a;
        if ((rc = launch_gemm<kEpiResid, CLASP_OPROJ_CW, CLASP_OPROJ_KW, CLASP_OPROJ_NACC, CLASP_R2_OPROJ>(ctx, g, st, CLASP_KERNEL_O_PROJ))) return rc;
    }
    {
        GemmArgs g{};
        if (c.dtype == CLASP_BF16) {  // interleaved gate|up: 2F/16 tiles of one stream
            g.W[0] = ctx->w_gate_up[l]; g.N = 2 * F;
        } else {  // fp32: gate rows followed by up rows
            g.W[0] = ctx->w_gate_up[l]; g.W[1] = static_cast<const float*>(ctx->w_gate_up[l]) + (size_t)F * d; g.N = F;
        }
        g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = g.N / 16;
        g.A = ctx->op_a; g.n_rows = n; g.K = d; g.R = R;
        g.ss_parts = ctx->ss_a; g.n_parts = d / 16; g.inv_dim = 1.0f / d; g.eps = c.rms_eps;
        g.next_op = ctx->op_act;
        if ((rc = launch_gemm<kEpiSwiglu, CLASP_GATEUP_CW, CLASP_GATEUP_KW, CLASP_GATEUP_NACC, CLASP_R2_GATEUP>(ctx, g, st, CLASP_KERNEL_GATE_UP))) return rc;
    }
    if (down_split > 1 && c.dtype == CLASP_BF16) {
        GemmArgs g{};
        g.W[0] = ctx->w_down[l]; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = d / 16;
        g.A = ctx->op_act; g.n_rows = n; g.N = d; g.K = F; g.R = R;
        g.out = ctx->down_parts; g.ldo = d; g.ldr = kMaxRows * d;
        TimerScope timer(ctx, CLASP_KERNEL_DOWN, st, false);
        const dim3 block(CLASP_DOWNP_CW * CLASP_DOWNP_KW * 64);
        if (R == 1)
            launch_timed(timer, gemm_bf16_kernel<1, CLASP_DOWNP_CW, CLASP_DOWNP_KW, kEpiPartial,
                                                 CLASP_STREAM_DEPTH / CLASP_DOWNP_NACC, CLASP_ACT_SPLIT, CLASP_DOWNP_NACC>,
                         dim3((d / 16 + CLASP_DOWNP_CW * CLASP_DOWNP_NACC - 1) / (CLASP_DOWNP_CW * CLASP_DOWNP_NACC), down_split),
                         block, 0, st, g);
        else
            launch_timed(timer, gemm_bf16_kernel<2, CLASP_DOWNP_CW, CLASP_DOWNP_KW, kEpiPartial, CLASP_R2_DEPTH,
                                                 CLASP_ACT_SPLIT, CLASP_R2_NACC>,
                         dim3((d / 16 + CLASP_DOWNP_CW * CLASP_R2_NACC - 1) / (CLASP_DOWNP_CW * CLASP_R2_NACC), down_split),
                         block, 0, st, g);
        CLASP_LAUNCH_CHECK();
    } else {
        GemmArgs g{};
        g.W[0] = ctx->w_down[l]; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = d / 16;
        g.A = ctx->op_act; g.n_rows = n; g.N = d; g.K = F; g.R = R;
        g.out = h_out; g.ldo = d; g.resid = ctx->a_buf; g.ldr = d;
        g.next_op = next_op; g.next_gain = next_gain; g.next_ss = next_ss;
        g.capture = capture; g.ldc = d;
        if ((rc = launch_gemm<kEpiResid, CLASP_DOWN_CW, CLASP_DOWN_KW, CLASP_DOWN_NACC>(ctx, g, st, CLASP_KERNEL_DOWN))) return rc;
    }
    return CLASP_OK;
}

int launch_embed(const clasp_ctx* ctx, const int32_t* tokens, int n, int R, float* h, const float* gain,
                 float* capture, hipStream_t st) {
    const clasp_config& c = ctx->cfg;
    if (c.dtype == CLASP_BF16)
        hipLaunchKernelGGL((embed_kernel<kDtBf16>), dim3(n, (c.d_model + 255) / 256), dim3(256), 0, st, tokens, ctx->embed, c.vocab, c.d_model, h,
                           ctx->op_h, R, gain, ctx->ss_h, capture);
    else
        hipLaunchKernelGGL((embed_kernel<kDtF32>), dim3(n, (c.d_model + 255) / 256), dim3(256), 0, st, tokens, ctx->embed, c.vocab, c.d_model, h,
                           ctx->op_h, R, gain, ctx->ss_h, capture);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

// final norm (already folded into op_h / ss_h by the last layer's epilogue) -> lm_head -> greedy head
int run_head(const clasp_ctx* ctx, int n, int R, float* logits_out, int32_t* argmax_out, float* margin_out,
             float* prob_out, hipStream_t st) {
    const clasp_config& c = ctx->cfg;
    GemmArgs g{};
    g.W[0] = ctx->lm_head; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = c.vocab / 16;
    g.A = ctx->op_h; g.n_rows = n; g.N = c.vocab; g.K = c.d_model; g.R = R;
    g.ss_parts = ctx->ss_h; g.n_parts = c.d_model / 16; g.inv_dim = 1.0f / c.d_model; g.eps = c.rms_eps;
    int rc;
    const bool want_head = argmax_out || margin_out || prob_out;
    if (c.dtype == CLASP_BF16) {
        // logits are only written when the caller asked for them; the greedy head comes from per-tile pieces
        g.out = logits_out; g.ldo = c.vocab;
        g.head_parts = static_cast<f32x4*>(ctx->head_parts);
        if ((rc = launch_gemm<kEpiHead, CLASP_HEAD_CW, CLASP_HEAD_KW>(ctx, g, st, CLASP_KERNEL_LM_HEAD))) return rc;
        if (want_head) {
            hipLaunchKernelGGL(head_reduce_kernel, dim3(n), dim3(1024), 0, st, static_cast<const f32x4*>(ctx->head_parts),
                               c.vocab / 16, argmax_out, margin_out, prob_out);
            CLASP_LAUNCH_CHECK();
        }
        return CLASP_OK;
    }
    float* logits = logits_out ? logits_out : ctx->logits;
    g.out = logits; g.ldo = c.vocab;
    if ((rc = launch_gemm<kEpiScale, 1, 1>(ctx, g, st, CLASP_KERNEL_LM_HEAD))) return rc;
    if (want_head) {
        hipLaunchKernelGGL(argmax_kernel, dim3(n), dim3(1024), 0, st, logits, c.vocab, argmax_out, margin_out, prob_out);
        CLASP_LAUNCH_CHECK();
    }
    return CLASP_OK;
}

// The layers a skip set keeps on one row at position `pos`. Returns the index of the ctx->h buffer that holds the
// result (the state before the final norm); op_h / ss_h hold its operand for the head.
int masked_layers(clasp_ctx* ctx, const uint8_t* mask, const int32_t* token, int pos, hipStream_t st, int* h_index) {
    const int L = ctx->cfg.n_layers;
    std::vector<int>& kept = ctx->kept;
    kept.clear();  // capacity n_layers since clasp_create
    for (int l = 0; l < L; ++l)
        if (!mask || !mask[l]) kept.push_back(l);
    int rc;
    const float* gain0 = kept.empty() ? ctx->final_norm : ctx->attn_norm[kept[0]];
    if ((rc = launch_embed(ctx, token, 1, 1, ctx->h[0], gain0, nullptr, st))) return rc;
    for (size_t k = 0; k < kept.size(); ++k) {
        const float* gain = (k + 1 < kept.size()) ? ctx->attn_norm[kept[k + 1]] : ctx->final_norm;
        if ((rc = run_layer(ctx, kept[k], 1, 1, 1, pos, ctx->h[k & 1], ctx->h[(k + 1) & 1], ctx->op_h, gain, ctx->ss_h,
                            nullptr, st)))
            return rc;
    }
    *h_index = (int)(kept.size() & 1);
    return CLASP_OK;
}

// ... then the head: greedy token (+ top-1 probability) and / or the logits.
int draft_forward(clasp_ctx* ctx, const uint8_t* mask, const int32_t* token, int pos, float* logits_out,
                  int32_t* argmax_out, float* top1_prob_out, hipStream_t st) {
    int h_index = 0;
    const int rc = masked_layers(ctx, mask, token, pos, st, &h_index);
    if (rc) return rc;
    return run_head(ctx, 1, 1, logits_out, argmax_out, nullptr, top1_prob_out, st);
}

// Algorithm 1 over the layers lo .. hi-1 (tables indexed from the window's first layer), everything outside kept.
int dp_select_window(clasp_ctx* ctx, const float* states, size_t layer_stride, int pos, int M, int lo, int hi,
                     uint8_t* mask_out, float* score_out, uint8_t* choice_out, float* g_final_out, hipStream_t st) {
    const clasp_config& c = ctx->cfg;
    const int L = hi - lo, d = c.d_model;
    const int down_split = (c.dtype == CLASP_BF16 && c.d_ffn / 32 >= CLASP_DOWNP_KS * CLASP_DOWNP_KW * 4) ? CLASP_DOWNP_KS : 1;
    uint8_t* choice = choice_out ? choice_out : ctx->choice;
    const int cells = (L + 1) * (M + 1);
    hipLaunchKernelGGL(dp_table_init_kernel, dim3((cells + 255) / 256), dim3(256), 0, st, score_out, choice, cells);
    CLASP_LAUNCH_CHECK();
    const float* x0 = states + (size_t)lo * layer_stride;
    // Cells (i, j) from which (L, M) cannot be reached (j < M - (L - i): too few layers left to skip) decide nothing;
    // they are computed only when the caller asked for the tables. first_cell(i) = first cell of level i that is needed.
    const bool full_table = score_out || choice_out;
    auto first_cell = [&](int i) { return full_table ? 0 : std::max(0, M - (L - i)); };
    // candidates level i pushes through its layer: cells max(1, first_cell(i)) .. min(i-1, M) of level i-1
    auto rows_of = [&](int i) { return i > L ? 0 : std::min(i - 1, M) - std::max(1, first_cell(i)) + 1; };
    // 16-row groups of a level's launches: levels with at most 16 candidates (the first 17 always; without tables also
    // the last ones) take the one-group kernels, which are the faster ones
    auto groups_of = [&](int i) { return rows_of(i) > 16 ? 2 : 1; };
    int rc;
    for (int i = 1; i <= L; ++i) {
        const int ell = (i - 1 < M) ? i - 1 : M;
        const int j0 = first_cell(i), jc0 = std::max(1, j0), n_comp = ell - jc0 + 1;
        const int jn0 = std::max(1, first_cell(i + 1));  // first cell whose state the next level pushes through a layer
        const float* g_prev = (i == 1) ? x0 : ctx->g[(i - 1) & 1];
        float* g_cur = ctx->g[i & 1];
        if (n_comp > 0) {  // candidates g(i-1, jc0..ell) through the window's layer i-1, all at position `pos`
            if ((rc = run_layer(ctx, lo + i - 1, n_comp, groups_of(i), 0, pos, g_prev + (size_t)jc0 * d, ctx->G, nullptr, nullptr,
                                nullptr, nullptr, st, down_split)))
                return rc;
        }
        SelectArgs s{};
        s.i = i; s.M = M; s.d = d; s.R = groups_of(i + 1);  // the operand it writes is the next level's
        s.j0 = j0; s.jc0 = jc0; s.jn0 = jn0;
        s.x_i = x0 + (size_t)i * layer_stride;
        s.g_prev = g_prev; s.g_cur = g_cur;
        if (down_split > 1) {  // candidates = residual rows (a_buf) + the K-slices the down projection left behind
            s.G = ctx->a_buf; s.parts = ctx->down_parts; s.n_parts = down_split; s.part_stride = (size_t)kMaxRows * d;
        } else {
            s.G = ctx->G;
        }
        s.op = (i < L) ? ctx->op_h : nullptr;
        s.gain = (i < L) ? ctx->attn_norm[lo + i] : nullptr;
        s.ss = ctx->ss_h;
        s.scores = score_out; s.choice = choice;
        const int cells_i = ((i < M) ? i : M) + 1 - j0;
        if (c.dtype == CLASP_BF16)
            hipLaunchKernelGGL((dp_select_kernel<kDtBf16>), dim3(cells_i), dim3(1024), 0, st, s);
        else
            hipLaunchKernelGGL((dp_select_kernel<kDtF32>), dim3(cells_i), dim3(1024), 0, st, s);
        CLASP_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(dp_backtrack_kernel, dim3(2), dim3(256), 0, st, choice, L, M, mask_out, lo, c.n_layers,
                       ctx->g[L & 1], g_final_out, d);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

// ---- prompt processing with many rows per pass ---------------------------------------------------------------------
#ifndef CLASP_PREFILL_BIG
#define CLASP_PREFILL_BIG 1  // 256 x 256 tiles fed by direct global -> LDS loads where the grid is large enough
#endif
// The big tiles are taken when they give at least this fraction of the CUs a workgroup: half (measured at the 8B
// shape: 512 tokens 18.9 -> 15.9 ms, 3072 tokens 63.3 -> 50.3 ms against "every CU"; a third costs short passes).
#ifndef CLASP_PREFILL_BIG_FILL_NUM
#define CLASP_PREFILL_BIG_FILL_NUM 1
#endif
#ifndef CLASP_PREFILL_BIG_FILL_DEN
#define CLASP_PREFILL_BIG_FILL_DEN 2
#endif
constexpr int kPrefillMaxChunk = 8192;
// Passes of at least this many rows (640: measured break-even at the 8B shape is between 512 and 640) run their GEMMs on fp16 MFMAs: one fp16 plane per activation instead of the bf16
// hi / lo pair (half the matrix-core work) against an fp16 copy of the layer's weights made at the start of the layer
// (one more read and write of the layer per pass, which shorter passes would not earn back). 0 = never.
#ifndef CLASP_PREFILL_F16_ROWS
#define CLASP_PREFILL_F16_ROWS 640
#endif

struct PrefillWs {
    float *h, *a_buf, *ss_h, *ss_a, *rstd_h, *rstd_a, *parts;
    void *op_h, *op_a, *op_attn, *op_act, *q_frag;
    char* w16;  // fp16 copy of one layer's packed matrices (q, k, v, o, gate|up, down in this order), or null
};

bool prefill_uses_f16(int rows) { return CLASP_PREFILL_F16_ROWS > 0 && rows >= CLASP_PREFILL_F16_ROWS; }
constexpr int kPrefillSplitRows = 1024, kPrefillMaxSplit = 4;  // K-split of short passes: rows it applies to, slices

size_t carve_prefill(const clasp_config& c, int chunk, char* base, PrefillWs* ws) {
    Carver w{base};
    const size_t C = chunk, d = c.d_model, qd = (size_t)c.n_heads * c.head_dim;
    PrefillWs t;
    t.h = w.take<float>(C * d * 4);
    t.a_buf = w.take<float>(C * d * 4);
    t.ss_h = w.take<float>((d / 16) * C * 4);
    t.ss_a = w.take<float>((d / 16) * C * 4);
    t.rstd_h = w.take<float>(C * 4);
    t.rstd_a = w.take<float>(C * 4);
    t.op_h = w.take<void>(C * d * 4);
    t.op_a = w.take<void>(C * d * 4);
    t.op_attn = w.take<void>(C * qd * 4);
    t.op_act = w.take<void>(C * (size_t)c.d_ffn * 4);
    t.q_frag = w.take<void>(C * qd * 2);
    t.parts = w.take<float>((size_t)kPrefillMaxSplit * std::min<size_t>(C, kPrefillSplitRows) * d * 4);
    const size_t kvd = (size_t)c.n_kv_heads * c.head_dim;
    t.w16 = prefill_uses_f16(chunk) ? w.take<char>((2 * qd * d + 2 * kvd * d + 3 * d * (size_t)c.d_ffn) * 2) : nullptr;
    if (ws) *ws = t;
    return w.off;
}

// Which GEMM kernel a projection of the prompt pass takes (measured at the 8B shape):
//  * o_proj, gate|up, down: 256 x 256 tiles fed by direct global -> LDS loads when they give at least half of the CUs a
//    workgroup (gate|up from 257 rows on, the projections onto d_model from 1793 rows on), else 128 x 128 tiles, two
//    workgroups per CU;
//  * q/k/v: in fp16 passes 256 x 192 tiles of the same kernel (two full rounds of CUs at 4096 rows) under the same
//    condition; in bf16 passes (hi + lo planes: its epilogue does not fit the big tile's register budget) 128 x 128
//    tiles with three lighter workgroups per CU;
//  * any of them: 64 x 128 tiles when even the 128 x 128 grid has fewer workgroups than CUs.
//  F16: the pass runs on fp16 operands (p.g.A is an fp16 plane, p.g.W an fp16 copy of the weights).
template <int EPI, bool F16>
int launch_prefill_gemm(const clasp_ctx* ctx, const PrefillGemmArgs& p, hipStream_t st, float* parts = nullptr) {
    const int tiles = p.g.N / 16;
    if constexpr (EPI != kEpiQkv || F16) {
        // q/k/v (fp16 passes only: with the bf16 planes its epilogue does not fit the registers): 192 columns per workgroup
        constexpr int RN = EPI == kEpiQkv ? 6 : 8;
        const int nrb = (p.g.R * 16 + kPrefillBigRows - 1) / kPrefillBigRows, total = nrb * ((tiles + 2 * RN - 1) / (2 * RN));
        // (the fp16 variant of the big tile walks the contraction in pairs of k-steps)
        if (CLASP_PREFILL_BIG && total * CLASP_PREFILL_BIG_FILL_DEN >= ctx->n_cu * CLASP_PREFILL_BIG_FILL_NUM && (!F16 || (p.g.K / 32) % 2 == 0)) {
            static bool opted_in = false;  // more than 64 KiB of LDS per workgroup has to be requested once per kernel
            auto kernel = prefill_gemm256_kernel<EPI, F16, RN>;
            constexpr size_t big_lds = prefill_big_lds<F16, RN>();
            if (!opted_in) {
                if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)big_lds) !=
                    hipSuccess)
                    return CLASP_E_HIP;
                opted_in = true;
            }
            hipLaunchKernelGGL(kernel, dim3((total + 7) / 8 * 8), dim3(512), big_lds, st, p);
            CLASP_LAUNCH_CHECK();
            return CLASP_OK;
        }
    }
    auto launch = [&](auto kernel, size_t lds, int rows, bool& opted) -> int {
        if (!opted) {  // more than 64 KiB of LDS per workgroup has to be requested once per kernel
            if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                return CLASP_E_HIP;
            opted = true;
        }
        const int total = ((p.g.R * 16 + rows - 1) / rows) * ((tiles + 7) / 8);
        hipLaunchKernelGGL(kernel, dim3((total + 7) / 8 * 8), dim3(256), lds, st, p);
        CLASP_LAUNCH_CHECK();
        return CLASP_OK;
    };
    static bool opted_in[2] = {false, false};
    // 64-row tiles when 128-row tiles would not give every CU a workgroup (prompts of a few hundred tokens)
    const int total128 = ((p.g.R * 16 + kPrefillRows - 1) / kPrefillRows) * ((tiles + 7) / 8);
    if (total128 < ctx->n_cu || (EPI == kEpiResid && p.g.n_rows <= kPrefillSplitRows && total128 < 2 * ctx->n_cu)) {
        if constexpr (EPI == kEpiResid) {
            // ... and when even those leave most of the three workgroup slots per CU empty, the contraction is split over
            // gridDim.y workgroups as well (o_proj and down at 512 rows: 256 workgroups of 128 / 448 k-steps otherwise);
            // the slices are summed in order by a second kernel that also runs the epilogue
            const int total = ((p.g.R * 16 + 63) / 64) * ((tiles + 7) / 8);
            int split = (3 * ctx->n_cu) / (total > 0 ? total : 1);
            split = split > kPrefillMaxSplit ? kPrefillMaxSplit : split;
            while (split >= 2 && p.g.K / 32 < 16 * split) --split;  // at least 16 k-steps per slice
            if (parts && split >= 2 && p.g.n_rows <= kPrefillSplitRows) {
                static bool split_opted_in = false;
                auto kernel = prefill_gemm_kernel<kEpiPartial, 2, 4, 2, 3, F16>;
                constexpr size_t lds = prefill_gemm_lds_bytes<2, 4, 2, F16>();
                if (!split_opted_in) {
                    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                        return CLASP_E_HIP;
                    split_opted_in = true;
                }
                PrefillGemmArgs q = p;
                q.k_split = split;
                q.slab = (size_t)p.g.n_rows * p.g.ldo;
                q.g.out = parts;
                hipLaunchKernelGGL(kernel, dim3((total + 7) / 8 * 8, split), dim3(256), lds, st, q);
                CLASP_LAUNCH_CHECK();
                q.g.out = p.g.out;
                hipLaunchKernelGGL(prefill_reduce_kernel, dim3(p.g.n_rows, (p.g.N + 255) / 256), dim3(256), 0, st, q, parts);
                CLASP_LAUNCH_CHECK();
                return CLASP_OK;
            }
        }
        constexpr size_t lds64 = prefill_gemm_lds_bytes<2, 4, 2, F16>();
        return launch(prefill_gemm_kernel<EPI, 2, 4, 2, 3, F16>, lds64, 64, opted_in[0]);
    }
    constexpr int D = EPI == kEpiQkv ? 1 : 2, WPS = EPI == kEpiQkv ? 3 : 2;
    constexpr size_t lds128 = prefill_gemm_lds_bytes<4, 4, D, F16>();
    return launch(prefill_gemm_kernel<EPI, 4, 4, D, WPS, F16>, lds128, kPrefillRows, opted_in[1]);
}

// Attention of a chunk: long prefixes share the key / value blocks of a workgroup through LDS, short ones (a few blocks
// per query, the ring would stay mostly empty) let every wavefront read them itself.
#ifndef CLASP_PREFILL_ATTN_LDS_WAVES
#define CLASP_PREFILL_ATTN_LDS_WAVES 8
#endif
#ifndef CLASP_PREFILL_ATTN_LDS_MIN_BLOCKS
#define CLASP_PREFILL_ATTN_LDS_MIN_BLOCKS 32
#endif
int launch_prefill_attn(const clasp_ctx* ctx, const PrefillAttnArgs& a, hipStream_t st) {
    const clasp_config& c = ctx->cfg;
    const int n_qt = a.R * ctx->group;
    const int nblk = (a.pos0 + a.n_rows + 31) / 32;
    if (CLASP_PREFILL_ATTN_LDS_WAVES && nblk >= CLASP_PREFILL_ATTN_LDS_MIN_BLOCKS) {
        constexpr int NW = CLASP_PREFILL_ATTN_LDS_WAVES ? CLASP_PREFILL_ATTN_LDS_WAVES : 4;
        const dim3 grid(c.n_kv_heads, (n_qt + NW * kPrefillAttnNT - 1) / (NW * kPrefillAttnNT));
        static bool opted_in[2] = {false, false};
        auto launch = [&](auto kernel, size_t lds, bool& opted) -> int {
            if (!opted) {
                if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                    return CLASP_E_HIP;
                opted = true;
            }
            hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), lds, st, a);
            CLASP_LAUNCH_CHECK();
            return CLASP_OK;
        };
        if (c.head_dim == 64) return launch(prefill_attn_lds_kernel<64, NW>, (size_t)kPrefillAttnStages * 8 * 1024, opted_in[0]);
        return launch(prefill_attn_lds_kernel<128, NW>, (size_t)kPrefillAttnStages * 16 * 1024, opted_in[1]);
    }
    const int per_wg = kPrefillAttnWaves * kPrefillAttnNT;
    const dim3 grid(c.n_kv_heads, (n_qt + per_wg - 1) / per_wg);
    if (c.head_dim == 64) hipLaunchKernelGGL(prefill_attn_kernel<64>, grid, dim3(kPrefillAttnWaves * 64), 0, st, a);
    else hipLaunchKernelGGL(prefill_attn_kernel<128>, grid, dim3(kPrefillAttnWaves * 64), 0, st, a);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

// The full model over n rows at positions pos0.. (n <= the chunk the workspace was carved for): leaves their keys and
// values in the cache. The last layer stops after its q/k/v projection: nothing after it feeds the cache.
int prefill_chunk(const clasp_ctx* ctx, const PrefillWs& ws, int ld, const int32_t* tokens, int n, int pos0,
                  hipStream_t st) {
    const clasp_config& c = ctx->cfg;
    const int d = c.d_model, F = c.d_ffn, L = c.n_layers, R = (n + 15) / 16;
    const bool f16 = ws.w16 && prefill_uses_f16(n);
    int rc;
    hipLaunchKernelGGL(prefill_embed_kernel, dim3(n, (d + 255) / 256), dim3(256), 0, st, tokens,
                       static_cast<const bf16*>(ctx->embed), c.vocab, d, ws.h, ws.op_h, R, ctx->attn_norm[0], ws.ss_h, ld,
                       (int)f16);
    CLASP_LAUNCH_CHECK();
    auto gemm = [&](auto epi, const PrefillGemmArgs& p, float* parts) -> int {
        constexpr int EPI = decltype(epi)::value;
        return f16 ? launch_prefill_gemm<EPI, true>(ctx, p, st, parts) : launch_prefill_gemm<EPI, false>(ctx, p, st, parts);
    };
    for (int l = 0; l < L; ++l) {
        // this layer's matrices, as packed or as the fp16 copy made here (the last layer only runs q/k/v)
        const void* W[6] = {ctx->wq[l], ctx->wk[l], ctx->wv[l], ctx->wo[l], ctx->w_gate_up[l], ctx->w_down[l]};
        if (f16) {
            const size_t bytes[6] = {(size_t)ctx->q_dim * d * 2, (size_t)ctx->kv_dim * d * 2, (size_t)ctx->kv_dim * d * 2,
                                     (size_t)d * ctx->q_dim * 2, (size_t)2 * F * d * 2,       (size_t)d * F * 2};
            const int n_mat = l == L - 1 ? 3 : 6;
            ConvertArgs cv{};
            size_t off = 0;
            for (int m = 0; m < 6; ++m) {
                cv.src[m] = static_cast<const u32x4*>(W[m]);
                cv.dst[m] = reinterpret_cast<u32x4*>(ws.w16 + off);
                if (m < n_mat) off += bytes[m];
                cv.end[m] = off / 16;
                W[m] = cv.dst[m];
            }
            hipLaunchKernelGGL(prefill_convert_f16_kernel, dim3(ctx->n_cu * 8), dim3(256), 0, st, cv);
            CLASP_LAUNCH_CHECK();
        }
        hipLaunchKernelGGL(prefill_rstd_kernel, dim3((n + 63) / 64), dim3(64, 16), 0, st, ws.ss_h, d / 16, ld, n, 1.0f / d,
                           c.rms_eps, ws.rstd_h);
        CLASP_LAUNCH_CHECK();
        {
            PrefillGemmArgs p{};
            GemmArgs& g = p.g;
            g.W[0] = W[0]; g.W[1] = W[1]; g.W[2] = W[2];
            g.tile_end[0] = ctx->q_dim / 16; g.tile_end[1] = (ctx->q_dim + ctx->kv_dim) / 16; g.tile_end[2] = ctx->qkv_dim / 16;
            g.A = ws.op_h; g.n_rows = n; g.N = ctx->qkv_dim; g.K = d; g.R = R;
            p.rstd = ws.rstd_h; p.op_f16 = f16;
            QkvOut& o = g.qkv;
            o.n_heads = c.n_heads; o.n_kv_heads = c.n_kv_heads; o.head_dim = c.head_dim;
            o.pos0 = pos0; o.mode = 1; o.t_max = c.max_seq; o.rope = ctx->rope;
            o.q_scale = 1.4426950408889634f / sqrtf((float)c.head_dim);
            o.q_frag = ws.q_frag;
            o.k_cache = ctx->k_cache + (size_t)l * ctx->kv_layer_bytes;
            o.v_cache = ctx->v_cache + (size_t)l * ctx->kv_layer_bytes;
            if ((rc = gemm(std::integral_constant<int, kEpiQkv>{}, p, nullptr))) return rc;
        }
        if (l == L - 1) break;
        {
            PrefillAttnArgs a{};
            a.q_frag = ws.q_frag;
            a.Kc = ctx->k_cache + (size_t)l * ctx->kv_layer_bytes;
            a.Vt = ctx->v_cache + (size_t)l * ctx->kv_layer_bytes;
            a.out_op = ws.op_attn;
            a.n_rows = n; a.R = R; a.n_heads = c.n_heads; a.n_kv_heads = c.n_kv_heads; a.pos0 = pos0; a.t_max = c.max_seq;
            a.op_f16 = f16;
            if ((rc = launch_prefill_attn(ctx, a, st))) return rc;
        }
        {
            PrefillGemmArgs p{};
            GemmArgs& g = p.g;
            g.W[0] = W[3]; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = d / 16;
            g.A = ws.op_attn; g.n_rows = n; g.N = d; g.K = ctx->q_dim; g.R = R;
            g.out = ws.a_buf; g.ldo = d; g.resid = ws.h; g.ldr = d;
            g.next_op = ws.op_a; g.next_gain = ctx->mlp_norm[l]; g.next_ss = ws.ss_a; p.ld_ss = ld; p.op_f16 = f16;
            if ((rc = gemm(std::integral_constant<int, kEpiResid>{}, p, ws.parts))) return rc;
        }
        hipLaunchKernelGGL(prefill_rstd_kernel, dim3((n + 63) / 64), dim3(64, 16), 0, st, ws.ss_a, d / 16, ld, n, 1.0f / d,
                           c.rms_eps, ws.rstd_a);
        CLASP_LAUNCH_CHECK();
        {
            PrefillGemmArgs p{};
            GemmArgs& g = p.g;
            g.W[0] = W[4]; g.N = 2 * F; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = g.N / 16;
            g.A = ws.op_a; g.n_rows = n; g.K = d; g.R = R;
            p.rstd = ws.rstd_a; p.op_f16 = f16;
            g.next_op = ws.op_act;
            if ((rc = gemm(std::integral_constant<int, kEpiSwiglu>{}, p, nullptr))) return rc;
        }
        {
            PrefillGemmArgs p{};
            GemmArgs& g = p.g;
            g.W[0] = W[5]; g.tile_end[0] = g.tile_end[1] = g.tile_end[2] = d / 16;
            g.A = ws.op_act; g.n_rows = n; g.N = d; g.K = F; g.R = R;
            g.out = ws.h; g.ldo = d; g.resid = ws.a_buf; g.ldr = d;
            g.next_op = ws.op_h; g.next_gain = ctx->attn_norm[l + 1]; g.next_ss = ws.ss_h; p.ld_ss = ld; p.op_f16 = f16;
            if ((rc = gemm(std::integral_constant<int, kEpiResid>{}, p, ws.parts))) return rc;
        }
    }
    return CLASP_OK;
}

}  // namespace

extern "C" {

const char* clasp_strerror(int code) {
    switch (code) {
        case CLASP_OK: return "ok";
        case CLASP_E_INVALID_ARG: return "invalid argument";
        case CLASP_E_UNSUPPORTED: return "unsupported shape";
        case CLASP_E_HIP: return "HIP runtime error";
        case CLASP_E_WORKSPACE: return "workspace too small";
        default: return "unknown error";
    }
}

size_t clasp_packed_bytes(int rows, int cols, int dtype) {
    if (rows <= 0 || cols <= 0 || rows % 16) return 0;
    if (dtype == CLASP_BF16) return (cols % 32) ? 0 : (size_t)rows * cols * 2;
    if (dtype == CLASP_F32) return (size_t)rows * cols * 4;
    return 0;
}

int clasp_pack_matrix(const void* src, void* dst, int rows, int cols, int dtype, int rope_head_dim, void* stream) {
    if (!src || !dst || src == dst || rope_head_dim < 0) return CLASP_E_INVALID_ARG;
    if (rope_head_dim && (rope_head_dim % 16 || rows % rope_head_dim)) return CLASP_E_UNSUPPORTED;
    const size_t bytes = clasp_packed_bytes(rows, cols, dtype);
    if (!bytes) return CLASP_E_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == CLASP_F32) {
        if (hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess) return CLASP_E_HIP;
        return CLASP_OK;
    }
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(2048), dim3(256), 0, st, reinterpret_cast<const u32x4*>(src),
                       reinterpret_cast<u32x4*>(dst), rows, cols, rope_head_dim);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

int clasp_pack_gate_up(const void* gate, const void* up, void* dst, int d_ffn, int d_model, int dtype, void* stream) {
    if (!gate || !up || !dst || gate == dst || up == dst) return CLASP_E_INVALID_ARG;
    const size_t bytes = clasp_packed_bytes(d_ffn, d_model, dtype);
    if (!bytes) return CLASP_E_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == CLASP_F32) {
        if (hipMemcpyAsync(dst, gate, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess ||
            hipMemcpyAsync(static_cast<char*>(dst) + bytes, up, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess)
            return CLASP_E_HIP;
        return CLASP_OK;
    }
    hipLaunchKernelGGL(pack_gate_up_bf16_kernel, dim3(2048), dim3(256), 0, st, reinterpret_cast<const u32x4*>(gate),
                       reinterpret_cast<const u32x4*>(up), reinterpret_cast<u32x4*>(dst), d_ffn, d_model);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

size_t clasp_workspace_bytes(const clasp_config* cfg) {
    if (check_config(cfg) != CLASP_OK) return 0;
    return carve(*cfg, nullptr, nullptr);
}

size_t clasp_kv_cache_bytes(const clasp_config* cfg) {
    if (check_config(cfg) != CLASP_OK) return 0;
    return (size_t)cfg->n_layers * cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * (cfg->dtype == CLASP_BF16 ? 2 : 4);
}

int clasp_create(const clasp_config* cfg, const clasp_weights* w, void* workspace, size_t workspace_bytes,
                 void* k_cache, void* v_cache, clasp_ctx** out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !workspace || !k_cache || !v_cache || !out) return CLASP_E_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(k_cache) & 15) ||
        (reinterpret_cast<uintptr_t>(v_cache) & 15))
        return CLASP_E_INVALID_ARG;
    if (workspace_bytes < carve(*cfg, nullptr, nullptr)) return CLASP_E_WORKSPACE;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->mlp_norm || !w->wq || !w->wk || !w->wv ||
        !w->wo || !w->w_gate_up || !w->w_down)
        return CLASP_E_INVALID_ARG;
    auto misaligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; };  // 16-byte vector loads
    if (misaligned(w->embed) || misaligned(w->lm_head) || misaligned(w->final_norm)) return CLASP_E_INVALID_ARG;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const void* ptrs[8] = {w->attn_norm[l], w->mlp_norm[l], w->wq[l], w->wk[l], w->wv[l], w->wo[l], w->w_gate_up[l], w->w_down[l]};
        for (const void* ptr : ptrs)
            if (!ptr || misaligned(ptr)) return CLASP_E_INVALID_ARG;
    }
    clasp_ctx* ctx = new (std::nothrow) clasp_ctx();
    if (!ctx) return CLASP_E_INVALID_ARG;
    ctx->cfg = *cfg;
    ctx->q_dim = cfg->n_heads * cfg->head_dim;
    ctx->kv_dim = cfg->n_kv_heads * cfg->head_dim;
    ctx->qkv_dim = ctx->q_dim + 2 * ctx->kv_dim;
    ctx->group = cfg->n_heads / cfg->n_kv_heads;
    ctx->esz = cfg->dtype == CLASP_BF16 ? 2 : 4;
    ctx->embed = w->embed; ctx->lm_head = w->lm_head; ctx->final_norm = w->final_norm;
    const int L = cfg->n_layers;
    ctx->attn_norm.assign(w->attn_norm, w->attn_norm + L);
    ctx->mlp_norm.assign(w->mlp_norm, w->mlp_norm + L);
    ctx->wq.assign(w->wq, w->wq + L); ctx->wk.assign(w->wk, w->wk + L); ctx->wv.assign(w->wv, w->wv + L);
    ctx->wo.assign(w->wo, w->wo + L); ctx->w_gate_up.assign(w->w_gate_up, w->w_gate_up + L);
    ctx->w_down.assign(w->w_down, w->w_down + L);
    ctx->kept.reserve(L);
    ctx->k_cache = static_cast<char*>(k_cache);
    ctx->v_cache = static_cast<char*>(v_cache);
    ctx->kv_layer_bytes = (size_t)cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * ctx->esz;
    carve(*cfg, static_cast<char*>(workspace), ctx);
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            ctx->n_cu = cus;
        ctx->device = dev;
        ctx->static_scratch = static_scratch_ptr();
        if (!ctx->static_scratch) {
            delete ctx;
            return CLASP_E_HIP;
        }
    }

    const size_t kvb = clasp_kv_cache_bytes(cfg);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, 0, reinterpret_cast<u32x4*>(k_cache), kvb / 16);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, 0, reinterpret_cast<u32x4*>(v_cache), kvb / 16);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, 0, reinterpret_cast<u32x4*>(workspace),
                       carve(*cfg, nullptr, nullptr) / 16);
    hipLaunchKernelGGL(rope_table_kernel, dim3(1024), dim3(256), 0, 0, ctx->rope, cfg->max_seq, cfg->head_dim / 2,
                       (double)cfg->rope_base);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(0) != hipSuccess) {
        delete ctx;
        return CLASP_E_HIP;
    }
    *out = ctx;
    return CLASP_OK;
}

int clasp_destroy(clasp_ctx* ctx) {
    if (!ctx) return CLASP_E_INVALID_ARG;
    delete ctx;
    return CLASP_OK;
}

int clasp_kernel_timer_begin(clasp_ctx* ctx, int kind, int capacity, int every) {
    if (!ctx || kind < 0 || kind >= CLASP_KERNEL_KINDS || capacity < 1 || capacity > (1 << 20) || every < 1)
        return CLASP_E_INVALID_ARG;
    if (ctx->timer_kind >= 0) return CLASP_E_INVALID_ARG;
    ctx->timer_start.resize(capacity);
    ctx->timer_stop.resize(capacity);
    for (int i = 0; i < capacity; ++i)
        if (hipEventCreate(&ctx->timer_start[i]) != hipSuccess || hipEventCreate(&ctx->timer_stop[i]) != hipSuccess)
            return CLASP_E_HIP;
    ctx->timer_used = ctx->timer_seen = 0;
    ctx->timer_every = every;
    ctx->timer_kind = kind;
    return CLASP_OK;
}

int clasp_kernel_timer_end(clasp_ctx* ctx, float* total_ms, int* launches) {
    if (!ctx || !total_ms || !launches || ctx->timer_kind < 0) return CLASP_E_INVALID_ARG;
    float sum = 0.f;
    int rc = CLASP_OK;
    for (size_t i = 0; i < ctx->timer_used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(ctx->timer_stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, ctx->timer_start[i], ctx->timer_stop[i]) != hipSuccess)
            rc = CLASP_E_HIP;
        sum += ms;
    }
    for (size_t i = 0; i < ctx->timer_start.size(); ++i) {
        (void)hipEventDestroy(ctx->timer_start[i]);
        (void)hipEventDestroy(ctx->timer_stop[i]);
    }
    *total_ms = sum;
    *launches = (int)ctx->timer_used;
    ctx->timer_start.clear();
    ctx->timer_stop.clear();
    ctx->timer_kind = -1;
    ctx->timer_used = 0;
    return rc;
}

int clasp_kv_load(clasp_ctx* ctx, int layer, const float* K, const float* V, int n_tokens, void* stream) {
    if (!ctx || !K || !V) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (layer < 0 || layer >= c.n_layers || n_tokens < 0 || n_tokens > c.max_seq) return CLASP_E_INVALID_ARG;
    if (n_tokens == 0) return CLASP_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void* Kc = ctx->k_cache + (size_t)layer * ctx->kv_layer_bytes;
    void* Vt = ctx->v_cache + (size_t)layer * ctx->kv_layer_bytes;
    if (c.dtype == CLASP_BF16)
        hipLaunchKernelGGL((kv_load_kernel<kDtBf16>), dim3(1024), dim3(256), 0, st, K, V, Kc, Vt, n_tokens, c.n_kv_heads,
                           c.head_dim, c.max_seq);
    else
        hipLaunchKernelGGL((kv_load_kernel<kDtF32>), dim3(1024), dim3(256), 0, st, K, V, Kc, Vt, n_tokens, c.n_kv_heads,
                           c.head_dim, c.max_seq);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

int clasp_kv_read(clasp_ctx* ctx, int layer, int pos0, int n_tokens, float* K, float* V, void* stream) {
    if (!ctx || !K || !V) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (layer < 0 || layer >= c.n_layers || pos0 < 0 || n_tokens < 0 || (long long)pos0 + n_tokens > c.max_seq)
        return CLASP_E_INVALID_ARG;
    if (n_tokens == 0) return CLASP_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const void* Kc = ctx->k_cache + (size_t)layer * ctx->kv_layer_bytes;
    const void* Vt = ctx->v_cache + (size_t)layer * ctx->kv_layer_bytes;
    if (c.dtype == CLASP_BF16)
        hipLaunchKernelGGL((kv_read_kernel<kDtBf16>), dim3(1024), dim3(256), 0, st, Kc, Vt, K, V, pos0, n_tokens,
                           c.n_kv_heads, c.head_dim, c.max_seq);
    else
        hipLaunchKernelGGL((kv_read_kernel<kDtF32>), dim3(1024), dim3(256), 0, st, Kc, Vt, K, V, pos0, n_tokens,
                           c.n_kv_heads, c.head_dim, c.max_seq);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

int clasp_verify_forward(clasp_ctx* ctx, const int32_t* tokens, int n_tokens, int pos0, float* hidden_out,
                         int32_t* argmax_out, float* margin_out, float* logits_out, void* stream) {
    if (!ctx || !tokens) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (n_tokens < 1 || n_tokens > c.max_rows || pos0 < 0 || (long long)pos0 + n_tokens > c.max_seq)
        return CLASP_E_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = n_tokens, R = (n + 15) / 16, L = c.n_layers, d = c.d_model;
    const size_t cap_stride = (size_t)n * d;
    int rc;
    if ((rc = launch_embed(ctx, tokens, n, R, ctx->h[0], ctx->attn_norm[0], hidden_out, st))) return rc;
    for (int l = 0; l < L; ++l) {
        const float* gain = (l + 1 < L) ? ctx->attn_norm[l + 1] : ctx->final_norm;
        float* cap = hidden_out ? hidden_out + (size_t)(l + 1) * cap_stride : nullptr;
        if ((rc = run_layer(ctx, l, n, R, 1, pos0, ctx->h[l & 1], ctx->h[(l + 1) & 1], ctx->op_h, gain, ctx->ss_h, cap, st)))
            return rc;
    }
    if (argmax_out || margin_out || logits_out)
        return run_head(ctx, n, R, logits_out, argmax_out, margin_out, nullptr, st);
    return CLASP_OK;
}

size_t clasp_prefill_workspace_bytes(const clasp_config* cfg, int chunk_rows) {
    if (check_config(cfg) != CLASP_OK || cfg->dtype != CLASP_BF16) return 0;
    if (chunk_rows < kPrefillRows || chunk_rows > kPrefillMaxChunk || chunk_rows % kPrefillRows) return 0;
    return carve_prefill(*cfg, chunk_rows, nullptr, nullptr);
}

int clasp_prefill(clasp_ctx* ctx, const int32_t* tokens, int n_tokens, int pos0, int chunk_rows, void* workspace,
                  size_t workspace_bytes, void* stream) {
    if (!ctx || !tokens || !workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (c.dtype != CLASP_BF16) return CLASP_E_UNSUPPORTED;
    if (n_tokens < 1 || pos0 < 0 || (long long)pos0 + n_tokens > c.max_seq) return CLASP_E_INVALID_ARG;
    const size_t need = clasp_prefill_workspace_bytes(&c, chunk_rows);
    if (!need) return CLASP_E_INVALID_ARG;
    if (workspace_bytes < need) return CLASP_E_WORKSPACE;
    PrefillWs ws;
    carve_prefill(c, chunk_rows, static_cast<char*>(workspace), &ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int s = 0; s < n_tokens; s += chunk_rows) {
        const int n = n_tokens - s < chunk_rows ? n_tokens - s : chunk_rows;
        const int rc = prefill_chunk(ctx, ws, chunk_rows, tokens + s, n, pos0 + s, st);
        if (rc) return rc;
    }
    return CLASP_OK;
}

int clasp_prefill_static(clasp_ctx* ctx, const int32_t* tokens, int n_tokens, int pos0, int chunk_rows, void* stream) {
    if (!ctx || !tokens) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (c.dtype != CLASP_BF16) return CLASP_E_UNSUPPORTED;
    if (n_tokens < 1 || pos0 < 0 || (long long)pos0 + n_tokens > c.max_seq) return CLASP_E_INVALID_ARG;
    const size_t need = clasp_prefill_workspace_bytes(&c, chunk_rows);
    if (!need) return CLASP_E_INVALID_ARG;
    if (need > kStaticScratchBytes) return CLASP_E_WORKSPACE;  // model x chunk_rows beyond the static array
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return CLASP_E_HIP;
    if (dev != ctx->device || !ctx->static_scratch) return CLASP_E_INVALID_ARG;  // the array of another GPU
    // Every buffer of a pass is written before it is read (rows beyond n_tokens in a 16-row group only feed results
    // that are never stored), so what the previous call left in the array needs no clearing.
    return clasp_prefill(ctx, tokens, n_tokens, pos0, chunk_rows, ctx->static_scratch, kStaticScratchBytes, stream);
}

size_t clasp_static_scratch_bytes(void) { return kStaticScratchBytes; }

int clasp_draft_step(clasp_ctx* ctx, const uint8_t* mask, const int32_t* token, int pos, int32_t* next_token_out,
                     float* top1_prob_out, void* stream) {
    if (!ctx || !token || !next_token_out) return CLASP_E_INVALID_ARG;
    if (pos < 0 || pos >= ctx->cfg.max_seq) return CLASP_E_INVALID_ARG;
    return draft_forward(ctx, mask, token, pos, nullptr, next_token_out, top1_prob_out, static_cast<hipStream_t>(stream));
}

int clasp_sample_token(clasp_ctx* ctx, const float* logits, float temperature, const float* u, int32_t* token_out,
                       void* stream) {
    if (!ctx || !logits || !u || !token_out || !(temperature > 0.f)) return CLASP_E_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(sample_kernel, dim3(1), dim3(kSampleThreads), 0, st, logits, ctx->cfg.vocab, 1.0f / temperature, u,
                       token_out);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

int clasp_draft_sample(clasp_ctx* ctx, const uint8_t* mask, const int32_t* token, int pos, float temperature,
                       const float* u, float* logits_out, int32_t* next_token_out, void* stream) {
    if (!ctx || !token || !next_token_out || !u || !logits_out || !(temperature > 0.f)) return CLASP_E_INVALID_ARG;
    if (pos < 0 || pos >= ctx->cfg.max_seq) return CLASP_E_INVALID_ARG;
    int rc;
    if ((rc = draft_forward(ctx, mask, token, pos, logits_out, nullptr, nullptr, static_cast<hipStream_t>(stream))))
        return rc;
    return clasp_sample_token(ctx, logits_out, temperature, u, next_token_out, stream);
}

int clasp_spec_accept(clasp_ctx* ctx, const float* p_logits, const float* q_logits, size_t ld, const int32_t* tokens,
                      int n_draft, float temperature, const float* u_accept, const float* u_final,
                      int32_t* n_accepted_out, int32_t* next_token_out, void* stream) {
    if (!ctx || !p_logits || !q_logits || !tokens || !u_accept || !u_final || !n_accepted_out || !next_token_out)
        return CLASP_E_INVALID_ARG;
    if (!(temperature > 0.f) || n_draft < 1 || n_draft > ctx->cfg.max_rows - 1 || ld < (size_t)ctx->cfg.vocab)
        return CLASP_E_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(spec_accept_kernel, dim3(1), dim3(kSampleThreads), 0, st, p_logits, q_logits, ld, tokens, n_draft,
                       ctx->cfg.vocab, 1.0f / temperature, u_accept, u_final, n_accepted_out, next_token_out);
    CLASP_LAUNCH_CHECK();
    return CLASP_OK;
}

int clasp_dp_select_window(clasp_ctx* ctx, const float* states, size_t layer_stride, int pos, int M, int layer_lo,
                           int layer_hi, uint8_t* mask_out, float* score_out, uint8_t* choice_out, float* g_final_out,
                           void* stream) {
    if (!ctx || !states || !mask_out) return CLASP_E_INVALID_ARG;
    const clasp_config& c = ctx->cfg;
    if (layer_lo < 0 || layer_hi > c.n_layers || layer_lo >= layer_hi) return CLASP_E_INVALID_ARG;
    if (M < 0 || M > layer_hi - layer_lo || M > c.max_rows || pos < 0 || pos >= c.max_seq || layer_stride < (size_t)c.d_model)
        return CLASP_E_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(states) & 15) || (layer_stride & 3)) return CLASP_E_INVALID_ARG;  // float4 loads
    return dp_select_window(ctx, states, layer_stride, pos, M, layer_lo, layer_hi, mask_out, score_out, choice_out,
                            g_final_out, static_cast<hipStream_t>(stream));
}

int clasp_dp_select(clasp_ctx* ctx, const float* states, size_t layer_stride, int pos, int M, uint8_t* mask_out,
                    float* score_out, uint8_t* choice_out, float* g_final_out, void* stream) {
    if (!ctx) return CLASP_E_INVALID_ARG;
    return clasp_dp_select_window(ctx, states, layer_stride, pos, M, 0, ctx->cfg.n_layers, mask_out, score_out, choice_out,
                                  g_final_out, stream);
}

int clasp_skip_cosine(clasp_ctx* ctx, const uint8_t* masks, int n_masks, const int32_t* token, int pos, const float* target,
                      float* cos_out, void* stream) {
    if (!ctx || !masks || !token || !target || !cos_out || n_masks < 1) return CLASP_E_INVALID_ARG;
    if (pos < 0 || pos >= ctx->cfg.max_seq) return CLASP_E_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int L = ctx->cfg.n_layers;
    for (int m = 0; m < n_masks; ++m) {
        int h_index = 0;
        const int rc = masked_layers(ctx, masks + (size_t)m * L, token, pos, st, &h_index);
        if (rc) return rc;
        hipLaunchKernelGGL(cosine_kernel, dim3(1), dim3(1024), 0, st, ctx->h[h_index], target, ctx->cfg.d_model, cos_out + m);
        CLASP_LAUNCH_CHECK();
    }
    return CLASP_OK;
}

}  // extern "C"
