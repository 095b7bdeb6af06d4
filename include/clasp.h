/*
 * clasp.h -- C ABI of the MI355X (gfx950) CLaSp hot path: self-speculative decoding with an in-context
 * layer-skip search (dynamic program over (layer, skip count)), the layer-skipped draft forward and the full
 * verify forward that feeds it.
 *
 * General rules
 *   - Plain C types only. "dev" pointers are device (HBM) addresses owned by the caller (e.g. PyTorch tensors);
 *     "host" pointers are ordinary host memory. The library borrows every pointer for the duration of the call;
 *     weights, workspace and KV caches are borrowed for the lifetime of the context.
 *   - After clasp_create the library allocates no device memory: everything lives in the caller's workspace.
 *   - Every call is asynchronous on the given HIP stream (a hipStream_t passed as void*, NULL = default
 *     stream); the caller synchronises. Calls on one context must not overlap, and calls into the library from
 *     several host threads must be serialised by the caller (launch set-up keeps process-wide state).
 *   - Every function returns CLASP_OK (0) or a negative CLASP_E_* code; nothing aborts or throws.
 *   - One GPU, the current HIP device at clasp_create time.
 *
 * Model: pre-norm LLaMA decoder (RMSNorm, q/k/v projections, rotary embedding with half-split pairing, grouped
 * query attention over a KV cache, output projection, SwiGLU MLP, untied lm_head), the model family the paper
 * evaluates (Experiments, "Model and Testbed"). h_{l+1} = f_l(h_l) as in Sec. 3.4.
 *
 * Data layouts
 *   - dtype CLASP_BF16: matrices are bf16 in the packed tile order written by clasp_pack_matrix; activations,
 *     residual stream, hidden states, scores and logits are fp32. The projections multiply bf16 weights by activations
 *     split into two bf16 numbers (hi + lo, 16 significant bits), accumulating in fp32. Attention runs on fp16
 *     matrix instructions: queries, cached keys / values and softmax weights are fp16 (2 bytes per element like bf16,
 *     11 significant bits instead of 8; the paper's own runs are FP16, Experiments), accumulation is fp32. Conversions
 *     to fp16 saturate: a key, value or scaled query beyond +-65504 is stored as +-65504, never as an infinity.
 *   - dtype CLASP_F32: matrices are fp32 row-major [out_features][in_features] (clasp_pack_matrix is a copy);
 *     everything is fp32.
 *   - embed is always row-major [vocab][d_model] in the model dtype. RMSNorm gains are fp32 [d_model], 16-byte
 *     aligned like every other device pointer handed to the library.
 *   - KV cache, per K and per V: clasp_kv_cache_bytes() bytes, [layer][kv_head] major, 4 bytes per element for fp32
 *     models and 2 (fp16) for bf16 models; inside a head the order is the library's own (fp32: K [max_seq][head_dim],
 *     V [head_dim][max_seq]; bf16 models: blocks of 32 positions in MFMA operand order), so contents from elsewhere go
 *     in through clasp_kv_load. Keys are stored
 *     after rotation. Validity is the caller's length counter: the library reads positions below the `pos` it is
 *     given and never beyond. clasp_create zero-fills both caches.
 */
#ifndef CLASP_H
#define CLASP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct clasp_ctx clasp_ctx;

enum { CLASP_F32 = 0, CLASP_BF16 = 1 };

enum {
    CLASP_OK = 0,
    CLASP_E_INVALID_ARG = -1, /* NULL required pointer, size or index out of range                     */
    CLASP_E_UNSUPPORTED = -2, /* shape outside what the kernels are built for (see clasp_create)         */
    CLASP_E_HIP = -3,         /* a HIP runtime call or kernel launch failed                              */
    CLASP_E_WORKSPACE = -4    /* workspace smaller than clasp_workspace_bytes()                          */
};

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_seq;  /* KV cache capacity in tokens, multiple of 32                                      */
    int32_t max_rows; /* most rows one launch carries (verify rows, or skip budget M), 1..32              */
    int32_t dtype;    /* CLASP_F32 or CLASP_BF16                                                         */
    float rms_eps, rope_base;
} clasp_config;

/* All pointers are dev pointers; the per-layer members are HOST arrays of n_layers dev pointers. */
typedef struct {
    const void *embed;      /* [vocab][d_model] row-major, model dtype                                    */
    const void *lm_head;    /* [vocab][d_model], packed                                                   */
    const float *final_norm;
    const float *const *attn_norm; /* gains of the norm in front of attention                             */
    const float *const *mlp_norm;  /* gains of the norm in front of the MLP                               */
    const void *const *wq;     /* [n_heads*head_dim][d_model], packed                                     */
    const void *const *wk;     /* [n_kv_heads*head_dim][d_model], packed                                  */
    const void *const *wv;     /* [n_kv_heads*head_dim][d_model], packed                                  */
    const void *const *wo;     /* [d_model][n_heads*head_dim], packed                                     */
    const void *const *w_gate_up; /* gate and up projections, [2*d_ffn][d_model], from clasp_pack_gate_up          */
    const void *const *w_down; /* [d_model][d_ffn], packed                                                */
} clasp_weights;

/* Bytes of a packed [rows][cols] matrix (equals rows*cols*elem size; rows % 16 == 0 and, for bf16,
 * cols % 32 == 0 are required, 0 is returned otherwise). */
size_t clasp_packed_bytes(int rows, int cols, int dtype);

/* Re-orders a row-major [rows][cols] dev matrix `src` into the library's streaming order in `dst` (dev, distinct
 * from src, clasp_packed_bytes() bytes). bf16: tiles of 16 output features x 32 inputs, each tile stored so that
 * one 64-lane wavefront reads it with a single coalesced 16-byte-per-lane load in MFMA operand order; tiles of
 * one 16-feature group are contiguous along the input dimension. fp32: plain copy.
 * rope_head_dim: 0 for every matrix except wq and wk, which take the model's head_dim: their output features are
 * regrouped per head so that a rotary pair (e, e + head_dim/2) falls into one tile (ignored for fp32). */
int clasp_pack_matrix(const void *src, void *dst, int rows, int cols, int dtype, int rope_head_dim, void *stream);

/* Packs the row-major dev matrices gate and up ([d_ffn][d_model] each) into ONE matrix dst of 2 * clasp_packed_bytes(
 * d_ffn, d_model, dtype) bytes. bf16: the two projections are interleaved, 8 gate features and the 8 matching up
 * features per 16-feature tile, so that one weight stream feeds the fused SwiGLU; fp32: gate rows, then up rows. */
int clasp_pack_gate_up(const void *gate, const void *up, void *dst, int d_ffn, int d_model, int dtype, void *stream);

/* Device bytes clasp_create needs in `workspace` (256-byte aligned), and bytes of ONE of the two KV caches. */
size_t clasp_workspace_bytes(const clasp_config *cfg);
size_t clasp_kv_cache_bytes(const clasp_config *cfg);

/* Builds a context. Requirements, else CLASP_E_UNSUPPORTED: n_heads % n_kv_heads == 0; d_model, d_ffn,
 * n_heads*head_dim multiples of 32 (bf16) or 16 (fp32); vocab % 16 == 0; head_dim 64 or 128 (bf16), even (fp32);
 * 1 <= max_rows <= 32; max_seq % 32 == 0. Zero-fills the KV caches and builds the rotary table (synchronous). */
int clasp_create(const clasp_config *cfg, const clasp_weights *weights, void *workspace, size_t workspace_bytes,
                 void *k_cache, void *v_cache, clasp_ctx **out);
int clasp_destroy(clasp_ctx *ctx);

/*
 * Verification (Sec. 3.1 stage 2; Sec. 3.4: the verify pass's per-layer hidden states are the DP's objective):
 * the full model over n_tokens rows at positions pos0..pos0+n_tokens-1, causal among themselves, attending cache
 * positions 0..pos0-1. Writes the rows' keys/values into every layer's cache at their positions.
 *   tokens      dev int32 [n_tokens]; ids outside [0, vocab) are clamped
 *   n_tokens    1..max_rows;  pos0 >= 0, pos0 + n_tokens <= max_seq
 *   hidden_out  dev fp32 [n_layers+1][n_tokens][d_model] or NULL: state l = input of layer l, state n_layers =
 *               output of the last layer before the final norm
 *   argmax_out  dev int32 [n_tokens] or NULL: greedy next token per row (lowest index on ties)
 *   margin_out  dev fp32 [n_tokens] or NULL: top-1 minus top-2 logit
 *   logits_out  dev fp32 [n_tokens][vocab] or NULL
 * Plain greedy decoding of one token is this call with n_tokens = 1; prefill is this call in chunks.
 */
int clasp_verify_forward(clasp_ctx *ctx, const int32_t *tokens, int n_tokens, int pos0, float *hidden_out,
                         int32_t *argmax_out, float *margin_out, float *logits_out, void *stream);

/*
 * Prompt processing with many rows per pass (the full-model forward of Sec. 3.1 over the prompt, whose lasting
 * product is the KV cache that verification, layer optimisation (Sec. 3.4) and drafting read): the full model over
 * n_tokens rows at positions pos0..pos0+n_tokens-1, causal among themselves, attending cache positions 0..pos0-1,
 * in passes of chunk_rows rows through compute-bound MFMA GEMMs and causal flash attention. Writes the rows'
 * keys/values into every layer's cache and nothing else; the states and the next token of the prompt's last token
 * come from clasp_verify_forward on that token (or on the last few) afterwards. bf16 models only
 * (CLASP_E_UNSUPPORTED otherwise). Passes of fewer than 640 rows compute as clasp_verify_forward does (bf16 weights,
 * hi + lo bf16 activation operands, fp32 accumulation) and leave the same cache up to rounding order. Passes of 640
 * rows or more (chunk_rows >= 640 and that many rows left) run their projections on fp16 matrix instructions: each
 * activation is rounded to one fp16 number (11 significant bits instead of the pair's 16; values beyond +-65504, which
 * an un-normalised hidden state times its gain or a SwiGLU product of a trained model may in principle reach, saturate
 * there instead of becoming infinities), the layer's weights are converted to fp16 into the workspace at the start of
 * the layer (exact for every bf16 weight of magnitude >= 2^-17, rounding to multiples of 2^-24 below), accumulation
 * stays fp32, attention is the same fp16 kernel family as elsewhere. That halves the matrix-core work of a pass; the
 * cache stays inside the 2e-2 of the fp64 reference that every result of a bf16 model is held to.
 *   tokens       dev int32 [n_tokens]; ids outside [0, vocab) are clamped
 *   n_tokens     >= 1;  pos0 >= 0, pos0 + n_tokens <= max_seq
 *   chunk_rows   rows per pass: a multiple of 128 in 128..8192 (larger = fewer passes over the weights: from 4096 on
 *                every projection of an 8B-shaped model fills the chip with 256 x 256 tiles, and 8192 is a few per cent
 *                faster still on prompts that long)
 *   workspace    dev, 256-byte aligned, >= clasp_prefill_workspace_bytes(cfg, chunk_rows) bytes, caller-owned, only
 *                used during the call (on `stream`); for chunk_rows >= 640 it includes room for one layer's weights
 * clasp_prefill_workspace_bytes returns 0 for an unsupported configuration or chunk_rows.
 */
size_t clasp_prefill_workspace_bytes(const clasp_config *cfg, int chunk_rows);
int clasp_prefill(clasp_ctx *ctx, const int32_t *tokens, int n_tokens, int pos0, int chunk_rows, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * clasp_prefill for callers that cannot allocate device memory and hold no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same passes, same kernels and the same cache contents
 * as clasp_prefill with this chunk_rows, but the pass's working buffers live in a static device array inside the
 * library (clasp_static_scratch_bytes() = 32 MiB per GPU that loads the library, held until the process ends) whose
 * address on the context's GPU clasp_create looked up. The call allocates and frees nothing.
 *   CLASP_E_WORKSPACE   clasp_prefill_workspace_bytes(cfg, chunk_rows) exceeds the array (8B-shaped models fit with
 *                       chunk_rows = 128; wider models or longer passes need clasp_prefill with a caller workspace)
 *   CLASP_E_INVALID_ARG also when the current HIP device is not the one the context was created on
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two contexts, two threads)
 * race, and must be serialised by the caller. Nothing in the array has to start at zero, and nothing is carried from
 * one call to the next.
 */
int clasp_prefill_static(clasp_ctx *ctx, const int32_t *tokens, int n_tokens, int pos0, int chunk_rows, void *stream);
size_t clasp_static_scratch_bytes(void);

/*
 * Layer optimisation (Sec. 3.4, Eq. 2, Algorithm 1; batching of the candidates of one layer: Sec. 3.6).
 * For the token at position `pos` with stored verify states x_0..x_L, runs the dynamic program
 *   D(i,j) = max{ cos(x_i, g(i-1,j-1)), cos(x_i, f_{i-1}(g(i-1,j))) },  i = 1..L, j = 1..min(i, M)
 * keeping the skip candidate on ties, and backtracks from (L, M) to the skip set. All candidates of one layer go
 * through f_{i-1} in one batched pass that reads the layer's weights and the shared KV prefix once; each candidate
 * attends cache positions 0..pos-1 plus its own key/value and no other candidate. Writes no KV.
 *   states       dev fp32, 16-byte aligned, state l at states + l*layer_stride (elements, multiple of 4),
 *                l = 0..n_layers;  0 <= pos < max_seq
 *   M            skip budget, 0 <= M <= min(n_layers, max_rows)
 *   mask_out     dev uint8 [n_layers]: 1 = layer skipped; exactly M ones
 *   score_out    dev fp32 [(n_layers+1)][(M+1)][2] or NULL: (cosine of the computed candidate, cosine of the skip
 *                candidate) per cell, NaN where a candidate does not exist
 *   choice_out   dev uint8 [(n_layers+1)][(M+1)] or NULL: 0 computed kept, 1 skip kept, 255 no such cell
 *   g_final_out  dev fp32 [d_model] or NULL: g(L, M)
 * Without score_out and choice_out the cells from which (L, M) cannot be reached (j < M - (L - i)) are left out: they
 * decide nothing, and the last M levels then push fewer candidates through their layer. g_final_out is the same up to
 * fp32 rounding order (launches with fewer rows may take kernels that slice the contraction differently), mask_out is
 * the same unless a comparison is tied within that rounding.
 */
int clasp_dp_select(clasp_ctx *ctx, const float *states, size_t layer_stride, int pos, int M, uint8_t *mask_out,
                    float *score_out, uint8_t *choice_out, float *g_final_out, void *stream);

/*
 * The same search restricted to the layers layer_lo .. layer_hi-1 (Sec. 3.5 fixes the first and last layers of the
 * model and searches the ones between): layers outside the window are always kept, the dynamic program starts from
 * state layer_lo and matches states layer_lo+1 .. layer_hi; M <= layer_hi - layer_lo. mask_out covers all n_layers;
 * score_out / choice_out are [(layer_hi-layer_lo+1)][(M+1)]([2]) tables indexed from the window's first layer.
 * clasp_dp_select is this call with the window 0 .. n_layers.
 */
int clasp_dp_select_window(clasp_ctx *ctx, const float *states, size_t layer_stride, int pos, int M, int layer_lo,
                           int layer_hi, uint8_t *mask_out, float *score_out, uint8_t *choice_out, float *g_final_out,
                           void *stream);

/*
 * The objective of Eq. 1 for given skip sets (what Sec. 3.5 compares between brute-force search, random choice and
 * the dynamic program): for each of n_masks masks, the token goes through the layers the mask keeps at position
 * `pos` (as in clasp_draft_step, including the write of its key/value at `pos` in the kept layers), and the cosine
 * of the resulting last hidden state (before the final norm) with `target` is stored.
 *   masks    host uint8 [n_masks][n_layers], 1 = skip;  token dev int32 [1];  target dev fp32 [d_model]
 *   cos_out  dev fp32 [n_masks]: <h, target> / (max(|h|, 1e-12) max(|target|, 1e-12))
 */
int clasp_skip_cosine(clasp_ctx *ctx, const uint8_t *masks, int n_masks, const int32_t *token, int pos,
                      const float *target, float *cos_out, void *stream);

/*
 * Drafting (Sec. 3.1 stage 1, Sec. 3.3): one token through the layers the skip set keeps, at position `pos`,
 * attending cache positions 0..pos-1; writes the token's key/value at `pos` into the kept layers' caches only.
 *   mask           host uint8 [n_layers], 1 = skip (NULL = keep all)
 *   token          dev int32 [1]
 *   next_token_out dev int32 [1]: greedy next token;  top1_prob_out dev fp32 [1] or NULL: its softmax probability
 */
int clasp_draft_step(clasp_ctx *ctx, const uint8_t *mask, const int32_t *token, int pos, int32_t *next_token_out,
                     float *top1_prob_out, void *stream);

/*
 * Stochastic decoding (the Temperature = 1 setting of Sec. 4; the method stays speculative sampling, Sec. 4.1, so
 * the output is distributed exactly as the full model's). Every random draw takes a uniform number in [0, 1) from
 * the caller (dev fp32), so a run is reproducible from its inputs. temperature > 0 divides the logits.
 *
 * clasp_sample_token: token_out[0] ~ softmax(logits / temperature), by inverting the cumulative distribution in
 *   index order with u[0].  logits dev fp32 [vocab].
 * clasp_draft_sample: clasp_draft_step, but the next token is drawn from the draft model's distribution with u[0]
 *   and the draft model's logits are kept for the acceptance test.  logits_out dev fp32 [vocab] (required).
 * clasp_spec_accept: one round's acceptance. tokens dev int32 [n_draft+1] = pending token, drafts; p_logits dev fp32
 *   rows 0..n_draft (full model, clasp_verify_forward's logits_out over the same rows), q_logits rows 0..n_draft-1
 *   (clasp_draft_sample's), both with `ld` elements between rows (ld >= vocab). Draft i (token after row i) is kept
 *   when u_accept[i] * q_i(x) < p_i(x); at the first rejection a the replacement is drawn from max(0, p_a - q_a)
 *   renormalised, and when all are kept the bonus token is drawn from p_n; both draws use u_final[0].
 *   n_accepted_out, next_token_out dev int32 [1].  1 <= n_draft <= max_rows - 1.
 */
int clasp_sample_token(clasp_ctx *ctx, const float *logits, float temperature, const float *u, int32_t *token_out,
                       void *stream);
int clasp_draft_sample(clasp_ctx *ctx, const uint8_t *mask, const int32_t *token, int pos, float temperature,
                       const float *u, float *logits_out, int32_t *next_token_out, void *stream);
int clasp_spec_accept(clasp_ctx *ctx, const float *p_logits, const float *q_logits, size_t ld, const int32_t *tokens,
                      int n_draft, float temperature, const float *u_accept, const float *u_final,
                      int32_t *n_accepted_out, int32_t *next_token_out, void *stream);

/* Installs cache contents for one layer: K, V dev fp32 [n_tokens][n_kv_heads][head_dim] (keys already rotated) are
 * converted to the cache's element type (fp32, or saturating fp16 for bf16 models) and layout at positions 0..n_tokens-1. For callers that hold a cache from elsewhere
 * (and for tests that feed synthetic cache contents). */
int clasp_kv_load(clasp_ctx *ctx, int layer, const float *K, const float *V, int n_tokens, void *stream);

/* The inverse: cache positions pos0..pos0+n_tokens-1 of one layer as dev fp32 [n_tokens][n_kv_heads][head_dim]
 * (keys as stored, i.e. rotated; values of the cache dtype widened exactly). For callers that move a cache elsewhere
 * and for tests that compare cache contents. */
int clasp_kv_read(clasp_ctx *ctx, int layer, int pos0, int n_tokens, float *K, float *V, void *stream);

/* Measurement aid: between begin and end, every `every`-th launch of the chosen kernel kind inside the calls above
 * gets a pair of HIP events (up to `capacity` launches; host-side event objects only). The GEMM kinds attach the pair
 * to the launch itself, so it holds the kernel's own begin and end time stamps; attention (which may be two launches)
 * is bracketed by two recorded events, which adds a few microseconds. clasp_kernel_timer_end waits for the events and
 * returns the summed elapsed time and the number of launches timed. */
enum {
    CLASP_KERNEL_QKV = 0,      /* RMSNorm-scaled q/k/v projection                      */
    CLASP_KERNEL_ATTENTION = 1,
    CLASP_KERNEL_O_PROJ = 2,   /* output projection + residual                         */
    CLASP_KERNEL_GATE_UP = 3,  /* gate and up projections + SwiGLU (the largest kernel) */
    CLASP_KERNEL_DOWN = 4,     /* down projection + residual                           */
    CLASP_KERNEL_LM_HEAD = 5,
    CLASP_KERNEL_KINDS = 6
};
int clasp_kernel_timer_begin(clasp_ctx *ctx, int kind, int capacity, int every);
int clasp_kernel_timer_end(clasp_ctx *ctx, float *total_ms, int *launches);

const char *clasp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CLASP_H */
