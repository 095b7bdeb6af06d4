// Small kernels around the GEMMs and attention: weight packing, rotary table, embedding gather, cache loading,
// the DP's cosine/select step (Algorithm 1), backtracking, and greedy argmax over the logits.
#pragma once
#include "clasp_common.h"

namespace clasp {

// ---- weight packing: row-major bf16 [N][K] -> fragments (tile of 16 features x 32 inputs = 64 lanes x 8 bf16) ----
// dst fragment index = tile*(K/32) + k/32; lane q*16 + c holds W[feature(tile, c)][(k/32)*32 + q*8 .. +8].
// feature(tile, c) = tile*16 + c, except for rotary matrices (rope_hd > 0: wq, wk), where the features of each head
// are regrouped so that tile u of a head holds features 8u..8u+7 (c < 8) and their rotary partners
// rope_hd/2 + 8u.. (c >= 8): the projection's epilogue can then rotate a pair inside one tile.
__global__ void pack_bf16_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int N, int K, int rope_hd) {
    const size_t total = (size_t)N * K / 8;  // 16-byte vectors
    const int KS = K >> 5;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(v & 63);
        const size_t frag = v >> 6;
        const int s = (int)(frag % KS);
        const size_t tile = frag / KS;
        const int c = lane & 15, q = lane >> 4;
        size_t row = tile * 16 + c;
        if (rope_hd > 0) {
            const int tph = rope_hd >> 4;
            const size_t head = tile / tph;
            const int u = (int)(tile % tph);
            row = head * rope_hd + (c < 8 ? u * 8 + c : (rope_hd >> 1) + u * 8 + (c - 8));
        }
        dst[v] = src[(row * K + (size_t)s * 32 + q * 8) / 8];
    }
}

// gate|up interleave: packed tile t holds gate features 8t..8t+7 (lanes c < 8) and up features 8t..8t+7 (c >= 8), so
// that one weight stream feeds the SwiGLU epilogue and the tile count is 2*F/16 (finer, better balanced work).
__global__ void pack_gate_up_bf16_kernel(const u32x4* __restrict__ gate, const u32x4* __restrict__ up,
                                         u32x4* __restrict__ dst, int F, int K) {
    const size_t total = (size_t)2 * F * K / 8;
    const int KS = K >> 5;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(v & 63);
        const size_t frag = v >> 6;
        const int s = (int)(frag % KS);
        const size_t tile = frag / KS;
        const int c = lane & 15, q = lane >> 4;
        const size_t row = tile * 8 + (c & 7);
        const u32x4* src = (c < 8) ? gate : up;
        dst[v] = src[(row * K + (size_t)s * 32 + q * 8) / 8];
    }
}

// ---- rotary table: (cos, sin)(pos * base^(-2e/hd)) evaluated in double, stored as float2 ------------------------
__global__ void rope_table_kernel(float2* table, int max_seq, int half, double base) {
    const size_t total = (size_t)max_seq * half;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(i % half);
        const double pos = (double)(i / half);
        const double theta = pos * pow(base, -(double)e / (double)half);
        table[i] = make_float2((float)cos(theta), (float)sin(theta));
    }
}

__global__ void fill_zero_kernel(u32x4* p, size_t n_vec) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}

// ---- embedding gather: h_0 of each row, plus everything layer 0 consumes ------------------------------------------
// Grid (rows, ceil(d / 256)): one column per thread, so the token -> table -> store chain is walked once.
template <int DT>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* tokens, const void* table, int vocab, int d,
                                                    float* h, void* op, int R, const float* gain, float* ss,
                                                    float* capture) {
    const int row = blockIdx.x, c = blockIdx.y * 256 + threadIdx.x;  // d % 16 == 0: a 16-column tile is all in or out
    if (c >= d) return;
    int tok = tokens[row];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    float v;
    if constexpr (DT == kDtBf16) v = from_bf16(reinterpret_cast<const bf16*>(table)[(size_t)tok * d + c]);
    else v = reinterpret_cast<const float*>(table)[(size_t)tok * d + c];
    h[(size_t)row * d + c] = v;
    if (capture) capture[(size_t)row * d + c] = v;
    store_operand<DT>(op, R, d, row, c, v * (gain ? gain[c] : 1.0f));
    const float sq = sum16(v * v);
    if ((c & 15) == 0) ss[(size_t)(c >> 4) * kMaxRows + row] = sq;
}

// ---- install cache contents given as fp32 [T][n_kv][hd] -----------------------------------------------------------
template <int DT>
__global__ void kv_load_kernel(const float* K, const float* V, void* Kc, void* Vt, int T, int nkv, int hd, int t_max) {
    const size_t total = (size_t)T * nkv * hd;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(i % hd);
        const int kvh = (int)((i / hd) % nkv);
        const size_t t = i / ((size_t)hd * nkv);
        const size_t ko = ((size_t)kvh * t_max + t) * hd + e, vo = ((size_t)kvh * hd + e) * t_max + t;
        if constexpr (DT == kDtBf16) {
            const size_t head = (size_t)kvh * t_max * hd;
            reinterpret_cast<kv_t*>(Kc)[head + kfrag_offset(hd, (int)t, e)] = to_kv(K[i]);
            reinterpret_cast<kv_t*>(Vt)[head + vfrag_offset(hd, (int)t, e)] = to_kv(V[i]);
        } else {
            reinterpret_cast<float*>(Kc)[ko] = K[i];
            reinterpret_cast<float*>(Vt)[vo] = V[i];
        }
    }
}

// ---- read cache contents back as fp32 [T][n_kv][hd] (positions pos0 .. pos0+T-1) ------------------------------------
template <int DT>
__global__ void kv_read_kernel(const void* Kc, const void* Vt, float* K, float* V, int pos0, int T, int nkv, int hd,
                               int t_max) {
    const size_t total = (size_t)T * nkv * hd;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(i % hd);
        const int kvh = (int)((i / hd) % nkv);
        const size_t t = pos0 + i / ((size_t)hd * nkv);
        if constexpr (DT == kDtBf16) {
            const size_t head = (size_t)kvh * t_max * hd;
            K[i] = from_kv(reinterpret_cast<const kv_t*>(Kc)[head + kfrag_offset(hd, (int)t, e)]);
            V[i] = from_kv(reinterpret_cast<const kv_t*>(Vt)[head + vfrag_offset(hd, (int)t, e)]);
        } else {
            K[i] = reinterpret_cast<const float*>(Kc)[((size_t)kvh * t_max + t) * hd + e];
            V[i] = reinterpret_cast<const float*>(Vt)[((size_t)kvh * hd + e) * t_max + t];
        }
    }
}

// ---- the DP's score / select step for layer index i (Algorithm 1, Eq. 2) -------------------------------------------
// Workgroup j = blockIdx.x handles cell (i, j), j = 0..min(i, M):
//   j = 0          g(i,0) = x_i
//   1 <= j <= ell  (ell = min(i-1, M)): keep the computed candidate G[j-1] = f_{i-1}(g(i-1,j)) if its cosine with x_i
//                  is strictly larger than that of the skip candidate g(i-1,j-1), else the skip candidate
//   j = i <= M     g(i,i) = g(i-1,i-1) (all layers so far skipped)
// and emits g(i,j), j >= 1, as row j-1 of the next layer's input (fp32 + GEMM operand + sums of squares).
struct SelectArgs {
    int i, M, d, R;
    const float* x_i;     // [d]
    const float* g_prev;  // g(i-1, .) rows, [M+1][d]
    const float* G;       // computed candidates, row j-1 for cell j, [ell][d]; or, when n_parts > 0, the residual
                          // rows to which the n_parts K-slices of the down projection still have to be added
    const float* parts;   // [n_parts][part_stride] partial sums of the down projection, rows of length d
    int n_parts;
    size_t part_stride;
    float* g_cur;         // g(i, .) rows, [M+1][d]
    void* op;             // next layer's operand (null when i == L)
    const float* gain;    // next layer's attention-norm gains
    float* ss;
    float* scores;    // [(L+1)][(M+1)][2] or null
    uint8_t* choice;  // [(L+1)][(M+1)]
    // cells of this launch: j = j0 + blockIdx.x. Row 0 of G belongs to cell jc0 (>= 1), row 0 of the next layer's operand
    // to cell jn0 (>= 1; cells below it feed nothing). The full table has j0 = 0, jc0 = jn0 = 1; a search that only
    // needs the skip set leaves out the cells from which (L, M) cannot be reached.
    int j0, jc0, jn0;
};

// One workgroup of 1024 threads per cell; a thread owns the 4-column chunks threadIdx.x, threadIdx.x + 1024, ...
// Everything a thread reads - x_i, the skip candidate, the computed candidate with its K-slices, the next layer's
// gains - is requested before the first value is used (NP, the number of K-slices, is a compile-time constant for that
// reason: a loop over a run-time count waits for every slice before it asks for the next), so a cell costs one trip to
// memory, the block reduction of the five dot products, and the stores. The first kSelectKeep chunks of a thread stay
// in registers (d <= 8192); chunks beyond them are read again after the decision.
#ifndef CLASP_SELECT_KEEP
#define CLASP_SELECT_KEEP 2
#endif
constexpr int kSelectKeep = CLASP_SELECT_KEEP;

template <int DT, bool HAS_COMP, int NP>
__device__ __forceinline__ void select_cell(const SelectArgs& a, int j, float (*red)[5]) {
    const int d = a.d, nc = d / 4, tid = threadIdx.x;
    float* dst = a.g_cur + (size_t)j * d;
    const f32x4* x4 = reinterpret_cast<const f32x4*>(a.x_i);
    const f32x4* skip4 = reinterpret_cast<const f32x4*>(a.g_prev + (size_t)(j - 1) * d);
    // the computed candidate: a finished row, or residual + K-slices of the down projection added in slice order
    const f32x4* comp4 = reinterpret_cast<const f32x4*>(a.G + (size_t)(j - a.jc0) * d);
    const f32x4* part4 = reinterpret_cast<const f32x4*>(a.parts + (size_t)(j - a.jc0) * d);
    const size_t ps4 = a.part_stride / 4;
    const bool feeds = a.op && j >= a.jn0;  // this cell is row j - jn0 of the next layer's input
    const f32x4* gain4 = feeds ? reinterpret_cast<const f32x4*>(a.gain) : nullptr;
    const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f}, ones = f32x4{1.f, 1.f, 1.f, 1.f};
    auto load_comp = [&](int c) -> f32x4 {
        f32x4 v = comp4[c];
        if constexpr (NP >= 0) {
            f32x4 p[NP > 0 ? NP : 1];
#pragma unroll
            for (int k = 0; k < NP; ++k) p[k] = part4[k * ps4 + c];
#pragma unroll
            for (int k = 0; k < NP; ++k) v += p[k];
        } else {
            for (int k = 0; k < a.n_parts; ++k) v += part4[k * ps4 + c];
        }
        return v;
    };
    float acc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};  // x.x, s.x, s.s, c.x, c.c
    auto dots = [&](const f32x4& x, const f32x4& s, const f32x4& g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[0] = fmaf(x[e], x[e], acc[0]);
            acc[1] = fmaf(s[e], x[e], acc[1]);
            acc[2] = fmaf(s[e], s[e], acc[2]);
            acc[3] = fmaf(g[e], x[e], acc[3]);
            acc[4] = fmaf(g[e], g[e], acc[4]);
        }
    };
    f32x4 s_keep[kSelectKeep], g_keep[kSelectKeep], gn_keep[kSelectKeep];
#pragma unroll
    for (int u = 0; u < kSelectKeep; ++u) {
        const int c = tid + u * 1024;
        const bool live = c < nc;
        const int cc = live ? c : 0;  // a thread without a chunk reads chunk 0 and adds zeros
        f32x4 x = x4[cc], s = skip4[cc], g = zero;
        if constexpr (HAS_COMP) g = load_comp(cc);
        gn_keep[u] = gain4 ? gain4[cc] : ones;
        if (!live) x = s = g = zero;
        s_keep[u] = s;
        g_keep[u] = g;
        dots(x, s, g);
    }
    for (int c = tid + kSelectKeep * 1024; c < nc; c += 1024) {
        f32x4 g = zero;
        if constexpr (HAS_COMP) g = load_comp(c);
        dots(x4[c], skip4[c], g);
    }
    const int wave = tid >> 6, nw = blockDim.x >> 6;
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        acc[k] = wave_sum(acc[k]);
        if ((tid & 63) == 0) red[wave][k] = acc[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        float t = 0.f;
        for (int w = 0; w < nw; ++w) t += red[w][k];
        acc[k] = t;
    }
    const float nx = fmaxf(sqrtf(acc[0]), 1e-12f);
    const float sig_s = acc[1] / (fmaxf(sqrtf(acc[2]), 1e-12f) * nx);
    const float sig_c = HAS_COMP ? acc[3] / (fmaxf(sqrtf(acc[4]), 1e-12f) * nx) : __builtin_nanf("");
    const bool keep_comp = HAS_COMP && (sig_c > sig_s);
    if (tid == 0) {
        const size_t cell = (size_t)a.i * (a.M + 1) + j;
        a.choice[cell] = keep_comp ? 0 : 1;
        if (a.scores) {
            a.scores[cell * 2] = sig_c;
            a.scores[cell * 2 + 1] = sig_s;
        }
    }
    auto emit = [&](int c, const f32x4& v, const f32x4& gn) {
        reinterpret_cast<f32x4*>(dst)[c] = v;
        if (feeds) {
            store_operand4<DT>(a.op, a.R, d, j - a.jn0, c * 4, v * gn);
            float sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];  // 4 lanes cover one 16-column tile
            sq += __shfl_xor(sq, 1);
            sq += __shfl_xor(sq, 2);
            if ((c & 3) == 0) a.ss[(size_t)(c >> 2) * kMaxRows + (j - a.jn0)] = sq;
        }
    };
#pragma unroll
    for (int u = 0; u < kSelectKeep; ++u) {
        const int c = tid + u * 1024;
        if (c < nc) emit(c, keep_comp ? g_keep[u] : s_keep[u], gn_keep[u]);
    }
    for (int c = tid + kSelectKeep * 1024; c < nc; c += 1024) {
        f32x4 v = skip4[c];
        if constexpr (HAS_COMP) {
            if (keep_comp) v = load_comp(c);
        }
        emit(c, v, gain4 ? gain4[c] : ones);
    }
}

template <int DT>
__global__ __launch_bounds__(1024) void dp_select_kernel(SelectArgs a) {
    __shared__ float red[16][5];
    const int j = a.j0 + blockIdx.x, d = a.d;
    if (j == 0) {
        float* dst = a.g_cur;
        const f32x4* x4 = reinterpret_cast<const f32x4*>(a.x_i);
        for (int c = threadIdx.x; c < d / 4; c += blockDim.x) reinterpret_cast<f32x4*>(dst)[c] = x4[c];
        return;
    }
    const bool has_comp = j <= min(a.i - 1, a.M);  // cells of a launch never lie below jc0
    if (!has_comp) select_cell<DT, false, 0>(a, j, red);
    else if (a.n_parts == 0) select_cell<DT, true, 0>(a, j, red);
    else if (a.n_parts == 4) select_cell<DT, true, 4>(a, j, red);
    else select_cell<DT, true, -1>(a, j, red);
}

__global__ void dp_table_init_kernel(float* scores, uint8_t* choice, int cells) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < cells; c += gridDim.x * blockDim.x) {
        choice[c] = 255;
        if (scores) {
            scores[2 * c] = __builtin_nanf("");
            scores[2 * c + 1] = __builtin_nanf("");
        }
    }
}

// Backtracking from (L, M): a kept skip candidate at (i, j) means layer i-1 is skipped.
// The tables cover the L layers of the searched window, which starts at layer `lo` of the model's L_all layers; the
// mask covers all of them (layers outside the window are never skipped).
__global__ void dp_backtrack_kernel(const uint8_t* choice, int L, int M, uint8_t* mask, int lo, int L_all,
                                    const float* g_last, float* g_final, int d) {
    if (blockIdx.x == 0) {
        for (int l = threadIdx.x; l < L_all; l += blockDim.x) mask[l] = 0;
        __syncthreads();
        if (threadIdx.x == 0) {
            int i = L, j = M;
            while (i > 0 && j > 0) {
                if (choice[(size_t)i * (M + 1) + j] == 1) {
                    mask[lo + i - 1] = 1;
                    --j;
                }
                --i;
            }
        }
    } else if (g_final) {
        for (int c = threadIdx.x; c < d; c += blockDim.x) g_final[c] = g_last[(size_t)M * d + c];
    }
}

// ---- cosine of two vectors (the DP's objective, Eq. 1, for a given skip set) ------------------------------------------
// out[0] = <a, b> / (max(|a|, 1e-12) max(|b|, 1e-12)), fixed-order sums. One workgroup.
__global__ __launch_bounds__(1024) void cosine_kernel(const float* a, const float* b, int d, float* out) {
    __shared__ float red[16];
    float ab = 0.f, aa = 0.f, bb = 0.f;
    for (int c = threadIdx.x; c < d; c += 1024) {
        const float x = a[c], y = b[c];
        ab += x * y;
        aa += x * x;
        bb += y * y;
    }
    ab = block_sum(ab, red);
    aa = block_sum(aa, red);
    bb = block_sum(bb, red);
    if (threadIdx.x == 0) out[0] = ab / (fmaxf(sqrtf(aa), 1e-12f) * fmaxf(sqrtf(bb), 1e-12f));
}

// ---- greedy head ----------------------------------------------------------------------------------------------
// bf16 path: merges the per-tile pieces the lm_head epilogue left behind ([32][tiles] x (max, index, second max, sum of
// exp(logit - max))) into argmax (lowest index on ties), top-1 minus top-2 logit and the softmax probability of the
// top-1. One workgroup per row.
__global__ __launch_bounds__(1024) void head_reduce_kernel(const f32x4* parts, int n_tiles, int32_t* argmax_out,
                                                           float* margin_out, float* prob_out) {
    __shared__ float s_v1[16], s_v2[16], s_se[16];
    __shared__ int s_i1[16];
    const int row = blockIdx.x;
    float v1 = -INFINITY, v2 = -INFINITY, se = 0.f;
    int i1 = 0x7fffffff;
    auto merge = [](float& a1, int& ai, float& a2, float& ase, float b1, int bi, float b2, float bse) {
        const float m = fmaxf(a1, b1);
        const float fa = (a1 == -INFINITY) ? 0.f : expf(a1 - m), fb = (b1 == -INFINITY) ? 0.f : expf(b1 - m);
        ase = ase * fa + bse * fb;
        if (b1 > a1 || (b1 == a1 && bi < ai)) {
            a2 = fmaxf(a1, b2);
            a1 = b1;
            ai = bi;
        } else {
            a2 = fmaxf(a2, b1);
        }
    };
    // eight pieces per thread requested together (a vocabulary of 128k has 8016 tiles: one trip to memory instead of
    // eight), merged in the order of the tile index as before
    constexpr int kU = 8;
    for (int t0 = threadIdx.x; t0 < n_tiles; t0 += blockDim.x * kU) {
        f32x4 p[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int t = t0 + u * blockDim.x;
            p[u] = parts[(size_t)row * n_tiles + min(t, n_tiles - 1)];
        }
#pragma unroll
        for (int u = 0; u < kU; ++u)
            if (t0 + u * (int)blockDim.x < n_tiles) merge(v1, i1, v2, se, p[u][0], __float_as_int(p[u][1]), p[u][2], p[u][3]);
    }
    for (int o = 1; o < 64; o <<= 1) {
        const float b1 = __shfl_xor(v1, o), b2 = __shfl_xor(v2, o), bs = __shfl_xor(se, o);
        const int bi = __shfl_xor(i1, o);
        merge(v1, i1, v2, se, b1, bi, b2, bs);
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_v1[wave] = v1; s_v2[wave] = v2; s_i1[wave] = i1; s_se[wave] = se; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < nw; ++w) merge(v1, i1, v2, se, s_v1[w], s_i1[w], s_v2[w], s_se[w]);
        if (argmax_out) argmax_out[row] = i1;
        if (margin_out) margin_out[row] = v1 - v2;
        if (prob_out) prob_out[row] = 1.0f / se;
    }
}

// fp32 path: the same three results straight from the logits.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* logits, int vocab, int32_t* argmax_out,
                                                      float* margin_out, float* prob_out) {
    __shared__ float s_v1[16], s_v2[16], s_sum[16];
    __shared__ int s_i1[16];
    const float* lg = logits + (size_t)blockIdx.x * vocab;
    float v1 = -INFINITY, v2 = -INFINITY;
    int i1 = 0x7fffffff;
    for (int c = threadIdx.x; c < vocab; c += blockDim.x) {
        const float v = lg[c];
        if (v > v1) { v2 = v1; v1 = v; i1 = c; }
        else if (v > v2) v2 = v;
    }
    auto merge = [](float& a1, int& ai, float& a2, float b1, int bi, float b2) {
        if (b1 > a1 || (b1 == a1 && bi < ai)) {
            a2 = fmaxf(a1, b2);
            a1 = b1;
            ai = bi;
        } else {
            a2 = fmaxf(a2, b1);
        }
    };
    for (int o = 1; o < 64; o <<= 1) {
        const float b1 = __shfl_xor(v1, o), b2 = __shfl_xor(v2, o);
        const int bi = __shfl_xor(i1, o);
        merge(v1, i1, v2, b1, bi, b2);
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_v1[wave] = v1; s_v2[wave] = v2; s_i1[wave] = i1; }
    __syncthreads();
    v1 = s_v1[0]; v2 = s_v2[0]; i1 = s_i1[0];
    for (int w = 1; w < nw; ++w) merge(v1, i1, v2, s_v1[w], s_i1[w], s_v2[w]);
    float sum = 0.f;
    if (prob_out) {
        for (int c = threadIdx.x; c < vocab; c += blockDim.x) sum += expf(lg[c] - v1);
        sum = wave_sum(sum);
        if ((threadIdx.x & 63) == 0) s_sum[wave] = sum;
        __syncthreads();
        sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += s_sum[w];
    }
    if (threadIdx.x == 0) {
        if (argmax_out) argmax_out[blockIdx.x] = i1;
        if (margin_out) margin_out[blockIdx.x] = v1 - v2;
        if (prob_out) prob_out[blockIdx.x] = 1.0f / sum;
    }
}

}  // namespace clasp
