// Skinny GEMMs of the decoder layer: Y[rows <= 32][N] = X[rows][K] . W[N][K]^T with the weights streamed from HBM
// exactly once per launch for all rows (Sec. 3.6 of the paper batches the DP's candidate states of one layer into
// one pass for this reason). The contraction is HBM-bound (arithmetic intensity = rows flop/byte), so the kernels
// are organised around keeping 16-byte-per-lane weight loads in flight; MFMA does the arithmetic because the
// vector ALUs could not keep up with 16..32 rows at 8 TB/s.
//
// bf16 kernel: a wavefront streams a k-slice of one tile of 16 output features (contiguous in the packed weight
// order) with a register double buffer of P fragments; the activation fragments (hi and lo planes) come from L2/L1
// in the same order. Partial tiles are reduced in a fixed order (deterministic, independent of the number of rows)
// through LDS and, when K is also split across workgroups, through a scratch buffer; then the epilogue runs.
//
// Epilogues (they produce what the NEXT kernel consumes, so that no separate norm / rotary / activation kernels
// exist):
//   kEpiScale   out = acc * rstd(row)                       (lm_head; fp32 path q/k/v; RMSNorm's 1/rms factor
//                                                            commutes with the contraction, its gains are already
//                                                            folded into the activation fragments)
//   kEpiResid   out = resid + acc; optionally a copy (hidden-state capture), the next GEMM's operand
//               (out * gain, in operand layout) and per-tile partial sums of out^2 for the next 1/rms
//   kEpiSwiglu  gate and up projections interleaved in one packed matrix (8 gate + 8 up features per tile):
//               operand of the down projection = silu(g*rstd) * (u*rstd)
//   kEpiPartial raw partial sums of this workgroup's K slice, out[blockIdx.y][row][col]: K is split over gridDim.y
//               workgroups and the consumer (the DP's select kernel, which reads whole rows anyway) adds the slices
//               in a fixed order together with the residual; there is no cross-workgroup traffic inside the kernel
//   kEpiHead    lm_head: logits = acc * rstd (stored only if asked for) and, per tile and row, the running pieces of
//               the greedy head: largest logit, its index, second largest, sum of exp(logit - largest); a small
//               kernel merges the tiles' pieces
//   kEpiQkv     q/k/v projection for the MFMA attention kernel: scales by rstd, applies the rotary embedding to q
//               and k (the packed wq/wk put the two halves of a rotary pair into one 16-feature tile), and writes
//               q as ready-made MFMA fragments, k and v into the KV cache (verify/draft rows) or into the small
//               per-launch self block (DP candidates, which must not touch the cache)
#pragma once
#include <type_traits>

#include "clasp_common.h"

namespace clasp {

constexpr int kEpiScale = 0, kEpiResid = 1, kEpiSwiglu = 2, kEpiQkv = 3, kEpiPartial = 4, kEpiHead = 5;

struct QkvOut {
    int n_heads, n_kv_heads, head_dim, pos0, mode, t_max;
    const float2* rope;  // [max_seq][head_dim/2] (cos, sin)
    float q_scale;       // softmax scale * log2(e), folded into q
    void* q_frag;        // [n_kv_heads][2*group][head_dim/32][64][8] kv_t (see attention kernel)
    void* k_cache;       // this layer, per KV head t_max/32 blocks in fragment order (kfrag_offset)
    void* v_cache;       // this layer, same (vfrag_offset)
    void* k_self;        // [n_kv_heads] one block each: the DP candidates' own keys
    void* v_self;        // [n_kv_heads] one block each
};

struct GemmArgs {
    const void* W[3];   // up to three matrices stacked along N (q|k|v); fp32 kEpiSwiglu: W[0] = gate, W[1] = up
    int tile_end[3];    // exclusive end tile (16 features) of each stacked matrix
    const void* A;      // activation operand: bf16 hi/lo fragments, or fp32 row-major [rows][K]
    int n_rows, N, K, R;
    const float* ss_parts;  // [n_parts][32] partial sums of squares of the un-normalised input rows
    int n_parts;
    float inv_dim, eps;
    float* out;  // fp32 [rows][ldo]
    int ldo;
    const float* resid;  // fp32 [rows][ldr]
    int ldr;
    void* next_op;           // operand for the next GEMM (its K = this N), may be null
    const float* next_gain;  // [N] gains folded into next_op (null = 1)
    float* next_ss;          // [N/16][32] partial sums of squares of `out`, may be null
    float* capture;          // optional copy of out, [rows][ldc]
    int ldc;
    QkvOut qkv;  // kEpiQkv only
    f32x4* head_parts;  // kEpiHead: [32][N/16] (max, index bits, second max, sum exp)
    // single-row kernel fed by split attention (A unused): row 0's input features are the merged attention outputs,
    // feature x belongs to head x / attn_hd; query j of KV head v left `attn_split` pieces
    // (O^T[attn_hd], max, sum) at attn_partial + ((v * attn_split + s) * 16 + j) * (attn_hd + 2)
    const float* attn_partial;
    int attn_split, attn_group, attn_hd;
};

// (largest, index, second largest) of two disjoint sets; equal maxima keep the lower index.
__device__ __forceinline__ void top2_merge(float& a1, int& ai, float& a2, float b1, int bi, float b2) {
    if (b1 > a1 || (b1 == a1 && bi < ai)) {
        a2 = fmaxf(a1, b2);
        a1 = b1;
        ai = bi;
    } else {
        a2 = fmaxf(a2, b1);
    }
}

// rstd[row] = 1 / sqrt(sum_p parts[p][row] * inv_dim + eps), fixed summation order. Needs blockDim % 32 == 0. Every
// thread issues 16 loads before it adds anything, so up to 16 * blockDim / 32 partials (256 for a 512-thread
// workgroup) cost one memory round trip; rows that do not exist are not read.
__device__ __forceinline__ void compute_rstd(const GemmArgs& g, float* rstd_s, float* tmp /* [blockDim] */) {
    const int row = threadIdx.x & 31, sub = threadIdx.x >> 5, nsub = blockDim.x >> 5;
    float s = 0.f;
    for (int base = 0; base < g.n_parts; base += 16 * nsub) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int p = base + sub + u * nsub;
            v[u] = (p < g.n_parts && row < g.n_rows) ? g.ss_parts[(size_t)p * kMaxRows + row] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) s += v[u];
    }
    tmp[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x < 32) {
        float t = 0.f;
        for (int u = 0; u < nsub; ++u) t += tmp[u * 32 + threadIdx.x];
        rstd_s[threadIdx.x] = 1.0f / sqrtf(t * g.inv_dim + g.eps);
    }
    __syncthreads();
}

// The same reduction in three steps, for kernels that hide the round trip of the partials behind their weight stream:
// thread t adds the partials p = t/32 + u*nsub (nsub = blockDim/32, fixed order) of row t%32;
//   rstd_issue  requests the first NLD of them (all of them when n_parts <= NLD * nsub);
//   rstd_stash  adds them up (fetching any remaining ones the slow way) and leaves the thread's sum in tmp[t];
//   rstd_finish, run by one whole wavefront after a workgroup barrier that follows rstd_stash, adds the nsub sums of
//   each row in order and writes rstd_s; the same wavefront may read rstd_s right after it.
template <int NLD>
__device__ __forceinline__ void rstd_issue(const GemmArgs& g, float (&v)[NLD]) {
    const int row = threadIdx.x & 31, sub = threadIdx.x >> 5, nsub = blockDim.x >> 5;
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
        const int p = sub + u * nsub;
        v[u] = (p < g.n_parts && row < g.n_rows) ? g.ss_parts[(size_t)p * kMaxRows + row] : 0.f;
    }
}
template <int NLD>
__device__ __forceinline__ void rstd_stash(const GemmArgs& g, const float (&v)[NLD], float* tmp /* [blockDim] */) {
    const int row = threadIdx.x & 31, sub = threadIdx.x >> 5, nsub = blockDim.x >> 5;
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < NLD; ++u) s += v[u];
    for (int p = sub + NLD * nsub; p < g.n_parts; p += nsub)
        if (row < g.n_rows) s += g.ss_parts[(size_t)p * kMaxRows + row];
    tmp[threadIdx.x] = s;
}
__device__ __forceinline__ void rstd_finish(const GemmArgs& g, const float* tmp, float* rstd_s) {
    const int lane = threadIdx.x & 63, nsub = blockDim.x >> 5;
    if (lane < 32) {
        float t = 0.f;
        for (int u = 0; u < nsub; ++u) t += tmp[u * 32 + lane];
        rstd_s[lane] = 1.0f / sqrtf(t * g.inv_dim + g.eps);
    }
    // LDS operations of one wavefront complete in program order; the fences keep the compiler from moving the
    // readers of rstd_s above the store
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int R, int NACC, int P, int SPLIT>
struct GemmStage {
    u32x4 b[NACC][P];
    u32x4 a[P][R][SPLIT];
};

// af[rg] points at this lane's 16 bytes inside a plane of row group rg. Lanes whose row does not exist read the last
// live row instead (same cache line as a live lane, so no extra traffic): their products land in output rows that are
// never stored, and unconditional loads keep the load stream free of exec-mask merges, which would make every stage
// wait for the previous one.
template <int R, int NACC, int P, int SPLIT>
__device__ __forceinline__ void gemm_issue(GemmStage<R, NACC, P, SPLIT>& st, const u32x4* const (&w)[NACC],
                                           const u32x4* const (&af)[R], int s, int ks1) {
#pragma unroll
    for (int u = 0; u < P; ++u) {
        const int ss = min(s + u, ks1 - 1);
#pragma unroll
        for (int a = 0; a < NACC; ++a) st.b[a][u] = load_stream(w[a] + (size_t)ss * 64);
#pragma unroll
        for (int rg = 0; rg < R; ++rg)
#pragma unroll
            for (int h = 0; h < SPLIT; ++h) st.a[u][rg][h] = af[rg][((size_t)ss * R * 2 + h) * 64];
    }
}

// WT = false: accumulator tile D[row][feature], a lane holds rows 4*(lane/16) .. +3 of feature lane%16.
// WT = true (weights as the first operand): D[feature][row], a lane holds features 4*(lane/16) .. +3 of row lane%16,
// i.e. four consecutive columns of one output row: what the epilogues that write rows (residual, K-slices) want.
template <int R, int NACC, int P, int SPLIT, bool WT = false>
__device__ __forceinline__ void gemm_compute(const GemmStage<R, NACC, P, SPLIT>& st, f32x4 (&acc)[NACC][R], int s,
                                             int ks1) {
#pragma unroll
    for (int u = 0; u < P; ++u) {
        if (s + u < ks1) {
#pragma unroll
            for (int rg = 0; rg < R; ++rg)
#pragma unroll
                for (int h = 0; h < SPLIT; ++h)
#pragma unroll
                    for (int a = 0; a < NACC; ++a) {
                        if constexpr (WT)
                            acc[a][rg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(st.b[a][u]),
                                                                                 as_bf16x8(st.a[u][rg][h]), acc[a][rg], 0, 0, 0);
                        else
                            acc[a][rg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(st.a[u][rg][h]),
                                                                                 as_bf16x8(st.b[a][u]), acc[a][rg], 0, 0, 0);
                    }
        }
    }
}

// Inputs of the epilogue that do not depend on the contraction (residual values, gain, rotary factors). The
// epilogue wavefront requests them before the main loop so that the tail of the kernel has no dependent global load.
struct EpiPre {
    float resid[4];
    float2 cs[4];
    float gain;
};

template <int EPI>
__device__ __forceinline__ void epi_prefetch(const GemmArgs& g, int tile, int lane, int rg, EpiPre& pre) {
    const int c = lane & 15, col = tile * 16 + c, row0 = rg * 16 + (lane >> 4) * 4;
    if constexpr (EPI == kEpiResid) {
        pre.gain = g.next_gain ? g.next_gain[col] : 1.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) pre.resid[r] = (row0 + r < g.n_rows) ? g.resid[(size_t)(row0 + r) * g.ldr + col] : 0.f;
    } else if constexpr (EPI == kEpiQkv) {
        const QkvOut& o = g.qkv;
        const int HALF = o.head_dim >> 1, tph = o.head_dim >> 4;
        const int tl = tile - (tile < g.tile_end[0] ? 0 : g.tile_end[0]);  // q or k tile inside its matrix
        const int e = (tl % tph) * 8 + (c & 7);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            pre.cs[r] = (tile < g.tile_end[1] && row < g.n_rows) ? o.rope[(size_t)(o.pos0 + (o.mode ? row : 0)) * HALF + e]
                                                                  : make_float2(1.f, 0.f);
        }
    }
}

// q/k/v epilogue of one lane: 4 rows x 1 feature of tile `tile` (see kEpiQkv above).
__device__ __forceinline__ void qkv_epilogue(const GemmArgs& g, int tile, int lane, int rg, const f32x4& sum,
                                             const float* rstd_s, const EpiPre& pre) {
    const QkvOut& o = g.qkv;
    const int HD = o.head_dim, HALF = HD >> 1, tph = HD >> 4;  // tiles per head
    const int c = lane & 15, row0 = rg * 16 + (lane >> 4) * 4;
    const int G = o.n_heads / o.n_kv_heads;
    const int which = tile < g.tile_end[0] ? 0 : (tile < g.tile_end[1] ? 1 : 2);
    const int tl = tile - (which == 0 ? 0 : g.tile_end[which - 1]);
    const int head = tl / tph, u = tl % tph;
    kv_t* kc = reinterpret_cast<kv_t*>(o.k_cache);
    kv_t* vc = reinterpret_cast<kv_t*>(o.v_cache);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = row0 + r;
        const float own = sum[r] * rstd_s[row & 31];
        const float partner = __shfl_xor(own, 8);
        if (which == 2) {  // v: plain feature order
            const int x = u * 16 + c;
            if (row < g.n_rows) {
                const kv_t v = to_kv(own);
                if (o.mode) vc[(size_t)head * o.t_max * HD + vfrag_offset(HD, o.pos0 + row, x)] = v;
                else reinterpret_cast<kv_t*>(o.v_self)[(size_t)head * 32 * HD + vfrag_offset(HD, row, x)] = v;
            }
            continue;
        }
        // q / k: lanes 0..7 hold feature e = 8u + c, lanes 8..15 its rotary partner e + HALF
        const int e = u * 8 + (c & 7), x = e + ((c & 8) ? HALF : 0);
        if (row < g.n_rows) {
            const int pos = o.pos0 + (o.mode ? row : 0);
            const float2 cs = pre.cs[r];
            const float rot = own * cs.x + ((c & 8) ? partner : -partner) * cs.y;
            if (which == 0) {
                const int kvh = head / G, qi = row * G + head % G;
                const size_t off = (((((size_t)kvh * (2 * G) + (qi >> 4)) * (HD >> 5) + (x >> 5)) * 64) +
                                    ((x >> 3) & 3) * 16 + (qi & 15)) * 8 + (x & 7);
                reinterpret_cast<kv_t*>(o.q_frag)[off] = to_kv(rot * o.q_scale);
            } else if (o.mode) {
                kc[(size_t)head * o.t_max * HD + kfrag_offset(HD, pos, x)] = to_kv(rot);
            } else {
                reinterpret_cast<kv_t*>(o.k_self)[(size_t)head * 32 * HD + kfrag_offset(HD, row, x)] = to_kv(rot);
            }
        }
    }
}

// Epilogue of one (tile, row group) for one lane: 4 rows x 1 feature; sum[a] = finished accumulators.
template <int EPI, int NACC>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, int tile, int lane, int rg, const f32x4 (&sum)[NACC],
                                              const float* rstd_s, const EpiPre& pre) {
    const int col = tile * 16 + (lane & 15);
    const int row0 = rg * 16 + (lane >> 4) * 4;
    if constexpr (EPI == kEpiScale) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            if (row < g.n_rows) g.out[(size_t)row * g.ldo + col] = sum[0][r] * rstd_s[row];
        }
    } else if constexpr (EPI == kEpiQkv) {
        qkv_epilogue(g, tile, lane, rg, sum[0], rstd_s, pre);
    } else if constexpr (EPI == kEpiHead) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            if (row >= g.n_rows) continue;  // uniform over the 16 lanes that share a row; the shuffles stay inside them
            const float x = sum[0][r] * rstd_s[row];
            if (g.out) g.out[(size_t)row * g.ldo + col] = x;
            float v1 = x, v2 = -INFINITY;
            int i1 = col;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                const float b1 = __shfl_xor(v1, o), b2 = __shfl_xor(v2, o);
                const int bi = __shfl_xor(i1, o);
                top2_merge(v1, i1, v2, b1, bi, b2);
            }
            const float se = sum16(expf(x - v1));
            if ((lane & 15) == 0) g.head_parts[(size_t)row * (g.N >> 4) + tile] = f32x4{v1, __int_as_float(i1), v2, se};
        }
    } else if constexpr (EPI == kEpiPartial) {
        float* slab = g.out + (size_t)blockIdx.y * g.ldr;  // ldr = elements per slab
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            if (row < g.n_rows) slab[(size_t)row * g.ldo + col] = sum[0][r];
        }
    } else if constexpr (EPI == kEpiResid) {
        const float gain = pre.gain;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            float v = 0.f;
            if (row < g.n_rows) {
                v = pre.resid[r] + sum[0][r];
                g.out[(size_t)row * g.ldo + col] = v;
                if (g.capture) g.capture[(size_t)row * g.ldc + col] = v;
            }
            if (g.next_op) store_operand<kDtBf16>(g.next_op, g.R, 0, row, col, v * gain);
            if (g.next_ss) {
                const float sq = sum16(v * v);
                if ((lane & 15) == 0) g.next_ss[(size_t)tile * kMaxRows + row] = sq;
            }
        }
    } else {
        // the packed gate|up matrix interleaves the two projections: lanes 0..7 of a tile hold gate features
        // 8*tile .. 8*tile+7, lanes 8..15 the matching up features
        const int c = lane & 15;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + r;
            const float own = sum[0][r] * rstd_s[row & 31];
            const float up = __shfl_xor(own, 8);
            const float v = (row < g.n_rows) ? own / (1.0f + expf(-own)) * up : 0.f;
            if (c < 8) store_operand<kDtBf16>(g.next_op, g.R, 0, row, tile * 8 + c, v);
        }
    }
}

// The residual and K-slice epilogues on a transposed accumulator tile (gemm_compute<.., WT = true>): a lane owns columns
// tile*16 + 4*(lane/16) .. +3 of row rg*16 + lane%16, so the residual, the output row, the captured state and the
// next GEMM's operand move as 16-byte (operand planes: 8-byte) pieces, and a row's sum of squares over the tile needs
// two shuffles. With one feature per lane the same epilogue took 12-16 stores of 2 or 4 bytes and 16 shuffles per lane
// at the very end of the kernel, where nothing overlaps them.
struct EpiPreT {
    f32x4 resid, gain;
    f32x4 cs[2];  // rotary (cos, sin) of the lane's four features
};

template <int EPI>
__device__ __forceinline__ void epi_prefetch_t(const GemmArgs& g, int tile, int lane, int rg, EpiPreT& pre) {
    if constexpr (EPI == kEpiResid) {
        const int row = rg * 16 + (lane & 15), col0 = tile * 16 + (lane >> 4) * 4;
        pre.gain = g.next_gain ? *reinterpret_cast<const f32x4*>(g.next_gain + col0) : f32x4{1.f, 1.f, 1.f, 1.f};
        pre.resid = row < g.n_rows ? *reinterpret_cast<const f32x4*>(g.resid + (size_t)row * g.ldr + col0)
                                   : f32x4{0.f, 0.f, 0.f, 0.f};
    } else if constexpr (EPI == kEpiQkv) {
        const QkvOut& o = g.qkv;
        const int HALF = o.head_dim >> 1, tph = o.head_dim >> 4;
        const int tl = tile - (tile < g.tile_end[0] ? 0 : g.tile_end[0]);  // q or k tile inside its matrix
        const int q4 = lane >> 4, row = rg * 16 + (lane & 15);
        const int e0 = (tl % tph) * 8 + (q4 & 1) * 4;
        pre.cs[0] = pre.cs[1] = f32x4{1.f, 0.f, 1.f, 0.f};
        if (tile < g.tile_end[1] && row < g.n_rows) {
            const f32x4* rp = reinterpret_cast<const f32x4*>(o.rope + (size_t)(o.pos0 + (o.mode ? row : 0)) * HALF + e0);
            pre.cs[0] = rp[0];
            pre.cs[1] = rp[1];
        }
    }
}

// q/k/v epilogue of one lane on a transposed tile: 4 features x 1 row. Tile features 0..7 are rotary features
// e = 8u .. 8u+7 of a head, 8..15 their partners e + head_dim/2 (the packing of wq / wk), so the partner of a lane's
// values sits 32 lanes away; q and k leave as 8-byte pieces of their fragments, v (stored transposed) element by element.
__device__ __forceinline__ void qkv_epilogue_t(const GemmArgs& g, int tile, int lane, int rg, const f32x4& sum,
                                               const float* rstd_s, const EpiPreT& pre) {
    typedef __attribute__((ext_vector_type(4))) _Float16 kvx4;
    static_assert(sizeof(kv_t) == 2, "8-byte pieces of four cache elements");
    const QkvOut& o = g.qkv;
    const int HD = o.head_dim, HALF = HD >> 1, tph = HD >> 4;  // tiles per head
    const int q4 = lane >> 4, row = rg * 16 + (lane & 15);
    const int G = o.n_heads / o.n_kv_heads;
    const int which = tile < g.tile_end[0] ? 0 : (tile < g.tile_end[1] ? 1 : 2);
    const int tl = tile - (which == 0 ? 0 : g.tile_end[which - 1]);
    const int head = tl / tph, u = tl % tph;
    const float rs = rstd_s[row & 31];
    f32x4 own, partner;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        own[i] = sum[i] * rs;
        partner[i] = __shfl_xor(own[i], 32);
    }
    if (row >= g.n_rows) return;
    if (which == 2) {  // v: plain feature order
        kv_t* base = o.mode ? reinterpret_cast<kv_t*>(o.v_cache) + (size_t)head * o.t_max * HD
                            : reinterpret_cast<kv_t*>(o.v_self) + (size_t)head * 32 * HD;
        const int t = o.mode ? o.pos0 + row : row;
#pragma unroll
        for (int i = 0; i < 4; ++i) base[vfrag_offset(HD, t, u * 16 + q4 * 4 + i)] = to_kv(own[i]);
        return;
    }
    const bool upper = q4 >= 2;
    const int x0 = u * 8 + (q4 & 1) * 4 + (upper ? HALF : 0);
    const float qs = which == 0 ? o.q_scale : 1.0f;
    kvx4 out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float cs_x = pre.cs[i >> 1][(i & 1) * 2], cs_y = pre.cs[i >> 1][(i & 1) * 2 + 1];
        const float rot = own[i] * cs_x + (upper ? partner[i] : -partner[i]) * cs_y;
        out[i] = which == 0 ? to_kv(rot * qs) : to_kv(rot);
    }
    if (which == 0) {
        const int kvh = head / G, qi = row * G + head % G;
        const size_t off = (((((size_t)kvh * (2 * G) + (qi >> 4)) * (HD >> 5) + (x0 >> 5)) * 64) +
                            ((x0 >> 3) & 3) * 16 + (qi & 15)) * 8 + (x0 & 7);
        *reinterpret_cast<kvx4*>(reinterpret_cast<kv_t*>(o.q_frag) + off) = out;
    } else if (o.mode) {
        *reinterpret_cast<kvx4*>(reinterpret_cast<kv_t*>(o.k_cache) + (size_t)head * o.t_max * HD +
                                 kfrag_offset(HD, o.pos0 + row, x0)) = out;
    } else {
        *reinterpret_cast<kvx4*>(reinterpret_cast<kv_t*>(o.k_self) + (size_t)head * 32 * HD + kfrag_offset(HD, row, x0)) = out;
    }
}

template <int EPI>
__device__ __forceinline__ void gemm_epilogue_t(const GemmArgs& g, int tile, int lane, int rg, const f32x4& sum,
                                                const float* rstd_s, const EpiPreT& pre) {
    static_assert(EPI == kEpiResid || EPI == kEpiPartial || EPI == kEpiQkv, "row-writing epilogues only");
    const int row = rg * 16 + (lane & 15), col0 = tile * 16 + (lane >> 4) * 4;
    if constexpr (EPI == kEpiQkv) {
        qkv_epilogue_t(g, tile, lane, rg, sum, rstd_s, pre);
    } else if constexpr (EPI == kEpiPartial) {
        float* slab = g.out + (size_t)blockIdx.y * g.ldr;  // ldr = elements per slab
        if (row < g.n_rows) *reinterpret_cast<f32x4*>(slab + (size_t)row * g.ldo + col0) = sum;
    } else {
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
        if (row < g.n_rows) {
            v = pre.resid + sum;
            *reinterpret_cast<f32x4*>(g.out + (size_t)row * g.ldo + col0) = v;
            if (g.capture) {  // the caller's buffer: 16-byte stores only if it is aligned for them
                float* cp = g.capture + (size_t)row * g.ldc + col0;
                if ((reinterpret_cast<uintptr_t>(g.capture) & 15) == 0 && (g.ldc & 3) == 0) {
                    *reinterpret_cast<f32x4*>(cp) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) cp[e] = v[e];
                }
            }
        }
        if (g.next_op) store_operand4<kDtBf16>(g.next_op, g.R, 0, row, col0, v * pre.gain);
        if (g.next_ss) {
            float sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
            sq += __shfl_xor(sq, 16);
            sq += __shfl_xor(sq, 32);
            if (lane < 16) g.next_ss[(size_t)tile * kMaxRows + row] = sq;
        }
    }
}

// Workgroup = CW x KW wavefronts: wavefront (cw, kw) streams NACC neighbouring column tiles, starting at tile
// (blockIdx.x*CW + cw)*NACC, over k-slice kw of KW equal slices; with NACC = 2 one activation fragment feeds two weight
// fragments, which halves the activation loads per weight byte. The CW wavefronts that share a k-slice read the same
// activation fragments at about the same time (one L2 fetch, the rest hit in L1); the KW partial tiles of a column
// tile are summed through LDS in slice order.
// (Cross-workgroup split-K inside one kernel is not used: agent-scope release fences cost far more than they save
// on this part, every one of them writes the whole L2 back.)
template <int R, int CW, int KW, int EPI, int P, int SPLIT, int NACC = 1>
__global__ __launch_bounds__(CW * KW * 64) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int NW = CW * KW;
    __shared__ f32x4 red[KW][CW][NACC][R][64];
    __shared__ float rstd_s[kMaxRows];
    __shared__ float tmp_s[NW * 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cw = wave % CW, kw = wave / CW;
    const int n_tiles = g.N >> 4;
    const int tile0 = (blockIdx.x * CW + cw) * NACC;
    const int KS = g.K >> 5;
    const int nslice = gridDim.y * KW, slice = blockIdx.y * KW + kw;  // gridDim.y > 1 only with kEpiPartial
    const int ks0 = (int)(((long long)KS * slice) / nslice), ks1 = (int)(((long long)KS * (slice + 1)) / nslice);

    int tile[NACC];
    const u32x4* w[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a) {
        tile[a] = min(tile0 + a, n_tiles - 1);  // tiles beyond the last shadow it, their result is dropped
        int mi = 0, tl = tile[a];
        if constexpr (EPI == kEpiScale || EPI == kEpiQkv) {
            if (tile[a] >= g.tile_end[0]) { mi = 1; tl = tile[a] - g.tile_end[0]; }
            if (tile[a] >= g.tile_end[1]) { mi = 2; tl = tile[a] - g.tile_end[1]; }
        }
        w[a] = reinterpret_cast<const u32x4*>(g.W[mi]) + (size_t)tl * KS * 64 + lane;
    }
    const u32x4* af[R];
#pragma unroll
    for (int rg = 0; rg < R; ++rg) {  // row of this lane, clamped to the last live row; may sit in an earlier group
        const int row = min(rg * 16 + (lane & 15), g.n_rows - 1);
        af[rg] = reinterpret_cast<const u32x4*>(g.A) + (size_t)(row >> 4) * 128 + (row & 15) * 4 + (lane >> 4);
    }

    f32x4 acc[NACC][R];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int rg = 0; rg < R; ++rg) acc[a][rg] = f32x4{0.f, 0.f, 0.f, 0.f};

    GemmStage<R, NACC, P, SPLIT> st0, st1;
    int s = ks0;
    if (s < ks1) gemm_issue<R, NACC, P, SPLIT>(st0, w, af, s, ks1);  // weights first: independent of rstd

    constexpr bool kWT = (EPI == kEpiResid || EPI == kEpiPartial || EPI == kEpiQkv);  // row-writing epilogues take transposed tiles
    typename std::conditional<kWT, EpiPreT, EpiPre>::type pre[NACC][R];
    if (kw == 0) {
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int rg = 0; rg < R; ++rg) {
                if constexpr (kWT) epi_prefetch_t<EPI>(g, tile[a], lane, rg, pre[a][rg]);
                else epi_prefetch<EPI>(g, tile[a], lane, rg, pre[a][rg]);
            }
    }
    if constexpr (EPI != kEpiResid && EPI != kEpiPartial) compute_rstd(g, rstd_s, tmp_s);

    while (s < ks1) {
        if (s + P < ks1) gemm_issue<R, NACC, P, SPLIT>(st1, w, af, s + P, ks1);
        gemm_compute<R, NACC, P, SPLIT, kWT>(st0, acc, s, ks1);
        s += P;
        if (s >= ks1) break;
        if (s + P < ks1) gemm_issue<R, NACC, P, SPLIT>(st0, w, af, s + P, ks1);
        gemm_compute<R, NACC, P, SPLIT, kWT>(st1, acc, s, ks1);
        s += P;
    }

    f32x4 sum[NACC][R];
    if constexpr (KW > 1) {
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int rg = 0; rg < R; ++rg) red[kw][cw][a][rg][lane] = acc[a][rg];
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int a = 0; a < NACC; ++a)
#pragma unroll
                for (int rg = 0; rg < R; ++rg) {
                    sum[a][rg] = red[0][cw][a][rg][lane];
                    for (int k = 1; k < KW; ++k) sum[a][rg] += red[k][cw][a][rg][lane];
                }
        }
    } else {
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int rg = 0; rg < R; ++rg) sum[a][rg] = acc[a][rg];
    }

    if (kw != 0) return;

#pragma unroll
    for (int a = 0; a < NACC; ++a) {
        if (tile0 + a >= n_tiles) continue;
#pragma unroll
        for (int rg = 0; rg < R; ++rg) {
            if constexpr (kWT) {
                gemm_epilogue_t<EPI>(g, tile[a], lane, rg, sum[a][rg], rstd_s, pre[a][rg]);
            } else {
                f32x4 fin[1];
                fin[0] = sum[a][rg];
                gemm_epilogue<EPI, 1>(g, tile[a], lane, rg, fin, rstd_s, pre[a][rg]);
            }
        }
    }
}

// Single-row variant (draft steps, plain decoding): with one live row an activation fragment is the same 16 bytes in all
// 16 lanes of a lane group, and fetching it with per-lane global loads (two per weight load: hi and lo plane) costs the
// load pipeline more than the weights do. Here every wavefront first copies row 0 of ITS k-slice (64 bytes per plane
// and k-step) into a private LDS region, one 16-byte piece per lane and load, and the main loop reads the fragments
// back with broadcast LDS reads, which run beside the weight stream instead of inside it. One column tile per
// workgroup, KW wavefronts split K; the register stages hold weights only. `nks_max` = LDS k-steps reserved per
// wavefront (>= ceil(K/32/KW), <= 16*kGemvLoads/SPLIT); dynamic LDS = KW * nks_max * SPLIT * 64 bytes.
// ASRC = 1 (output projection of a draft step): the row is not read from an operand but merged here from the pieces
// that split attention left per (KV head, prefix split, query): the arithmetic of attn_combine_kernel with the splits taken in order, so
// the attention kernel needs neither a second launch nor a single workgroup per KV head.
constexpr int kGemvLoads = 8;
constexpr int kGemvMaxSplit = 8;
template <int KW, int EPI, int P, int SPLIT, int ASRC = 0>
__global__ __launch_bounds__(KW * 64) void gemv_bf16_kernel(GemmArgs g, int nks_max) {
    extern __shared__ u32x4 a_lds[];
    __shared__ f32x4 red[KW][64];
    __shared__ float rstd_s[kMaxRows];
    __shared__ float tmp_s[KW * 64];
    constexpr bool kNeedsRstd = EPI != kEpiResid && EPI != kEpiPartial;
    const int kw = threadIdx.x >> 6, lane = threadIdx.x & 63, q = lane >> 4;
    const int tile = blockIdx.x, KS = g.K >> 5;
    const int ks0 = (KS * kw) / KW, ks1 = (KS * (kw + 1)) / KW, nks = ks1 - ks0;

    int mi = 0, tl = tile;
    if constexpr (EPI == kEpiScale || EPI == kEpiQkv) {
        if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
        if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
    }
    const u32x4* w0 = reinterpret_cast<const u32x4*>(g.W[mi]) + (size_t)tl * KS * 64 + lane;
    u32x4 wb[2][P];
    auto issue = [&](u32x4 (&buf)[P], int s) {
#pragma unroll
        for (int u = 0; u < P; ++u) buf[u] = load_stream(w0 + (size_t)min(s + u, ks1 - 1) * 64);
    };
    int s = ks0;
    if (s < ks1) issue(wb[0], s);  // weights first: independent of everything else

    // piece e of the slice = (k-step e / (4*SPLIT), plane (e / 4) % SPLIT, 16-byte quarter e % 4) of row 0
    const int n_el = nks * SPLIT * 4;
    u32x4* mine = a_lds + (size_t)kw * nks_max * SPLIT * 4;
    EpiPre pre;
    float ssv[16];
    if constexpr (ASRC == 0) {
        u32x4 av[kGemvLoads];
        const u32x4* A = reinterpret_cast<const u32x4*>(g.A);
#pragma unroll
        for (int i = 0; i < kGemvLoads; ++i) {
            const int e = min(lane + i * 64, max(n_el - 1, 0));
            av[i] = A[((size_t)(ks0 + e / (4 * SPLIT)) * 2 + (e / 4) % SPLIT) * 64 + (e & 3)];
        }
        if (kw == 0) epi_prefetch<EPI>(g, tile, lane, 0, pre);
        if constexpr (kNeedsRstd) rstd_issue(g, ssv);
        if (s + P < ks1) issue(wb[1], s + P);
#pragma unroll
        for (int i = 0; i < kGemvLoads; ++i)
            if (lane + i * 64 < n_el) mine[lane + i * 64] = av[i];
    } else {
        // (k-step, quarter) pp of the slice = 8 consecutive features of one head; lane takes pp = lane, lane + 64, ..
        const int HD = g.attn_hd, S = g.attn_split;
        const size_t sstride = (size_t)16 * (HD + 2);
        struct Piece { float2 ml[kGemvMaxSplit], ov[kGemvMaxSplit][4]; };
        auto fetch = [&](Piece& pc, int pp) {  // requests of the pieces that exist; nothing is added yet
            const int x0 = (ks0 + (pp >> 2)) * 32 + (pp & 3) * 8, head = x0 / HD, e0 = x0 - head * HD;
            const int kvh = head / g.attn_group, qi = head - kvh * g.attn_group;
            const float* base = g.attn_partial + ((size_t)kvh * S * 16 + qi) * (HD + 2);
#pragma unroll
            for (int sp = 0; sp < kGemvMaxSplit; ++sp) {
                if (sp < S) {
                    pc.ml[sp] = *reinterpret_cast<const float2*>(base + sp * sstride + HD);
#pragma unroll
                    for (int i = 0; i < 4; ++i) pc.ov[sp][i] = reinterpret_cast<const float2*>(base + sp * sstride + e0)[i];
                }
            }
        };
        auto merge_store = [&](const Piece& pc, int pp) {  // the merge of attn_combine_kernel, splits in order, then hi/lo into LDS
            float mstar = -INFINITY;
#pragma unroll
            for (int sp = 0; sp < kGemvMaxSplit; ++sp)
                if (sp < S) mstar = fmaxf(mstar, pc.ml[sp].x);
            float L = 0.f, O[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) O[i] = 0.f;
#pragma unroll
            for (int sp = 0; sp < kGemvMaxSplit; ++sp) {
                if (sp < S) {
                    const float f = (pc.ml[sp].x == -INFINITY) ? 0.f : exp2f(pc.ml[sp].x - mstar);
                    L += f * pc.ml[sp].y;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        O[2 * i] += f * pc.ov[sp][i].x;
                        O[2 * i + 1] += f * pc.ov[sp][i].y;
                    }
                }
            }
            bf16x8 hi, lo;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float v = O[i] / L;
                hi[i] = to_bf16(v);
                lo[i] = to_bf16(v - from_bf16(hi[i]));
            }
            const int sl = pp >> 2, qq = pp & 3;
            mine[(sl * SPLIT) * 4 + qq] = as_u32x4(hi);
            if constexpr (SPLIT == 2) mine[(sl * SPLIT + 1) * 4 + qq] = as_u32x4(lo);
        };
        Piece pc;
        if (lane < nks * 4) fetch(pc, lane);  // ahead of the second weight stage, like the operand loads above
        if (kw == 0) epi_prefetch<EPI>(g, tile, lane, 0, pre);
        if (s + P < ks1) issue(wb[1], s + P);
        if (lane < nks * 4) merge_store(pc, lane);
        for (int pp = lane + 64; pp < nks * 4; pp += 64) {
            fetch(pc, pp);
            merge_store(pc, pp);
        }
    }
    if constexpr (kNeedsRstd) rstd_stash(g, ssv, tmp_s);
    // the region is private to this wavefront and its LDS operations complete in program order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](const u32x4 (&buf)[P], int s0) {
#pragma unroll
        for (int u = 0; u < P; ++u) {
            if (s0 + u < ks1) {
#pragma unroll
                for (int h = 0; h < SPLIT; ++h)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(mine[((s0 + u - ks0) * SPLIT + h) * 4 + q]),
                                                                  as_bf16x8(buf[u]), acc, 0, 0, 0);
            }
        }
    };
    while (s < ks1) {  // two register stages: one being consumed, the other in flight
        compute(wb[0], s);
        s += P;
        if (s >= ks1) break;
        if (s + P < ks1) issue(wb[0], s + P);
        compute(wb[1], s);
        s += P;
        if (s + P < ks1) issue(wb[1], s + P);
    }

    red[kw][lane] = acc;
    __syncthreads();
    if (kw != 0) return;
    if constexpr (kNeedsRstd) rstd_finish(g, tmp_s, rstd_s);
    f32x4 fin[1];
    fin[0] = red[0][lane];
    for (int k = 1; k < KW; ++k) fin[0] += red[k][lane];
    gemm_epilogue<EPI, 1>(g, tile, lane, 0, fin, rstd_s, pre);
}

// Few-row kernel (1..kFewRows rows) for projections with more column tiles than the GPU has CUs (gate|up, lm_head):
// persistent workgroups walk over tiles blockIdx.x, blockIdx.x + gridDim.x, ..; the live rows of every wavefront's
// k-slice sit in a private LDS region (dynamic LDS: KW * KSW * SPLIT * 64 * rows bytes; lanes of rows that do not exist
// read the last live row), so the registers are free for NST = KSW/P weight stages, a whole tile slice per wavefront: the
// stage just consumed is refilled with the same stage of the NEXT tile, which keeps NST-1 stages in flight across the
// per-tile reduction barrier. KW wavefronts stream; one more wavefront does nothing but the epilogues (it is always
// early at the barrier, so no streaming wavefront ever waits for an epilogue; the partial tiles are double-buffered in
// LDS, and an epilogue has two tile times to finish). Needs K/32 <= KW*KSW.
constexpr int kFewRows = 8;
template <int KSW, int KW, int EPI, int P, int SPLIT>
__global__ __launch_bounds__((KW + 1) * 64) void gemv_persistent_bf16_kernel(GemmArgs g) {
    static_assert(KSW % P == 0, "a tile slice is a whole number of stages");
    constexpr int NST = KSW / P;
    extern __shared__ u32x4 a_s[];  // [KW][KSW * SPLIT * 4 * rows]
    __shared__ f32x4 red[2][KW][64];
    __shared__ float rstd_s[kMaxRows];
    __shared__ float tmp_s[(KW + 1) * 64];
    constexpr bool kNeedsRstd = EPI != kEpiResid && EPI != kEpiPartial;
    const int kw = threadIdx.x >> 6, lane = threadIdx.x & 63, q = lane >> 4;
    const int n_tiles = g.N >> 4, KS = g.K >> 5;
    float ssv[16];
    if constexpr (kNeedsRstd) rstd_issue(g, ssv);

    if (kw == KW) {  // the epilogue wavefront
        if constexpr (kNeedsRstd) rstd_stash(g, ssv, tmp_s);
        int it = 0;
        for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x, ++it) {
            EpiPre pre;
            epi_prefetch<EPI>(g, tile, lane, 0, pre);
            __syncthreads();  // the KW partial tiles of `tile` are in red[it & 1]
            if constexpr (kNeedsRstd) {
                if (it == 0) rstd_finish(g, tmp_s, rstd_s);
            }
            f32x4(&rb)[KW][64] = red[it & 1];
            f32x4 fin[1];
            fin[0] = rb[0][lane];
            for (int k = 1; k < KW; ++k) fin[0] += rb[k][lane];
            gemm_epilogue<EPI, 1>(g, tile, lane, 0, fin, rstd_s, pre);
        }
        return;
    }

    const int ks0 = (KS * kw) / KW, nks = (KS * (kw + 1)) / KW - ks0;  // nks <= KSW (checked on the host)
    auto wptr = [&](int tile) -> const u32x4* {
        int mi = 0, tl = tile;
        if constexpr (EPI == kEpiScale || EPI == kEpiQkv) {
            if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
            if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
        }
        return reinterpret_cast<const u32x4*>(g.W[mi]) + ((size_t)tl * KS + ks0) * 64 + lane;
    };
    u32x4 wb[NST][P];
    auto issue = [&](u32x4 (&buf)[P], int tile, int j) {  // stage j of `tile`: k-steps j*P .. j*P+P-1 of the slice
        const u32x4* w = wptr(tile);
#pragma unroll
        for (int u = 0; u < P; ++u) buf[u] = load_stream(w + (size_t)min(j * P + u, max(nks - 1, 0)) * 64);
    };
    int tile = blockIdx.x;
    if (tile < n_tiles) {
#pragma unroll
        for (int j = 0; j < NST; ++j) issue(wb[j], tile, j);  // the whole first slice
    }
    // the live rows of this wavefront's k-slice into its LDS region: piece e = ((k-step, plane, 16-byte quarter), row),
    // row fastest, so that the 16 lanes of a quarter read 16 consecutive pieces
    const int nr = g.n_rows;
    u32x4* mine = a_s + (size_t)kw * (KSW * SPLIT * 4) * nr;
    {
        const int n_el = nks * SPLIT * 4 * nr;
        const u32x4* A = reinterpret_cast<const u32x4*>(g.A);
        constexpr int NLD = (KSW * SPLIT * 4 * kFewRows + 63) / 64;
        u32x4 av[NLD];
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = min(lane + i * 64, max(n_el - 1, 0)), row = e % nr, t = e / nr;
            if (i == 0 || lane + i * 64 < n_el)
                av[i] = A[((size_t)(ks0 + t / (4 * SPLIT)) * 2 + (t / 4) % SPLIT) * 64 + row * 4 + (t & 3)];
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (lane + i * 64 < n_el) mine[lane + i * 64] = av[i];
        if constexpr (kNeedsRstd) rstd_stash(g, ssv, tmp_s);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the region is private to this wavefront
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    const u32x4* mine_r = mine + q * nr + min(lane & 15, nr - 1);  // this lane's quarter and (clamped) row

    for (int it = 0; tile < n_tiles; tile += gridDim.x, ++it) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        const int next_tile = tile + gridDim.x;
#pragma unroll
        for (int j = 0; j < NST; ++j) {
#pragma unroll
            for (int u = 0; u < P; ++u) {
                if (j * P + u < nks) {
#pragma unroll
                    for (int h = 0; h < SPLIT; ++h)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(mine_r[((j * P + u) * SPLIT + h) * 4 * nr]),
                                                                      as_bf16x8(wb[j][u]), acc, 0, 0, 0);
                }
            }
            if (next_tile < n_tiles) issue(wb[j], next_tile, j);  // refill what was just consumed
        }
        red[it & 1][kw][lane] = acc;
        __syncthreads();
    }
}

// Resident-activation variant for one row group (rows <= 16) and K/32 <= KW*KSW: wavefront kw keeps ITS k-slice of the
// activation fragments (hi and lo) in registers for the whole kernel, and the workgroup walks over column tiles
// blockIdx.x, blockIdx.x + gridDim.x, ... streaming nothing but weights: one 16-byte load per lane per MFMA pair.
// The register double buffer runs across tile boundaries (the next tile's first fragments are requested before the
// current tile's last ones are consumed), the per-tile reduction over the KW slices goes through a double-buffered
// LDS tile with one barrier per tile, and the epilogue duty rotates over the wavefronts.
template <int KSW, int KW, int EPI, int P, int SPLIT>
__global__ __launch_bounds__(KW * 64) void gemm_bf16_resident_kernel(GemmArgs g) {
    static_assert(KSW % P == 0 && (KSW / P) % 2 == 0, "a tile must take an even number of register stages");
    constexpr int NACC = 1;
    constexpr int NST = KSW / P;
    __shared__ f32x4 red[2][KW][NACC][64];
    __shared__ float rstd_s[kMaxRows];
    __shared__ float tmp_s[KW * 64];
    const int kw = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_tiles = g.N >> 4, KS = g.K >> 5;
    const int ks0 = (KS * kw) / KW, nks = (KS * (kw + 1)) / KW - ks0;  // nks <= KSW (checked on the host)

    // this wavefront's slice of the activations, resident for the whole kernel
    u32x4 areg[KSW][SPLIT];
    {
        const u32x4* af = reinterpret_cast<const u32x4*>(g.A) + min(lane & 15, g.n_rows - 1) * 4 + (lane >> 4);
#pragma unroll
        for (int i = 0; i < KSW; ++i)  // rows that do not exist mirror the last live row, steps beyond the slice its last step
#pragma unroll
            for (int h = 0; h < SPLIT; ++h) areg[i][h] = af[((size_t)(ks0 + min(i, max(nks - 1, 0))) * 2 + h) * 64];
    }

    auto wptr = [&](int tile, int which) -> const u32x4* {
        int mi = which, tl = tile;
        if constexpr (EPI == kEpiScale || EPI == kEpiQkv) {
            if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
            if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
        }
        return reinterpret_cast<const u32x4*>(g.W[mi]) + ((size_t)tl * KS + ks0) * 64 + lane;
    };
    u32x4 wb[2][NACC][P];
    auto issue = [&](u32x4 (&buf)[NACC][P], int tile, int j) {  // stage j of `tile`: k-steps j*P .. j*P+P-1 of the slice
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
            const u32x4* w = wptr(tile, a);
#pragma unroll
            for (int u = 0; u < P; ++u) buf[a][u] = load_stream(w + (size_t)min(j * P + u, nks - 1) * 64);
        }
    };

    int tile = blockIdx.x;
    if (tile < n_tiles && nks > 0) issue(wb[0], tile, 0);
    if constexpr (EPI != kEpiResid) compute_rstd(g, rstd_s, tmp_s);

    for (int it = 0; tile < n_tiles; tile += gridDim.x, ++it) {
        f32x4 acc[NACC];
#pragma unroll
        for (int a = 0; a < NACC; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int next_tile = tile + gridDim.x;
        EpiPre pre;
        if (kw == it % KW) epi_prefetch<EPI>(g, tile, lane, 0, pre);
#pragma unroll
        for (int j = 0; j < NST; ++j) {
            // request the next stage (of this tile, or the first one of the next tile) before consuming this one
            if (nks > 0) {
                if (j + 1 < NST) issue(wb[(j + 1) & 1], tile, j + 1);
                else if (next_tile < n_tiles) issue(wb[0], next_tile, 0);
            }
#pragma unroll
            for (int u = 0; u < P; ++u) {
                if (j * P + u < nks) {
#pragma unroll
                    for (int h = 0; h < SPLIT; ++h)
#pragma unroll
                        for (int a = 0; a < NACC; ++a)
                            acc[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(areg[j * P + u][h]),
                                                                             as_bf16x8(wb[j & 1][a][u]), acc[a], 0, 0, 0);
                }
            }
        }
        f32x4(&rb)[KW][NACC][64] = red[it & 1];
#pragma unroll
        for (int a = 0; a < NACC; ++a) rb[kw][a][lane] = acc[a];
        __syncthreads();
        if (kw == it % KW) {
            f32x4 fin[NACC];
#pragma unroll
            for (int a = 0; a < NACC; ++a) {
                fin[a] = rb[0][a][lane];
                for (int k = 1; k < KW; ++k) fin[a] += rb[k][a][lane];
            }
            gemm_epilogue<EPI, NACC>(g, tile, lane, 0, fin, rstd_s, pre);
        }
    }
}

// fp32 path (small models / exactness checks): row-major fp32 weights, plain FMA. One workgroup (4 wavefronts) per
// tile of 16 output features, each wavefront takes 4 of them and splits K across its lanes.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
    constexpr int NACC = (EPI == kEpiSwiglu) ? 2 : 1;
    __shared__ float rstd_s[kMaxRows];
    __shared__ float tmp_s[256];
    __shared__ float vals[NACC][16][kMaxRows];
    const int tile = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if constexpr (EPI != kEpiResid) compute_rstd(g, rstd_s, tmp_s);

    int mi = 0, tl = tile;
    if constexpr (EPI == kEpiScale) {
        if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
        if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
    }
    const float* A = reinterpret_cast<const float*>(g.A);
    for (int c = 0; c < 4; ++c) {
        const int cl = wave * 4 + c;
        const float* wrow[NACC];
        wrow[0] = reinterpret_cast<const float*>(g.W[mi]) + ((size_t)tl * 16 + cl) * g.K;
        if constexpr (NACC == 2) wrow[1] = reinterpret_cast<const float*>(g.W[1]) + ((size_t)tl * 16 + cl) * g.K;
        float acc[NACC][kMaxRows];
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int r = 0; r < kMaxRows; ++r) acc[a][r] = 0.f;
        for (int k = lane; k < g.K; k += 64) {
            float wv[NACC];
#pragma unroll
            for (int a = 0; a < NACC; ++a) wv[a] = wrow[a][k];
#pragma unroll
            for (int r = 0; r < kMaxRows; ++r) {
                if (r < g.n_rows) {
                    const float x = A[(size_t)r * g.K + k];
#pragma unroll
                    for (int a = 0; a < NACC; ++a) acc[a][r] = fmaf(wv[a], x, acc[a][r]);
                }
            }
        }
#pragma unroll
        for (int a = 0; a < NACC; ++a)
#pragma unroll
            for (int r = 0; r < kMaxRows; ++r) {
                const float t = wave_sum(acc[a][r]);
                if (lane == 0) vals[a][cl][r] = t;
            }
    }
    __syncthreads();
    // epilogue: one (row, column) pair per thread per pass; 16 consecutive lanes share a row
    for (int idx = threadIdx.x; idx < 16 * kMaxRows; idx += 256) {
        const int row = idx >> 4, cl = idx & 15, col = tile * 16 + cl;
        float v = 0.f;
        if constexpr (EPI == kEpiScale) {
            if (row < g.n_rows) g.out[(size_t)row * g.ldo + col] = vals[0][cl][row] * rstd_s[row];
        } else if constexpr (EPI == kEpiResid) {
            if (row < g.n_rows) {
                v = g.resid[(size_t)row * g.ldr + col] + vals[0][cl][row];
                g.out[(size_t)row * g.ldo + col] = v;
                if (g.capture) g.capture[(size_t)row * g.ldc + col] = v;
                if (g.next_op)
                    store_operand<kDtF32>(g.next_op, g.R, g.N, row, col, v * (g.next_gain ? g.next_gain[col] : 1.0f));
            }
            if (g.next_ss) {
                const float sq = sum16(v * v);
                if (cl == 0) g.next_ss[(size_t)tile * kMaxRows + row] = sq;
            }
        } else {
            if (row < g.n_rows) {
                const float gt = vals[0][cl][row] * rstd_s[row], up = vals[1][cl][row] * rstd_s[row];
                v = gt / (1.0f + expf(-gt)) * up;
                store_operand<kDtF32>(g.next_op, g.R, g.N, row, col, v);
            }
        }
    }
}

}  // namespace clasp
