// Grouped-query attention of the candidate / verify / draft rows over the layer's shared KV cache.
//
// All rows of a launch read the cached prefix ONCE: the rows times the query heads of one KV group form the N
// dimension of S^T = K . Q^T, so a key fragment loaded from HBM serves every row (this is the paper's Sec. 3.6
// point: the DP's candidate states share one KV cache instead of duplicating it).
//   mode 0 (DP candidates): every row sits at position pos0 and sees cache positions 0..pos0-1 plus its own
//                           key/value, which live in a small per-launch self block; the cache is not touched.
//   mode 1 (verify / draft): row r sits at pos0 + r; its key/value is in the cache at that position already (the
//                           projection kernel wrote it) and it sees cache positions 0..pos0+r.
//
// bf16 kernel: flash-decoding on MFMA. Queries arrive rotated, scaled and in MFMA operand order from the q/k/v
// projection's epilogue. Keys are the M dimension of S^T (a lane then holds 4 keys x 1 query, and the two 16-key
// tiles of a 32-key block are interleaved so that the exponentiated scores of a lane are already the 8-key B
// fragment of O^T = V^T . P^T); V is cached transposed so that its fragments are 16-byte loads too. Wavefronts of a
// workgroup take 32-key blocks round-robin and are merged through LDS in a fixed order; several workgroups may split
// a long prefix (grid.z); attn_combine_kernel then merges their partial results in split order.
// fp32 kernel: plain loops, rotary embedding applied in the kernel, exact softmax over all visible keys.
#pragma once
#include "clasp_common.h"

namespace clasp {

struct AttnArgs {
    const float* qkv;  // fp32 path: [rows][ld_qkv]: q heads | k heads | v heads, un-rotated
    int ld_qkv;
    int n_rows, n_heads, n_kv_heads, head_dim;
    int pos0, mode;
    const float2* rope;  // [max_seq][head_dim/2] (cos, sin)
    void* Kc;            // this layer: fp32 [n_kv_heads][t_max][head_dim]; bf16: fragment order (kfrag_offset)
    void* Vt;            // this layer: fp32 [n_kv_heads][head_dim][t_max]; bf16: fragment order (vfrag_offset)
    int t_max;
    void* out_op;  // operand of the output projection (K = n_heads*head_dim)
    int R;
    int n_split;
    float* partial;      // [n_kv_heads][query groups][n_split][NT*16][head_dim+2] when n_split > 1
    float scale;         // 1/sqrt(head_dim)
    // bf16 path: written by the q/k/v projection's epilogue
    const void* q_frag;
    const void* k_self;  // [n_kv_heads] one 32-position block each: the DP candidates' own keys / values
    const void* v_self;
};

#ifndef CLASP_ATTN_DOUBLE_NT
#define CLASP_ATTN_DOUBLE_NT 1  // query tiles up to which a workgroup keeps two whole fragment sets
#endif

// Keys and values of a long prefix are read once per launch and should not displace anything (streaming loads); a
// short prefix is read by the sibling workgroups of its KV head within microseconds and fits in L2 many times over,
// where plain loads let the siblings hit (measured: 1.5 us per layer at T = 512, the other way round from 8k tokens on).
template <bool STREAM>
__device__ __forceinline__ u32x4 load_kv(const u32x4* p) {
    if constexpr (STREAM) return load_stream(p);
    else return *p;
}

constexpr float kLog2e = 1.4426950408889634f;

template <int HD, int NT>
struct AttnState {
    float m[NT], l[NT];
    f32x4 o[NT][HD / 16];
};

// Fragments of one 32-key block: k[u][kk] = A fragment of key tile u (16 keys), k-step kk; v[c] = A fragment of V^T
// rows c*16..c*16+15.
template <int HD>
struct AttnFrags {
    kvx8 k[2][HD / 32], v[HD / 16];
};

// All of a block's key and value fragments are requested together (and, in the pipelined loop, one block ahead), so
// that neither the value loads nor the next block wait behind the softmax.
template <int HD, class KF, class VF>
__device__ __forceinline__ void attn_load(AttnFrags<HD>& f, KF kf, VF vf) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int kk = 0; kk < HD / 32; ++kk) f.k[u][kk] = kf(u, kk);
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) f.v[c] = vf(c);
}

// One 32-key block in two steps, so that a pipelined loop can re-use the key registers for the next block's keys as
// soon as the scores exist, and the value registers as soon as the block is accumulated.
// attn_scores: S^T = K Q^T for NT query tiles, online softmax update (running max / sum, rescaling of O^T), leaves the
//              exponentiated scores as the B fragments pf[t] of the second product.
//   valid(u, r, t) -> whether key (lane/16)*8 + u*4 + r of the block is visible to query t*16 + lane%16
// attn_pv:     O^T += V^T P^T.
//   masked (wave-uniform) = false promises that valid() holds for every key of the block and every query of the
//   wavefront (a block below the diagonal of a causal pass), and the comparisons are left out.
// The exponentials are the hardware's 2^x (v_exp_f32: arguments are <= 0, results in [0, 1], tiny ones may flush to 0).
// O^T and the running sum are only rescaled in blocks where some query's running maximum grows (for the others the
// factor is exactly 1): after the first few blocks of a long prefix that is rare, and the rescaling is a third of the
// vector work of a block.
// attn_qk: the raw scores S^T = K Q^T of one block (MFMAs only); attn_softmax: everything between the two products.
template <int HD, int NT>
__device__ __forceinline__ void attn_qk(f32x4 (&s)[2][NT], const kvx8 (&qf)[NT][HD / 32], const kvx8 (&kfr)[2][HD / 32]) {
    constexpr int KK = HD / 32;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int t = 0; t < NT; ++t) s[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                s[u][t] = mfma_kv(kfr[u][kk], qf[t][kk], s[u][t]);
        }
    }
}

template <int HD, int NT, class VALID>
__device__ __forceinline__ void attn_softmax(AttnState<HD, NT>& st, f32x4 (&s)[2][NT], VALID valid, kvx8 (&pf)[NT], bool masked) {
    constexpr int CT = HD / 16;
    if (masked) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (!valid(u, r, t)) s[u][t][r] = -INFINITY;
    }
    float m_safe[NT], m_new[NT];
    bool grew = false;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[u][t][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        m_new[t] = fmaxf(st.m[t], mx);
        m_safe[t] = (m_new[t] == -INFINITY) ? 0.f : m_new[t];
        grew = grew || m_new[t] > st.m[t];
    }
    if (__builtin_amdgcn_ballot_w64(grew) != 0) {  // wave-uniform: some query's maximum grew
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float alpha = __builtin_amdgcn_exp2f(st.m[t] - m_safe[t]);
            st.l[t] *= alpha;
            st.m[t] = m_new[t];
#pragma unroll
            for (int c = 0; c < CT; ++c) st.o[t][c] *= alpha;
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[u][t][r] - m_safe[t]);
                psum += p;
                pf[t][u * 4 + r] = (kv_t)p;  // p in [0, 1]
            }
        st.l[t] += psum;
    }
}

template <int HD, int NT, class VALID>
__device__ __forceinline__ void attn_scores(AttnState<HD, NT>& st, const kvx8 (&qf)[NT][HD / 32],
                                            const kvx8 (&kfr)[2][HD / 32], VALID valid, kvx8 (&pf)[NT], bool masked = true) {
    f32x4 s[2][NT];
    attn_qk<HD, NT>(s, qf, kfr);
    attn_softmax<HD, NT>(st, s, valid, pf, masked);
}

template <int HD, int NT>
__device__ __forceinline__ void attn_pv(AttnState<HD, NT>& st, const kvx8 (&vfr)[HD / 16], const kvx8 (&pf)[NT]) {
#pragma unroll
    for (int c = 0; c < HD / 16; ++c) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
            st.o[t][c] = mfma_kv(vfr[c], pf[t], st.o[t][c]);
    }
}

template <int HD, int NT, class VALID>
__device__ __forceinline__ void attn_compute(AttnState<HD, NT>& st, const kvx8 (&qf)[NT][HD / 32],
                                             const AttnFrags<HD>& f, VALID valid, bool masked = true) {
    kvx8 pf[NT];
    attn_scores<HD, NT>(st, qf, f.k, valid, pf, masked);
    attn_pv<HD, NT>(st, f.v, pf);
}

// q_frag: queries of one KV head (query index qi = row*group + head%group) as MFMA B fragments,
// [kv_head][qi/16][x/32][lane = ((x%32)/8)*16 + qi%16][x%8], written by the q/k/v projection's epilogue.
template <int HD, int NT, int NW, bool STREAM>
__global__ __launch_bounds__(NW * 64) void attn_bf16_kernel(AttnArgs a) {
    constexpr int KK = HD / 32, CT = HD / 16;
    extern __shared__ float lds_dyn[];  // NW*HD*17 floats: per-wavefront O^T tiles (+1 column against bank conflicts)
    typedef float (*MgT)[HD][17];
    MgT mg_o = reinterpret_cast<MgT>(lds_dyn);
    __shared__ float mg_m[NW][16], mg_l[NW][16], mg_f[NW][16];
    const int kvh = blockIdx.x, qg = blockIdx.y, split = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int G = a.n_heads / a.n_kv_heads, nQ = a.n_rows * G;
    const int q_base = qg * NT * 16;
    const int m16 = lane & 15, q4 = lane >> 4;
    const kv_t* Kc = reinterpret_cast<const kv_t*>(a.Kc);
    const kv_t* Vt = reinterpret_cast<const kv_t*>(a.Vt);

    // query fragments straight from HBM/L2 (already rotated, scaled and in B-operand order)
    kvx8 qf[NT][KK];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(a.q_frag) + ((size_t)kvh * (2 * G) + qg * NT) * KK * 64 + lane;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[t][kk] = as_kvx8(qp[(t * KK + kk) * 64]);
    }
    // visibility: query qi of row r sees cache keys <= limit (verify/draft: pos0 + r, its own position, whose
    // key/value the projection kernel has just written; DP candidates: pos0 - 1) and, for DP candidates, its own
    // entry of the self block
    int limit[NT], qrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int qi = q_base + t * 16 + m16;
        qrow[t] = qi < nQ ? qi / G : -1;
        limit[t] = qi < nQ ? (a.mode ? a.pos0 + qrow[t] : a.pos0 - 1) : -1;
    }

    AttnState<HD, NT> st;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        st.m[t] = -INFINITY;
        st.l[t] = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) st.o[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int n_cache = a.pos0 + (a.mode ? a.n_rows : 0);  // cache positions any row may see
    const int nblk = (n_cache + 31) >> 5;
    const int b0 = (int)(((long long)nblk * split) / a.n_split), b1 = (int)(((long long)nblk * (split + 1)) / a.n_split);
    const u32x4* Kh = reinterpret_cast<const u32x4*>(Kc + (size_t)kvh * a.t_max * HD) + lane;
    const u32x4* Vh = reinterpret_cast<const u32x4*>(Vt + (size_t)kvh * a.t_max * HD) + lane;
    auto load_blk = [&](AttnFrags<HD>& f, int blk) {
        const u32x4* kp = Kh + (size_t)blk * (2 * KK * 64);
        const u32x4* vp = Vh + (size_t)blk * (CT * 64);
        attn_load<HD>(f, [&](int u, int kk) { return as_kvx8(load_kv<STREAM>(kp + (u * KK + kk) * 64)); },
                      [&](int c) { return as_kvx8(load_kv<STREAM>(vp + c * 64)); });
    };
    auto compute_blk = [&](const AttnFrags<HD>& f, int blk) {
        const int kb = blk << 5;
        attn_compute<HD, NT>(st, qf, f, [&](int u, int r, int t) { return kb + q4 * 8 + u * 4 + r <= limit[t]; });
    };
    int blk = b0 + wave;
    if constexpr (NT <= CLASP_ATTN_DOUBLE_NT || (NW <= 4 && NT <= 3)) {  // registers allow a second fragment set (four wavefronts: one per SIMD, the whole register file each): the next block is in flight during the MFMAs
        AttnFrags<HD> f0, f1;
        if (blk < b1) load_blk(f0, blk);
        while (blk < b1) {
            if (blk + NW < b1) load_blk(f1, blk + NW);
            compute_blk(f0, blk);
            blk += NW;
            if (blk >= b1) break;
            if (blk + NW < b1) load_blk(f0, blk + NW);
            compute_blk(f1, blk);
            blk += NW;
        }
    } else {
        // one fragment set, re-used in flight: the next block's keys are requested as soon as this block's scores
        // exist (they land during the softmax and the second product), its values as soon as the block is accumulated
        AttnFrags<HD> f;
        auto load_k = [&](int b) {
            const u32x4* kp = Kh + (size_t)b * (2 * KK * 64);
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) f.k[u][kk] = as_kvx8(load_kv<STREAM>(kp + (u * KK + kk) * 64));
        };
        auto load_v = [&](int b) {
            const u32x4* vp = Vh + (size_t)b * (CT * 64);
#pragma unroll
            for (int c = 0; c < CT; ++c) f.v[c] = as_kvx8(load_kv<STREAM>(vp + c * 64));
        };
        if (blk < b1) {
            load_k(blk);
            load_v(blk);
        }
        for (; blk < b1; blk += NW) {
            const int kb = blk << 5;
            kvx8 pf[NT];
            attn_scores<HD, NT>(st, qf, f.k, [&](int u, int r, int t) { return kb + q4 * 8 + u * 4 + r <= limit[t]; }, pf);
            if (blk + NW < b1) load_k(blk + NW);
            attn_pv<HD, NT>(st, f.v, pf);
            if (blk + NW < b1) load_v(blk + NW);
        }
    }
    if (!a.mode && split == a.n_split - 1 && wave == (b1 - b0) % NW) {  // DP candidates: own key/value only
        const u32x4* kp = reinterpret_cast<const u32x4*>(a.k_self) + (size_t)kvh * (2 * KK * 64) + lane;
        const u32x4* vp = reinterpret_cast<const u32x4*>(a.v_self) + (size_t)kvh * (CT * 64) + lane;
        AttnFrags<HD> f;
        attn_load<HD>(f, [&](int u, int kk) { return as_kvx8(kp[(u * KK + kk) * 64]); },
                      [&](int c) { return as_kvx8(vp[c * 64]); });
        attn_compute<HD, NT>(st, qf, f, [&](int u, int r, int t) { return q4 * 8 + u * 4 + r == qrow[t]; });
    }

    // merge the wavefronts' running (max, sum, O^T), one query tile at a time, fixed order
    float* part = a.partial + ((((size_t)kvh * gridDim.y + qg) * a.n_split + split) * NT * 16) * (HD + 2);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float l = st.l[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lane < 16) {
            mg_m[wave][lane] = st.m[t];
            mg_l[wave][lane] = l;
        }
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) mg_o[wave][c * 16 + q4 * 4 + r][m16] = st.o[t][c][r];
        __syncthreads();
        if (tid < 16) {  // per query: global max, rescale factors, total sum
            float mstar = -INFINITY;
            for (int w = 0; w < NW; ++w) mstar = fmaxf(mstar, mg_m[w][tid]);
            float L = 0.f;
            for (int w = 0; w < NW; ++w) {
                const float mw = mg_m[w][tid];
                const float f = (mw == -INFINITY) ? 0.f : exp2f(mw - mstar);
                mg_f[w][tid] = f;
                L += f * mg_l[w][tid];
            }
            mg_m[0][tid] = mstar;
            mg_l[0][tid] = L;
        }
        __syncthreads();
        for (int idx = tid; idx < HD * 16; idx += NW * 64) {
            const int e = idx >> 4, j = idx & 15, qi = q_base + t * 16 + j;
            if (qi < nQ) {
                float O = 0.f;
                for (int w = 0; w < NW; ++w) O += mg_f[w][j] * mg_o[w][e][j];
                if (a.n_split == 1) {
                    const int row = qi / G, h = kvh * G + qi % G;
                    store_operand<kDtBf16>(a.out_op, a.R, 0, row, h * HD + e, O / mg_l[0][j]);
                } else {
                    float* p = part + (size_t)(t * 16 + j) * (HD + 2);
                    p[e] = O;
                    if (e == 0) {
                        p[HD] = mg_m[0][j];
                        p[HD + 1] = mg_l[0][j];
                    }
                }
            }
        }
        __syncthreads();
    }
}

// Merges the n_split partial results of one query and writes the output-projection operand. Grid (kv heads, queries),
// kCombineWaves wavefronts: every thread first takes the largest of the splits' maxima (the same few words for the whole
// workgroup), then wavefront w adds the rescaled sums of splits w, w + kCombineWaves, .. for two head-dim elements per
// lane (all of a wavefront's loads in flight together), and the wavefronts' sums are added in order through LDS.
constexpr int kCombineWaves = 4;
__global__ __launch_bounds__(kCombineWaves * 64) void attn_combine_kernel(AttnArgs a, int nt, int qgroups) {
    __shared__ float sL[kCombineWaves];
    __shared__ float2 sO[kCombineWaves][64];
    const int kvh = blockIdx.x, qi = blockIdx.y, HD = a.head_dim;
    const int G = a.n_heads / a.n_kv_heads;
    const int qg = qi / (nt * 16), ql = qi % (nt * 16);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t sstride = (size_t)nt * 16 * (HD + 2);
    const float* pq = a.partial + (((size_t)kvh * qgroups + qg) * a.n_split) * sstride + (size_t)ql * (HD + 2);
    float mstar = -INFINITY;
#pragma unroll 8
    for (int s = 0; s < a.n_split; ++s) mstar = fmaxf(mstar, pq[s * sstride + HD]);
    float L = 0.f;
    float2 O = make_float2(0.f, 0.f);
    const bool live = 2 * lane < HD;  // head_dim 64: half of the lanes carry elements
#pragma unroll 4
    for (int s = wave; s < a.n_split; s += kCombineWaves) {
        const float2 ml = *reinterpret_cast<const float2*>(pq + s * sstride + HD);
        const float2 ov = live ? *reinterpret_cast<const float2*>(pq + s * sstride + 2 * lane) : make_float2(0.f, 0.f);
        const float f = (ml.x == -INFINITY) ? 0.f : exp2f(ml.x - mstar);
        L += f * ml.y;
        O.x += f * ov.x;
        O.y += f * ov.y;
    }
    if (lane == 0) sL[wave] = L;
    sO[wave][lane] = O;
    __syncthreads();
    if (wave == 0 && live) {
        float Lt = sL[0];
        float2 Ot = sO[0][lane];
        for (int w = 1; w < kCombineWaves; ++w) {
            Lt += sL[w];
            Ot.x += sO[w][lane].x;
            Ot.y += sO[w][lane].y;
        }
        const int row = qi / G, h = kvh * G + qi % G;
        store_operand<kDtBf16>(a.out_op, a.R, 0, row, h * HD + 2 * lane, Ot.x / Lt);
        store_operand<kDtBf16>(a.out_op, a.R, 0, row, h * HD + 2 * lane + 1, Ot.y / Lt);
    }
}

// fp32 path: one workgroup per (query head, row); plain loops, exact softmax over all visible keys.
// Dynamic LDS: (head_dim + n_keys) floats with n_keys = pos0 + 32.
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a) {
    extern __shared__ float lds[];
    __shared__ float red[8];
    const int h = blockIdx.x, r = blockIdx.y, HD = a.head_dim, HALF = HD / 2;
    const int G = a.n_heads / a.n_kv_heads, kvh = h / G;
    const int pos = a.pos0 + (a.mode ? r : 0);
    const int n_self = a.mode ? r + 1 : 1;  // visible self keys: rows 0..r, or only row r
    const int self0 = a.mode ? 0 : r;
    const int n_keys = a.pos0 + n_self;
    float* q = lds;
    float* sc = lds + HD;
    const float* Kc = reinterpret_cast<const float*>(a.Kc) + (size_t)kvh * a.t_max * HD;
    const float* Vt = reinterpret_cast<const float*>(a.Vt) + (size_t)kvh * HD * a.t_max;
    for (int e = threadIdx.x; e < HALF; e += blockDim.x) {
        const float* qp = a.qkv + (size_t)r * a.ld_qkv + h * HD;
        const float2 cs = a.rope[(size_t)pos * HALF + e];
        q[e] = qp[e] * cs.x - qp[e + HALF] * cs.y;
        q[e + HALF] = qp[e + HALF] * cs.x + qp[e] * cs.y;
    }
    __syncthreads();
    float mx = -INFINITY;
    for (int t = threadIdx.x; t < n_keys; t += blockDim.x) {
        float s = 0.f;
        if (t < a.pos0) {
            const float* kp = Kc + (size_t)t * HD;
            for (int e = 0; e < HD; ++e) s = fmaf(q[e], kp[e], s);
        } else {
            const int sr = self0 + (t - a.pos0);
            const int spos = a.pos0 + (a.mode ? sr : 0);
            const float* kp = a.qkv + (size_t)sr * a.ld_qkv + (a.n_heads + kvh) * HD;
            for (int e = 0; e < HALF; ++e) {
                const float2 cs = a.rope[(size_t)spos * HALF + e];
                s = fmaf(q[e], kp[e] * cs.x - kp[e + HALF] * cs.y, s);
                s = fmaf(q[e + HALF], kp[e + HALF] * cs.x + kp[e] * cs.y, s);
            }
        }
        s *= a.scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float den = 0.f;
    for (int t = threadIdx.x; t < n_keys; t += blockDim.x) {
        const float p = expf(sc[t] - mx);
        sc[t] = p;
        den += p;
    }
    den = block_sum(den, red + 4);
    for (int e = threadIdx.x; e < HD; e += blockDim.x) {
        float o = 0.f;
        const float* vp = Vt + (size_t)e * a.t_max;
        for (int t = 0; t < a.pos0; ++t) o = fmaf(sc[t], vp[t], o);
        for (int t = a.pos0; t < n_keys; ++t) {
            const int sr = self0 + (t - a.pos0);
            o = fmaf(sc[t], a.qkv[(size_t)sr * a.ld_qkv + (a.n_heads + a.n_kv_heads + kvh) * HD + e], o);
        }
        store_operand<kDtF32>(a.out_op, a.R, a.n_heads * HD, r, h * HD + e, o / den);
    }
    if (a.mode && h % G == 0) {  // this row's key/value into the cache
        float* Kw = reinterpret_cast<float*>(a.Kc) + ((size_t)kvh * a.t_max + pos) * HD;
        float* Vw = reinterpret_cast<float*>(a.Vt) + (size_t)kvh * HD * a.t_max + pos;
        const float* kp = a.qkv + (size_t)r * a.ld_qkv + (a.n_heads + kvh) * HD;
        const float* vp = kp + a.n_kv_heads * HD;
        for (int e = threadIdx.x; e < HALF; e += blockDim.x) {
            const float2 cs = a.rope[(size_t)pos * HALF + e];
            Kw[e] = kp[e] * cs.x - kp[e + HALF] * cs.y;
            Kw[e + HALF] = kp[e + HALF] * cs.x + kp[e] * cs.y;
            Vw[(size_t)e * a.t_max] = vp[e];
            Vw[(size_t)(e + HALF) * a.t_max] = vp[e + HALF];
        }
    }
}

}  // namespace clasp
