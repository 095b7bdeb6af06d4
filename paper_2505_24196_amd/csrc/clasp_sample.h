// Stochastic decoding (the paper's Temperature = 1 setting, Sec. 4; "still speculative sampling", Sec. 4.1): draws from
// softmax(logits / T) by inverting the cumulative distribution with a uniform number the caller supplies, and the
// speculative-sampling acceptance rule over one round of drafts. One 1024-thread workgroup per call: the work is a
// few passes over [rows][vocab] fp32 logits (megabytes), nothing next to the forward passes around it.
// Every sum runs in a fixed order (thread t owns the contiguous chunk of ceil(V/1024) entries starting at
// t*ceil(V/1024)), so the same inputs give the same token on every run.
#pragma once
#include "clasp_common.h"

namespace clasp {

constexpr int kSampleThreads = 1024;

struct SampleShared {
    float red[kSampleThreads / 64];
    float part[kSampleThreads];   // per-thread chunk sums, then exclusive prefixes
    float wave_tot[kSampleThreads / 64];
    int pick;
};

__device__ __forceinline__ float block_max(float v, float* scratch) {
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    float t = scratch[0];
    for (int w = 1; w < nw; ++w) t = fmaxf(t, scratch[w]);
    return t;
}

struct RowStat {
    float m, s;  // max logit, sum over v of exp((logit_v - m) * inv_t)
};

__device__ __forceinline__ RowStat row_stat(const float* lg, int V, float inv_t, SampleShared& sh) {
    const int C = (V + kSampleThreads - 1) / kSampleThreads;
    const int lo = min(threadIdx.x * C, V), hi = min(lo + C, V);
    float m = -INFINITY;
    for (int v = lo; v < hi; ++v) m = fmaxf(m, lg[v]);
    m = block_max(m, sh.red);
    float s = 0.f;
    for (int v = lo; v < hi; ++v) s += expf((lg[v] - m) * inv_t);
    s = block_sum(s, sh.red);
    return RowStat{m, s};
}

// Inverse-CDF draw from the non-negative weights w(0..V-1): the index v with c_{v-1} <= u * c_last < c_v, c = running
// sums in index order. Returns the index to every thread (-1 when all weights are zero).
template <class WF>
__device__ __forceinline__ int block_draw(WF w, int V, float u, SampleShared& sh) {
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int C = (V + kSampleThreads - 1) / kSampleThreads;
    const int lo = min(t * C, V), hi = min(lo + C, V);
    float local = 0.f;
    for (int v = lo; v < hi; ++v) local += w(v);
    __syncthreads();
    sh.part[t] = local;
    if (t == 0) sh.pick = -1;
    __syncthreads();
    if (lane == 0) {
        float s = 0.f;
        for (int k = 0; k < 64; ++k) s += sh.part[wave * 64 + k];
        sh.wave_tot[wave] = s;
    }
    __syncthreads();
    float excl = 0.f, total = 0.f;
    for (int k = 0; k < kSampleThreads / 64; ++k) {
        if (k < wave) excl += sh.wave_tot[k];
        total += sh.wave_tot[k];
    }
    {
        float s = 0.f;
        for (int k = 0; k < lane; ++k) s += sh.part[wave * 64 + k];
        excl += s;
    }
    __syncthreads();
    sh.part[t] = excl;  // non-decreasing in t
    __syncthreads();
    if (!(total > 0.f)) return -1;
    const float target = u * total;
    const bool owner = excl <= target && (t == kSampleThreads - 1 || target < sh.part[t + 1]);
    if (owner) {  // exactly one thread; its chunk has positive weight unless it is the last thread
        float run = excl;
        int pick = -1, last = -1;
        for (int v = lo; v < hi; ++v) {
            const float wv = w(v);
            run += wv;
            if (wv > 0.f) last = v;
            if (target < run) { pick = v; break; }
        }
        sh.pick = pick >= 0 ? pick : last;  // the running sum here may end an ulp short of the next thread's prefix
    }
    __syncthreads();
    int pick = sh.pick;
    if (pick < 0) {  // rounding left u * c_last at or beyond the last running sum: last index of positive weight
        int last = -1;
        for (int v = lo; v < hi; ++v)
            if (w(v) > 0.f) last = v;
        pick = (int)block_max((float)last, sh.red);  // indices < 2^24 are exact in fp32
    }
    return pick;
}

// token_out[0] ~ softmax(logits / T) with the uniform number u[0].
__global__ __launch_bounds__(kSampleThreads) void sample_kernel(const float* logits, int V, float inv_t, const float* u,
                                                                int32_t* token_out) {
    __shared__ SampleShared sh;
    const RowStat st = row_stat(logits, V, inv_t, sh);
    const int tok = block_draw([&](int v) { return expf((logits[v] - st.m) * inv_t); }, V, u[0], sh);
    if (threadIdx.x == 0) token_out[0] = tok;
}

// One round of speculative sampling. tokens[0] is the round's pending token, tokens[1..n] the drafts; p row i / q row
// i are the full / draft model's logits for the token after row i. Draft i is kept when
// u_accept[i] * q_i(x) < p_i(x); the first rejected position a draws its replacement from max(0, p_a - q_a), and when
// all n are kept the bonus token comes from p_n; both draws use u_final[0].
__global__ __launch_bounds__(kSampleThreads) void spec_accept_kernel(const float* p_logits, const float* q_logits,
                                                                     size_t ld, const int32_t* tokens, int n, int V,
                                                                     float inv_t, const float* u_accept,
                                                                     const float* u_final, int32_t* n_accepted_out,
                                                                     int32_t* next_token_out) {
    __shared__ SampleShared sh;
    int a = n;
    RowStat ps{}, qs{};
    for (int i = 0; i < n; ++i) {  // every thread takes the same branches: all inputs of the test are block-uniform
        const float* p = p_logits + (size_t)i * ld;
        const float* q = q_logits + (size_t)i * ld;
        ps = row_stat(p, V, inv_t, sh);
        qs = row_stat(q, V, inv_t, sh);
        const int x = min(max(tokens[i + 1], 0), V - 1);
        const float px = expf((p[x] - ps.m) * inv_t) / ps.s, qx = expf((q[x] - qs.m) * inv_t) / qs.s;
        if (!(u_accept[i] * qx < px)) {
            a = i;
            break;
        }
    }
    const float* p = p_logits + (size_t)a * ld;
    int tok = -1;
    if (a < n) {
        const float* q = q_logits + (size_t)a * ld;
        const float ip = 1.0f / ps.s, iq = 1.0f / qs.s;
        tok = block_draw(
            [&](int v) { return fmaxf(expf((p[v] - ps.m) * inv_t) * ip - expf((q[v] - qs.m) * inv_t) * iq, 0.f); }, V,
            u_final[0], sh);
    } else {
        ps = row_stat(p, V, inv_t, sh);
    }
    if (tok < 0) tok = block_draw([&](int v) { return expf((p[v] - ps.m) * inv_t); }, V, u_final[0], sh);
    if (threadIdx.x == 0) {
        n_accepted_out[0] = a;
        next_token_out[0] = tok;
    }
}

}  // namespace clasp
