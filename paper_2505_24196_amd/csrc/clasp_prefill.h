// Prompt processing ("prefill") with many rows per pass: the full model over hundreds or thousands of prompt tokens
// at once, whose only lasting product is the KV cache that verification, the layer-skip search and drafting (Sec. 3.1,
// 3.6 of the paper) read afterwards. With C rows per pass the GEMMs do C flop per weight byte, beyond the ridge of the
// part (~310) from a few hundred rows on, so unlike the decode-time kernels these are organised around the matrix
// cores and around getting operands to them:
//   * prefill_gemm256_kernel: 256 x 256 workgroup tiles, 4 x 2 wavefronts with 64 x 128 accumulators; both operands
//     are stored in MFMA fragment order already (weights as packed for the decode kernels, activations as the operand
//     planes every producer writes), so staging is a copy of whole KiB fragments, done by direct global -> LDS loads
//     into a ring of three or four stages.
//   * prefill_gemm_kernel: 128 x 128 or 64 x 128 tiles staged through registers, for the q/k/v projection and for
//     passes too short for the big tile; prefill_reduce_kernel finishes a K-split of very short passes.
//   * prefill_attn_lds_kernel / prefill_attn_kernel: causal flash attention over the fragment-order cache; a wavefront
//     owns two tiles of 16 queries (row x head of one KV group); long prefixes share each 32-key block among the eight
//     wavefronts of a workgroup through a ring of LDS stages, short ones are read by every wavefront itself.
// Passes of fewer than 640 rows keep the decode path's hi + lo bf16 activation split (two MFMAs per fragment pair), so
// that the cache a short prompt leaves behind equals the row-limited path's up to rounding order. Longer passes are
// bound by the matrix cores, where the split doubles the work: they run on fp16 operands instead (one fp16 plane per
// activation, 11 significant bits; the layer's bf16 weights converted to fp16, which represents them exactly down to
// 2^-17, by prefill_convert_f16_kernel at the start of each layer; fp32 accumulation). Epilogues write exactly what
// the decode kernels' epilogues write (rotated, scaled query fragments; keys and values into the cache; residual
// stream, next operand in the pass's format, sum-of-squares partials; SwiGLU operand).
#pragma once
#include "clasp_attn.h"
#include "clasp_common.h"
#include "clasp_gemm.h"

namespace clasp {

struct PrefillGemmArgs {
    GemmArgs g;          // W, tile_end, A, n_rows, N, K, R, out/ldo, resid/ldr, next_op, next_gain, next_ss, qkv
    const float* rstd;   // [n_rows] 1/rms of the input rows (projections that follow a norm), else null
    int ld_ss;           // row capacity of next_ss: next_ss[tile][ld_ss]
    // kEpiPartial (prefill_gemm_kernel with gridDim.y = k_split > 1): slice y of the contraction leaves its raw sums in
    // g.out + y * slab ([rows][g.ldo]); prefill_reduce_kernel adds the slices in order and runs the residual epilogue
    int k_split;
    size_t slab;
    int op_f16;          // format of next_op: one fp16 plane (passes that run on fp16 MFMAs) or the bf16 hi / lo planes
};

// rstd[row] = 1 / sqrt(sum_p ss[p][row] / dim + eps). Block (64, 16): thread (x, y) adds parts y, y + 16, .. of row
// blockIdx.x*64 + x (coalesced over rows, loads issued eight at a time), the sixteen sums are added in y order.
__global__ __launch_bounds__(1024) void prefill_rstd_kernel(const float* ss, int n_parts, int ld, int n_rows, float inv_dim,
                                                            float eps, float* rstd) {
    __shared__ float part[16][64];
    const int row = blockIdx.x * 64 + threadIdx.x, y = threadIdx.y;
    float s = 0.f;
    if (row < n_rows) {
        for (int p0 = y; p0 < n_parts; p0 += 16 * 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = (p0 + 16 * u < n_parts) ? ss[(size_t)(p0 + 16 * u) * ld + row] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
    }
    part[y][threadIdx.x] = s;
    __syncthreads();
    if (y == 0 && row < n_rows) {
        float t = 0.f;
        for (int k = 0; k < 16; ++k) t += part[k][threadIdx.x];
        rstd[row] = 1.0f / sqrtf(t * inv_dim + eps);
    }
}

// Embedding gather for a chunk: h_0, the first layer's operand (times its norm gains) and sum-of-squares partials.
// Grid (rows, ceil(d / 256)).
__global__ __launch_bounds__(256) void prefill_embed_kernel(const int32_t* tokens, const bf16* table, int vocab, int d,
                                                            float* h, void* op, int R, const float* gain, float* ss,
                                                            int ld_ss, int op_f16) {
    const int row = blockIdx.x, c = blockIdx.y * 256 + threadIdx.x;
    if (c >= d) return;
    int tok = tokens[row];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const float v = from_bf16(table[(size_t)tok * d + c]);
    h[(size_t)row * d + c] = v;
    store_operand_fmt(op, R, row, c, v * gain[c], op_f16);
    const float sq = sum16(v * v);
    if ((c & 15) == 0) ss[(size_t)(c >> 4) * ld_ss + row] = sq;
}

// The GEMMs below multiply with the weight fragment as the MFMA's first operand and the activation fragment as its
// second, so a finished 16 x 16 accumulator tile is D[feature][row]: lane holds row rt*16 + lane%16 and the four
// consecutive features tile*16 + (lane/16)*4 + r. Four consecutive features of one row are contiguous in everything an
// epilogue touches (residual stream, operand planes, query fragments, key cache), so each of its loads and stores
// moves 8 or 16 bytes per lane (with the other orientation, four rows of one feature per lane, they were 2 or 4 bytes
// wide and four times as many).
//
// What the epilogues of one feature tile read from memory, for all RM row tiles of a wavefront. The compiler cannot move
// a load across the epilogue's stores (they might alias), so loads issued tile by tile would each wait out a memory
// latency in turn; instead the batch of the next feature tile is requested before the current one is stored.
template <int EPI, int RM>
struct PrefillEpilogueBatch {
    f32x4 gain;           // kEpiResid: the next norm's gains of the lane's four features
    f32x4 resid[RM];      // kEpiResid: the residual values of those features in the lane's row of each row tile
    f32x4 rope[RM][2];    // kEpiQkv: (cos, sin) x 4 of the lane's four rotary pairs at its rows' positions (q and k tiles)
};

template <int EPI, int RM>
__device__ __forceinline__ void prefill_epilogue_fetch(const PrefillGemmArgs& p, int rt0, int tile, int n_tiles, int lane,
                                                       PrefillEpilogueBatch<EPI, RM>& b) {
    const GemmArgs& g = p.g;
    const int f0 = (lane >> 4) * 4, col0 = tile * 16 + f0;
    const bool there = tile < n_tiles;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f}, one = {1.f, 1.f, 1.f, 1.f};
    if constexpr (EPI == kEpiResid) b.gain = g.next_gain && there ? *reinterpret_cast<const f32x4*>(g.next_gain + col0) : one;
#pragma unroll
    for (int i = 0; i < RM; ++i) {
        const int row = (rt0 + i) * 16 + (lane & 15);
        const bool live = row < g.n_rows;
        if constexpr (EPI == kEpiResid)
            b.resid[i] = live && there ? *reinterpret_cast<const f32x4*>(g.resid + (size_t)row * g.ldr + col0) : zero;
        if constexpr (EPI == kEpiQkv) {
            const QkvOut& o = g.qkv;
            const int HALF = o.head_dim >> 1, tph = o.head_dim >> 4;
            // a q or k tile starts a whole number of heads after its matrix's first tile; pairs e0 .. e0 + 3
            const int tl = tile - (tile < g.tile_end[0] ? 0 : g.tile_end[0]);
            const int e0 = (tl % tph) * 8 + (f0 & 7);
            const f32x4* cs = reinterpret_cast<const f32x4*>(o.rope + (size_t)(o.pos0 + row) * HALF + e0);
            const bool rotated = live && tile < g.tile_end[1];
            b.rope[i][0] = rotated ? cs[0] : zero;
            b.rope[i][1] = rotated ? cs[1] : zero;
        }
    }
}

// One finished accumulator tile (row tile rt, feature tile `tile`), lane layout as described above. Every lane runs the
// same shuffles; only stores are predicated. resid / gain / rope: the lane's entries of PrefillEpilogueBatch for this tile.
template <int EPI>
__device__ __forceinline__ void prefill_epilogue(const PrefillGemmArgs& p, int rt, int tile, int lane, const f32x4& acc,
                                                 float rstd, const f32x4& resid, const f32x4& gain, const f32x4 (&rope)[2]) {
    const GemmArgs& g = p.g;
    const int row = rt * 16 + (lane & 15), f0 = (lane >> 4) * 4, col0 = tile * 16 + f0;
    const bool live = row < g.n_rows;
    if constexpr (EPI == kEpiQkv) {
        const QkvOut& o = g.qkv;
        const int HD = o.head_dim, HALF = HD >> 1, tph = HD >> 4, KK = HD >> 5;
        const int G = o.n_heads / o.n_kv_heads;
        const int which = tile < g.tile_end[0] ? 0 : (tile < g.tile_end[1] ? 1 : 2);
        const int tl = tile - (which == 0 ? 0 : (which == 1 ? g.tile_end[0] : g.tile_end[1]));
        const int head = tl / tph, u = tl % tph;
        // q / k tiles hold the rotary pairs (e, e + HALF), e = u*8 .. u*8 + 7: features 0..7 of the tile are the first
        // halves, features 8..15 their partners, i.e. the lane 32 further on holds this lane's partners
        const bool second = f0 >= 8;
        f32x4 own, partner;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            own[r] = acc[r] * rstd;
            partner[r] = __shfl_xor(own[r], 32);
        }
        if (!live) return;
        const int pos = o.pos0 + row;
        if (which == 2) {
            kv_t* vc = reinterpret_cast<kv_t*>(o.v_cache) + (size_t)head * o.t_max * HD;
#pragma unroll
            for (int r = 0; r < 4; ++r) vc[vfrag_offset(HD, pos, u * 16 + f0 + r)] = to_kv(own[r]);
            return;
        }
        typedef __attribute__((ext_vector_type(4))) _Float16 kvx4;
        const int x0 = u * 8 + (f0 & 7) + (second ? HALF : 0);  // four consecutive elements x0 .. x0 + 3 of the head
        const float scale = which == 0 ? o.q_scale : 1.0f;
        kvx4 out;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float cs = rope[r >> 1][(r & 1) * 2], sn = rope[r >> 1][(r & 1) * 2 + 1];
            out[r] = to_kv((own[r] * cs + (second ? partner[r] : -partner[r]) * sn) * scale);
        }
        if (which == 0) {
            // query index inside its KV head: row * G + head % G; g.R * G tiles of 16 queries per KV head
            const int kvh = head / G, qi = row * G + head % G;
            const size_t off = (((((size_t)kvh * (g.R * G) + (qi >> 4)) * KK + (x0 >> 5)) * 64) +
                                ((x0 >> 3) & 3) * 16 + (qi & 15)) * 8 + (x0 & 7);
            *reinterpret_cast<kvx4*>(reinterpret_cast<kv_t*>(o.q_frag) + off) = out;
        } else {
            kv_t* kc = reinterpret_cast<kv_t*>(o.k_cache) + (size_t)head * o.t_max * HD;
            *reinterpret_cast<kvx4*>(kc + kfrag_offset(HD, pos, x0)) = out;
        }
    } else if constexpr (EPI == kEpiPartial) {
        float* slab = g.out + (size_t)blockIdx.y * p.slab;
        if (live) *reinterpret_cast<f32x4*>(slab + (size_t)row * g.ldo + col0) = acc;
    } else if constexpr (EPI == kEpiResid) {
        const f32x4 v = live ? resid + acc : f32x4{0.f, 0.f, 0.f, 0.f};
        if (live) *reinterpret_cast<f32x4*>(g.out + (size_t)row * g.ldo + col0) = v;
        if (g.next_op) store_operand4_fmt(g.next_op, g.R, row, col0, v * gain, p.op_f16);  // rows that do not exist: zeros
        // sum of squares over the tile's 16 features: the lane's four, then the four lanes of the row
        float sq = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        sq += __shfl_xor(sq, 16);
        sq += __shfl_xor(sq, 32);
        if (g.next_ss && f0 == 0 && live) g.next_ss[(size_t)tile * p.ld_ss + row] = sq;
    } else {  // kEpiSwiglu: features 0..7 of a tile are gate features 8*tile .., features 8..15 the matching up features
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float own = acc[r] * rstd;  // 0 for a row that does not exist
            const float up = __shfl_xor(own, 32);
            v[r] = live ? own / (1.0f + expf(-own)) * up : 0.f;
        }
        if (f0 < 8) store_operand4_fmt(g.next_op, g.R, row, tile * 8 + f0, v, p.op_f16);
    }
}

// All accumulator tiles of a wavefront: row tiles rt0 .. rt0 + RM - 1 (those below g.R) x feature tiles tile0 ..
// tile0 + RN - 1 (those below n_tiles), feature tile by feature tile, the next one's inputs in flight meanwhile.
template <int EPI, int RM, int RN>
__device__ __forceinline__ void prefill_epilogue_all(const PrefillGemmArgs& p, int rt0, int tile0, int n_tiles, int lane,
                                                     const f32x4 (&acc)[RM][RN]) {
    const GemmArgs& g = p.g;
    float rstd[RM];  // 1/rms of the lane's row in each row tile (projections that follow a norm), 0 for rows that do not exist
#pragma unroll
    for (int i = 0; i < RM; ++i) {
        const int row = (rt0 + i) * 16 + (lane & 15);
        rstd[i] = (EPI == kEpiQkv || EPI == kEpiSwiglu) && row < g.n_rows ? p.rstd[row] : 0.f;
    }
    // (the residual epilogue of the 256 x 256 tile, whose 32 accumulator tiles leave no room for a second batch of
    // 20 registers, fetches each feature tile's batch right before it is used)
    constexpr bool AHEAD = !(EPI == kEpiResid && RM * RN >= 32);
    PrefillEpilogueBatch<EPI, RM> batch[2];
    prefill_epilogue_fetch<EPI, RM>(p, rt0, tile0, n_tiles, lane, batch[0]);
#pragma unroll
    for (int j = 0; j < RN; ++j) {
        if (AHEAD && j + 1 < RN) prefill_epilogue_fetch<EPI, RM>(p, rt0, tile0 + j + 1, n_tiles, lane, batch[(j + 1) & 1]);
        if (!AHEAD && j > 0) prefill_epilogue_fetch<EPI, RM>(p, rt0, tile0 + j, n_tiles, lane, batch[j & 1]);
        const PrefillEpilogueBatch<EPI, RM>& b = batch[j & 1];
        if (tile0 + j >= n_tiles) continue;
#pragma unroll
        for (int i = 0; i < RM; ++i)
            if (rt0 + i < g.R) prefill_epilogue<EPI>(p, rt0 + i, tile0 + j, lane, acc[i][j], rstd[i], b.resid[i], b.gain, b.rope[i]);
    }
}

constexpr int kPrefillRM = 4;                      // 16-row tiles per wavefront (2 in the small-tile variant)
constexpr int kPrefillRows = 2 * kPrefillRM * 16;  // rows of the 128-row workgroup tile; chunk sizes are multiples of it

// D = k-steps a stage is requested ahead of its use (register sets in flight); D + 1 LDS stages
template <int RM, int RN, int D, bool F16 = false>
constexpr size_t prefill_gemm_lds_bytes() {
    return (size_t)(D + 1) * (2 * (F16 ? 1 : 2) * RM + 2 * RN) * 1024;
}

// acc += (activation fragment a) x (weight fragment b) on the matrix cores, operands bf16 or fp16 as the pass runs
template <bool F16>
__device__ __forceinline__ f32x4 prefill_mma(const u32x4& a, const u32x4& b, const f32x4& acc) {
    // weights first: the tile comes out as D[feature][row] (see the epilogue)
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, b), __builtin_bit_cast(f16x8, a), acc, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(b), as_bf16x8(a), acc, 0, 0, 0);
}

// Workgroup = 2 x 2 wavefronts; wavefront (wm, wn) accumulates row tiles wm*RM .. +RM-1 times feature tiles wn*RN ..
// +RN-1 of the workgroup tile (RM = 4: 128 rows; RM = 2: 64 rows, for passes so short that 128-row tiles would leave
// CUs without a workgroup). Per k-step the workgroup stages 4*RM activation fragments (row tiles x hi/lo) and 2*RN weight
// fragments of 1 KiB each: requested into registers at the top of a k-step, written to a free LDS stage after the
// MFMAs of the D-th k-step from there (D register sets alternate, D + 1 LDS stages), one barrier per k-step. Two
// workgroups share a CU (<= 256 registers per lane, <= 80 KiB of LDS each), so one computes while the other waits for
// LDS, memory or its barrier; WPS = wavefronts per SIMD the register budget is cut for (3 with RN = 4, D = 1: 48 KiB of
// LDS and 152 registers, three workgroups per CU).
// Workgroups are numbered so that the ones resident on an XCD at the same time share weight columns: the XCD's L2
// then sees each weight fragment from HBM once and serves the sibling row blocks.
template <int EPI, int RM, int RN, int D, int WPS, bool F16 = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPS, WPS))) void prefill_gemm_kernel(PrefillGemmArgs p) {
    constexpr int NSTAGE = D + 1, ROWS = 2 * RM * 16;
    constexpr int NP = F16 ? 1 : 2;  // planes of an activation fragment: fp16, or bf16 hi + lo
    constexpr int A_FR = 2 * NP * RM, B_FR = 2 * RN, FR = A_FR + B_FR, NL = FR / 4;
    static_assert(FR % 4 == 0 && (D == 1 || D == 2), "fragments are dealt to four wavefronts");
    extern __shared__ u32x4 prefill_lds[];  // [NSTAGE][FR][64]
    const GemmArgs& g = p.g;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, wm = w >> 1, wn = w & 1;
    const int KS_all = g.K >> 5, n_tiles = g.N >> 4;
    // this workgroup's slice of the contraction (all of it unless gridDim.y > 1)
    const int ks0 = (int)(((long long)KS_all * blockIdx.y) / gridDim.y), KS = (int)(((long long)KS_all * (blockIdx.y + 1)) / gridDim.y) - ks0;
    const int nrb = (g.R * 16 + ROWS - 1) / ROWS, ncb = (n_tiles + B_FR - 1) / B_FR;
    // block id -> (row block, column block): ids congruent mod 8 run on one XCD; give each XCD a contiguous range
    const int total = nrb * ncb, per_xcd = (total + 7) >> 3;
    const int pid = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (pid >= total) return;
    const int rb = pid % nrb, cb = pid / nrb;

    // loader role: fragments w, w + 4, .. of the stage
    const u32x4* src[NL];
    size_t step[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const int f = w + 4 * j;
        if (f < A_FR) {  // activation fragment: row tile f/NP, plane f%NP; fetched in the order the MFMA lanes want it
            const int rg = min(rb * (2 * RM) + f / NP, g.R - 1);
            // bf16 planes are row-major (lane q*16 + r takes row r, 16-byte piece q); the fp16 plane is in lane order
            src[j] = reinterpret_cast<const u32x4*>(g.A) + ((size_t)rg * NP + f % NP) * 64 +
                     (F16 ? lane : (lane & 15) * 4 + (lane >> 4));
            step[j] = (size_t)g.R * NP * 64;
        } else {
            const int tile = min(cb * B_FR + (f - A_FR), n_tiles - 1);
            int mi = 0, tl = tile;
            if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
            if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
            src[j] = reinterpret_cast<const u32x4*>(g.W[mi]) + (size_t)tl * KS_all * 64 + lane;
            step[j] = 64;
        }
        src[j] += (size_t)ks0 * step[j];
    }
    auto issue = [&](u32x4 (&r)[NL]) {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            r[j] = *src[j];
            src[j] += step[j];
        }
    };
    auto commit = [&](const u32x4 (&r)[NL], int buf) {
#pragma unroll
        for (int j = 0; j < NL; ++j) prefill_lds[((size_t)buf * FR + (w + 4 * j)) * 64 + lane] = r[j];
    };

    f32x4 acc[RM][RN];
#pragma unroll
    for (int i = 0; i < RM; ++i)
#pragma unroll
        for (int j = 0; j < RN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](int buf) {
        const u32x4* L = prefill_lds + (size_t)buf * FR * 64 + lane;
        u32x4 bf[RN];
#pragma unroll
        for (int j = 0; j < RN; ++j) bf[j] = L[(A_FR + wn * RN + j) * 64];
        // the next row tile's fragment(s) are requested before this tile's MFMAs are issued (the scheduling fences
        // keep the compiler from sinking the reads below them): LDS latency hides behind the MFMAs
        u32x4 a[NP];
#pragma unroll
        for (int h = 0; h < NP; ++h) a[h] = L[(wm * RM * NP + h) * 64];
#pragma unroll
        for (int i = 0; i < RM; ++i) {
            u32x4 c[NP];
#pragma unroll
            for (int h = 0; h < NP; ++h) c[h] = a[h];
            if (i + 1 < RM) {
#pragma unroll
                for (int h = 0; h < NP; ++h) a[h] = L[((wm * RM + i + 1) * NP + h) * 64];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < NP; ++h)
#pragma unroll
                for (int j = 0; j < RN; ++j) acc[i][j] = prefill_mma<F16>(c[h], bf[j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // stage s is requested at the top of k-step s - D, committed to LDS stage s % (D + 1) after the MFMAs of k-step
    // s - 1 (the barrier that ended k-step s - 2 freed that stage) and consumed in k-step s
    u32x4 r0[NL], r1[D == 2 ? NL : 1];
    issue(r0);
    commit(r0, 0);
    if constexpr (D == 1) {
        __syncthreads();
        for (int s = 0; s < KS; ++s) {
            if (s + 1 < KS) issue(r0);
            compute(s & 1);
            if (s + 1 < KS) commit(r0, (s + 1) & 1);
            __syncthreads();
        }
    } else {
        if (KS > 1) issue(r0);  // stage 1
        __syncthreads();
        int buf = 0;
        auto iteration = [&](int s, u32x4 (&cur)[NL], u32x4 (&nxt)[NL]) {  // cur holds stage s + 1, nxt is free
            if (s + 2 < KS) issue(nxt);
            compute(buf);
            buf = buf == NSTAGE - 1 ? 0 : buf + 1;
            if (s + 1 < KS) commit(cur, buf);
            __syncthreads();
        };
        for (int s = 0; s < KS; s += 2) {
            iteration(s, r0, r1);
            if (s + 1 < KS) iteration(s + 1, r1, r0);
        }
    }

    prefill_epilogue_all<EPI, RM, RN>(p, rb * (2 * RM) + wm * RM, cb * B_FR + wn * RN, n_tiles, lane, acc);
}

// Sum of the k_split slices a split contraction left behind, in slice order, plus the residual epilogue (output, next
// operand, sum-of-squares partials). Grid (rows, ceil(N / 256)), one column per thread.
__global__ __launch_bounds__(256) void prefill_reduce_kernel(PrefillGemmArgs p, const float* parts) {
    const GemmArgs& g = p.g;
    const int row = blockIdx.x, c = blockIdx.y * 256 + threadIdx.x;
    if (c >= g.N) return;  // N % 16 == 0: a 16-column tile is all in or out
    float v = g.resid[(size_t)row * g.ldr + c];
    for (int s = 0; s < p.k_split; ++s) v += parts[(size_t)s * p.slab + (size_t)row * g.ldo + c];
    g.out[(size_t)row * g.ldo + c] = v;
    if (g.next_op) store_operand_fmt(g.next_op, g.R, row, c, v * (g.next_gain ? g.next_gain[c] : 1.0f), p.op_f16);
    const float sq = sum16(v * v);
    if (g.next_ss && (c & 15) == 0) g.next_ss[(size_t)(c >> 4) * p.ld_ss + row] = sq;
}

// ---- 256 x 256 tile fed by direct global -> LDS loads ---------------------------------------------------------------
// What binds the kernel above is operand delivery: a 128 x 256 tile pulls 32 KiB per k-step through L2 for 4 MFLOP, most
// of it with Infinity-Cache / HBM latency, and registers + LDS keep only one or two k-steps in flight. Here a workgroup
// of 4 x 2 wavefronts (64 x 128 accumulators each) owns a 256 x 256 tile (48 KiB per k-step for 8 MFLOP), and the
// fragments go straight from global memory into a ring of three LDS stages with global_load_lds_dwordx4 (per lane a
// global address, destination = wave-uniform LDS base + lane * 16, which is exactly a fragment): no staging registers,
// two k-steps (96 KiB per CU) in flight while the third is consumed. The loads are written as inline assembly
// because their completion has to be awaited stage by stage (s_waitcnt vmcnt(N): the N loads of the later stages may
// stay in flight); nothing else in the loop touches global memory, and the counter is drained before the epilogue.
// (The same loop on 32 x 32 x 16 MFMAs, whose operands a lane can gather from two neighbouring fragments, measured 12 %
// slower.)
// With fp16 operands a k-step is 16 + 16 fragments (32 KiB) and the ring has four stages: one being read into registers
// a k-step ahead of its MFMAs, three in flight (see the loop).
constexpr int kPrefillBigRows = 256;
#ifndef CLASP_PREFILL_GROUP_ROWS
#define CLASP_PREFILL_GROUP_ROWS 4
#endif
#ifndef CLASP_PREFILL_REGPIPE
#define CLASP_PREFILL_REGPIPE 1
#endif
#ifndef CLASP_PREFILL_F16_STAGES
#define CLASP_PREFILL_F16_STAGES 4
#endif
template <bool F16>
constexpr int prefill_big_stages() { return F16 ? CLASP_PREFILL_F16_STAGES : 3; }
// RN = feature tiles per wavefront: 8 (256 columns per workgroup) or 6 (192 columns: the q/k/v projection, whose 384
// feature tiles make 512 workgroups = two full rounds of CUs that way, and whose epilogue needs the registers)
template <bool F16, int RN = 8>
constexpr int prefill_big_frags() {  // activation + weight fragments per k-step, padded to eight wavefronts' equal shares
    return (4 * kPrefillRM * (F16 ? 1 : 2) + 2 * RN + 7) / 8 * 8;
}
template <bool F16, int RN = 8>
constexpr size_t prefill_big_lds() { return (size_t)prefill_big_stages<F16>() * prefill_big_frags<F16, RN>() * 1024; }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // all but the newest N vector-memory operations of this wavefront are done
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// ... all but the newest `stages` (0..4, wave-uniform) groups of NL operations
template <int NL>
__device__ __forceinline__ void wait_all_but_stages(int stages) {
    static_assert(4 * NL < 64, "the counter has six bits");
    if (stages >= 4) wait_vmcnt<4 * NL>();
    else if (stages == 3) wait_vmcnt<3 * NL>();
    else if (stages == 2) wait_vmcnt<2 * NL>();
    else if (stages == 1) wait_vmcnt<NL>();
    else wait_vmcnt<0>();
}

// lds_byte_addr must be the same in every lane (the hardware takes it from M0, a reserved register that the compiler
// sets itself before each of its own uses); lane l's 16 bytes land at + l * 16.
__device__ __forceinline__ void load_to_lds_16(const u32x4* g, unsigned lds_byte_addr) {
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(g) : "memory");
}

// The same with the global address split into a wave-uniform base (a scalar register pair, advanced with scalar
// arithmetic) and a 32-bit byte offset per lane.
__device__ __forceinline__ void load_to_lds_16(const void* uniform_base, unsigned lane_offset, unsigned lds_byte_addr) {
    const uintptr_t b = reinterpret_cast<uintptr_t>(uniform_base);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b), hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
    const unsigned long long sb = ((unsigned long long)hi << 32) | lo;
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(base), "v"(lane_offset), "s"(sb) : "memory");
}

template <int EPI, bool F16 = false, int RN = 8>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_gemm256_kernel(PrefillGemmArgs p) {
    constexpr int NP = F16 ? 1 : 2;  // planes of an activation fragment: fp16, or bf16 hi + lo
    // FR: slots of a stage (1 KiB each); the last FR - A_FR - B_FR of them are padding that receives copies of the last
    // weight fragment, so that every wavefront issues the same number of loads per stage
    constexpr int RM = kPrefillRM, A_FR = 4 * RM * NP, B_FR = 2 * RN, FR = prefill_big_frags<F16, RN>(), NL = FR / 8;
    constexpr int NSTAGE = prefill_big_stages<F16>(), AHEAD = NSTAGE - 1;
    static_assert(FR >= A_FR + B_FR && FR % 8 == 0, "fragments are dealt to eight wavefronts");
    static_assert((F16 && CLASP_PREFILL_REGPIPE) || AHEAD == 2 || AHEAD == 3,
                  "the waits of the plain loop are written out for two or three stages in flight");
    extern __shared__ u32x4 prefill_lds[];  // [NSTAGE][FR][64]
    const GemmArgs& g = p.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w >> 1, wn = w & 1;
    const int KS = g.K >> 5, n_tiles = g.N >> 4;
    const int nrb = (g.R * 16 + kPrefillBigRows - 1) / kPrefillBigRows, ncb = (n_tiles + B_FR - 1) / B_FR;
    const int total = nrb * ncb, per_xcd = (total + 7) >> 3;
    const int pid = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (pid >= total) return;
    // consecutive ids walk the row blocks of a group of GR first, then the column blocks: the workgroups an XCD runs at
    // the same time then cover GR x (32 / GR) tiles and share GR + 32 / GR operand panels in its L2
    constexpr int GR = CLASP_PREFILL_GROUP_ROWS;
    const int grp = pid / (GR * ncb), in_grp = pid - grp * (GR * ncb), rows_grp = min(GR, nrb - grp * GR);
    const int rb = grp * GR + in_grp % rows_grp, cb = in_grp / rows_grp;

    // this wavefront's fragments w, w + 8, .. of a stage: a wave-uniform address each (kept in scalar registers) plus
    // one of two per-lane offsets (activation fragments are fetched in the order the MFMA lanes want them)
    static_assert(A_FR % 8 == 0, "a wavefront's j-th fragment is an activation fragment in all wavefronts or in none");
    const char* src[NL];
    size_t step[NL];
    // bf16 planes are row-major (lane q*16 + r takes row r, 16-byte piece q); the fp16 plane is in lane order
    const unsigned lane_off_b = (unsigned)lane * 16;
    const unsigned lane_off_a = F16 ? lane_off_b : (unsigned)((lane & 15) * 4 + (lane >> 4)) * 16;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
        const int f = w + 8 * j;
        if (f < A_FR) {
            const int rg = min(rb * (A_FR / NP) + f / NP, g.R - 1);
            src[j] = reinterpret_cast<const char*>(g.A) + ((size_t)rg * NP + f % NP) * 1024;
            step[j] = (size_t)g.R * NP * 1024;
        } else {
            const int tile = min(cb * B_FR + min(f - A_FR, B_FR - 1), n_tiles - 1);
            int mi = 0, tl = tile;
            if (tile >= g.tile_end[0]) { mi = 1; tl = tile - g.tile_end[0]; }
            if (tile >= g.tile_end[1]) { mi = 2; tl = tile - g.tile_end[1]; }
            src[j] = reinterpret_cast<const char*>(g.W[mi]) + (size_t)tl * KS * 1024;
            step[j] = 1024;
        }
    }
    const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)prefill_lds);
    auto issue = [&](int buf) {  // this wavefront's NL fragments of the next stage in line
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            load_to_lds_16(src[j], 8 * j < A_FR ? lane_off_a : lane_off_b, lds_base + (unsigned)((buf * FR + w + 8 * j) * 1024));
            src[j] += step[j];
        }
    };

    f32x4 acc[RM][RN];
#pragma unroll
    for (int i = 0; i < RM; ++i)
#pragma unroll
        for (int j = 0; j < RN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](int buf) {
        const u32x4* L = prefill_lds + (size_t)buf * FR * 64 + lane;
        u32x4 bf[RN];
#pragma unroll
        for (int j = 0; j < RN; ++j) bf[j] = L[(A_FR + wn * RN + j) * 64];
        u32x4 a[NP];
#pragma unroll
        for (int h = 0; h < NP; ++h) a[h] = L[(wm * RM * NP + h) * 64];
#pragma unroll
        for (int i = 0; i < RM; ++i) {
            u32x4 c[NP];
#pragma unroll
            for (int h = 0; h < NP; ++h) c[h] = a[h];
            if (i + 1 < RM) {
#pragma unroll
                for (int h = 0; h < NP; ++h) a[h] = L[((wm * RM + i + 1) * NP + h) * 64];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < NP; ++h)
#pragma unroll
                for (int j = 0; j < RN; ++j) acc[i][j] = prefill_mma<F16>(c[h], bf[j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if constexpr (F16 && CLASP_PREFILL_REGPIPE) {
        // fp16 operands leave room for a second set of fragment registers: the fragments of stage s + 1 are read from
        // LDS while the MFMAs of stage s run from registers, so LDS reads and matrix cores overlap inside a wavefront
        // instead of alternating in lockstep across the workgroup behind the barrier. A stage's LDS slot is free once
        // every wavefront holds it in registers (the barrier of the k-step that multiplies it), so all NSTAGE slots
        // are in use: one being read, the others in flight.
        static_assert(NSTAGE >= 3 && NSTAGE <= 5, "wait_all_but_stages handles up to four stages in flight");
        u32x4 a0[RM], b0[RN], a1[RM], b1[RN];
        auto fetch = [&](int buf, u32x4 (&a)[RM], u32x4 (&b)[RN]) {
            const u32x4* L = prefill_lds + (size_t)buf * FR * 64 + lane;
#pragma unroll
            for (int j = 0; j < RN; ++j) b[j] = L[(A_FR + wn * RN + j) * 64];
#pragma unroll
            for (int i = 0; i < RM; ++i) a[i] = L[(wm * RM + i) * 64];
        };
#pragma unroll
        for (int t = 0; t < NSTAGE; ++t)
            if (t < KS) issue(t);
        wait_all_but_stages<NL>(min(KS, NSTAGE) - 1);  // own loads of stage 0 have landed
        __syncthreads();
        fetch(0, a0, b0);
        int buf = 0;  // LDS slot of stage s
        auto mma = [&](const u32x4 (&a)[RM], const u32x4 (&b)[RN]) {
#pragma unroll
            for (int i = 0; i < RM; ++i)
#pragma unroll
                for (int j = 0; j < RN; ++j) acc[i][j] = prefill_mma<true>(a[i], b[j], acc[i][j]);
        };
        // k-step s < KS - 1: stage s + 1 goes to the other register set while stage s is multiplied. Every path through
        // it reads before it multiplies: a k-step that could skip the reads would make the compiler wait for them in
        // front of the MFMAs on the common path as well (the wait counters are merged where paths meet).
        auto kstep = [&](int s, const u32x4 (&ca)[RM], const u32x4 (&cb_)[RN], u32x4 (&na)[RM], u32x4 (&nb)[RN]) {
            const int later = KS - 1 - s;
            // own loads of stage s + 1 have landed; stages s + 2 .. s + NSTAGE - 1 (where they exist) may stay in flight
            wait_all_but_stages<NL>(min(later - 1, NSTAGE - 2));
            __syncthreads();  // everybody's have, and every wavefront has stage s in registers
            if (s + NSTAGE < KS) issue(buf);
            buf = buf == NSTAGE - 1 ? 0 : buf + 1;
            // the RM + RN reads of stage s + 1 are spread between the RM * RN MFMAs of stage s (two or three MFMAs after
            // each read, pinned by scheduling fences): issued in one burst by all eight wavefronts after the barrier they
            // would fill the LDS queue, and a wavefront whose read is not accepted cannot issue the MFMAs behind it
            const u32x4* L = prefill_lds + (size_t)buf * FR * 64 + lane;
            constexpr int NR = RM + RN, NM = RM * RN;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NR; ++t) {
                if (t < RN) nb[t] = L[(A_FR + wn * RN + t) * 64];
                else na[t - RN] = L[(wm * RM + t - RN) * 64];
#pragma unroll
                for (int m = t * NM / NR; m < (t + 1) * NM / NR; ++m)
                    acc[m / RN][m % RN] = prefill_mma<true>(ca[m / RN], cb_[m % RN], acc[m / RN][m % RN]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // KS is even (the launcher sends other contractions to the smaller tiles): pairs of k-steps alternate the two
        // register sets, and the last pair ends without a read
        for (int s = 0; s + 2 < KS; s += 2) {
            kstep(s, a0, b0, a1, b1);
            kstep(s + 1, a1, b1, a0, b0);
        }
        kstep(KS - 2, a0, b0, a1, b1);
        mma(a1, b1);
    } else {
    // stage s lives in LDS stage s % NSTAGE; it is requested AHEAD k-steps before its use, right after the barrier that
    // tells that every wavefront has finished reading the stage it replaces
#pragma unroll
    for (int t = 0; t < AHEAD; ++t)
        if (t < KS) issue(t);
    int buf = 0;
    for (int s = 0; s < KS; ++s) {
        // own loads of stage s have landed: the stages requested after it (at most AHEAD - 1, fewer at the end) may
        // stay in flight
        const int later = KS - 1 - s;
        if (later >= AHEAD - 1) wait_vmcnt<(AHEAD - 1) * NL>();
        else if (AHEAD == 3 && later == 1) wait_vmcnt<NL>();
        else wait_vmcnt<0>();
        __syncthreads();  // everybody's have, and stage s - 1 is no longer read
        if (s + AHEAD < KS) issue(buf == 0 ? NSTAGE - 1 : buf - 1);  // (s + AHEAD) % NSTAGE
        compute(buf);
        buf = buf == NSTAGE - 1 ? 0 : buf + 1;
    }
    }
    wait_vmcnt<0>();
    // nothing of the epilogue is scheduled into the last k-steps, where both fragment sets and all accumulators are live
    __builtin_amdgcn_sched_barrier(0);
    prefill_epilogue_all<EPI, RM, RN>(p, rb * (A_FR / NP) + wm * RM, cb * B_FR + wn * RN, n_tiles, lane, acc);
}
// ---- weights of one layer as fp16 ------------------------------------------------------------------------------------
// Element-wise bf16 -> fp16 of up to six packed matrices (fragment order is kept: the copy is read exactly like the
// original). Exact for every weight of magnitude >= 2^-17; smaller ones round to the fp16 subnormal grid (2^-24).
struct ConvertArgs {
    const u32x4* src[6];
    u32x4* dst[6];
    size_t end[6];  // running total of 16-byte units after each matrix
};

__global__ __launch_bounds__(256) void prefill_convert_f16_kernel(ConvertArgs c) {
    const size_t total = c.end[5];
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const u32x4* sp = c.src[0];
        u32x4* dp = c.dst[0];
        size_t first = 0;
#pragma unroll
        for (int k = 1; k < 6; ++k)
            if (i >= c.end[k - 1]) { sp = c.src[k]; dp = c.dst[k]; first = c.end[k - 1]; }
        const size_t j = i - first;
        const u32x4 v = __builtin_nontemporal_load(sp + j);
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const f16 a = (f16)__uint_as_float(v[e] << 16), b = (f16)__uint_as_float(v[e] & 0xffff0000u);
            o[e] = (unsigned)__builtin_bit_cast(unsigned short, a) | ((unsigned)__builtin_bit_cast(unsigned short, b) << 16);
        }
        dp[j] = o;
    }
}

// ---- causal attention over the cache for a chunk of rows ----------------------------------------------------------
struct PrefillAttnArgs {
    const void* q_frag;  // [n_kv_heads][R*G tiles][head_dim/32][64][8], rotated and scaled by the q/k/v epilogue
    const void* Kc;      // this layer's cache, fragment order; the chunk's own keys / values are already in it
    const void* Vt;
    void* out_op;        // operand of the output projection, R row groups
    int n_rows, R, n_heads, n_kv_heads, pos0, t_max;
    int op_f16;          // format of out_op, as PrefillGemmArgs::op_f16
};

constexpr int kPrefillAttnNT = 2, kPrefillAttnWaves = 4;

// Smallest cache position limit among a wavefront's queries (-1 if one of them does not exist): blocks that end at or
// below it are visible to all of them and need no masking.
template <int NT>
__device__ __forceinline__ int prefill_attn_min_limit(const int (&limit)[NT]) {
    int v = limit[0];
#pragma unroll
    for (int t = 1; t < NT; ++t) v = min(v, limit[t]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) v = min(v, __shfl_xor(v, off));
    return __builtin_amdgcn_readfirstlane(v);
}

// Grid (n_kv_heads, ceil(query tiles / 8)). Query qi = row * G + head % G of KV head kvh sees cache positions
// 0 .. pos0 + row.
template <int HD>
__global__ __launch_bounds__(kPrefillAttnWaves * 64) void prefill_attn_kernel(PrefillAttnArgs a) {
    constexpr int NT = kPrefillAttnNT, KK = HD / 32, CT = HD / 16;
    const int kvh = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int G = a.n_heads / a.n_kv_heads, nQ = a.n_rows * G, n_qt = a.R * G;
    // workgroups are handed out in blockIdx order: the last queries (most keys) go first, so that the CUs that finish
    // early pick up the short ones
    const int t0 = ((int)(gridDim.y - 1 - blockIdx.y) * kPrefillAttnWaves + wave) * NT;  // first query tile of this wavefront
    if (t0 * 16 >= nQ) return;
    const int m16 = lane & 15, q4 = lane >> 4;

    kvx8 qf[NT][KK];
    int limit[NT];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(a.q_frag) + (size_t)kvh * n_qt * KK * 64 + lane;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int qt = min(t0 + t, n_qt - 1), qi = (t0 + t) * 16 + m16;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[t][kk] = as_kvx8(qp[((size_t)qt * KK + kk) * 64]);
            limit[t] = qi < nQ ? a.pos0 + qi / G : -1;
        }
    }
    // last position any query of the wavefront sees (queries ascend with the tile index)
    const int last_q = min((t0 + NT) * 16, nQ) - 1;
    const int nblk = ((a.pos0 + last_q / G) >> 5) + 1;

    AttnState<HD, NT> st;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        st.m[t] = -INFINITY;
        st.l[t] = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) st.o[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const u32x4* Kh = reinterpret_cast<const u32x4*>(reinterpret_cast<const kv_t*>(a.Kc) + (size_t)kvh * a.t_max * HD) + lane;
    const u32x4* Vh = reinterpret_cast<const u32x4*>(reinterpret_cast<const kv_t*>(a.Vt) + (size_t)kvh * a.t_max * HD) + lane;
    auto load_blk = [&](AttnFrags<HD>& f, int blk) {
        const u32x4* kp = Kh + (size_t)blk * (2 * KK * 64);
        const u32x4* vp = Vh + (size_t)blk * (CT * 64);
        attn_load<HD>(f, [&](int u, int kk) { return as_kvx8(kp[(u * KK + kk) * 64]); },
                      [&](int c) { return as_kvx8(vp[c * 64]); });
    };
    const int min_limit = prefill_attn_min_limit<NT>(limit);
    auto compute_blk = [&](const AttnFrags<HD>& f, int blk) {
        const int kb = blk << 5;
        attn_compute<HD, NT>(st, qf, f, [&](int u, int r, int t) { return kb + q4 * 8 + u * 4 + r <= limit[t]; },
                             kb + 31 > min_limit);
    };
    AttnFrags<HD> f0, f1;
    load_blk(f0, 0);
    for (int blk = 0; blk < nblk; blk += 2) {
        if (blk + 1 < nblk) load_blk(f1, blk + 1);
        compute_blk(f0, blk);
        if (blk + 1 >= nblk) break;
        if (blk + 2 < nblk) load_blk(f0, blk + 2);
        compute_blk(f1, blk + 1);
    }

    // O^T tile: lane holds features c*16 + q4*4 + r of query m16
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float l = st.l[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int qi = (t0 + t) * 16 + m16;
        if (qi >= nQ) continue;
        const float inv = 1.0f / l;
        const int row = qi / G, h = kvh * G + qi % G;
#pragma unroll
        for (int c = 0; c < CT; ++c)
            store_operand4_fmt(a.out_op, a.R, row, h * HD + c * 16 + q4 * 4, st.o[t][c] * inv, a.op_f16);
    }
}

// ---- the same attention with the key / value blocks shared through LDS ----------------------------------------------
// In the kernel above every wavefront streams the whole visible prefix of its KV head from L2 for its 32 queries; at
// long prefixes that is what binds it (4096 rows x 32k tokens: 34 GB through L2 per layer). Here the NW wavefronts of a
// workgroup (NW x 32 queries) walk the prefix together: each 32-key block goes from global memory straight into a
// ring of eight LDS stages (global_load_lds_dwordx4, a quarter or an eighth of the block's fragments per wavefront,
// six blocks in flight) and every wavefront reads its fragments from there, one block ahead of the one it multiplies.
// One barrier per block; the ring is kept full to the end by re-requesting the last block, so the number of loads
// to wait for is the same in every step.
constexpr int kPrefillAttnStages = 8;

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64) void prefill_attn_lds_kernel(PrefillAttnArgs a) {
    constexpr int NT = kPrefillAttnNT, KK = HD / 32, CT = HD / 16, FRB = 2 * KK + CT, PER = FRB / NW;
    constexpr int NSTAGE = kPrefillAttnStages;
    static_assert(FRB % NW == 0 && (NSTAGE - 2) * PER <= 63, "loads per wavefront and block; vmcnt holds 6 bits");
    extern __shared__ u32x4 attn_lds[];  // [NSTAGE][FRB][64]
    const int kvh = blockIdx.x, lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int G = a.n_heads / a.n_kv_heads, nQ = a.n_rows * G, n_qt = a.R * G;
    // workgroups are handed out in blockIdx order: the last queries (most keys) go first, so that the CUs that finish
    // early pick up the short ones
    const int t_wg = (int)(gridDim.y - 1 - blockIdx.y) * NW * NT;  // first query tile of the workgroup
    if (t_wg * 16 >= nQ) return;
    const int t0 = t_wg + wave * NT;
    const int m16 = lane & 15, q4 = lane >> 4;

    kvx8 qf[NT][KK];
    int limit[NT];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(a.q_frag) + (size_t)kvh * n_qt * KK * 64 + lane;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int qt = min(t0 + t, n_qt - 1), qi = (t0 + t) * 16 + m16;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[t][kk] = as_kvx8(qp[((size_t)qt * KK + kk) * 64]);
            limit[t] = qi < nQ ? a.pos0 + qi / G : -1;
        }
    }
    // blocks any query of the workgroup sees (queries ascend with the tile index)
    const int last_q = min((t_wg + NW * NT) * 16, nQ) - 1;
    const int nblk = ((a.pos0 + last_q / G) >> 5) + 1;

    AttnState<HD, NT> st;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        st.m[t] = -INFINITY;
        st.l[t] = 0.f;
#pragma unroll
        for (int c = 0; c < CT; ++c) st.o[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const u32x4* Kh = reinterpret_cast<const u32x4*>(reinterpret_cast<const kv_t*>(a.Kc) + (size_t)kvh * a.t_max * HD) + lane;
    const u32x4* Vh = reinterpret_cast<const u32x4*>(reinterpret_cast<const kv_t*>(a.Vt) + (size_t)kvh * a.t_max * HD) + lane;
    const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) char*)attn_lds);
    auto issue = [&](int blk, int stage) {  // this wavefront's PER fragments of block min(blk, nblk - 1)
        const int b = min(blk, nblk - 1);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int f = wave + NW * j;  // fragments 0 .. 2*KK-1: keys, then values
            const u32x4* src = f < 2 * KK ? Kh + ((size_t)b * (2 * KK) + f) * 64 : Vh + ((size_t)b * CT + (f - 2 * KK)) * 64;
            load_to_lds_16(src, lds_base + (unsigned)((stage * FRB + f) * 1024));
        }
    };
    // Software pipeline of a wavefront over the blocks (step b, after the barrier that tells that blocks <= b + 2 are
    // complete in LDS and that nobody reads the slot of block b - 1 any more):
    //   scores of block b + 1 (MFMAs; its keys were read from LDS during step b - 1)
    //   values of block b: LDS -> registers (needed at the end of this step)
    //   softmax of block b's scores, computed in step b - 1 (vector work, while the MFMAs above execute)
    //   keys of block b + 2: LDS -> the key registers the MFMAs above have consumed
    //   O^T += V^T P^T of block b (MFMAs)
    // so that the matrix cores work on one block's scores while the vector units exponentiate the previous block's,
    // instead of the two taking turns. Blocks b + 3 .. b + NSTAGE - 1 are in flight (the newest requested right after
    // the barrier, into the slot of block b - 1). Blocks beyond the last are clamped copies of it: their loads keep the
    // counts constant, their scores are never used.
    static_assert(NSTAGE == 8, "five blocks in flight at the barrier");
    auto read_keys = [&](kvx8 (&k)[2][KK], int stage) {
        const u32x4* L = attn_lds + (size_t)stage * FRB * 64 + lane;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) k[u][kk] = as_kvx8(L[(u * KK + kk) * 64]);
    };
    auto read_values = [&](kvx8 (&v)[CT], int stage) {
        const u32x4* L = attn_lds + (size_t)stage * FRB * 64 + lane;
#pragma unroll
        for (int c = 0; c < CT; ++c) v[c] = as_kvx8(L[(2 * KK + c) * 64]);
    };
    auto next_stage = [&](int stage) { return stage == NSTAGE - 1 ? 0 : stage + 1; };
#pragma unroll 1
    for (int b = 0; b < NSTAGE - 1; ++b) issue(b, b);
    const int min_limit = prefill_attn_min_limit<NT>(limit);
    kvx8 kreg[2][KK], vreg[CT];
    f32x4 s0[2][NT], s1[2][NT];
    wait_vmcnt<(NSTAGE - 3) * PER>();  // blocks 0 and 1 have landed (own loads; the barrier covers the others')
    __syncthreads();
    read_keys(kreg, 0);
    attn_qk<HD, NT>(s0, qf, kreg);
    read_keys(kreg, 1);
    int stage = 0;  // of block blk
    auto step = [&](int blk, f32x4 (&s_cur)[2][NT], f32x4 (&s_nxt)[2][NT]) {
        wait_vmcnt<(NSTAGE - 4) * PER>();
        __syncthreads();
        issue(blk + NSTAGE - 1, stage == 0 ? NSTAGE - 1 : stage - 1);
        attn_qk<HD, NT>(s_nxt, qf, kreg);  // block blk + 1
        read_values(vreg, stage);
        const int kb = blk << 5;
        kvx8 pf[NT];
        attn_softmax<HD, NT>(st, s_cur, [&](int u, int r, int t) { return kb + q4 * 8 + u * 4 + r <= limit[t]; }, pf,
                             kb + 31 > min_limit);
        read_keys(kreg, next_stage(next_stage(stage)));  // block blk + 2
        attn_pv<HD, NT>(st, vreg, pf);
        stage = next_stage(stage);
    };
#pragma unroll 1
    for (int blk = 0; blk < nblk; blk += 2) {
        step(blk, s0, s1);
        if (blk + 1 < nblk) step(blk + 1, s1, s0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float l = st.l[t];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int qi = (t0 + t) * 16 + m16;
        if (qi >= nQ) continue;
        const float inv = 1.0f / l;
        const int row = qi / G, h = kvh * G + qi % G;
#pragma unroll
        for (int c = 0; c < CT; ++c)
            store_operand4_fmt(a.out_op, a.R, row, h * HD + c * 16 + q4 * 4, st.o[t][c] * inv, a.op_f16);
    }
}

}  // namespace clasp

