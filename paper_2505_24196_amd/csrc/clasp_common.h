// Shared device-side definitions for the CLaSp gfx950 kernels: vector types, the bf16 MFMA operand ("fragment")
// layout that every producer writes and every GEMM reads, and small wavefront helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace clasp {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kMaxRows = 32;      // rows (tokens / DP candidates) one launch may carry
constexpr int kWave = 64;         // CDNA wavefront
constexpr int kDtF32 = 0, kDtBf16 = 1;

// ---- bf16 activation operand layout -----------------------------------------------------------------------
// An activation matrix X[rows <= 16*R][K] that a GEMM will contract over K is kept in HBM per k-step s (32
// consecutive k) and row group rg (16 rows) as two planes of 16 rows x 32 bf16, row-major: "hi" = round(x) and
// "lo" = round(x - hi). MFMA lane (q*16 + r) fetches X[rg*16 + r][s*32 + q*8 .. +8] of each plane with one 16-byte
// load and feeds it to v_mfma_f32_16x16x32_bf16 unchanged; lanes whose row does not exist fetch nothing, so the
// traffic follows the number of live rows. hi + lo carries 16 mantissa bits: the activations lose next to nothing
// against fp32 while the weights stay bf16.
__device__ __forceinline__ size_t frag_elem_offset(int R, int row, int k) {
    const int s = k >> 5, rg = row >> 4, r = row & 15;
    return ((((size_t)s * R + rg) * 2) * 16 + r) * 32 + (k & 31);  // hi plane; the lo plane sits 512 elements on
}
constexpr int kLoPlane = 512;

// ---- attention operand type (bf16 models) ---------------------------------------------------------------------
// Keys, values, queries and the softmax weights enter the attention MFMAs as fp16 (v_mfma_f32_16x16x32_f16, the rate
// of the bf16 instruction): 11 significant bits instead of bf16's 8 at the same 2 bytes per element, which is what keeps
// a 32-layer random-init model inside 2e-2 of an fp64 reference when the cache is the model's own (the paper's runs
// are FP16 throughout, Experiments). Conversions saturate at the largest finite fp16 number, so an outlier becomes
// +-65504 instead of an infinity that would turn a whole softmax row into NaN.
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef f16 kv_t;
typedef f16x8 kvx8;
__device__ __forceinline__ kv_t to_kv(float x) { return (kv_t)fminf(fmaxf(x, -65504.f), 65504.f); }
__device__ __forceinline__ float from_kv(kv_t x) { return (float)x; }
__device__ __forceinline__ kvx8 as_kvx8(u32x4 v) { return __builtin_bit_cast(kvx8, v); }
__device__ __forceinline__ f32x4 mfma_kv(kvx8 a, kvx8 b, f32x4 acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
}

// ---- KV cache layout (bf16 models; elements are kv_t) ------------------------------------------------------------
// Per KV head the cache is a sequence of 32-position blocks, each stored as the MFMA operand fragments the
// attention kernel consumes, so that every wavefront-wide load is one contiguous KiB (gathers of 64-byte row pieces
// cost this part several times more issue time than they move data):
//   K block: [u = 2 key tiles][kk = head_dim/32 k-steps][64 lanes][8]; lane q*16 + m of tile u holds
//            K[position 8*(m/4) + 4*u + m%4][kk*32 + q*8 .. +8]   (the two 16-key tiles interleave in groups of 4 so
//            that a lane's exponentiated scores are directly the 8-key fragment of the P.V product)
//   V block: [c = head_dim/16 feature tiles][64 lanes][8]; lane q*16 + m holds V[position q*8 .. +8][c*16 + m]
// Offsets are in elements from the head's base (head stride = t_max * head_dim).
__device__ __forceinline__ size_t kfrag_offset(int HD, int t, int x) {
    const int o = t & 31, u = (o >> 2) & 1, m = ((o >> 3) << 2) | (o & 3);
    return ((((size_t)(t >> 5) * 2 + u) * (HD >> 5) + (x >> 5)) * 64 + ((x >> 3) & 3) * 16 + m) * 8 + (x & 7);
}
__device__ __forceinline__ size_t vfrag_offset(int HD, int t, int x) {
    return ((((size_t)(t >> 5) * (HD >> 4) + (x >> 4)) * 64) + ((t >> 3) & 3) * 16 + (x & 15)) * 8 + (t & 7);
}

__device__ __forceinline__ bf16 to_bf16(float x) { return static_cast<bf16>(x); }  // round-to-nearest-even
__device__ __forceinline__ float from_bf16(bf16 x) { return static_cast<float>(x); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 as_u32x4(bf16x8 v) { return __builtin_bit_cast(u32x4, v); }

// Streaming (no-reuse) 16-byte load: weights and KV are read once per launch, keep them out of the way of the
// small activation working set that every workgroup re-reads from L2.
__device__ __forceinline__ u32x4 load_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }

// Sum over the 16 lanes that share lane/16 (xor butterflies stay inside the 16-lane row).
__device__ __forceinline__ float sum16(float v) {
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8);
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
    v = sum16(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// Deterministic block-wide sum (fixed tree): every thread gets the total. `scratch` holds >= blockDim/64 floats.
__device__ __forceinline__ float block_sum(float v, float* scratch) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < nw; ++w) t += scratch[w];
    return t;
}

// Store one activation element for a later GEMM: bf16 hi/lo fragment order, or fp32 row-major [row][ld].
template <int DT>
__device__ __forceinline__ void store_operand(void* buf, int R, int ld, int row, int k, float v) {
    if constexpr (DT == kDtBf16) {
        bf16* p = reinterpret_cast<bf16*>(buf) + frag_elem_offset(R, row, k);
        const bf16 hi = to_bf16(v);
        p[0] = hi;
        p[kLoPlane] = to_bf16(v - from_bf16(hi));
    } else {
        reinterpret_cast<float*>(buf)[(size_t)row * ld + k] = v;
    }
}

// Four consecutive elements k..k+3 (k % 4 == 0) of one row.
template <int DT>
__device__ __forceinline__ void store_operand4(void* buf, int R, int ld, int row, int k, f32x4 v) {
    if constexpr (DT == kDtBf16) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        bf16* p = reinterpret_cast<bf16*>(buf) + frag_elem_offset(R, row, k);
        bf16x4 hi, lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hi[i] = to_bf16(v[i]);
            lo[i] = to_bf16(v[i] - from_bf16(hi[i]));
        }
        *reinterpret_cast<bf16x4*>(p) = hi;
        *reinterpret_cast<bf16x4*>(p + kLoPlane) = lo;
    } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(buf) + (size_t)row * ld + k) = v;
    }
}

// ---- fp16 activation operand layout (prompt passes of many rows) ----------------------------------------------
// One KiB per (k-step, row group) holding 16 rows x 32 halves, a single fp16 value (11 significant bits) per element
// instead of the hi / lo pair, read by v_mfma_f32_16x16x32_f16 against weights converted to fp16 (every bf16 weight of
// magnitude >= 2^-17 is an fp16 number). Inside the KiB the order is the MFMA operand's own: lane q*16 + r owns the 16
// bytes X[rg*16 + r][s*32 + q*8 .. +8] at byte offset lane * 16, so a wavefront fetches a fragment with consecutive
// lanes on consecutive addresses, exactly like a weight fragment.
__device__ __forceinline__ size_t frag16_elem_offset(int R, int row, int k) {
    const int s = k >> 5, rg = row >> 4, r = row & 15, q = (k >> 3) & 3;
    return ((((size_t)s * R + rg) * 4 + q) * 16 + r) * 8 + (k & 7);
}

// Operand element in the format a prompt pass runs in: fp16 plane (f16 != 0) or the bf16 hi / lo planes.
__device__ __forceinline__ void store_operand_fmt(void* buf, int R, int row, int k, float v, int f16_plane) {
    if (f16_plane) reinterpret_cast<f16*>(buf)[frag16_elem_offset(R, row, k)] = to_kv(v);
    else store_operand<kDtBf16>(buf, R, 0, row, k, v);
}

__device__ __forceinline__ void store_operand4_fmt(void* buf, int R, int row, int k, f32x4 v, int f16_plane) {
    if (f16_plane) {
        typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
        f16x4 h;
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = to_kv(v[i]);
        *reinterpret_cast<f16x4*>(reinterpret_cast<f16*>(buf) + frag16_elem_offset(R, row, k)) = h;
    } else {
        store_operand4<kDtBf16>(buf, R, 0, row, k, v);
    }
}

}  // namespace clasp
