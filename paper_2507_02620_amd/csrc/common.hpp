// Shared device-side vocabulary of the stage kernels (gfx950 / CDNA4, wave64).
//
// MFMA operand convention used everywhere in this library ("fragment"): one 16 x KT tile of a
// row-major matrix, held as 16 bytes per lane.  Lane l = g*16 + r (r = l % 16, g = l / 16) holds
// row r, elements [g*EPF, g*EPF + EPF) of the tile's KT = 4*EPF columns.
//   bf16 : EPF = 8, KT = 32, one v_mfma_f32_16x16x32_bf16 per fragment pair
//   f32  : EPF = 4, KT = 16, four v_mfma_f32_16x16x4_f32 (element e of both fragments feeds MFMA e;
//          the contraction index is then g*4 + e on both sides, so the sum is the same)
// mma(A, B, C) computes C[i][j] += sum_k A[i][k] * B[j][k] for two fragments A (rows i) and B (rows j);
// the 16x16 fp32 result lives as 4 values per lane: lane l holds C[i = (l/16)*4 + v][j = l % 16], v = 0..3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define FS_WAVE 64
#define FS_ANC_WORDS 16 /* 64-bit words per ancestor-mask row: FS_MAX_TREE / 64 */

template <typename T>
struct Elem;

template <>
struct Elem<float> {
    using frag_t = f32x4;
    using out4_t = f32x4;
    static constexpr int EPF = 4;
    static constexpr int KT = 16;
    static __device__ __forceinline__ f32x4 mma(frag_t a, frag_t b, f32x4 c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ frag_t zero() { return frag_t{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ float sumsq(frag_t a) { return a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3]; }
    static __device__ __forceinline__ out4_t pack4(float a, float b, float c, float d) { return out4_t{a, b, c, d}; }
    static __device__ __forceinline__ float to_f(float v) { return v; }
    static __device__ __forceinline__ float from_f(float v) { return v; }
};

template <>
struct Elem<bf16_t> {
    using frag_t = bf16x8;
    using out4_t = bf16x4;
    static constexpr int EPF = 8;
    static constexpr int KT = 32;
    static __device__ __forceinline__ f32x4 mma(frag_t a, frag_t b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ frag_t zero() {
        frag_t z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.f;
        return z;
    }
    static __device__ __forceinline__ float sumsq(frag_t a) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float f = (float)a[e];
            s += f * f;
        }
        return s;
    }
    static __device__ __forceinline__ out4_t pack4(float a, float b, float c, float d) {
        return out4_t{(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
    }
    static __device__ __forceinline__ float to_f(bf16_t v) { return (float)v; }
    static __device__ __forceinline__ bf16_t from_f(float v) { return (bf16_t)v; }
};

// "Fragment-major" activation layout: the [rows][K] matrix is stored as [rows/16][K/KT][64 lanes][EPF], i.e.
// already in MFMA operand order, so that a consumer's fragment load is one contiguous KiB per wave (like the
// re-tiled weights) instead of sixteen 64-byte row pieces.  Producers write 4 consecutive columns per lane.
template <typename T>
static __device__ __forceinline__ size_t frag_major_index(int m, int k, int nkt) {
    using E = Elem<T>;
    return ((((size_t)(m >> 4) * nkt + k / E::KT) * 64) + ((k % E::KT) / E::EPF) * 16 + (m & 15)) * E::EPF + (k % E::EPF);
}

// Small index lists that travel as kernel arguments (no device allocation, no copy, capturable).
struct IdxList {
    int n;
    short v[1024];
};

// Direct-to-LDS loads (__builtin_amdgcn_global_load_lds) take address-space-qualified pointers; the LDS one is wave-uniform,
// the hardware adds lane * 16.
#define FS_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define FS_GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
// s_waitcnt immediate (gfx9 encoding): vmcnt = n (6 bits), lgkmcnt = l (4 bits: at most l LDS reads still in flight), expcnt untouched
#define FS_WAIT_VM_LGKM(n, l) __builtin_amdgcn_s_waitcnt(0x0070 | ((n) & 15) | (((n) >> 4) << 14) | ((l) << 8))

static __device__ __forceinline__ float wave_xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask, FS_WAVE)); }
static __device__ __forceinline__ float wave_xor_add(float v, int mask) { return v + __shfl_xor(v, mask, FS_WAVE); }
