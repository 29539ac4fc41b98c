// Device helpers shared by the online kernels: 16-byte row loads dotted with a
// token held in LDS, and the token's int8 code.
#pragma once

#include "common.h"

// ------------------------------------------------------------------ row . x
// 16-byte vector of T and its dot product with a 16-byte vector of x.
template <typename T> struct RowVec;
template <> struct RowVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ float dot(const td_u32x4& w, const td_u32x4& x, float acc) {
        acc = fmaf(__uint_as_float(w.x), __uint_as_float(x.x), acc);
        acc = fmaf(__uint_as_float(w.y), __uint_as_float(x.y), acc);
        acc = fmaf(__uint_as_float(w.z), __uint_as_float(x.z), acc);
        acc = fmaf(__uint_as_float(w.w), __uint_as_float(x.w), acc);
        return acc;
    }
};
typedef __bf16 td_bf16x2 __attribute__((ext_vector_type(2)));

// acc + w.lo*x.lo + w.hi*x.hi on two packed bf16 pairs, fp32 accumulation (v_dot2_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t x, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(td_bf16x2, w), __builtin_bit_cast(td_bf16x2, x), acc,
                                           false);
}
template <> struct RowVec<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ float dot(const td_u32x4& w, const td_u32x4& x, float acc) {
        acc = dot2_bf16(w.x, x.x, acc);
        acc = dot2_bf16(w.y, x.y, acc);
        acc = dot2_bf16(w.z, x.z, acc);
        acc = dot2_bf16(w.w, x.w, acc);
        return acc;
    }
};

// R rows at once (their loads are independent, so they overlap in flight).
// rows[i] may be null for i past the end of the matrix; such rows return 0.
// xs points at n values of x (LDS or global).  Result valid in every lane.
template <typename T, int R>
__device__ __forceinline__ void rows_dot(const T* const (&rows)[R], const T* xs, int n, int lane,
                                         float (&out)[R]) {
    constexpr int V = RowVec<T>::N;
    float acc[R];
#pragma unroll
    for (int i = 0; i < R; ++i) acc[i] = 0.0f;
    if (n % V == 0) {
        const int nv = n / V;
        const td_u32x4* xv = reinterpret_cast<const td_u32x4*>(xs);
#pragma unroll 2
        for (int v = lane; v < nv; v += TD_WAVE) {
            td_u32x4 w[R];
#pragma unroll
            for (int i = 0; i < R; ++i)
                w[i] = rows[i] ? td_load_stream16(reinterpret_cast<const td_u32x4*>(rows[i]) + v)
                               : td_u32x4{0, 0, 0, 0};
            const td_u32x4 xx = xv[v];
#pragma unroll
            for (int i = 0; i < R; ++i) acc[i] = RowVec<T>::dot(w[i], xx, acc[i]);
        }
    } else {
        for (int k = lane; k < n; k += TD_WAVE) {
            const float xx = td_load<T>(xs + k);
#pragma unroll
            for (int i = 0; i < R; ++i)
                if (rows[i]) acc[i] = fmaf(td_load<T>(rows[i] + k), xx, acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) out[i] = td_wave_sum(acc[i]);
}

// int8 rows against the int8 token code: exact int32 sums.
template <int R>
__device__ __forceinline__ void rows_dot_i8(const int8_t* const (&rows)[R], const int8_t* xq, int n, int lane,
                                            int (&out)[R]) {
    int acc[R];
#pragma unroll
    for (int i = 0; i < R; ++i) acc[i] = 0;
    if (n % 16 == 0) {
        const int nv = n / 16;
        const td_u32x4* xv = reinterpret_cast<const td_u32x4*>(xq);
#pragma unroll 2
        for (int v = lane; v < nv; v += TD_WAVE) {
            td_u32x4 w[R];
#pragma unroll
            for (int i = 0; i < R; ++i)
                w[i] = rows[i] ? td_load_stream16(reinterpret_cast<const td_u32x4*>(rows[i]) + v)
                               : td_u32x4{0, 0, 0, 0};
            const td_u32x4 xx = xv[v];
#pragma unroll
            for (int i = 0; i < R; ++i) {
                acc[i] = __builtin_amdgcn_sdot4((int)w[i].x, (int)xx.x, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)w[i].y, (int)xx.y, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)w[i].z, (int)xx.z, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)w[i].w, (int)xx.w, acc[i], false);
            }
        }
    } else {
        for (int k = lane; k < n; k += TD_WAVE) {
            const int xx = xq[k];
#pragma unroll
            for (int i = 0; i < R; ++i)
                if (rows[i]) acc[i] += (int)rows[i][k] * xx;
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) out[i] = td_wave_sum_i(acc[i]);
}

// Exponent of the token's power-of-two quantisation step: floor(log2 m) - 6.
__device__ __forceinline__ int token_exponent(float m) {
    if (!(m > 0.0f)) return 0;
    int ex;
    (void)frexpf(m, &ex);  // m = f * 2^ex, 0.5 <= f < 1
    return ex - 1 - 6;
}

__device__ __forceinline__ int8_t quantize_value(float v, int e) {
    float q = rintf(ldexpf(v, -e));
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int8_t)(int)q;
}

