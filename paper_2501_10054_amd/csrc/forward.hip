// Online path of the partially-linear FFN (Sec. "Inference Runtime"):
//   speculative result  y = W'x + b'
//   predictor           int8 sketch of W1 against an int8 code of x, range test,
//                       flagged neurons compacted into a list
//   result fixing       for each flagged neuron j: z_j = W1[j].x + b1_j,
//                       y += (sigma(z_j) - (a_j z_j + c_j)) * W2[:, j]
// plus the unmodified FFN on the same row-streaming core (the dense baseline).
//
// Every kernel here is bound by HBM bandwidth: each weight row is read exactly
// once with 16-byte loads per lane, one wavefront per row, the token staged in
// LDS, and the per-row reduction done with cross-lane shuffles.
#include "common.h"
#include "rowdot.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace {

constexpr int kBlock = 256;                 // 4 wavefronts
constexpr int kWaves = kBlock / TD_WAVE;
constexpr int kPredRowsPerWave = 8;         // 4 waves x 8 rows = one 32-bit mask word per block
constexpr int kGemvRowsPerWave = 4;

// ------------------------------------------------------------ token staging
// Copies x (d values) into LDS; returns max|x_k| over the block (all threads).
template <typename T>
__device__ __forceinline__ float stage_token(const T* __restrict__ x, T* xs, int d, float* red) {
    float m = 0.0f;
    for (int k = threadIdx.x; k < d; k += kBlock) {
        const T v = x[k];
        xs[k] = v;
        m = fmaxf(m, fabsf(td_load<T>(&v)));
    }
    m = td_wave_max(m);
    if ((threadIdx.x & (TD_WAVE - 1)) == 0) red[threadIdx.x / TD_WAVE] = m;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = fmaxf(r, red[w]);
    return r;
}

// ----------------------------------------------- folded product + predictor
// Blocks [0, gemv_blocks) compute rows of W'x + b' into yacc (fp32).
// Blocks [gemv_blocks, gemv_blocks + pred_blocks) each own 32 consecutive
// neurons: they form the block's mask word and append the flagged indices to
// the token's list.
template <typename T>
__global__ void __launch_bounds__(kBlock)
fold_predict_kernel(const T* __restrict__ Wp, const float* __restrict__ bp, const int8_t* __restrict__ Q,
                    const float* __restrict__ tlo, const float* __restrict__ thi, const T* __restrict__ x,
                    float* __restrict__ yacc, uint32_t* __restrict__ mask, int32_t* __restrict__ count,
                    int32_t* __restrict__ list, int d, int h, int gemv_blocks) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* xs = reinterpret_cast<T*>(smem);
    int8_t* xq = reinterpret_cast<int8_t*>(smem + (((size_t)d * sizeof(T) + 15) & ~(size_t)15));
    __shared__ float red[kWaves];
    __shared__ uint32_t word_parts[kWaves];
    __shared__ int list_base;

    const int lane = threadIdx.x & (TD_WAVE - 1);
    const int wave = threadIdx.x / TD_WAVE;
    const float m = stage_token<T>(x, xs, d, red);

    if ((int)blockIdx.x < gemv_blocks) {
        __syncthreads();
        const int r0 = ((int)blockIdx.x * kWaves + wave) * kGemvRowsPerWave;
        const T* rows[kGemvRowsPerWave];
#pragma unroll
        for (int i = 0; i < kGemvRowsPerWave; ++i) rows[i] = (r0 + i < d) ? Wp + (size_t)(r0 + i) * d : nullptr;
        float out[kGemvRowsPerWave];
        rows_dot<T, kGemvRowsPerWave>(rows, xs, d, lane, out);
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < kGemvRowsPerWave; ++i)
                if (r0 + i < d) yacc[r0 + i] = out[i] + bp[r0 + i];
        }
        return;
    }

    // ---- predictor block
    const int e = token_exponent(m);
    for (int k = threadIdx.x; k < d; k += kBlock) xq[k] = quantize_value(td_load<T>(xs + k), e);
    __syncthreads();

    const int pb = (int)blockIdx.x - gemv_blocks;
    const int j0 = pb * 32 + wave * kPredRowsPerWave;
    const int8_t* rows[kPredRowsPerWave];
#pragma unroll
    for (int i = 0; i < kPredRowsPerWave; ++i) rows[i] = (j0 + i < h) ? Q + (size_t)(j0 + i) * d : nullptr;
    int acc[kPredRowsPerWave];
    rows_dot_i8<kPredRowsPerWave>(rows, xq, d, lane, acc);

    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < kPredRowsPerWave; ++i) {
        if (j0 + i < h) {
            const float v = ldexpf((float)acc[i], e);
            const bool inside = (v >= tlo[j0 + i]) && (v < thi[j0 + i]);
            if (!inside) bits |= 1u << i;
        }
    }
    if (lane == 0) word_parts[wave] = bits << (wave * kPredRowsPerWave);
    __syncthreads();
    uint32_t word = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) word |= word_parts[w];
    if (threadIdx.x == 0) {
        mask[pb] = word;
        const int n = __popc(word);
        list_base = n ? atomicAdd(count, n) : 0;
    }
    __syncthreads();
    if (threadIdx.x < 32 && ((word >> threadIdx.x) & 1u)) {
        const int rank = __popc(word & ((1u << threadIdx.x) - 1u));
        if (list_base + rank < h) list[list_base + rank] = pb * 32 + (int)threadIdx.x;
    }
}

// ------------------------------------------------------------ result fixing
// One wavefront per flagged neuron (grid-stride over the device-side count).
template <typename T>
__global__ void __launch_bounds__(kBlock)
fix_kernel(const T* __restrict__ W1, const T* __restrict__ b1, const T* __restrict__ W2T,
           const float* __restrict__ a, const float* __restrict__ c, const T* __restrict__ x,
           const int32_t* __restrict__ count, const int32_t* __restrict__ list, float* __restrict__ yacc, int d,
           int h, int act) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* xs = reinterpret_cast<T*>(smem);
    const int n = min(*count, h);
    const int lane = threadIdx.x & (TD_WAVE - 1);
    const int gw = (int)blockIdx.x * kWaves + threadIdx.x / TD_WAVE;
    const int total = (int)gridDim.x * kWaves;
    if ((int)blockIdx.x * kWaves >= n) return;  // whole block idle (uniform)
    for (int k = threadIdx.x; k < d; k += kBlock) xs[k] = x[k];
    __syncthreads();

    constexpr int V = RowVec<T>::N;
    for (int i = gw; i < n; i += total) {
        const int j = list[i];
        if (j < 0 || j >= h) continue;
        const T* rows[1] = {W1 + (size_t)j * d};
        float z[1];
        rows_dot<T, 1>(rows, xs, d, lane, z);
        float zj = z[0];
        if (b1) zj += td_load<T>(b1 + j);
        const float delta = td_act(zj, act) - fmaf(a[j], zj, c[j]);
        const T* w2 = W2T + (size_t)j * d;
        if (d % V == 0) {
            const int nv = d / V;
            for (int v = lane; v < nv; v += TD_WAVE) {
                const td_u32x4 w = td_load_stream16(reinterpret_cast<const td_u32x4*>(w2) + v);
                const T* wt = reinterpret_cast<const T*>(&w);
#pragma unroll
                for (int u = 0; u < V; ++u) unsafeAtomicAdd(yacc + (size_t)v * V + u, delta * td_load<T>(wt + u));
            }
        } else {
            for (int k = lane; k < d; k += TD_WAVE) unsafeAtomicAdd(yacc + k, delta * td_load<T>(w2 + k));
        }
    }
}

__global__ void __launch_bounds__(kBlock) zero_i32_kernel(int32_t* __restrict__ p, int n) {
    const int i = (int)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) p[i] = 0;
}

// fp32 accumulator -> output dtype (one block; optionally y / sqrt(mean(y^2) + eps))
template <typename T>
__global__ void __launch_bounds__(kBlock)
finish_kernel(const float* __restrict__ yacc, T* __restrict__ y, int d, int norm_out, float eps) {
    __shared__ float red[kWaves];
    float scale = 1.0f;
    if (norm_out) {
        float ss = 0.0f;
        for (int k = threadIdx.x; k < d; k += kBlock) ss += yacc[k] * yacc[k];
        ss = td_wave_sum(ss);
        if ((threadIdx.x & (TD_WAVE - 1)) == 0) red[threadIdx.x / TD_WAVE] = ss;
        __syncthreads();
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) tot += red[w];
        scale = 1.0f / sqrtf(tot / (float)d + eps);
    }
    for (int k = threadIdx.x; k < d; k += kBlock) td_store<T>(y + k, yacc[k] * scale);
}

// -------------------------------------------------------------- dense FFN
// out[r] = post(rows[r] . x + bias[r]) for r < n_rows; x has n_in values.
template <typename T, bool kActivate>
__global__ void __launch_bounds__(kBlock)
dense_rows_kernel(const T* __restrict__ W, const T* __restrict__ bias, const T* __restrict__ x,
                  T* __restrict__ out, int n_rows, int n_in, int act, int x_in_lds) {
    extern __shared__ __align__(16) unsigned char smem[];
    const T* xs = x;
    if (x_in_lds) {
        T* s = reinterpret_cast<T*>(smem);
        for (int k = threadIdx.x; k < n_in; k += kBlock) s[k] = x[k];
        __syncthreads();
        xs = s;
    }
    const int lane = threadIdx.x & (TD_WAVE - 1);
    const int wave = threadIdx.x / TD_WAVE;
    const int r0 = ((int)blockIdx.x * kWaves + wave) * kGemvRowsPerWave;
    const T* rows[kGemvRowsPerWave];
#pragma unroll
    for (int i = 0; i < kGemvRowsPerWave; ++i) rows[i] = (r0 + i < n_rows) ? W + (size_t)(r0 + i) * n_in : nullptr;
    float o[kGemvRowsPerWave];
    rows_dot<T, kGemvRowsPerWave>(rows, xs, n_in, lane, o);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < kGemvRowsPerWave; ++i) {
            if (r0 + i < n_rows) {
                float v = o[i];
                if (bias) v += td_load<T>(bias + r0 + i);
                if (kActivate) v = td_act(v, act);
                td_store<T>(out + r0 + i, v);
            }
        }
    }
}

inline int div_up(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

template <typename T>
tardis_status_t forward_t(tardis_layer_s* L, const void* xv, int64_t n, void* yv, int norm_out, hipStream_t s) {
    const int d = (int)L->d, h = (int)L->h;
    const size_t xs_bytes = (((size_t)d * sizeof(T) + 15) & ~(size_t)15);
    const int gemv_blocks = div_up(d, kWaves * kGemvRowsPerWave);
    const int pred_blocks = div_up(h, 32);
    const int fix_blocks = 256;
    // a handful of tokens is faster through the single-token kernel (one launch each)
    // (a deterministic layer runs every call as decode groups on the counted fixed-point accumulators:
    //  the pass and prompt kernels add fp32 partial sums in an order that varies from run to run)
    if (!L->deterministic) {
        if (L->pf_scratch && n >= L->prefill_min_tokens) return td_forward_prefill(L, xv, n, yv, norm_out, s);
        if (n > L->batched_min_tokens && L->use_batched) return td_forward_batched(L, xv, n, yv, norm_out, s);
    }
    if (L->use_fused) {   // groups of 16, 8, 4, 2, 1 tokens share one pass over the weights
        TD_TRY(td_decode_fused(L, xv, n, yv, norm_out, s));
        L->last_n = n;
        return TARDIS_OK;
    }
    // (a fill kernel, not a memset node, so that the call can be captured in a graph)
    hipLaunchKernelGGL(zero_i32_kernel, dim3(div_up(n, kBlock)), dim3(kBlock), 0, s, L->counts, (int)n);
    for (int64_t t = 0; t < n; ++t) {
        const T* x = static_cast<const T*>(xv) + t * d;
        T* y = static_cast<T*>(yv) + t * d;
        float* yacc = L->yacc + t * d;
        uint32_t* mask = L->mask + t * L->mask_words;
        int32_t* count = L->counts + t;
        int32_t* list = L->list + t * h;
        hipLaunchKernelGGL(fold_predict_kernel<T>, dim3(gemv_blocks + pred_blocks), dim3(kBlock), xs_bytes + d, s,
                           static_cast<const T*>(L->Wp), L->bp, L->Q, L->tlo, L->thi, x, yacc, mask, count, list,
                           d, h, gemv_blocks);
        hipLaunchKernelGGL(fix_kernel<T>, dim3(fix_blocks), dim3(kBlock), xs_bytes, s,
                           static_cast<const T*>(L->W1), static_cast<const T*>(L->b1),
                           static_cast<const T*>(L->W2T), L->a, L->c, x, count, list, yacc, d, h, (int)L->act);
        hipLaunchKernelGGL(finish_kernel<T>, dim3(1), dim3(kBlock), 0, s, yacc, y, d, norm_out, kRmsEps);
    }
    TD_HIP(hipGetLastError());
    L->last_n = n;
    return TARDIS_OK;
}

template <typename T>
tardis_status_t dense_t(tardis_layer_s* L, const void* xv, int64_t n, void* yv, hipStream_t s) {
    const int d = (int)L->d, h = (int)L->h;
    const size_t lds_cap = 60 * 1024;
    const size_t x_bytes = (size_t)d * sizeof(T), hid_bytes = (size_t)h * sizeof(T);
    for (int64_t t = 0; t < n; ++t) {
        const T* x = static_cast<const T*>(xv) + t * d;
        T* y = static_cast<T*>(yv) + t * d;
        T* hid = reinterpret_cast<T*>(L->hidden) + t * h;
        const int l1 = x_bytes <= lds_cap, l2 = hid_bytes <= lds_cap;
        hipLaunchKernelGGL((dense_rows_kernel<T, true>), dim3(div_up(h, kWaves * kGemvRowsPerWave)), dim3(kBlock),
                           l1 ? x_bytes : 0, s, static_cast<const T*>(L->W1), static_cast<const T*>(L->b1), x, hid,
                           h, d, (int)L->act, l1);
        hipLaunchKernelGGL((dense_rows_kernel<T, false>), dim3(div_up(d, kWaves * kGemvRowsPerWave)), dim3(kBlock),
                           l2 ? hid_bytes : 0, s, static_cast<const T*>(L->W2), static_cast<const T*>(L->b2), hid,
                           y, d, h, 0, l2);
    }
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

}  // namespace

tardis_status_t td_forward(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s) {
    return L->dtype == TARDIS_BF16 ? forward_t<bf16_t>(L, x, n, y, norm_out, s)
                                   : forward_t<float>(L, x, n, y, norm_out, s);
}

tardis_status_t td_dense_forward(tardis_layer_s* L, const void* x, int64_t n, void* y, hipStream_t s) {
    if (L->pf_scratch && n >= L->prefill_min_tokens) return td_dense_prefill(L, x, n, y, s);
    return L->dtype == TARDIS_BF16 ? dense_t<bf16_t>(L, x, n, y, s) : dense_t<float>(L, x, n, y, s);
}
