// Shared declarations of libtardis: the layer handle, status helpers and the
// small device-side numeric helpers every kernel file uses.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/tardis.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits
typedef unsigned int td_u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte load

#define TD_WAVE 64

constexpr float kRmsEps = 1e-6f;

#define TD_HIP(expr)                                                              \
    do {                                                                          \
        hipError_t e__ = (expr);                                                  \
        if (e__ != hipSuccess)                                                    \
            return (e__ == hipErrorOutOfMemory) ? TARDIS_ERR_OOM : TARDIS_ERR_HIP; \
    } while (0)

#define TD_TRY(expr)                          \
    do {                                      \
        tardis_status_t s__ = (expr);         \
        if (s__ != TARDIS_OK) return s__;     \
    } while (0)

// One-time set-up that may be reached from several host threads (kernel attributes are raised
// when the first layer is folded): `fn` runs under a lock until it has succeeded once.
struct td_once {
    std::mutex lock;
    bool done = false;
    template <typename F> tardis_status_t run(F fn) {
        std::lock_guard<std::mutex> guard(lock);
        if (done) return TARDIS_OK;
        const tardis_status_t st = fn();
        if (st == TARDIS_OK) done = true;
        return st;
    }
};

// What the single-launch stack kernel needs of one layer (a copy lives in device memory, filled when
// the layer is folded).
struct td_stack_layer_dev {
    const bf16_t* Wp;
    const float* bp;
    const int8_t* Q;
    const float* tlo;
    const float* thi;
    const bf16_t* W1;
    const bf16_t* b1;
    const bf16_t* W2T;
    const float* a;
    const float* c;
    uint32_t* mask;
    bf16_t* xnext;
    float* yfix;       // the layer's accumulator copies (zero between launches)
    int32_t* sync;     // the layer's counters (zero between launches)
    int32_t h, npb, act, reserved;
};

// Everything one folded layer owns.  Pointers are device memory.
struct tardis_layer_s {
    int64_t d, h;
    int32_t dtype, act;
    int64_t max_batch;
    int64_t mask_words;  // ceil(h/32)
    // borrowed from the caller
    const void* W1;  // h x d
    const void* b1;  // h or null
    const void* b2;  // d or null
    // owned
    void* W2T;     // h x d, neuron-major copy of W2
    void* W2;      // d x h, copy of W2 as given (dense baseline)
    void* Wp;      // d x d folded matrix
    uint8_t* Wp8;      // d x d e4m3 codes of the folded matrix (8-bit storage only, else null): Wp = code * scale
    float* wp8_scale;  // d power-of-two row scales of Wp8
    float* bp;     // d folded bias
    int8_t* Q;     // h x d predictor codes, one byte each (absent when only the packed 4-bit form is kept)
    uint8_t* Q4;   // packed 4-bit sketch, h x d/2 bytes: one 16-byte vector per group of 32 columns (or null)
    uint8_t* M4;   // 4-bit sketch: h x ceil(d/32) group multipliers, one byte each (or null)
    int32_t sketch_bits;   // 8, or 4 / 3 / 2: grouped codes in 4-bit slots
    float margin;          // fraction of a range's width the predictor's test is narrowed by at either end
    float* tlo;    // h
    float* thi;    // h
    float* a;      // h
    float* c;      // h
    // working memory of the online calls (sized by max_batch)
    float* yacc;       // max_batch x d fp32 accumulator
    uint32_t* mask;    // max_batch x mask_words
    int32_t* counts;   // max_batch flagged-neuron counters
    int32_t* list;     // max_batch x h flagged indices
    float* hidden;     // max_batch x h activations for the dense baseline
    int32_t* sync;     // small block of device counters (zero between calls)
    void* zeros_h;     // h zero elements of the layer dtype (stands in for a missing b1)
    void* xnext;       // max_batch x d, layer dtype: normalised output handed to the next stacked layer
    float* yfix;       // dec_copies x kDecodeMaxTokens x d fp32 repair accumulators of the fused decode kernel (zero between calls)
    const tardis_layer_s* next_layer;   // the layer that runs after this one (hint, may be null; not owned)
    int32_t prefetch_bytes;             // bytes of that layer's predictor rows each finished block requests
    int32_t strict_release;             // the signalling thread of a decode block also executes an agent-scope release fence
    int32_t prefetch_shape;             // next-layer warming by order of arrival: first16 | last16 << 8 (sixteenths of prefetch_bytes; 0 = flat)
    int32_t dec_blocks;   // grid of the fused decode kernel
    int32_t dec_threads;  // block size of the fused decode kernel (512 or 1024)
    int32_t dec_copies;   // number of repair accumulator copies
    int32_t use_fused;    // fused single-launch decode path available for this layer
    // working memory of the batched path (one pass of up to 64 tokens); null if unused
    int8_t* bt_xq;                 // 64 x d int8 token codes
    int32_t* bt_e;                 // 64 token exponents
    unsigned long long* bt_tokmask;  // h: which tokens of the pass flagged each neuron
    int32_t* bt_ulist;             // h: neurons flagged by at least one token
    int32_t* bt_ucount;            // 1
    bf16_t* bt_delta;              // 64 x h repair factors
    float* bt_partial;             // partial products of the scatter step
    int32_t use_batched;
    void* pf_scratch;              // prompt path: int8 tokens, exponents, int32 sums, pre-activations, delta, fp32 y
    int32_t prefill_min_tokens;    // calls with at least this many tokens take the prompt path (if it has scratch)
    int32_t prefill_chunk;         // ... in chunks of at most this many tokens (what the scratch is sized for)
    int32_t* rec_count;            // two-kernel path: flagged neurons per predictor block,
    uint32_t* rec_jb;              //   neuron index and
    uint32_t* rec_tb;              //   token bits of each record (dec_blocks x neurons per block),
    float* rec_delta;              //   and kDecodeMaxTokens deltas per record
    int32_t defer_min_tokens;      // groups of at least this many tokens take the two-kernel path (4, 8; 99 = never)
    int32_t batched_min_tokens;    // token counts up to this go through the single-token path
    int64_t last_n;    // token count of the most recent online call
    int32_t fx;        // decode kernels accumulate the repair in counted fixed-point words (deterministic results)
    int32_t deterministic;   // every online call runs as decode groups on those accumulators
    float* fx_bound;   // K1, K2 of the accumulators' magnitude bound (device, 2 floats)
    td_stack_layer_dev* stack_desc;   // device copy of this layer's entry for the single-launch stack kernel (or null)
    int32_t stack_fused;              // knob: one-token stacks of such layers run in one launch
    int32_t stack_spin_limit;         // knob: polls a block of that launch spends on one layer's counter before it gives up
    int32_t poisoned;  // a launch of an online call failed half way: counters and accumulators may be left armed
};

static inline size_t td_elem_size(int32_t dtype) { return dtype == TARDIS_BF16 ? 2 : 4; }

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float td_bf16_to_f32(bf16_t v) {
    return __uint_as_float(((uint32_t)v) << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t td_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// 16-byte load of data that is read once (weights streamed from HBM)
__device__ __forceinline__ td_u32x4 td_load_stream16(const void* p) {
    return __builtin_nontemporal_load(static_cast<const td_u32x4*>(p));
}

template <typename T> __device__ __forceinline__ float td_load(const T* p);
template <> __device__ __forceinline__ float td_load<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float td_load<bf16_t>(const bf16_t* p) { return td_bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void td_store(T* p, float v);
template <> __device__ __forceinline__ void td_store<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void td_store<bf16_t>(bf16_t* p, float v) { *p = td_f32_to_bf16(v); }

__device__ __forceinline__ float td_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int td_wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float td_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// sigma(z) for the four supported activations (fp32)
__device__ __forceinline__ float td_act(float z, int act) {
    switch (act) {
        case TARDIS_ACT_GELU_ERF:
            return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f));
        case TARDIS_ACT_GELU_TANH: {
            float u = 0.79788456080286535588f * (z + 0.044715f * z * z * z);
            return 0.5f * z * (1.0f + tanhf(u));
        }
        case TARDIS_ACT_RELU:
            return z > 0.0f ? z : 0.0f;
        default:
            return z;
    }
}

// fp64 version for the offline fit
__device__ __forceinline__ double td_act_f64(double z, int act) {
    switch (act) {
        case TARDIS_ACT_GELU_ERF:
            return 0.5 * z * (1.0 + erf(z * 0.70710678118654752440));
        case TARDIS_ACT_GELU_TANH: {
            double u = 0.79788456080286535588 * (z + 0.044715 * z * z * z);
            return 0.5 * z * (1.0 + tanh(u));
        }
        case TARDIS_ACT_RELU:
            return z > 0.0 ? z : 0.0;
        default:
            return z;
    }
}

// ---------------------------------------------------------------- internal launchers
// (each validates nothing: the C-ABI layer in api.cpp has already done so)

// offline.hip
tardis_status_t td_transpose(const void* src, void* dst, int64_t rows, int64_t cols, int32_t dtype, hipStream_t s);
// bits = 8: Q (required).  bits = 4, 3, 2 (codes up to 7, 3, 1 in 4-bit slots): M4 (required), Q
// (effective one-byte codes, optional) and Q4 (packed, optional, needs d % 32 == 0).  margin: fraction
// of every range's width taken off at either end for the predictor's test.
tardis_status_t td_build_sketch(const void* W1, const void* b1, const float* lo, const float* hi, int64_t h,
                                int64_t d, int32_t dtype, int32_t bits, float margin, int8_t* Q, uint8_t* Q4,
                                uint8_t* M4, float* tlo, float* thi, hipStream_t s);
// one-byte effective codes (multiplier * 4-bit code) from the packed 4-bit sketch
tardis_status_t td_unpack_sketch4(const uint8_t* Q4, const uint8_t* M4, int64_t h, int64_t d, int8_t* Q,
                                  hipStream_t s);
// Wp8 / wp8_scale non-null (bf16 layers): W' is stored as e4m3 codes with a power-of-two scale per row, and Wp
// receives the same values as bf16
tardis_status_t td_fold(const tardis_ffn_desc* desc, const float* a, const float* c, void* Wp, float* bp,
                        uint8_t* Wp8, float* wp8_scale, hipStream_t s);
// step > 0: greedy range search with that increment; step <= 0: central quantile ranges
tardis_status_t td_calibrate(const tardis_ffn_desc* desc, const void* X, int64_t n, float coverage,
                             const float* cov_pn, float step, float* lo, float* hi, float* a, float* c,
                             hipStream_t s);
tardis_status_t td_estimate_errors(const tardis_ffn_desc* desc, const void* X, int64_t n, const float* lo,
                                   const float* hi, const float* a, const float* c, float* err, float* err_layer,
                                   hipStream_t s);
tardis_status_t td_assign_thresholds(const float* err, int64_t n, float t, float t_min, float t_max, float* out,
                                     hipStream_t s);
tardis_status_t td_fx_bounds(const tardis_layer_s* L, float* out2, hipStream_t s);
// gemm.hip:  C[m][n] = sum_k A[m][k] * B[n][k]  (+ C if accumulate) (+ row_bias[m]); C fp32, ldc = N
tardis_status_t td_gemm_nt(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K,
                           int32_t dtype, int accumulate, const void* row_bias, hipStream_t s);
// exact int8 x int8 -> int32 product of the same form (K a multiple of 16, operands 16-byte aligned)
tardis_status_t td_gemm_nt_i8(const int8_t* A, const int8_t* B, int32_t* C, int64_t M, int64_t N, int64_t K,
                              int splits, hipStream_t s);
// decode.hip
bool td_prefill_supported(const tardis_layer_s* L);
size_t td_prefill_scratch_bytes(const tardis_layer_s* L, int64_t n);
tardis_status_t td_forward_prefill(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s);
tardis_status_t td_dense_prefill(tardis_layer_s* L, const void* x, int64_t n, void* y, hipStream_t s);
bool td_layer_is_live(const tardis_layer_s* L);
tardis_status_t td_gemm_init();
int td_gemm_tile_rows(int64_t M);
tardis_status_t td_gemm_nt_split(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K, int32_t dtype,
                                 int accumulate, const void* row_bias, int splits, hipStream_t s);
tardis_status_t td_decode_init();
bool td_decode_fused_supported(const tardis_layer_s* L);
constexpr int kDecodeMaxTokens = 16;  // tokens one weight pass of the decode kernel can be shared between
// n consecutive tokens (bf16 layers the fused kernels support) as groups of 16, 8, 4, 2, 1 with the
// layer's own working memory
tardis_status_t td_decode_fused(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s);
// looks up the current device's static decode working memory (once per device)
tardis_status_t td_static_scratch_setup();
tardis_status_t td_mask_union(const tardis_layer_s* L, int64_t n, uint32_t* union_mask, int32_t* union_count,
                              hipStream_t s);
tardis_status_t td_mask_to_list(const tardis_layer_s* L, int64_t n, int32_t* counts, int32_t* list, hipStream_t s);
// stack.hip
tardis_status_t td_stack_init();
bool td_stack_decode_supported(const tardis_layer_s* L);
tardis_status_t td_stack_decode(tardis_layer_s* const* layers, int n_layers, const void* x, void* y, hipStream_t s);
// batched.hip
bool td_batched_supported(const tardis_layer_s* L);
size_t td_batched_partial_floats(const tardis_layer_s* L);
tardis_status_t td_batched_init();
tardis_status_t td_forward_batched(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s);
// forward.hip
// norm_out != 0: the output is y / sqrt(mean(y^2) + kRmsEps) per token (glue between stacked layers)
tardis_status_t td_forward(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s);
tardis_status_t td_dense_forward(tardis_layer_s* L, const void* x, int64_t n, void* y, hipStream_t s);
