// Many tokens at once (prompt processing), as dense matrix products.
//
// With hundreds of tokens the union of the flagged neurons is the whole layer (Sec. "Inference
// Runtime" notes that the method does not help prompt processing), so gathering rows per token
// gains nothing; the same per-token result is computed here from four matrix products on the
// matrix cores:
//     ACC = Xq Q^T            exact int32 (the predictor's integer sums of every token)
//     Z   = X W1^T            fp32 accumulate (the exact pre-activations)
//     Y   = X W'^T + D W2^T   with D[t][j] = sigma(z) - (a_j z + c_j) where token t flagged neuron j, else 0
// and y = Y + b' (then the optional RMS norm and the conversion).  Masks are bit-exact with the
// per-token path (same integer sums, same range test); D is rounded to bf16 for the last product.
#include "common.h"
#include "rowdot.h"

namespace {

// int8 code and exponent of every token (one block per token)
__global__ void __launch_bounds__(256)
quantize_rows_kernel(const bf16_t* __restrict__ X, int d, int8_t* __restrict__ XQ, int32_t* __restrict__ E) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const bf16_t* x = X + (size_t)t * d;
    float m = 0.0f;
    for (int k = threadIdx.x; k < d; k += 256) m = fmaxf(m, fabsf(td_bf16_to_f32(x[k])));
    m = td_wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const int e = token_exponent(m);
    for (int k = threadIdx.x; k < d; k += 256) XQ[(size_t)t * d + k] = quantize_value(td_bf16_to_f32(x[k]), e);
    if (threadIdx.x == 0) E[t] = e;
}

// range test, mask words and masked delta.  blockIdx.y = token; a thread covers 4 consecutive
// neurons (16-byte loads of the sums and pre-activations), 8 lanes assemble one mask word.
__global__ void __launch_bounds__(256)
delta_mask_kernel(const int32_t* __restrict__ ACC, const float* __restrict__ Z, const int32_t* __restrict__ E,
                  const float* __restrict__ tlo, const float* __restrict__ thi, const float* __restrict__ a,
                  const float* __restrict__ c, const bf16_t* __restrict__ b1, int act, int h,
                  bf16_t* __restrict__ D, uint32_t* __restrict__ mask, int mask_words) {
    const int t = blockIdx.y;
    const int j = ((int)blockIdx.x * 256 + (int)threadIdx.x) * 4;
    const int lane = threadIdx.x & 63;
    uint32_t nib = 0;
    if (j < h) {                                     // h % 4 == 0: all four or none
        const size_t at = (size_t)t * h + j;
        const int4 acc = *reinterpret_cast<const int4*>(ACC + at);
        const float4 z4 = *reinterpret_cast<const float4*>(Z + at);
        const float4 l4 = *reinterpret_cast<const float4*>(tlo + j), h4 = *reinterpret_cast<const float4*>(thi + j);
        const float4 a4 = *reinterpret_cast<const float4*>(a + j), c4 = *reinterpret_cast<const float4*>(c + j);
        const uint2 braw = *reinterpret_cast<const uint2*>(b1 + j);
        const int e = E[t];
        const int av[4] = {acc.x, acc.y, acc.z, acc.w};
        const float zv[4] = {z4.x, z4.y, z4.z, z4.w}, lv[4] = {l4.x, l4.y, l4.z, l4.w}, hv[4] = {h4.x, h4.y, h4.z, h4.w};
        const float aa[4] = {a4.x, a4.y, a4.z, a4.w}, cc[4] = {c4.x, c4.y, c4.z, c4.w};
        const float bv[4] = {__uint_as_float(braw.x << 16), __uint_as_float(braw.x & 0xffff0000u),
                             __uint_as_float(braw.y << 16), __uint_as_float(braw.y & 0xffff0000u)};
        bf16_t out[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float v = ldexpf((float)av[u], e);
            const bool flagged = !((v >= lv[u]) && (v < hv[u]));
            float dv = 0.0f;
            if (flagged) {
                const float z = zv[u] + bv[u];
                dv = td_act(z, act) - fmaf(aa[u], z, cc[u]);
                nib |= 1u << u;
            }
            out[u] = td_f32_to_bf16(dv);
        }
        uint2 packed;
        packed.x = (uint32_t)out[0] | ((uint32_t)out[1] << 16);
        packed.y = (uint32_t)out[2] | ((uint32_t)out[3] << 16);
        *reinterpret_cast<uint2*>(D + at) = packed;
    }
    uint32_t word = nib << (4 * (lane & 7));
    word |= __shfl_xor(word, 1);
    word |= __shfl_xor(word, 2);
    word |= __shfl_xor(word, 4);
    const int w = j >> 5;
    if ((lane & 7) == 0 && w < mask_words) mask[(size_t)t * mask_words + w] = word;
}

// y[t] = (Y[t] + b') (optionally RMS-normalised), one block per token
__global__ void __launch_bounds__(256)
finish_rows_kernel(const float* __restrict__ Y, const float* __restrict__ bp, int d, bf16_t* __restrict__ y,
                   int norm_out, float eps) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const float* row = Y + (size_t)t * d;
    float scale = 1.0f;
    if (norm_out) {
        float ss = 0.0f;
        for (int k = threadIdx.x; k < d; k += 256) {
            const float v = row[k] + bp[k];
            ss += v * v;
        }
        ss = td_wave_sum(ss);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
        __syncthreads();
        scale = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    }
    for (int k = threadIdx.x; k < d; k += 256) y[(size_t)t * d + k] = td_f32_to_bf16((row[k] + bp[k]) * scale);
}

// dense FFN, hidden activations: H = act(Z + b1), rounded to bf16 (4 neurons per thread)
__global__ void __launch_bounds__(256)
dense_hidden_kernel(const float* __restrict__ Z, const bf16_t* __restrict__ b1, int act, int h,
                    bf16_t* __restrict__ H) {
    const int t = blockIdx.y;
    const int j = ((int)blockIdx.x * 256 + (int)threadIdx.x) * 4;
    if (j >= h) return;
    const size_t at = (size_t)t * h + j;
    const float4 z4 = *reinterpret_cast<const float4*>(Z + at);
    const uint2 braw = *reinterpret_cast<const uint2*>(b1 + j);
    const float zv[4] = {z4.x, z4.y, z4.z, z4.w};
    const float bv[4] = {__uint_as_float(braw.x << 16), __uint_as_float(braw.x & 0xffff0000u),
                         __uint_as_float(braw.y << 16), __uint_as_float(braw.y & 0xffff0000u)};
    bf16_t out[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) out[u] = td_f32_to_bf16(td_act(zv[u] + bv[u], act));
    uint2 packed;
    packed.x = (uint32_t)out[0] | ((uint32_t)out[1] << 16);
    packed.y = (uint32_t)out[2] | ((uint32_t)out[3] << 16);
    *reinterpret_cast<uint2*>(H + at) = packed;
}

// dense FFN, output: y[t] = Y[t] + b2 (b2 may be null), one block per token
__global__ void __launch_bounds__(256)
dense_output_kernel(const float* __restrict__ Y, const bf16_t* __restrict__ b2, int d, bf16_t* __restrict__ y) {
    const int t = blockIdx.x;
    for (int k = threadIdx.x; k < d; k += 256)
        y[(size_t)t * d + k] = td_f32_to_bf16(Y[(size_t)t * d + k] + (b2 ? td_bf16_to_f32(b2[k]) : 0.0f));
}

}  // namespace

bool td_prefill_supported(const tardis_layer_s* L) {
    return L->dtype == TARDIS_BF16 && L->d % 128 == 0 && L->h >= 128 && L->h % 8 == 0 && L->Q != nullptr;
}

size_t td_prefill_scratch_bytes(const tardis_layer_s* L, int64_t n) {
    const size_t d = (size_t)L->d, h = (size_t)L->h, nn = (size_t)n;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    return up(nn * d) + up(nn * 4) + up(nn * h * 4) + up(nn * h * 4) + up(nn * h * 2) + up(nn * d * 4);
}

// one chunk of at most L->prefill_chunk tokens (the scratch is sized for that many)
static tardis_status_t prefill_chunk(tardis_layer_s* L, const bf16_t* x, int64_t n, bf16_t* y, uint32_t* mask,
                                     int norm_out, hipStream_t s) {
    const int64_t d = L->d, h = L->h;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    unsigned char* p = static_cast<unsigned char*>(L->pf_scratch);
    int8_t* xq = reinterpret_cast<int8_t*>(p);            p += up((size_t)n * d);
    int32_t* e = reinterpret_cast<int32_t*>(p);           p += up((size_t)n * 4);
    int32_t* acc = reinterpret_cast<int32_t*>(p);         p += up((size_t)n * h * 4);
    float* z = reinterpret_cast<float*>(p);               p += up((size_t)n * h * 4);
    bf16_t* dl = reinterpret_cast<bf16_t*>(p);            p += up((size_t)n * h * 2);
    float* yacc = reinterpret_cast<float*>(p);
    // products with few output tiles cut K into ranges (added atomically) so that >= 256 blocks run
    auto pick = [&](int64_t N, int64_t K) {
        const int64_t rows = td_gemm_tile_rows(n);
        const int64_t tiles = ((n + rows - 1) / rows) * ((N + 255) / 256);
        int sp = 1;
        while (sp < 8 && tiles * sp < 256 && K / (sp * 2) >= 1024) sp *= 2;
        return sp;
    };
    hipLaunchKernelGGL(quantize_rows_kernel, dim3((unsigned)n), dim3(256), 0, s, x, (int)d, xq, e);
    TD_TRY(td_gemm_nt_i8(xq, L->Q, acc, n, h, d, pick(h, d), s));                 // K in bytes decides the slices
    TD_TRY(td_gemm_nt_split(x, L->W1, z, n, h, d, TARDIS_BF16, 0, nullptr, pick(h, d * 2), s));
    hipLaunchKernelGGL(delta_mask_kernel, dim3((unsigned)((h + 1023) / 1024), (unsigned)n), dim3(256), 0, s, acc, z, e,
                       L->tlo, L->thi, L->a, L->c, static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h), (int)L->act,
                       (int)h, dl, mask, (int)L->mask_words);
    TD_TRY(td_gemm_nt_split(x, L->Wp, yacc, n, d, d, TARDIS_BF16, 0, nullptr, pick(d, d * 2), s));
    TD_TRY(td_gemm_nt_split(dl, L->W2, yacc, n, d, h, TARDIS_BF16, 1, nullptr, pick(d, h * 2), s));
    hipLaunchKernelGGL(finish_rows_kernel, dim3((unsigned)n), dim3(256), 0, s, yacc, L->bp, (int)d, y, norm_out,
                       kRmsEps);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

// Long prompts run in chunks of L->prefill_chunk tokens (tokens are independent): the scratch and
// the launch grids stay bounded whatever max_batch is.
tardis_status_t td_forward_prefill(tardis_layer_s* L, const void* xv, int64_t n, void* yv, int norm_out,
                                   hipStream_t s) {
    const bf16_t* x = static_cast<const bf16_t*>(xv);
    bf16_t* y = static_cast<bf16_t*>(yv);
    for (int64_t t0 = 0; t0 < n; t0 += L->prefill_chunk) {
        const int64_t nc = n - t0 < L->prefill_chunk ? n - t0 : L->prefill_chunk;
        TD_TRY(prefill_chunk(L, x + t0 * L->d, nc, y + t0 * L->d, L->mask + t0 * L->mask_words, norm_out, s));
    }
    L->last_n = n;
    return TARDIS_OK;
}

// The unmodified FFN on many tokens: two matrix-core products with the activation between them
// (the hidden activations are rounded to bf16, as the per-token dense kernels round them).
tardis_status_t td_dense_prefill(tardis_layer_s* L, const void* xv, int64_t n, void* yv, hipStream_t s) {
    const int64_t d = L->d, h = L->h;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    for (int64_t t0 = 0; t0 < n; t0 += L->prefill_chunk) {
        const int64_t nc = n - t0 < L->prefill_chunk ? n - t0 : L->prefill_chunk;
        unsigned char* p = static_cast<unsigned char*>(L->pf_scratch) + up((size_t)nc * d) + up((size_t)nc * 4) +
                           up((size_t)nc * h * 4);                        // (the layout of prefill_chunk)
        float* z = reinterpret_cast<float*>(p);               p += up((size_t)nc * h * 4);
        bf16_t* hid = reinterpret_cast<bf16_t*>(p);           p += up((size_t)nc * h * 2);
        float* yacc = reinterpret_cast<float*>(p);
        const bf16_t* x = static_cast<const bf16_t*>(xv) + t0 * d;
        auto pick = [&](int64_t N, int64_t K) {
            const int64_t rows = td_gemm_tile_rows(nc);
            const int64_t tiles = ((nc + rows - 1) / rows) * ((N + 255) / 256);
            int sp = 1;
            while (sp < 8 && tiles * sp < 256 && K / (sp * 2) >= 1024) sp *= 2;
            return sp;
        };
        TD_TRY(td_gemm_nt_split(x, L->W1, z, nc, h, d, TARDIS_BF16, 0, nullptr, pick(h, d * 2), s));
        hipLaunchKernelGGL(dense_hidden_kernel, dim3((unsigned)((h + 1023) / 1024), (unsigned)nc), dim3(256), 0, s, z,
                           static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h), (int)L->act, (int)h, hid);
        TD_TRY(td_gemm_nt_split(hid, L->W2, yacc, nc, d, h, TARDIS_BF16, 0, nullptr, pick(d, h * 2), s));
        hipLaunchKernelGGL(dense_output_kernel, dim3((unsigned)nc), dim3(256), 0, s, yacc,
                           static_cast<const bf16_t*>(L->b2), (int)d, static_cast<bf16_t*>(yv) + t0 * d);
    }
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
