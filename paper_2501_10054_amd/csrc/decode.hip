// Single-launch decode path (one token, bf16 storage): the whole online step of
// Sec. "Inference Runtime" -- speculative product, predictor, mask, result
// fixing -- in ONE kernel, so that a token costs one launch and every weight
// byte is requested exactly once.
//
// Work split.  The grid has G blocks; block b owns
//   * neurons   [b*npb, (b+1)*npb)   : predictor rows of Q, and the repair of
//                                      those of them that turn out flagged
//   * outputs   [b*rpb, (b+1)*rpb)   : rows of W' for the speculative product
// so no block ever waits for another: a neuron's flag is known inside the block
// that will repair it.  The repair needs y += delta_j * W2[:, j] over ALL
// outputs; each block sums its flagged neurons into a block-private fp32
// vector in LDS and adds that vector once, with fully coalesced fp32 atomics,
// into one of K accumulator copies.  The last block to finish (a device
// counter) adds the copies to the speculative result, converts to bf16, and
// re-arms the accumulators and the counter for the next call.
#include "common.h"
#include "rowdot.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace {

constexpr int kMaxNeuronsPerBlock = 512;
constexpr int kMaxCopies = 4;                  // repair accumulator copies (blocks spread over them)

__device__ __forceinline__ float load_coherent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte vectors it*64 + lane, it = 0..N-1, of one row (N*64 vectors long)
template <int N>
__device__ __forceinline__ void load_row(td_u32x4 (&dst)[N], const void* row, int lane) {
    const td_u32x4* p = static_cast<const td_u32x4*>(row) + lane;
#pragma unroll
    for (int it = 0; it < N; ++it) dst[it] = td_load_stream16(p + it * TD_WAVE);
}

template <int D, int BLOCK, int RQ>
__global__ void __launch_bounds__(BLOCK)
decode_fused_kernel(const bf16_t* __restrict__ Wp, const float* __restrict__ bp, const int8_t* __restrict__ Q,
                    const float* __restrict__ tlo, const float* __restrict__ thi, const bf16_t* __restrict__ W1,
                    const bf16_t* __restrict__ b1, const bf16_t* __restrict__ W2T, const float* __restrict__ a,
                    const float* __restrict__ c, const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                    float* __restrict__ yfold, float* __restrict__ yfix, int copies, uint32_t* __restrict__ mask,
                    int32_t* __restrict__ done, int h, int npb, int rpb, int act, int norm_out, float eps) {
    static_assert(D % 1024 == 0, "rows must be whole multiples of 64 lanes x 16 bytes");
    static_assert(D % BLOCK == 0 && BLOCK / TD_WAVE >= 4, "column ownership of the repair pass");
    constexpr int NW = BLOCK / TD_WAVE;
    constexpr int NVW = D / 8;                       // 16-byte vectors per bf16 row
    constexpr int IQ = D / 16 / TD_WAVE;             // per-lane vectors of an int8 row
    constexpr int IW = NVW / TD_WAVE;                // per-lane vectors of a bf16 row
    constexpr int XI = (NVW + BLOCK - 1) / BLOCK;    // per-thread vectors of the token

    __shared__ __align__(16) bf16_t xs[D];
    __shared__ __align__(16) int8_t xq[D];
    __shared__ float dl[NW];                         // delta_j of the neurons being repaired
    __shared__ int flist[kMaxNeuronsPerBlock];
    __shared__ uint32_t words[kMaxNeuronsPerBlock / 32];
    __shared__ float red[NW];
    __shared__ int nflag;
    __shared__ int is_last;

    const int tid = threadIdx.x;
    const int lane = tid & (TD_WAVE - 1);
    const int wave = tid / TD_WAVE;
    const int blk = blockIdx.x;
    const int j0 = blk * npb;                        // first neuron of this block
    const int jn = min(npb, h - j0);                 // neurons owned (may be <= 0)

    // ---- the token first (small), then the first batch of predictor rows and their range
    //      bounds, all in flight together
    td_u32x4 xv[XI];
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = min(it * BLOCK + tid, NVW - 1);
        xv[it] = reinterpret_cast<const td_u32x4*>(x)[v];
    }
    asm volatile("" ::: "memory");                   // keep the token's load ahead of the row loads
    td_u32x4 q[RQ][IQ];
    float tl[RQ], th[RQ];
#pragma unroll
    for (int i = 0; i < RQ; ++i) {   // rows past the end re-read a valid row; their result is ignored
        const int j = min(j0 + wave * RQ + i, h - 1);
        load_row<IQ>(q[i], Q + (size_t)j * D, lane);
        tl[i] = tlo[j];
        th[i] = thi[j];
    }
    const float bias_out = bp[min(blk * rpb + wave, D - 1)];

    // ---- stage the token, its max and its int8 code
    if (tid < kMaxNeuronsPerBlock / 32) words[tid] = 0u;
    if (tid == 0) nflag = 0;
    float m = 0.0f;
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = it * BLOCK + tid;
        if (v < NVW) {
            reinterpret_cast<td_u32x4*>(xs)[v] = xv[it];
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(td_bf16_to_f32(e8[u])));
        }
    }
    m = td_wave_max(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, red[w]);
    const int e = token_exponent(m);
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = it * BLOCK + tid;
        if (v < NVW) {
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u]), e)) << (8 * u);
                hi |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u + 4]), e)) << (8 * u);
            }
            reinterpret_cast<uint2*>(xq)[v] = make_uint2(lo, hi);
        }
    }
    __syncthreads();

    // ---- predictor rows: exact int32 dot products, range test, block-local list
    const td_u32x4* xq4 = reinterpret_cast<const td_u32x4*>(xq) + lane;
    for (int base = 0; base < jn; base += NW * RQ) {
        const int jb = base + wave * RQ;
        if (base > 0) {
#pragma unroll
            for (int i = 0; i < RQ; ++i) {
                const int j = min(j0 + jb + i, h - 1);
                load_row<IQ>(q[i], Q + (size_t)j * D, lane);
                tl[i] = tlo[j];
                th[i] = thi[j];
            }
        }
        int acc[RQ];
#pragma unroll
        for (int i = 0; i < RQ; ++i) acc[i] = 0;
#pragma unroll
        for (int it = 0; it < IQ; ++it) {
            const td_u32x4 xx = xq4[it * TD_WAVE];
#pragma unroll
            for (int i = 0; i < RQ; ++i) {
                acc[i] = __builtin_amdgcn_sdot4((int)q[i][it].x, (int)xx.x, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)q[i][it].y, (int)xx.y, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)q[i][it].z, (int)xx.z, acc[i], false);
                acc[i] = __builtin_amdgcn_sdot4((int)q[i][it].w, (int)xx.w, acc[i], false);
            }
        }
#pragma unroll
        for (int i = 0; i < RQ; ++i) {
            const int s = td_wave_sum_i(acc[i]);
            const int jl = jb + i;
            if (jl < jn && lane == 0) {
                const float v = ldexpf((float)s, e);
                const bool inside = (v >= tl[i]) && (v < th[i]);
                if (!inside) {
                    const int pos = atomicAdd(&nflag, 1);
                    flist[pos] = j0 + jl;
                    atomicOr(&words[jl >> 5], 1u << (jl & 31));
                }
            }
        }
    }

    const td_u32x4* xs4 = reinterpret_cast<const td_u32x4*>(xs) + lane;
    const int r0 = blk * rpb;
    const int rn = min(rpb, D - r0);                 // W' rows owned (may be <= 0)
    td_u32x4 wp[IW];
    const td_u32x4* wp_row = reinterpret_cast<const td_u32x4*>(Wp + (size_t)min(r0 + wave, D - 1) * D) + lane;
    // first half of this wave's W' row: requested before the block meets at the barrier, so that
    // the memory pipe stays busy while the flagged list is assembled
    constexpr int IWA = IW / 2;
#pragma unroll
    for (int it = 0; it < IWA; ++it) wp[it] = td_load_stream16(wp_row + it * TD_WAVE);

    __syncthreads();
    if (jn > 0 && tid < (jn + 31) / 32) mask[(j0 >> 5) + tid] = words[tid];
    const int nf = nflag;

    // ---- result fixing.  z_j and delta_j: one wavefront per flagged neuron (16-byte loads of
    //      W1[j], shuffle reduction).  y += delta_j * W2[:, j]: every thread owns the output
    //      columns tid, tid + BLOCK, ... and reads them from W2^T[j] with 2-byte loads (a
    //      wavefront reads 128 contiguous bytes), so the block's repair vector lives in
    //      registers and needs no LDS traffic.
    constexpr int CPT = D / BLOCK;                   // output columns per thread
    constexpr int FCH = (24 / CPT) < NW ? (24 / CPT) : NW;  // flagged neurons per pass (24 row registers)
    float yacc[CPT];
#pragma unroll
    for (int u = 0; u < CPT; ++u) yacc[u] = 0.0f;
    if (nf == 0) {
#pragma unroll
        for (int it = IWA; it < IW; ++it) wp[it] = td_load_stream16(wp_row + it * TD_WAVE);
    }
    for (int f0 = 0; f0 < nf; f0 += FCH) {
        asm volatile("" ::: "memory");   // re-read the token from LDS here instead of keeping it in registers
        const int fi = f0 + wave;
        const bool fixer = wave < FCH && fi < nf;
        td_u32x4 w1[IW];
        int jz = 0;
        float aj = 0.0f, cj = 0.0f, bj = 0.0f;
        if (fixer) {
            jz = flist[fi];
            load_row<IW>(w1, W1 + (size_t)jz * D, lane);
            aj = a[jz];
            cj = c[jz];
            bj = td_bf16_to_f32(b1[jz]);                // b1 is never null here (zeros if the layer has no bias)
        }
        uint16_t w2[FCH][CPT];                       // requested before z is known: one round trip in all
#pragma unroll
        for (int i = 0; i < FCH; ++i) {
            const int j = flist[min(f0 + i, nf - 1)];
            const bf16_t* row = W2T + (size_t)j * D + tid;
#pragma unroll
            for (int u = 0; u < CPT; ++u) w2[i][u] = __builtin_nontemporal_load(row + u * BLOCK);
        }
        // the second half of this wave's W' row is requested BEHIND the repair's loads (loads
        // return in order) and consumed after the repair, so that it streams in while the
        // repair's dependent steps run
        if (f0 == 0) {
            asm volatile("" ::: "memory");
#pragma unroll
            for (int it = IWA; it < IW; ++it) wp[it] = td_load_stream16(wp_row + it * TD_WAVE);
        }
        if (fixer) {
            float z = 0.0f;
#pragma unroll
            for (int it = 0; it < IW; ++it) z = RowVec<bf16_t>::dot(w1[it], xs4[it * TD_WAVE], z);
            z = td_wave_sum(z);
            z += bj;
            if (lane == 0) dl[wave] = td_act(z, act) - fmaf(aj, z, cj);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < FCH; ++i) {
            const float delta = (f0 + i < nf) ? dl[i] : 0.0f;
#pragma unroll
            for (int u = 0; u < CPT; ++u) yacc[u] = fmaf(delta, td_bf16_to_f32(w2[i][u]), yacc[u]);
        }
        __syncthreads();
    }

    // ---- one coalesced atomic pass per block into an accumulator copy (fire and forget)
    if (nf > 0) {
        float* dst = yfix + (size_t)(blk % copies) * D + tid;
#pragma unroll
        for (int u = 0; u < CPT; ++u)
            __hip_atomic_fetch_add(dst + u * BLOCK, yacc[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- speculative product rows (the first one from the registers loaded above)
    for (int ri = wave; ri < rn; ri += NW) {
        asm volatile("" ::: "memory");
        if (ri != wave) load_row<IW>(wp, Wp + (size_t)(r0 + ri) * D, lane);
        float s = 0.0f;
#pragma unroll
        for (int it = 0; it < IW; ++it) s = RowVec<bf16_t>::dot(wp[it], xs4[it * TD_WAVE], s);
        s = td_wave_sum(s);
        // written through to memory so that the finishing block, on any XCD, reads it
        if (lane == 0)
            __hip_atomic_store(yfold + r0 + ri, s + (ri == wave ? bias_out : bp[r0 + ri]), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- signal completion; every store and atomic of this block has been acknowledged
    //      (vmcnt drained by the workgroup-scope release) before the counter moves
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0)
        is_last = (__hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1);
    __syncthreads();
    if (!is_last) return;

    // ---- the last block to finish assembles y and re-arms the scratch
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int OI = (D / 4 + BLOCK - 1) / BLOCK;   // float4 pieces of y per thread
    f32x4 out[OI];
    float ss = 0.0f;
#pragma unroll
    for (int oi = 0; oi < OI; ++oi) {
        const int k4 = oi * BLOCK + tid;
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (k4 < D / 4) {
            v = reinterpret_cast<const f32x4*>(yfold)[k4];
            f32x4 part[kMaxCopies];
#pragma unroll
            for (int cidx = 0; cidx < kMaxCopies; ++cidx)      // all copies requested before any is used
                part[cidx] = cidx < copies ? reinterpret_cast<const f32x4*>(yfix + (size_t)cidx * D)[k4]
                                           : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int cidx = 0; cidx < kMaxCopies; ++cidx) {
                v += part[cidx];
                if (cidx < copies)
                    reinterpret_cast<f32x4*>(yfix + (size_t)cidx * D)[k4] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            }
        }
        out[oi] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    float scale = 1.0f;
    if (norm_out) {   // y / sqrt(mean(y^2) + eps): the glue between stacked layers
        ss = td_wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += red[w];
        scale = 1.0f / sqrtf(tot / (float)D + eps);
    }
#pragma unroll
    for (int oi = 0; oi < OI; ++oi) {
        const int k4 = oi * BLOCK + tid;
        if (k4 < D / 4) {
            const f32x4 v = out[oi] * scale;
            uint2 o;
            o.x = (uint32_t)td_f32_to_bf16(v.x) | ((uint32_t)td_f32_to_bf16(v.y) << 16);
            o.y = (uint32_t)td_f32_to_bf16(v.z) | ((uint32_t)td_f32_to_bf16(v.w) << 16);
            reinterpret_cast<uint2*>(y)[k4] = o;
        }
    }
    if (tid == 0) __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// flagged indices of every token, ascending, and their counts, from the mask words
__global__ void __launch_bounds__(256)
mask_to_list_kernel(const uint32_t* __restrict__ mask, int words, int h, int32_t* __restrict__ counts,
                    int32_t* __restrict__ list) {
    __shared__ int wave_tot[4];
    __shared__ int carry;
    const int t = blockIdx.x;
    const uint32_t* mw = mask + (size_t)t * words;
    int32_t* out = list ? list + (size_t)t * h : nullptr;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < words; base += 256) {
        const int w = base + threadIdx.x;
        const uint32_t bits = w < words ? mw[w] : 0u;
        const int n = __popc(bits);
        int incl = n;  // inclusive scan within the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int off = carry;
        for (int k = 0; k < wave; ++k) off += wave_tot[k];
        int pos = off + incl - n;
        if (out) {
            uint32_t b = bits;
            while (b) {
                const int bit = __ffs(b) - 1;
                b &= b - 1;
                const int j = w * 32 + bit;
                if (j < h && pos < h) out[pos] = j;
                ++pos;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) carry += wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        __syncthreads();
    }
    if (threadIdx.x == 0 && counts) counts[t] = carry;
}

template <int D, int BLOCK>
tardis_status_t launch_decode(tardis_layer_s* L, const void* x, void* y, float* yfold, uint32_t* mask,
                              int norm_out, hipStream_t s) {
    constexpr int RQ = 4;
    const int G = L->dec_blocks;
    const int h = (int)L->h;
    int npb = (h + G - 1) / G;
    npb = (npb + 31) / 32 * 32;
    const int rpb = (D + G - 1) / G;
    hipLaunchKernelGGL((decode_fused_kernel<D, BLOCK, RQ>), dim3(G), dim3(BLOCK), 0, s,
                       static_cast<const bf16_t*>(L->Wp), L->bp, L->Q, L->tlo, L->thi,
                       static_cast<const bf16_t*>(L->W1),
                       static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h), static_cast<const bf16_t*>(L->W2T), L->a, L->c, static_cast<const bf16_t*>(x),
                       static_cast<bf16_t*>(y), yfold, L->yfix, L->dec_copies, mask, L->sync, h, npb, rpb,
                       (int)L->act, norm_out, kRmsEps);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

}  // namespace

bool td_decode_fused_supported(const tardis_layer_s* L) {
    if (L->dtype != TARDIS_BF16) return false;
    if (!(L->d == 1024 || L->d == 2048 || L->d == 4096)) return false;   // wider rows exceed the register file
    const int G = L->dec_blocks;
    if (G < 1) return false;
    int64_t npb = (L->h + G - 1) / G;
    npb = (npb + 31) / 32 * 32;
    return npb <= kMaxNeuronsPerBlock;
}

tardis_status_t td_decode_fused(tardis_layer_s* L, const void* x, void* y, float* yfold, uint32_t* mask,
                                int norm_out, hipStream_t s) {
    if (L->dec_threads == 512) {
        switch (L->d) {
            case 1024: return launch_decode<1024, 512>(L, x, y, yfold, mask, norm_out, s);
            case 2048: return launch_decode<2048, 512>(L, x, y, yfold, mask, norm_out, s);
            case 4096: return launch_decode<4096, 512>(L, x, y, yfold, mask, norm_out, s);
        }
    }
    switch (L->d) {
        case 1024: return launch_decode<1024, 1024>(L, x, y, yfold, mask, norm_out, s);
        case 2048: return launch_decode<2048, 1024>(L, x, y, yfold, mask, norm_out, s);
        case 4096: return launch_decode<4096, 1024>(L, x, y, yfold, mask, norm_out, s);
    }
    return TARDIS_ERR_SHAPE;
}

tardis_status_t td_mask_to_list(const tardis_layer_s* L, int64_t n, int32_t* counts, int32_t* list, hipStream_t s) {
    hipLaunchKernelGGL(mask_to_list_kernel, dim3((unsigned)n), dim3(256), 0, s, L->mask, (int)L->mask_words,
                       (int)L->h, counts, list);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
