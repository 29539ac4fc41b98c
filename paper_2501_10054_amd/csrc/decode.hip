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

// TB tokens (1, 2 or 4) share one pass over the weights: x, y, yfold are TB x D, mask has TB rows of
// mask_words words, yfix is copies x TB x D.
//
// SK = 8: Q holds one int8 code per weight.  SK = 4: Q holds the packed 4-bit sketch, one 16-byte
// vector per group of 32 columns (byte b of dword w = code of column 4w+b in the low nibble, of column
// 16+4w+b in the high nibble), M4 one multiplier byte per group; the integer the range test sees is
// sum over groups of multiplier * (code . token code), the same number an int8 row of
// multiplier*code would give.
template <int D, int BLOCK, int RQ, int TB, int SK>
__global__ void __launch_bounds__(BLOCK)
decode_fused_kernel(const bf16_t* __restrict__ Wp, const float* __restrict__ bp, const int8_t* __restrict__ Q,
                    const uint8_t* __restrict__ M4, const float* __restrict__ tlo, const float* __restrict__ thi, const bf16_t* __restrict__ W1,
                    const bf16_t* __restrict__ b1, const bf16_t* __restrict__ W2T, const float* __restrict__ a,
                    const float* __restrict__ c, const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                    float* __restrict__ yfold, float* __restrict__ yfix, int copies, uint32_t* __restrict__ mask,
                    int mask_words, int32_t* __restrict__ done, int h, int npb, int rpb, int act, int norm_out,
                    float eps) {
    static_assert(D % 1024 == 0, "rows must be whole multiples of 64 lanes x 16 bytes");
    static_assert(D % BLOCK == 0 && BLOCK / TD_WAVE >= 4, "column ownership of the repair pass");
    static_assert(TB == 1 || TB == 2 || TB == 4, "tokens per pass");
    static_assert(SK == 8 || (SK == 4 && D % 2048 == 0), "a packed 4-bit row must fill whole wavefront loads");
    constexpr int NW = BLOCK / TD_WAVE;
    constexpr int NVW = D / 8;                       // 16-byte vectors per bf16 row
    constexpr int QROW = SK == 8 ? D : D / 2;        // bytes of one predictor row
    constexpr int IQ = QROW / 16 / TD_WAVE;          // per-lane vectors of a predictor row
    constexpr int IW = NVW / TD_WAVE;                // per-lane vectors of a bf16 row
    constexpr int XI = (TB * NVW + BLOCK - 1) / BLOCK;  // per-thread vectors of the tokens
    constexpr int MW = kMaxNeuronsPerBlock / 32;

    __shared__ __align__(16) bf16_t xs[TB * D];
    __shared__ __align__(16) int8_t xq[TB * D];
    __shared__ float dl[NW][TB];                     // delta of the neurons being repaired, per token
    __shared__ int flist[kMaxNeuronsPerBlock];       // neurons flagged by at least one token
    __shared__ unsigned char fbits[kMaxNeuronsPerBlock];  // which tokens flagged them
    __shared__ uint32_t words[TB][MW];
    __shared__ int tmax[TB];                         // max |x| per token (bit pattern of a non-negative float)
    __shared__ int nflag;
    __shared__ int is_last;

    const int tid = threadIdx.x;
    const int lane = tid & (TD_WAVE - 1);
    const int wave = tid / TD_WAVE;
    const int blk = blockIdx.x;
    const int j0 = blk * npb;                        // first neuron of this block
    const int jn = min(npb, h - j0);                 // neurons owned (may be <= 0)

    // ---- the tokens first (small), then the first batch of predictor rows and their range
    //      bounds, all in flight together
    td_u32x4 xv[XI];
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = min(it * BLOCK + tid, TB * NVW - 1);
        xv[it] = reinterpret_cast<const td_u32x4*>(x)[v];
    }
    asm volatile("" ::: "memory");                   // keep the tokens' loads ahead of the row loads
    td_u32x4 q[RQ][IQ];
    uint32_t mg[RQ][IQ];                             // group multipliers (4-bit sketch only)
    float tl[RQ], th[RQ];
    auto load_pred_rows = [&](const int jfirst) {    // rows past the end re-read a valid row; their result is ignored
#pragma unroll
        for (int i = 0; i < RQ; ++i) {
            const int j = min(jfirst + i, h - 1);
            load_row<IQ>(q[i], Q + (size_t)j * QROW, lane);
            if (SK == 4) {
#pragma unroll
                for (int it = 0; it < IQ; ++it) mg[i][it] = M4[(size_t)j * (D / 32) + it * TD_WAVE + lane];
            }
            tl[i] = tlo[j];
            th[i] = thi[j];
        }
    };
    load_pred_rows(j0 + wave * RQ);
    const float bias_out = bp[min(blk * rpb + wave, D - 1)];

    // ---- stage the tokens, their maxima and their int8 codes
    for (int k = tid; k < TB * MW; k += BLOCK) (&words[0][0])[k] = 0u;
    if (tid < TB) tmax[tid] = 0;
    if (tid == 0) nflag = 0;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = it * BLOCK + tid;
        if (v < TB * NVW) {
            reinterpret_cast<td_u32x4*>(xs)[v] = xv[it];
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
            float m = 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(td_bf16_to_f32(e8[u])));
            m = td_wave_max(m);                      // a wavefront's 64 vectors belong to one token
            if (lane == 0) atomicMax(&tmax[v / NVW], __float_as_int(m));
        }
    }
    __syncthreads();
    int ex[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) ex[t] = token_exponent(__int_as_float(tmax[t]));
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = it * BLOCK + tid;
        if (v < TB * NVW) {
            const int tok = v / NVW;
            int e = ex[0];
#pragma unroll
            for (int t = 1; t < TB; ++t) e = tok == t ? ex[t] : e;
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u]), e)) << (8 * u);
                hi |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u + 4]), e)) << (8 * u);
            }
            if (SK == 8) {
                reinterpret_cast<uint2*>(xq)[v] = make_uint2(lo, hi);
            } else {   // columns 0..15 of every group of 32 in the first half of the token's codes, 16..31 in the second
                const int i8 = v - tok * NVW, g = i8 >> 2, part = i8 & 3;
                const int at = tok * (D / 8) + (part < 2 ? 0 : D / 16) + g * 2 + (part & 1);
                reinterpret_cast<uint2*>(xq)[at] = make_uint2(lo, hi);
            }
        }
    }
    __syncthreads();

    // ---- predictor rows: exact int32 dot products, range test per token, block-local list of
    //      the neurons flagged by at least one token
    const td_u32x4* xq4 = reinterpret_cast<const td_u32x4*>(xq) + lane;
    for (int base = 0; base < jn; base += NW * RQ) {
        const int jb = base + wave * RQ;
        if (base > 0) load_pred_rows(j0 + jb);
        // two tokens at a time against the rows held in registers (register budget)
        constexpr int TP = TB < 2 ? TB : 2;
        uint32_t bits[RQ];
#pragma unroll
        for (int i = 0; i < RQ; ++i) bits[i] = 0u;
#pragma unroll
        for (int t0 = 0; t0 < TB; t0 += TP) {
            if (TB > 1) asm volatile("" ::: "memory");
            int acc[RQ][TP];
#pragma unroll
            for (int i = 0; i < RQ; ++i)
#pragma unroll
                for (int t = 0; t < TP; ++t) acc[i][t] = 0;
#pragma unroll
            for (int it = 0; it < IQ; ++it) {
                if (SK == 8) {
#pragma unroll
                    for (int t = 0; t < TP; ++t) {
                        const td_u32x4 xx = xq4[(t0 + t) * (D / 16) + it * TD_WAVE];
#pragma unroll
                        for (int i = 0; i < RQ; ++i) {
                            acc[i][t] = __builtin_amdgcn_sdot4((int)q[i][it].x, (int)xx.x, acc[i][t], false);
                            acc[i][t] = __builtin_amdgcn_sdot4((int)q[i][it].y, (int)xx.y, acc[i][t], false);
                            acc[i][t] = __builtin_amdgcn_sdot4((int)q[i][it].z, (int)xx.z, acc[i][t], false);
                            acc[i][t] = __builtin_amdgcn_sdot4((int)q[i][it].w, (int)xx.w, acc[i][t], false);
                        }
                    }
                } else {
                    // a nibble moved to the top of its byte is 16 * code as a signed byte: the group
                    // sums below are 16 times the true ones, taken out after the reduction
                    td_u32x4 xl[TP], xh[TP];
#pragma unroll
                    for (int t = 0; t < TP; ++t) {
                        xl[t] = xq4[(t0 + t) * (D / 16) + it * TD_WAVE];
                        xh[t] = xq4[(t0 + t) * (D / 16) + D / 32 + it * TD_WAVE];
                    }
#pragma unroll
                    for (int i = 0; i < RQ; ++i) {
                        const td_u32x4 w = q[i][it];
                        const td_u32x4 wl = (w << 4) & 0xF0F0F0F0u, wh = w & 0xF0F0F0F0u;
#pragma unroll
                        for (int t = 0; t < TP; ++t) {
                            int g = __builtin_amdgcn_sdot4((int)wl.x, (int)xl[t].x, 0, false);
                            g = __builtin_amdgcn_sdot4((int)wl.y, (int)xl[t].y, g, false);
                            g = __builtin_amdgcn_sdot4((int)wl.z, (int)xl[t].z, g, false);
                            g = __builtin_amdgcn_sdot4((int)wl.w, (int)xl[t].w, g, false);
                            g = __builtin_amdgcn_sdot4((int)wh.x, (int)xh[t].x, g, false);
                            g = __builtin_amdgcn_sdot4((int)wh.y, (int)xh[t].y, g, false);
                            g = __builtin_amdgcn_sdot4((int)wh.z, (int)xh[t].z, g, false);
                            g = __builtin_amdgcn_sdot4((int)wh.w, (int)xh[t].w, g, false);
                            acc[i][t] += (int)mg[i][it] * g;
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RQ; ++i) {
#pragma unroll
                for (int t = 0; t < TP; ++t) {
                    const int total = td_wave_sum_i(acc[i][t]);
                    const float v = ldexpf((float)(SK == 8 ? total : total >> 4), ex[t0 + t]);
                    const bool inside = (v >= tl[i]) && (v < th[i]);
                    bits[i] |= inside ? 0u : (1u << (t0 + t));
                }
            }
        }
#pragma unroll
        for (int i = 0; i < RQ; ++i) {
            const int jl = jb + i;
            if (jl < jn && lane == 0 && bits[i]) {
#pragma unroll
                for (int t = 0; t < TB; ++t)
                    if ((bits[i] >> t) & 1u) atomicOr(&words[t][jl >> 5], 1u << (jl & 31));
                const int pos = atomicAdd(&nflag, 1);
                flist[pos] = j0 + jl;
                fbits[pos] = (unsigned char)bits[i];
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
    if (jn > 0) {
        const int nw = (jn + 31) / 32;
        for (int k = tid; k < TB * nw; k += BLOCK) {
            const int t = k / nw, w = k % nw;
            mask[(size_t)t * mask_words + (j0 >> 5) + w] = words[t][w];
        }
    }
    const int nf = nflag;

    // ---- result fixing.  z and delta: one wavefront per flagged neuron (16-byte loads of
    //      W1[j], shuffle reduction), for the tokens that flagged it.  y += delta * W2[:, j]:
    //      every thread owns the output columns tid, tid + BLOCK, ... and reads them from
    //      W2^T[j] with 2-byte loads (a wavefront reads 128 contiguous bytes), so the block's
    //      repair vectors live in registers and need no LDS traffic.
    constexpr int CPT = D / BLOCK;                   // output columns per thread
    constexpr int WREG = TB == 1 ? 24 : 16;          // registers holding W2^T elements per pass
    constexpr int FCH = (WREG / CPT) < NW ? (WREG / CPT) : NW;  // flagged neurons per pass
    float yacc[TB][CPT];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int u = 0; u < CPT; ++u) yacc[t][u] = 0.0f;
    // the columns a thread owns are rotated by a block-dependent number of wavefronts, so that
    // the blocks' atomic passes do not all start on the same cache lines
    const int ctid = (tid + TD_WAVE * (blk >> 3)) & (BLOCK - 1);
    // one pass over up to FCH flagged neurons.  The first pass is straight-line code (no
    // loop-carried register state), and it also requests the second half of this wave's W' row
    // BEHIND the repair's loads (loads return in order): it is consumed after the repair and
    // streams in while the repair's dependent steps run.
    auto repair_pass = [&](auto first_tag, const int f0) {
        constexpr bool kFirst = decltype(first_tag)::value;
        asm volatile("" ::: "memory");   // re-read the tokens from LDS here instead of keeping them in registers
        const int fi = f0 + wave;
        const bool fixer = wave < FCH && fi < nf;
        td_u32x4 w1[IW];
        float aj = 0.0f, cj = 0.0f;
        uint32_t bj_raw = 0;
        if (fixer) {
            const int jz = flist[fi];
            load_row<IW>(w1, W1 + (size_t)jz * D, lane);
            aj = a[jz];
            cj = c[jz];
            bj_raw = b1[jz];                         // b1 is never null here (zeros if the layer has no bias)
        }
        uint16_t w2[FCH][CPT];                       // requested before z is known: one round trip in all
#pragma unroll
        for (int i = 0; i < FCH; ++i) {
            const int j = flist[min(f0 + i, nf - 1)];
            const bf16_t* row = W2T + (size_t)j * D + ctid;
#pragma unroll
            for (int u = 0; u < CPT; ++u) w2[i][u] = __builtin_nontemporal_load(row + u * BLOCK);
        }
        if (kFirst) {
            asm volatile("" ::: "memory");
#pragma unroll
            for (int it = IWA; it < IW; ++it) wp[it] = td_load_stream16(wp_row + it * TD_WAVE);
        }
        // nothing above may wait for a load: the conversion of b1 is pinned below this point
        asm volatile("" : "+v"(bj_raw), "+v"(aj), "+v"(cj));
        if (fixer) {
            const float bj = td_bf16_to_f32((bf16_t)bj_raw);
            const uint32_t zbits = fbits[fi];
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (TB > 1) asm volatile("" ::: "memory");   // one token's LDS reads at a time (register budget)
                float z = 0.0f;
#pragma unroll
                for (int it = 0; it < IW; ++it) z = RowVec<bf16_t>::dot(w1[it], xs4[t * NVW + it * TD_WAVE], z);
                z = td_wave_sum(z) + bj;
                const float dv = ((zbits >> t) & 1u) ? td_act(z, act) - fmaf(aj, z, cj) : 0.0f;
                if (lane == 0) dl[wave][t] = dv;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < FCH; ++i) {
            if (f0 + i < nf) {
#pragma unroll
                for (int t = 0; t < TB; ++t) {
                    const float delta = dl[i][t];
#pragma unroll
                    for (int u = 0; u < CPT; ++u)
                        yacc[t][u] = fmaf(delta, td_bf16_to_f32(w2[i][u]), yacc[t][u]);
                }
            }
        }
        __syncthreads();
    };
    if (nf == 0) {
#pragma unroll
        for (int it = IWA; it < IW; ++it) wp[it] = td_load_stream16(wp_row + it * TD_WAVE);
    } else {
        repair_pass(std::true_type{}, 0);
        for (int f0 = FCH; f0 < nf; f0 += FCH) repair_pass(std::false_type{}, f0);
    }

    // ---- one coalesced atomic pass per block and token into an accumulator copy (fire and forget)
    auto atomic_pass = [&]() {
        if (nf > 0) {
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                float* dst = yfix + ((size_t)(blk % copies) * TB + t) * D + ctid;
#pragma unroll
                for (int u = 0; u < CPT; ++u)
                    if (TB == 1 || yacc[t][u] != 0.0f)
                        __hip_atomic_fetch_add(dst + u * BLOCK, yacc[t][u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };
    atomic_pass();

    // ---- speculative product rows (the first one from the registers loaded above)
    for (int ri = wave; ri < rn; ri += NW) {
        asm volatile("" ::: "memory");
        if (ri != wave) load_row<IW>(wp, Wp + (size_t)(r0 + ri) * D, lane);
        const float bias = ri == wave ? bias_out : bp[r0 + ri];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            if (TB > 1) asm volatile("" ::: "memory");
            float s = 0.0f;
#pragma unroll
            for (int it = 0; it < IW; ++it) s = RowVec<bf16_t>::dot(wp[it], xs4[t * NVW + it * TD_WAVE], s);
            s = td_wave_sum(s);
            // written through to memory so that the finishing block, on any XCD, reads it
            if (lane == 0)
                __hip_atomic_store(yfold + (size_t)t * D + r0 + ri, s + bias, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
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
    constexpr int OI = (D / 4 + BLOCK - 1) / BLOCK;   // float4 pieces of one token's y per thread
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 out[TB][OI];
    f32x4 part[TB][OI][kMaxCopies];
#pragma unroll
    for (int t = 0; t < TB; ++t)                      // every load of every token requested before any is used
#pragma unroll
        for (int oi = 0; oi < OI; ++oi) {
            const int k4 = oi * BLOCK + tid;
            const bool live = k4 < D / 4;
            out[t][oi] = live ? reinterpret_cast<const f32x4*>(yfold + (size_t)t * D)[k4] : zero4;
#pragma unroll
            for (int cidx = 0; cidx < kMaxCopies; ++cidx)
                part[t][oi][cidx] = (live && cidx < copies)
                                        ? reinterpret_cast<const f32x4*>(yfix + ((size_t)cidx * TB + t) * D)[k4]
                                        : zero4;
        }
    float ss[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        ss[t] = 0.0f;
#pragma unroll
        for (int oi = 0; oi < OI; ++oi) {
            const int k4 = oi * BLOCK + tid;
            f32x4 v = out[t][oi];
#pragma unroll
            for (int cidx = 0; cidx < kMaxCopies; ++cidx) {
                v += part[t][oi][cidx];
                if (k4 < D / 4 && cidx < copies)
                    reinterpret_cast<f32x4*>(yfix + ((size_t)cidx * TB + t) * D)[k4] = zero4;
            }
            out[t][oi] = v;
            ss[t] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
    }
    float scale[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) scale[t] = 1.0f;
    if (norm_out) {   // y / sqrt(mean(y^2) + eps): the glue between stacked layers
        float* redt = &dl[0][0];                      // NW x TB floats, free by now
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            const float w = td_wave_sum(ss[t]);
            if (lane == 0) redt[wave * TB + t] = w;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            float tot = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) tot += redt[w * TB + t];
            scale[t] = 1.0f / sqrtf(tot / (float)D + eps);
        }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int oi = 0; oi < OI; ++oi) {
            const int k4 = oi * BLOCK + tid;
            if (k4 < D / 4) {
                const f32x4 v = out[t][oi] * scale[t];
                uint2 o;
                o.x = (uint32_t)td_f32_to_bf16(v.x) | ((uint32_t)td_f32_to_bf16(v.y) << 16);
                o.y = (uint32_t)td_f32_to_bf16(v.z) | ((uint32_t)td_f32_to_bf16(v.w) << 16);
                reinterpret_cast<uint2*>(y + (size_t)t * D)[k4] = o;
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

template <int D, int BLOCK, int TB, int SK>
tardis_status_t launch_decode(tardis_layer_s* L, const void* x, void* y, float* yfold, uint32_t* mask,
                              int norm_out, hipStream_t s) {
    constexpr int RQ = 4;
    const int G = L->dec_blocks;
    const int h = (int)L->h;
    int npb = (h + G - 1) / G;
    npb = (npb + 31) / 32 * 32;
    const int rpb = (D + G - 1) / G;
    const int8_t* codes = SK == 8 ? L->Q : reinterpret_cast<const int8_t*>(L->Q4);
    hipLaunchKernelGGL((decode_fused_kernel<D, BLOCK, RQ, TB, SK>), dim3(G), dim3(BLOCK), 0, s,
                       static_cast<const bf16_t*>(L->Wp), L->bp, codes, L->M4, L->tlo, L->thi,
                       static_cast<const bf16_t*>(L->W1),
                       static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h), static_cast<const bf16_t*>(L->W2T),
                       L->a, L->c, static_cast<const bf16_t*>(x), static_cast<bf16_t*>(y), yfold, L->yfix,
                       L->dec_copies, mask, (int)L->mask_words, L->sync, h, npb, rpb, (int)L->act, norm_out, kRmsEps);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

template <int D, int BLOCK, int SK>
tardis_status_t launch_tb(tardis_layer_s* L, const void* x, void* y, float* yfold, uint32_t* mask, int tokens,
                          int norm_out, hipStream_t s) {
    switch (tokens) {
        case 1: return launch_decode<D, BLOCK, 1, SK>(L, x, y, yfold, mask, norm_out, s);
        case 2: return launch_decode<D, BLOCK, 2, SK>(L, x, y, yfold, mask, norm_out, s);
        case 4: return launch_decode<D, BLOCK, 4, SK>(L, x, y, yfold, mask, norm_out, s);
    }
    return TARDIS_ERR_INVALID_ARG;
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

// `tokens` (1, 2 or 4) consecutive tokens in one launch
tardis_status_t td_decode_fused(tardis_layer_s* L, const void* x, void* y, float* yfold, uint32_t* mask,
                                int tokens, int norm_out, hipStream_t s) {
    if (L->Q4) {   // packed 4-bit sketch (d = 2048 or 4096 only)
        if (L->dec_threads == 512) {
            if (L->d == 2048) return launch_tb<2048, 512, 4>(L, x, y, yfold, mask, tokens, norm_out, s);
            if (L->d == 4096) return launch_tb<4096, 512, 4>(L, x, y, yfold, mask, tokens, norm_out, s);
        } else {
            if (L->d == 2048) return launch_tb<2048, 1024, 4>(L, x, y, yfold, mask, tokens, norm_out, s);
            if (L->d == 4096) return launch_tb<4096, 1024, 4>(L, x, y, yfold, mask, tokens, norm_out, s);
        }
        return TARDIS_ERR_SHAPE;
    }
    if (L->dec_threads == 512) {
        switch (L->d) {
            case 1024: return launch_tb<1024, 512, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
            case 2048: return launch_tb<2048, 512, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
            case 4096: return launch_tb<4096, 512, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
        }
    }
    switch (L->d) {
        case 1024: return launch_tb<1024, 1024, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
        case 2048: return launch_tb<2048, 1024, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
        case 4096: return launch_tb<4096, 1024, 8>(L, x, y, yfold, mask, tokens, norm_out, s);
    }
    return TARDIS_ERR_SHAPE;
}

tardis_status_t td_mask_to_list(const tardis_layer_s* L, int64_t n, int32_t* counts, int32_t* list, hipStream_t s) {
    hipLaunchKernelGGL(mask_to_list_kernel, dim3((unsigned)n), dim3(256), 0, s, L->mask, (int)L->mask_words,
                       (int)L->h, counts, list);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
