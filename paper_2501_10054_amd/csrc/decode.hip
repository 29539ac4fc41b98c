// Decode path (1 to 16 tokens per launch, bf16 storage): the whole online step of
// Sec. "Inference Runtime" -- speculative product, predictor, mask, result fixing --
// in ONE kernel for one or two tokens, so that a token costs one launch and every
// weight byte is requested exactly once; groups of 4, 8 and 16 tokens take a second
// kernel for the down projection (see DEFER below).
//
// Work split.  The grid has G blocks; block b owns
//   * neurons   [b*npb, (b+1)*npb)   : predictor rows of Q, and the repair of
//                                      those of them that turn out flagged
//   * outputs   [b*rpb, (b+1)*rpb)   : rows of W' for the speculative product
// so no block ever waits for another: a neuron's flag is known inside the block
// that will repair it.  The repair needs y += delta_j * W2[:, j] over ALL
// outputs; each thread keeps its columns of the block's sum over its flagged
// neurons in registers and adds them once, with fully coalesced fp32 atomics,
// into one of K accumulator copies.  The last block to finish (a device
// counter) adds the copies to the speculative result, converts to bf16, and
// re-arms the accumulators and the counter for the next call; the others spend
// that time warming the caches for the layer that runs next, if it is known.
#include <cstdlib>
#include <mutex>

#include "common.h"
#include "rowdot.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace {

constexpr int kMaxNeuronsPerBlock = 512;
constexpr int kMaxCopies = 4;                  // repair accumulator copies (blocks spread over them)

// Wait until every vector-memory operation this wavefront has issued (loads, stores, atomics
// without return) has been acknowledged.  No cache write-back or invalidation is involved.
__device__ __forceinline__ void td_wait_memory_acks() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float load_coherent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// four floats that blocks on other XCDs added to during this launch (device-coherent loads: no
// cache invalidation needed before them, which is what the agent-scope acquire would cost)
typedef float td_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ td_f32x4 load_coherent4(const float* p) {
    td_f32x4 v;
    v.x = load_coherent(p);
    v.y = load_coherent(p + 1);
    v.z = load_coherent(p + 2);
    v.w = load_coherent(p + 3);
    return v;
}

// acc + sum over 16 columns of w (sixteen e4m3 bytes) * x (sixteen bf16 in xa, xb), fp32
typedef float td_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot_e4m3_bf16(const td_u32x4& w, const td_u32x4& xa, const td_u32x4& xb, float acc) {
    const uint32_t wq[4] = {w.x, w.y, w.z, w.w};
    const uint32_t xq[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {   // dword q: columns 4q .. 4q+3
        const td_f32x2 f01 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wq[q], false);
        const td_f32x2 f23 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wq[q], true);
        acc = fmaf(f01.x, __uint_as_float(xq[2 * q] << 16), acc);
        acc = fmaf(f01.y, __uint_as_float(xq[2 * q] & 0xFFFF0000u), acc);
        acc = fmaf(f23.x, __uint_as_float(xq[2 * q + 1] << 16), acc);
        acc = fmaf(f23.y, __uint_as_float(xq[2 * q + 1] & 0xFFFF0000u), acc);
    }
    return acc;
}

// 16-byte vectors it*64 + lane, it = 0..N-1, of one row (N*64 vectors long)
template <int N>
__device__ __forceinline__ void load_row(td_u32x4 (&dst)[N], const void* row, int lane) {
    const td_u32x4* p = static_cast<const td_u32x4*>(row) + lane;
#pragma unroll
    for (int it = 0; it < N; ++it) dst[it] = td_load_stream16(p + it * TD_WAVE);
}

// Counted fixed-point accumulator.  Bits 0..15 count the contributions received, bits 16..63 hold
// their sum as a signed integer number of units.  The unit of a token is a power of two chosen from
// a bound on the magnitude of ANY partial sum of contributions to one output of that token,
//     |.| <= K1 * max|x| + K2        (K1, K2 per layer, computed when the layer is folded),
// so that the sum never leaves the 48-bit field: unit = 2^(e - 46) with 2^e > the bound.  Adding the
// 64-bit words with integer atomics adds both fields at once and exactly; the add that returns
// count == expected - 1 is the last one and its thread holds the finished sum.
struct FxAcc {
    static constexpr int kCountBits = 16;
    static constexpr int kValueBits = 46;            // bound / unit
    // exponent e with 2^e > bound (clamped so that every scale below is a normal float)
    static __device__ __forceinline__ int exponent(float k1, float k2, float xmax) {
        const float bound = fmaf(k1, xmax, k2);
        int e = 0;
        if (bound > 0.0f && bound < INFINITY) (void)frexpf(bound, &e);
        return min(max(e, -60), 120);
    }
    static __device__ __forceinline__ unsigned long long encode(float v, int e) {
        const long long q = __float2ll_rn(ldexpf(v, kValueBits - e));
        return (static_cast<unsigned long long>(q) << kCountBits) + 1ull;
    }
    static __device__ __forceinline__ bool completes(unsigned long long before, int expected) {
        return (int)(before & ((1u << kCountBits) - 1u)) == expected - 1;
    }
    static __device__ __forceinline__ float decode(unsigned long long total, int e) {
        return ldexpf((float)(static_cast<long long>(total) >> kCountBits), e - kValueBits);
    }
    static __device__ __forceinline__ unsigned long long add(unsigned long long* p, unsigned long long enc) {
        return __hip_atomic_fetch_add(p, enc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

// TB tokens (1, 2, 4, 8 or 16) share one pass over the weights: x, y, yfold are TB x D, mask has TB rows of
// mask_words words, yfix is copies x TB x D.
//
// SK = 8: Q holds one int8 code per weight.  SK = 4: Q holds the packed 4-bit sketch, one 16-byte
// vector per group of 32 columns (byte b of dword w = code of column 4w+b in the low nibble, of column
// 16+4w+b in the high nibble), M4 one multiplier byte per group; the integer the range test sees is
// sum over groups of multiplier * (code . token code), the same number an int8 row of
// multiplier*code would give.
//
// DEFER = true: the block stops after computing delta for its flagged neurons and writes one record
// per flagged neuron (index, token bits, TB deltas) instead of applying W2^T; the speculative rows
// go to yfold with plain stores and a second kernel (down_project_kernel) finishes the tokens.
// With many tokens per launch this replaces TB x d atomics per block by a column-sliced pass.
struct DeferOut {
    int32_t* count;    // flagged neurons of every block
    uint32_t* jb;      // blocks x cap: neuron index
    uint32_t* tb;      // blocks x cap: bit t set iff token t flagged the neuron
    float* delta;      // blocks x cap x TB
    int cap;           // record slots per block (= neurons per block)
};

// Device working memory of one decode call beyond its inputs and outputs: the layer's own
// buffers, or the library's static scratch (tardis_ffn_forward_static).
struct DecodeScratch {
    float* yfix;        // copies x kDecodeMaxTokens x d repair accumulators (zero between calls)
    int32_t* sync;      // completion counters (zero between calls)
    int32_t* rec_count; // records of the two-kernel path
    uint32_t* rec_jb;
    uint32_t* rec_tb;
    float* rec_delta;
};

// A block that has finished while the rest of the launch drains (atomics, the last block's
// assembly) requests `bytes` (whole 16-byte vectors, >= 16) of rows it will read first in the
// launch that follows - the predictor rows of its block index in the next layer.  The values are
// discarded; the point is that they sit in cache when that launch asks for them.
template <int BLOCK>
__device__ __forceinline__ void warm_rows(const unsigned char* __restrict__ p, int bytes, int tid) {
    constexpr int PFU = 256 * 1024 / (BLOCK * 16);   // up to 256 KB per block
    td_u32x4 v[PFU];
#pragma unroll
    for (int u = 0; u < PFU; ++u)                    // past the limit: re-read the last vector
        v[u] = *reinterpret_cast<const td_u32x4*>(p + min((u * BLOCK + tid) * 16, bytes - 16));
#pragma unroll
    for (int u = 0; u < PFU; ++u) asm volatile("" ::"v"(v[u]));
}

//
// NG > 0 (8 tokens): the predictor rows go through the int8 matrix cores instead of packed dot
// products: the block's rows form NG groups of 16, each group is shared by NW/NG wavefronts that
// split the columns, a wavefront multiplies its 16 rows x K-slice with the 8 tokens by
// v_mfma_i32_16x16x64_i8 (tokens 8..15 of the tile repeat tokens 0..7 and are ignored), and the
// partial sums meet in LDS.  Eight tokens of packed dot products would keep the vector ALUs busy
// for longer than the rows take to arrive.
//
// FX = true: the repair accumulators are 64-bit fixed-point words that also count their
// contributions (see FxAcc): every block adds to every column exactly once, integer adds commute,
// so the result does not depend on the order in which blocks finish (bit-identical from run to
// run), and the thread whose add completes a column's count holds that column's finished sum and
// writes y itself - no completion counter and no assembling block on the way out.
//
// WP8 = true (one kernel, fp32 accumulators only): the block's rows of W' are read in their 8-bit
// floating-point form (e4m3 codes, a power-of-two scale per row) - half the bytes of the bf16 rows;
// the values are the same numbers the bf16 copy of the matrix holds.
template <int D, int BLOCK, int RQ, int TB, int SK, bool DEFER, int NG, bool FX, bool WP8>
__global__ void __launch_bounds__(BLOCK)
decode_fused_kernel(const bf16_t* __restrict__ Wp, const float* __restrict__ bp, const int8_t* __restrict__ Q,
                    const uint8_t* __restrict__ M4, const float* __restrict__ tlo, const float* __restrict__ thi, const bf16_t* __restrict__ W1,
                    const bf16_t* __restrict__ b1, const bf16_t* __restrict__ W2T, const float* __restrict__ a,
                    const float* __restrict__ c, const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                    float* __restrict__ yfold, float* __restrict__ yfix, int copies, uint32_t* __restrict__ mask,
                    int mask_words, int32_t* __restrict__ done, int h, int npb, int rpb, int act, int norm_out,
                    float eps, DeferOut rec, int n_act, const unsigned char* __restrict__ pf_rows, int pf_bytes,
                    const float* __restrict__ fx_bound, int32_t* __restrict__ fx_exp, int strict_release, int pf_shape,
                    const uint8_t* __restrict__ Wp8, const float* __restrict__ wp8_scale) {
    // n_act <= TB tokens are real: the remaining slots of the group repeat the last real token and
    // none of their results reaches the caller's buffers
    static_assert(D % 1024 == 0, "rows must be whole multiples of 64 lanes x 16 bytes");
    static_assert(D % BLOCK == 0 && BLOCK / TD_WAVE >= 4, "column ownership of the repair pass");
    static_assert(TB == 1 || TB == 2 || TB == 4 || ((TB == 8 || TB == 16) && DEFER), "tokens per pass");
    static_assert(SK == 8 || (SK == 4 && D % 2048 == 0), "a packed 4-bit row must fill whole wavefront loads");
    static_assert(NG == 0 || (SK == 8 && (TB == 8 || TB == 16) && DEFER && (BLOCK / TD_WAVE) % NG == 0),
                  "matrix-core predictor");
    static_assert(TB < 16 || NG > 0, "sixteen tokens only with the matrix-core predictor");
    static_assert(!WP8 || (!DEFER && !FX && TB <= 2), "8-bit W' rows: one- and two-token launches with fp32 accumulators");
    constexpr int NW = BLOCK / TD_WAVE;
    constexpr int KQ = NW / (NG > 0 ? NG : 1);       // wavefronts sharing a group of 16 rows
    constexpr int KS = D / KQ;                       // columns of one wavefront's slice
    constexpr int NL = NG > 0 ? KS / 64 : 1;         // 16-byte vectors per lane of that slice
    constexpr int XP = NG > 0 ? D + 16 : D;          // LDS pitch of a token's int8 code (bank spread for the tile reads)
    constexpr int XSP = DEFER ? D + 8 : D;           // LDS pitch of a token in elements (same reason, W' tiles)
    constexpr int KW = D / NW;                       // columns of W' one wavefront multiplies on the deferred path
    static_assert(NG == 0 || (KS % 64 == 0 && NL >= 1), "slice of whole 64-column steps");
    constexpr int NVW = D / 8;                       // 16-byte vectors per bf16 row
    constexpr int QROW = SK == 8 ? D : D / 2;        // bytes of one predictor row
    constexpr int IQ = QROW / 16 / TD_WAVE;          // per-lane vectors of a predictor row
    constexpr int IW = NVW / TD_WAVE;                // per-lane vectors of a bf16 row
    static_assert(!DEFER || (KW % 32 == 0 && KW * 2 / 64 == IW), "W' slices of whole 32-column steps, IW vectors per lane");
    constexpr int XI = (TB * NVW + BLOCK - 1) / BLOCK;  // per-thread vectors of the tokens
    constexpr int MW = kMaxNeuronsPerBlock / 32;

    // TB x D bf16 tokens and their int8 codes: static LDS while they fit the 64 KiB a kernel may
    // declare, the dynamic segment for the larger groups
    constexpr bool kStaticTokens = !DEFER && (size_t)TB * D * 3 <= 56 * 1024;
    extern __shared__ __align__(16) unsigned char token_lds[];
    __shared__ __align__(16) bf16_t xs_fixed[kStaticTokens ? TB * D : 8];
    __shared__ __align__(16) int8_t xq_fixed[kStaticTokens ? TB * D : 16];
    bf16_t* xs = kStaticTokens ? xs_fixed : reinterpret_cast<bf16_t*>(token_lds);
    // sixteen tokens: the int8 codes live where the tokens will go once the predictor is done with
    // them (the tokens wait in registers meanwhile); both do not fit the LDS at once
    constexpr bool kAlias = TB == 16;
    int8_t* xq = kStaticTokens ? xq_fixed
                               : reinterpret_cast<int8_t*>(token_lds + (kAlias ? (size_t)0 : (size_t)TB * XSP * 2));
    __shared__ float dl[NW][TB];                     // delta of the neurons being repaired, per token
    __shared__ int flist[kMaxNeuronsPerBlock];       // neurons flagged by at least one token
    __shared__ unsigned short fbits[kMaxNeuronsPerBlock];  // which tokens flagged them
    __shared__ uint32_t words[TB][MW];
    __shared__ int tmax[TB];                         // max |x| per token (bit pattern of a non-negative float)
    __shared__ int nflag;
    __shared__ int is_last, arrival;
    // partial sums of the matrix-core predictor (int32) and, later, of the matrix-core W' product (fp32)
    __shared__ int pacc[DEFER ? NW : 1][16][DEFER ? TB : 1];
    float (*wpart)[16][DEFER ? TB : 1] = reinterpret_cast<float (*)[16][DEFER ? TB : 1]>(pacc);

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
        const int tok = v / NVW;
        xv[it] = reinterpret_cast<const td_u32x4*>(x)[min(tok, n_act - 1) * NVW + (v - tok * NVW)];
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
    td_u32x4 qm[NL];                                 // matrix-core path: row (lane % 16) of the group, 16 bytes per step
    float tl_own = 0.0f, th_own = 0.0f;              // ... and the bounds of neuron `tid` of the block
    auto load_pred_tile = [&]() {
        constexpr int NGD = NG > 0 ? NG : 1;         // (not instantiated for NG == 0; keeps the division defined)
        const int grp = wave % NGD, kq = wave / NGD;
        const int j = min(j0 + grp * 16 + (lane & 15), h - 1);
        const td_u32x4* p = reinterpret_cast<const td_u32x4*>(Q + (size_t)j * D + kq * KS) + (lane >> 4);
#pragma unroll
        for (int m = 0; m < NL; ++m) qm[m] = td_load_stream16(p + m * 4);
    };
    if constexpr (NG > 0) {
        // (sixteen tokens occupy 32 registers until they are staged: their rows are requested after that)
        if (!kAlias) load_pred_tile();
        const int jt = min(j0 + tid, h - 1);
        tl_own = tlo[jt];
        th_own = thi[jt];
    } else {
        load_pred_rows(j0 + wave * RQ);
    }
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
            if (!kAlias) reinterpret_cast<td_u32x4*>(xs + (size_t)(v / NVW) * XSP)[v % NVW] = xv[it];
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
            float m = 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(td_bf16_to_f32(e8[u])));
            m = td_wave_max(m);                      // a wavefront's 64 vectors belong to one token
            if (lane == 0) atomicMax(&tmax[v / NVW], __float_as_int(m));
        }
    }
    __syncthreads();
    int ex[NG > 0 ? 1 : TB];                         // the matrix-core path reads them from LDS where needed
    if constexpr (NG == 0) {
#pragma unroll
        for (int t = 0; t < TB; ++t) ex[t] = token_exponent(__int_as_float(tmax[t]));
    }
#pragma unroll
    for (int it = 0; it < XI; ++it) {
        const int v = it * BLOCK + tid;
        if (v < TB * NVW) {
            const int tok = v / NVW;
            int e;
            if constexpr (NG > 0) {
                e = token_exponent(__int_as_float(tmax[tok]));
            } else {
                e = ex[0];
#pragma unroll
                for (int t = 1; t < TB; ++t) e = tok == t ? ex[t] : e;
            }
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv[it]);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u]), e)) << (8 * u);
                hi |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u + 4]), e)) << (8 * u);
            }
            if (NG > 0) {
                reinterpret_cast<uint2*>(xq + (size_t)tok * XP)[v - tok * NVW] = make_uint2(lo, hi);
            } else if (SK == 8) {
                reinterpret_cast<uint2*>(xq)[v] = make_uint2(lo, hi);
            } else {   // columns 0..15 of every group of 32 in the first half of the token's codes, 16..31 in the second
                const int i8 = v - tok * NVW, g = i8 >> 2, part = i8 & 3;
                const int at = tok * (D / 8) + (part < 2 ? 0 : D / 16) + g * 2 + (part & 1);
                reinterpret_cast<uint2*>(xq)[at] = make_uint2(lo, hi);
            }
        }
    }
    if constexpr (NG > 0 && kAlias) load_pred_tile();
    __syncthreads();

    // ---- predictor rows: exact int32 dot products, range test per token, block-local list of
    //      the neurons flagged by at least one token
    const td_u32x4* xq4 = reinterpret_cast<const td_u32x4*>(xq) + lane;
    if constexpr (NG > 0) {
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        const int grp = wave % NG, kq = wave / NG;
        const int8_t* xrow = xq + (size_t)((lane & 15) & (TB - 1)) * XP + kq * KS + (lane >> 4) * 16;
        i32x4 acc4 = {0, 0, 0, 0};
#pragma unroll
        for (int m = 0; m < NL; ++m) {
            const td_u32x4 xb = *reinterpret_cast<const td_u32x4*>(xrow + m * 64);
            acc4 = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, qm[m]),
                                                         __builtin_bit_cast(i32x4, xb), acc4, 0, 0, 0);
        }
        if ((lane & 15) < TB) {   // lane: token lane % 16, rows 4 * (lane / 16) + i of the group
#pragma unroll
            for (int i = 0; i < 4; ++i) pacc[wave][4 * (lane >> 4) + i][lane & 15] = acc4[i];
        }
        (void)grp;
        if constexpr (kAlias) {   // the tokens again (from cache), now that the predictor rows' registers are free
            asm volatile("" ::: "memory");
#pragma unroll
            for (int it = 0; it < XI; ++it) {
                const int v = min(it * BLOCK + tid, TB * NVW - 1);
                const int tok = v / NVW;
                xv[it] = reinterpret_cast<const td_u32x4*>(x)[min(tok, n_act - 1) * NVW + (v - tok * NVW)];
            }
        }
    }
    for (int base = 0; NG == 0 && base < jn; base += NW * RQ) {
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
                    const float v = ldexpf((float)(SK == 8 ? total : total >> 4), ex[NG > 0 ? 0 : t0 + t]);
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
                if constexpr (!FX) {   // (FX: the list is built in ascending order from the words below)
                    const int pos = atomicAdd(&nflag, 1);
                    flist[pos] = j0 + jl;
                    fbits[pos] = (unsigned short)bits[i];
                }
            }
        }
    }

    auto xsv = [&](int t, int it) -> td_u32x4 {       // vector it*64 + lane of token t
        return reinterpret_cast<const td_u32x4*>(xs + (size_t)t * XSP)[it * TD_WAVE + lane];
    };
    const int r0 = blk * rpb;
    const int rn = min(rpb, D - r0);                 // W' rows owned (may be <= 0)
    constexpr int IWP = WP8 ? IW / 2 : IW;           // per-lane vectors of one row of W' as stored
    td_u32x4 wp[IWP > 0 ? IWP : 1];
    // one kernel: wavefront w holds row r0 + w whole.  Deferred path: the block's (up to 16) rows are one
    // matrix-core tile, wavefront w holds columns [w*KW, (w+1)*KW) of all of them - lane: row lane % 16,
    // 16 bytes at step it, k-group lane / 16 - so the tokens are read from LDS once per block, not per row
    const td_u32x4* wp_row =
        DEFER ? reinterpret_cast<const td_u32x4*>(Wp + (size_t)min(r0 + (lane & 15), D - 1) * D + wave * KW) + (lane >> 4)
        : WP8 ? reinterpret_cast<const td_u32x4*>(Wp8 + (size_t)min(r0 + wave, D - 1) * D) + lane
              : reinterpret_cast<const td_u32x4*>(Wp + (size_t)min(r0 + wave, D - 1) * D) + lane;
    constexpr int WSTEP = DEFER ? 4 : TD_WAVE;       // vectors between a lane's consecutive loads
    const float bias_own = DEFER ? bp[min(r0 + tid / TB, D - 1)] : 0.0f;   // thread (row, token) of the final sum
    // first half of this wave's W' row: requested before the block meets at the barrier, so that
    // the memory pipe stays busy while the flagged list is assembled
    constexpr int IWA = IWP / 2;
#pragma unroll
    for (int it = 0; it < IWA; ++it) wp[it] = td_load_stream16(wp_row + it * WSTEP);

    if constexpr (NG > 0) {
        __syncthreads();                             // the partial sums of every wavefront are in LDS
        if (tid < jn) {
            const int grp = tid >> 4, row = tid & 15;
            uint32_t bits = 0;
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                int total = 0;
#pragma unroll
                for (int kq = 0; kq < KQ; ++kq) total += pacc[kq * NG + grp][row][t];
                const float v = ldexpf((float)total, token_exponent(__int_as_float(tmax[t])));
                const bool inside = (v >= tl_own) && (v < th_own);
                bits |= inside ? 0u : (1u << t);
            }
            if (bits) {
#pragma unroll
                for (int t = 0; t < TB; ++t)
                    if ((bits >> t) & 1u) atomicOr(&words[t][tid >> 5], 1u << (tid & 31));
                if constexpr (!FX) {
                    const int pos = atomicAdd(&nflag, 1);
                    flist[pos] = j0 + tid;
                    fbits[pos] = (unsigned short)bits;
                }
            }
        }
        if constexpr (kAlias) {   // every wavefront is past its last read of the int8 codes: the tokens take their place
#pragma unroll
            for (int it = 0; it < XI; ++it) {
                const int v = it * BLOCK + tid;
                if (v < TB * NVW) reinterpret_cast<td_u32x4*>(xs + (size_t)(v / NVW) * XSP)[v % NVW] = xv[it];
            }
        }
    }
    __syncthreads();
    if constexpr (FX) {
        // the block's flagged neurons in ascending order, from the mask words: positions by
        // population count, so the order - and with it every floating-point sum over the list -
        // is the same in every run
        if (tid < kMaxNeuronsPerBlock && tid < jn) {
            const int w = tid >> 5, b = tid & 31;
            uint32_t tb = 0u, uw = 0u;
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                tb |= ((words[t][w] >> b) & 1u) << t;
                uw |= words[t][w];
            }
            if (tb) {
                int pos = __popc(uw & ((1u << b) - 1u));
                for (int ww = 0; ww < w; ++ww) {
                    uint32_t u = 0u;
#pragma unroll
                    for (int t = 0; t < TB; ++t) u |= words[t][ww];
                    pos += __popc(u);
                }
                flist[pos] = j0 + tid;
                fbits[pos] = (unsigned short)tb;
            }
        }
        if (tid == 0) {
            int tot = 0;
            for (int ww = 0; ww < MW; ++ww) {
                uint32_t u = 0u;
#pragma unroll
                for (int t = 0; t < TB; ++t) u |= words[t][ww];
                tot += __popc(u);
            }
            nflag = tot;
        }
        __syncthreads();
    }
    if (jn > 0) {
        const int nw = (jn + 31) / 32;
        for (int k = tid; k < TB * nw; k += BLOCK) {
            const int t = k / nw, w = k % nw;
            if (t < n_act) mask[(size_t)t * mask_words + (j0 >> 5) + w] = words[t][w];
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
    if constexpr (DEFER) {
        // ---- one wavefront per flagged neuron: exact z and delta for the tokens that flagged it
        if (tid == 0) rec.count[blk] = nf;
        if constexpr (FX) {   // the second kernel needs every token's fixed-point exponent
            if (blk == 0 && tid < TB)
                fx_exp[tid] = FxAcc::exponent(fx_bound[0], fx_bound[1], __int_as_float(tmax[tid]));
        }
        if (nf == 0) {
#pragma unroll
            for (int it = IWA; it < IWP; ++it) wp[it] = td_load_stream16(wp_row + it * WSTEP);
        }
        for (int f0 = 0; f0 < nf; f0 += NW) {
            asm volatile("" ::: "memory");
            const int fi = f0 + wave;
            const bool fixer = fi < nf;
            td_u32x4 w1[IW];
            float aj = 0.0f, cj = 0.0f;
            uint32_t bj_raw = 0;
            int jz = 0;
            if (fixer) {
                jz = flist[fi];
                load_row<IW>(w1, W1 + (size_t)jz * D, lane);
                aj = a[jz];
                cj = c[jz];
                bj_raw = b1[jz];
            }
            if (f0 == 0) {   // the rest of this wave's W' row streams in behind the first batch of W1 rows
                asm volatile("" ::: "memory");
#pragma unroll
                for (int it = IWA; it < IWP; ++it) wp[it] = td_load_stream16(wp_row + it * WSTEP);
            }
            asm volatile("" : "+v"(bj_raw), "+v"(aj), "+v"(cj));
            if (fixer) {
                const float bj = td_bf16_to_f32((bf16_t)bj_raw);
                const uint32_t zbits = fbits[fi];
                const size_t slot = (size_t)blk * rec.cap + fi;
#pragma unroll
                for (int t = 0; t < TB; ++t) {
                    asm volatile("" ::: "memory");
                    float dv = 0.0f;
                    if ((zbits >> t) & 1u) {
                        float z = 0.0f;
#pragma unroll
                        for (int it = 0; it < IW; ++it) z = RowVec<bf16_t>::dot(w1[it], xsv(t, it), z);
                        z = td_wave_sum(z) + bj;
                        dv = td_act(z, act) - fmaf(aj, z, cj);
                    }
                    if (lane == 0) rec.delta[slot * TB + t] = dv;
                }
                if (lane == 0) {
                    rec.jb[slot] = (uint32_t)jz;
                    rec.tb[slot] = zbits;
                }
            }
        }
        {   // speculative rows: 16 x KW slice of W' against the tokens on the matrix cores
            typedef float f32x4m __attribute__((ext_vector_type(4)));
            typedef __bf16 bf16x8m __attribute__((ext_vector_type(8)));
            asm volatile("" ::: "memory");
            const unsigned char* xb = reinterpret_cast<const unsigned char*>(xs) +
                                      (size_t)((lane & 15) & (TB - 1)) * XSP * 2 + (size_t)wave * KW * 2 + (lane >> 4) * 16;
            f32x4m accw = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int it = 0; it < IW; ++it) {
                const td_u32x4 tk = *reinterpret_cast<const td_u32x4*>(xb + it * 64);
                accw = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8m, wp[it]),
                                                               __builtin_bit_cast(bf16x8m, tk), accw, 0, 0, 0);
            }
            if ((lane & 15) < TB) {   // lane: token lane % 16, rows 4 * (lane / 16) + i
#pragma unroll
                for (int i = 0; i < 4; ++i) wpart[wave][4 * (lane >> 4) + i][lane & 15] = accw[i];
            }
            __syncthreads();
            if (tid < 16 * TB && tid / TB < rn) {
                const int row = tid / TB, t = tid % TB;
                float s = bias_own;
#pragma unroll
                for (int w = 0; w < NW; ++w) s += wpart[w][row][t];
                if (t < n_act) yfold[(size_t)t * D + r0 + row] = s;
            }
        }
        return;
    }

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
            for (int it = IWA; it < IWP; ++it) wp[it] = td_load_stream16(wp_row + it * WSTEP);
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
                for (int it = 0; it < IW; ++it) z = RowVec<bf16_t>::dot(w1[it], xsv(t, it), z);
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
        for (int it = IWA; it < IWP; ++it) wp[it] = td_load_stream16(wp_row + it * WSTEP);
    } else {
        repair_pass(std::true_type{}, 0);
        for (int f0 = FCH; f0 < nf; f0 += FCH) repair_pass(std::false_type{}, f0);
    }

    if constexpr (FX) {
        // ---- counted fixed-point accumulators.  Every block adds its repair vector to every column
        //      once (zeros included: the count is how a column knows it is finished); the block that
        //      owns rows [r0, r0 + rn) of W' adds the speculative value of those columns in the same
        //      word.  Columns of other blocks' rows go out now, while this block's W' rows are still
        //      arriving; its own columns follow the dot products.
        constexpr int kOwnMax = 64;                  // W' rows per block this path serves (launcher checks)
        __shared__ float ysp[TB][kOwnMax];
        unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(yfix);
        const int G = (int)gridDim.x;
        int fxe[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) fxe[t] = FxAcc::exponent(fx_bound[0], fx_bound[1], __int_as_float(tmax[t]));
        unsigned long long before[TB][CPT];
        bool own[CPT];
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int col = ctid + u * BLOCK;
            own[u] = col >= r0 && col < r0 + rn;
        }
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int u = 0; u < CPT; ++u)
                if (!own[u])
                    before[t][u] = FxAcc::add(acc64 + (size_t)t * D + ctid + u * BLOCK, FxAcc::encode(yacc[t][u], fxe[t]));
        for (int ri = wave; ri < rn; ri += NW) {
            asm volatile("" ::: "memory");
            if (ri != wave) load_row<IWP>(wp, Wp + (size_t)(r0 + ri) * D, lane);
            const float bias = ri == wave ? bias_out : bp[r0 + ri];
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                if (TB > 1) asm volatile("" ::: "memory");
                float sp = 0.0f;
#pragma unroll
                for (int it = 0; it < IW; ++it) sp = RowVec<bf16_t>::dot(wp[it], xsv(t, it), sp);
                sp = td_wave_sum(sp);
                if (lane == 0) ysp[t][ri] = sp + bias;
            }
        }
        if (tid == 0) is_last = 0;
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int u = 0; u < CPT; ++u)
                if (own[u]) {
                    yacc[t][u] += ysp[t][ctid + u * BLOCK - r0];
                    before[t][u] = FxAcc::add(acc64 + (size_t)t * D + ctid + u * BLOCK, FxAcc::encode(yacc[t][u], fxe[t]));
                }
        // ---- the add that completed a column's count holds its finished sum: write it, re-arm the word
        int finished = 0;
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int u = 0; u < CPT; ++u) {
                if (FxAcc::completes(before[t][u], G)) {
                    const int col = ctid + u * BLOCK;
                    const float v = FxAcc::decode(before[t][u] + FxAcc::encode(yacc[t][u], fxe[t]), fxe[t]);
                    acc64[(size_t)t * D + col] = 0ull;
                    if (norm_out)   // whole rows are needed: parked (written through) for the assembling block
                        __hip_atomic_store(yfold + (size_t)t * D + col, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else
                        y[(size_t)t * D + col] = td_f32_to_bf16(v);
                    ++finished;
                }
            }
        // a wavefront that completed nothing is not among the last to finish: it warms the caches for
        // the layer that runs next while the rest of the launch drains
        if (pf_rows != nullptr && jn > 0 && !__any(finished > 0))
            warm_rows<BLOCK>(pf_rows + (size_t)j0 * QROW, min(pf_bytes, jn * QROW), tid);
        if (!norm_out) return;
        // ---- stacked layers: the block that parks the last column normalises the rows
        finished = td_wave_sum_i(finished);
        if (finished > 0 && lane == 0) {
            td_wait_memory_acks();
            if (__hip_atomic_fetch_add(done, finished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + finished == TB * D)
                is_last = 1;
        }
        __syncthreads();
        if (!is_last) return;
        float* redt = &dl[0][0];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            float v[CPT];
            float ss = 0.0f;
#pragma unroll
            for (int u = 0; u < CPT; ++u) {
                v[u] = load_coherent(yfold + (size_t)t * D + tid + u * BLOCK);    // (parked by blocks on any XCD)
                ss += v[u] * v[u];
            }
            ss = td_wave_sum(ss);
            __syncthreads();
            if (lane == 0) redt[wave] = ss;
            __syncthreads();
            float tot = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) tot += redt[w];
            const float scale = 1.0f / sqrtf(tot / (float)D + eps);
#pragma unroll
            for (int u = 0; u < CPT; ++u) y[(size_t)t * D + tid + u * BLOCK] = td_f32_to_bf16(v[u] * scale);
        }
        if (tid == 0) __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
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
        if (ri != wave) {
            if constexpr (WP8) load_row<IWP>(wp, Wp8 + (size_t)(r0 + ri) * D, lane);
            else load_row<IWP>(wp, Wp + (size_t)(r0 + ri) * D, lane);
        }
        const float bias = ri == wave ? bias_out : bp[r0 + ri];
        float row_scale = 1.0f;
        if constexpr (WP8) row_scale = wp8_scale[r0 + ri];
#pragma unroll
        for (int t = 0; t < TB; ++t) {
            if (TB > 1) asm volatile("" ::: "memory");
            float s = 0.0f;
            if constexpr (WP8) {
                // vector it*64 + lane of the 8-bit row = 16 columns = two 16-byte vectors of the token
                const td_u32x4* xt = reinterpret_cast<const td_u32x4*>(xs + (size_t)t * XSP) + 2 * lane;
#pragma unroll
                for (int it = 0; it < IWP; ++it) s = dot_e4m3_bf16(wp[it], xt[it * 2 * TD_WAVE], xt[it * 2 * TD_WAVE + 1], s);
                s = td_wave_sum(s) * row_scale;
            } else {
#pragma unroll
                for (int it = 0; it < IWP; ++it) s = RowVec<bf16_t>::dot(wp[it], xsv(t, it), s);
                s = td_wave_sum(s);
            }
            // written through to memory so that the finishing block, on any XCD, reads it
            // (adding the value to the repair accumulators instead, so that the assembling block reads 16 KB
            //  less, was measured: 23.3 against 23.4 us per token - within the noise, not kept)
            if (lane == 0)
                __hip_atomic_store(yfold + (size_t)t * D + r0 + ri, s + bias, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // ---- signal completion.  Every wavefront first waits until its own stores and atomics have
    //      been acknowledged by memory (they are written through / executed memory-side, so
    //      acknowledged means visible to every XCD); only then does the block meet at the barrier
    //      and move the counter.  The fence alone does not do it: at workgroup scope it waits for
    //      LDS traffic only.
    td_wait_memory_acks();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
        // (strict_release: a formal agent-scope release by the signalling thread on top of the waits above)
        if (strict_release) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const int before = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        arrival = before;
        is_last = before == (int)gridDim.x - 1;
    }
    __syncthreads();
    if (!is_last) {
        // ---- this block is done, the memory system idles while the atomics drain and the last
        //      block assembles y: warm the caches with the predictor rows this block index reads
        //      first in the layer that runs next (pf_rows = that layer's codes, null if unknown).
        //      (Requesting them BEFORE the block signals - behind its own stores, waiting only for
        //      the older operations - was measured slower: 24.2 against 23.4 us per token.)
        if (pf_rows != nullptr && jn > 0) {
            // How much: the earlier a block finished (its number in the order of arrival at the counter), the
            // longer its wait for the launch to end - pf_shape holds, in sixteenths of pf_bytes, what the first
            // block to arrive asks for (low byte) and what the last would (next byte), linear in between; late
            // blocks ask for little, so that the launch does not end on their requests (0: pf_bytes for all).
            int want = pf_bytes;
            if (pf_shape != 0) {
                const int first16 = pf_shape & 255, last16 = (pf_shape >> 8) & 255;
                const int m16 = first16 - ((first16 - last16) * arrival) / (int)gridDim.x;
                want = max(16, ((pf_bytes >> 4) * m16) & ~15);
            }
            warm_rows<BLOCK>(pf_rows + (size_t)j0 * QROW, min(want, jn * QROW), tid);
        }
        return;
    }

    // ---- the last block to finish assembles y and re-arms the scratch (one cache invalidation,
    //      then 16-byte loads: faster here than four-byte device-coherent loads, many per thread)
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int OI = (D / 4 + BLOCK - 1) / BLOCK;   // float4 pieces of one token's y per thread
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 out[TB][OI];
    f32x4 part[TB][OI][kMaxCopies];
    if constexpr (TB == 1 && OI == 1) {
        // One token: 16-byte device-coherent loads (what an agent-scope atomic load is, four dwords wide) instead
        // of an agent-scope acquire, whose cache invalidation would also drop from this XCD's L2 the rows just
        // requested for the next layer.  (One statement for the loads and their wait: the compiler does not
        // know that the registers are in flight and would otherwise be free to copy them before the wait.
        // Copies the layer does not use re-read copy 0 and are discarded.)
        const int k4 = min(tid, D / 4 - 1);
        const f32x4* pa = reinterpret_cast<const f32x4*>(yfold) + k4;
        const f32x4* p0 = reinterpret_cast<const f32x4*>(yfix) + k4;
        const f32x4* p1 = reinterpret_cast<const f32x4*>(yfix + (size_t)(copies > 1 ? 1 : 0) * D) + k4;
        const f32x4* p2 = reinterpret_cast<const f32x4*>(yfix + (size_t)(copies > 2 ? 2 : 0) * D) + k4;
        const f32x4* p3 = reinterpret_cast<const f32x4*>(yfix + (size_t)(copies > 3 ? 3 : 0) * D) + k4;
        static_assert(kMaxCopies == 4, "one load per copy below");
        f32x4 va, v0, v1, v2, v3;
        asm volatile(
            "global_load_dwordx4 %0, %5, off sc1\n\t"
            "global_load_dwordx4 %1, %6, off sc1\n\t"
            "global_load_dwordx4 %2, %7, off sc1\n\t"
            "global_load_dwordx4 %3, %8, off sc1\n\t"
            "global_load_dwordx4 %4, %9, off sc1\n\t"
            "s_waitcnt vmcnt(0)"
            : "=&v"(va), "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
            : "v"(pa), "v"(p0), "v"(p1), "v"(p2), "v"(p3)
            : "memory");
        const bool live = tid < D / 4;
        out[0][0] = live ? va : zero4;
        part[0][0][0] = live ? v0 : zero4;
        part[0][0][1] = (live && copies > 1) ? v1 : zero4;
        part[0][0][2] = (live && copies > 2) ? v2 : zero4;
        part[0][0][3] = (live && copies > 3) ? v3 : zero4;
    } else if constexpr (TB == 2 && OI == 1) {
        // two tokens: the same, ten loads behind one wait
        const int k4 = min(tid, D / 4 - 1);
        const f32x4* pa[2];
        const f32x4* pc[2][kMaxCopies];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            pa[t] = reinterpret_cast<const f32x4*>(yfold + (size_t)t * D) + k4;
#pragma unroll
            for (int cidx = 0; cidx < kMaxCopies; ++cidx)
                pc[t][cidx] = reinterpret_cast<const f32x4*>(yfix + ((size_t)(cidx < copies ? cidx : 0) * TB + t) * D) + k4;
        }
        f32x4 va0, va1, v00, v01, v02, v03, v10, v11, v12, v13;
        asm volatile(
            "global_load_dwordx4 %0, %10, off sc1\n\t"
            "global_load_dwordx4 %1, %11, off sc1\n\t"
            "global_load_dwordx4 %2, %12, off sc1\n\t"
            "global_load_dwordx4 %3, %13, off sc1\n\t"
            "global_load_dwordx4 %4, %14, off sc1\n\t"
            "global_load_dwordx4 %5, %15, off sc1\n\t"
            "global_load_dwordx4 %6, %16, off sc1\n\t"
            "global_load_dwordx4 %7, %17, off sc1\n\t"
            "global_load_dwordx4 %8, %18, off sc1\n\t"
            "global_load_dwordx4 %9, %19, off sc1\n\t"
            "s_waitcnt vmcnt(0)"
            : "=&v"(va0), "=&v"(va1), "=&v"(v00), "=&v"(v01), "=&v"(v02), "=&v"(v03), "=&v"(v10), "=&v"(v11), "=&v"(v12), "=&v"(v13)
            : "v"(pa[0]), "v"(pa[1]), "v"(pc[0][0]), "v"(pc[0][1]), "v"(pc[0][2]), "v"(pc[0][3]), "v"(pc[1][0]), "v"(pc[1][1]), "v"(pc[1][2]), "v"(pc[1][3])
            : "memory");
        const bool live = tid < D / 4;
        out[0][0] = live ? va0 : zero4;
        out[1][0] = live ? va1 : zero4;
        part[0][0][0] = live ? v00 : zero4;
        part[0][0][1] = (live && copies > 1) ? v01 : zero4;
        part[0][0][2] = (live && copies > 2) ? v02 : zero4;
        part[0][0][3] = (live && copies > 3) ? v03 : zero4;
        part[1][0][0] = live ? v10 : zero4;
        part[1][0][1] = (live && copies > 1) ? v11 : zero4;
        part[1][0][2] = (live && copies > 2) ? v12 : zero4;
        part[1][0][3] = (live && copies > 3) ? v13 : zero4;
    } else {
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
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

// Second kernel of the deferred path: y_t = yfold_t + sum over the records of delta_t * W2^T[j].
// A block owns one slice of 256 output columns and the records of 16 predictor blocks, one
// wavefront per predictor block: a lane owns 4 columns (8-byte loads, 512 contiguous bytes per
// wavefront and row), eight rows in flight; each wavefront accumulates into its own TB x 256 floats
// of LDS (read-modify-write by the owning wavefront only, for the tokens whose bit is set), the
// block reduces over its wavefronts and adds TB x 256 floats to the accumulators in memory - 16
// times fewer atomics than one d-vector per predictor block and token.  The last block to finish
// assembles the tokens.
// FX = true: counted fixed-point accumulators (see FxAcc) instead of fp32 atomics and per-slice
// completion counters; the add that completes a column writes it.
template <int TB, int SL, bool FX>
__global__ void __launch_bounds__(1024)
down_project_kernel(const bf16_t* __restrict__ W2T, DeferOut rec, int nblk, int pbw, float* __restrict__ yfold,
                    float* __restrict__ yfix, bf16_t* __restrict__ y, int32_t* __restrict__ done, int D, int nslices,
                    int norm_out, float eps, int n_act, const unsigned char* __restrict__ pf_rows, int pf_bytes,
                    int pf_row_bytes, int npb, int h, const int32_t* __restrict__ fx_exp, int pf_shape) {
    constexpr int NW = 16, U = SL == 128 ? 48 : 16;  // wavefronts; rows in flight per wavefront (4- or 8-byte loads)
    constexpr int CPL = SL / TD_WAVE;                // columns per lane: 4 (8-byte loads) or 2 (4-byte loads)
    static_assert(CPL == 4 || CPL == 2, "slice width");
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef float f32xc __attribute__((ext_vector_type(CPL)));
    extern __shared__ __align__(16) float accL[];    // NW x TB x SL
    __shared__ int is_last, arrival;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slice = blockIdx.x % nslices, group = blockIdx.x / nslices;
    float* acc = accL + (size_t)wave * TB * SL + lane * CPL;
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int t = 0; t < TB; ++t) {
#pragma unroll
        for (int q = 0; q < CPL; ++q) acc[t * SL + q] = 0.0f;
    }
    // a block that is not the last to finish warms the caches for the next layer's first kernel:
    // the predictor rows of block index blockIdx.x there (same grid size as that kernel)
    // (how much follows the block's place `a` among the `cnt` blocks that share its counter, as in the
    //  single-token kernel; cnt = 0: the flat amount)
    auto warm_next = [&](int a = 0, int cnt = 0) {
        const int j0n = (int)blockIdx.x * npb, jnn = min(npb, h - j0n);
        int want = pf_bytes;
        if (pf_shape != 0 && cnt > 0) {
            const int first16 = pf_shape & 255, last16 = (pf_shape >> 8) & 255;
            want = max(16, ((pf_bytes >> 4) * (first16 - ((first16 - last16) * a) / cnt)) & ~15);
        }
        if (pf_rows != nullptr && (int)blockIdx.x < nblk && jnn > 0)
            warm_rows<1024>(pf_rows + (size_t)j0n * pf_row_bytes, min(want, jnn * pf_row_bytes), tid);
    };
    const bf16_t* base = W2T + (size_t)slice * SL + lane * CPL;
    // a wavefront takes `pbw` predictor blocks in turn
    for (int pi = 0; pi < pbw; ++pi) {
        const int pb = __builtin_amdgcn_readfirstlane((group * NW + wave) * pbw + pi);
        if (pb >= nblk) break;
        const uint32_t* jb = rec.jb + (size_t)pb * rec.cap;
        const uint32_t* tbp = rec.tb + (size_t)pb * rec.cap;
        const float* dl = rec.delta + (size_t)pb * rec.cap * TB;
        // the count and the first 64 records are requested together (a slot past the count holds stale
        // but in-bounds data and is never applied); lane r keeps record r and hands it out by readlane
        const int cnt = rec.count[pb];
        for (int c0 = 0; c0 < rec.cap; c0 += TD_WAVE) {
            const int mine = min(c0 + lane, rec.cap - 1);
            const uint32_t myj = jb[mine];
            const uint32_t myb = tbp[mine];
            float myd[TB];
#pragma unroll
            for (int t = 0; t < TB; ++t) myd[t] = dl[(size_t)mine * TB + t];
            const int here = min(cnt - c0, TD_WAVE);     // records of this batch of 64 (<= 0: none)
            if (here <= 0) break;
            for (int r0 = 0; r0 < here; r0 += U) {
                uint32_t w[U][CPL / 2];
#pragma unroll
                for (int u = 0; u < U; ++u) {   // slots past the end re-read the last record; they are not applied
                    const uint32_t j = __builtin_amdgcn_readlane(myj, min(r0 + u, here - 1));
                    if constexpr (CPL == 4) {
                        const unsigned long long v = __builtin_nontemporal_load(
                            reinterpret_cast<const unsigned long long*>(base + (size_t)j * D));
                        w[u][0] = (uint32_t)v;
                        w[u][1] = (uint32_t)(v >> 32);
                    } else {
                        w[u][0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(base + (size_t)j * D));
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (r0 + u < here) {
                        const int r = r0 + u;
                        const uint32_t bits = __builtin_amdgcn_readlane(myb, r);
                        f32xc wf;
#pragma unroll
                        for (int q = 0; q < CPL / 2; ++q) {
                            wf[2 * q] = __uint_as_float(w[u][q] << 16);
                            wf[2 * q + 1] = __uint_as_float(w[u][q] & 0xFFFF0000u);
                        }
                        if constexpr (TB <= 8) {
#pragma unroll
                            for (int t = 0; t < TB; ++t) {
                                if ((bits >> t) & 1u) {
                                    const float d = __builtin_bit_cast(
                                        float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, myd[t]), r));
                                    f32xc* a4 = reinterpret_cast<f32xc*>(acc + t * SL);
                                    *a4 = *a4 + wf * d;
                                }
                            }
                        } else {   // many tokens, one or two of them set: walk the set bits (all scalar)
                            uint32_t left = bits;
                            while (left) {
                                const int t = __builtin_ctz(left);
                                left &= left - 1;
                                const float d = __builtin_bit_cast(
                                    float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, myd[t]), r));
                                f32xc* a4 = reinterpret_cast<f32xc*>(acc + t * SL);
                                *a4 = *a4 + wf * d;
                            }
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    if constexpr (FX) {
        // ---- reduce over the wavefronts (fixed order); one counted fixed-point add per (token, column)
        //      of the slice, zeros included; the add that completes a column's count finishes it
        unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(yfix);
        const int ngroups = (int)gridDim.x / nslices;
        int finished = 0;
        if (tid == 0) is_last = 0;
        for (int k = tid; k < TB * SL; k += 1024) {
            const int t = k / SL, col = k % SL;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += accL[((size_t)w * TB + t) * SL + col];
            const int e = fx_exp[t];
            const size_t at = (size_t)t * D + slice * SL + col;
            const unsigned long long enc = FxAcc::encode(sum, e);
            const unsigned long long before = FxAcc::add(acc64 + at, enc);
            if (FxAcc::completes(before, ngroups)) {
                acc64[at] = 0ull;
                if (t < n_act) {                     // (else: a slot that repeats the last real token)
                    const float v = yfold[at] + FxAcc::decode(before + enc, e);
                    if (norm_out)
                        __hip_atomic_store(yfold + at, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else
                        y[at] = td_f32_to_bf16(v);
                }
                ++finished;
            }
        }
        if (!norm_out) {
            if (!__any(finished > 0)) warm_next();
            return;
        }
        finished = td_wave_sum_i(finished);
        __syncthreads();                             // is_last = 0 is in place
        if (finished > 0 && lane == 0) {
            td_wait_memory_acks();
            if (__hip_atomic_fetch_add(done, finished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + finished == TB * D)
                is_last = 1;
        }
        __syncthreads();
        if (!is_last) {
            warm_next();
            return;
        }
    }
    // ---- reduce over the wavefronts; one atomic per (token, column) of the slice
    for (int k = tid; FX == false && k < TB * SL; k += 1024) {
        const int t = k / SL, col = k % SL;
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += accL[((size_t)w * TB + t) * SL + col];
        if (sum != 0.0f)
            __hip_atomic_fetch_add(yfix + (size_t)t * D + slice * SL + col, sum, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
    }
    if constexpr (!FX) {
    td_wait_memory_acks();   // this wavefront's atomics have been performed before the block's counter moves
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    }
    if (!FX && !norm_out) {
        // ---- no row-wide quantity is needed: the last of the blocks that share this slice of
        //      columns assembles the slice (counter 1 + slice), all slices in parallel
        const int ngroups = (int)gridDim.x / nslices;
        if (tid == 0) {
            arrival = __hip_atomic_fetch_add(done + 1 + slice, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = arrival == ngroups - 1;
        }
        __syncthreads();
        if (!is_last) {
            warm_next(arrival, ngroups);
            return;
        }
        for (int k = tid; k < TB * (SL / 4); k += 1024) {
            const int t = k / (SL / 4), c4 = k % (SL / 4);
            const size_t at = (size_t)t * D + slice * SL + c4 * 4;
            const f32x4 fix4 = load_coherent4(yfix + at);
            *reinterpret_cast<f32x4*>(yfix + at) = zero4;
            if (t >= n_act) continue;                // a slot that repeats the last real token
            const f32x4 o4 = *reinterpret_cast<const f32x4*>(yfold + at) + fix4;
            uint2 o;
            o.x = (uint32_t)td_f32_to_bf16(o4.x) | ((uint32_t)td_f32_to_bf16(o4.y) << 16);
            o.y = (uint32_t)td_f32_to_bf16(o4.z) | ((uint32_t)td_f32_to_bf16(o4.w) << 16);
            *reinterpret_cast<uint2*>(y + at) = o;
        }
        if (tid == 0) __hip_atomic_store(done + 1 + slice, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if constexpr (!FX) {
        if (tid == 0) {
            arrival = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = arrival == (int)gridDim.x - 1;
        }
        __syncthreads();
        if (!is_last) {
            warm_next(arrival, (int)gridDim.x);
            return;
        }
    }

    // ---- the last block assembles the tokens (with their row-wide norm) and re-arms the scratch
    float* redt = accL;                              // NW x TB floats, free by now
    constexpr int TH = TB < 4 ? TB : 4;              // tokens assembled together
    for (int t0 = 0; t0 < TB; t0 += TH) {
        for (int k0 = 0; k0 < D / 4; k0 += 1024) {   // one pass when d = 4096
            const int k4 = k0 + tid;
            const bool live = k4 < D / 4;
            const int k4c = min(k4, D / 4 - 1);
            f32x4 v[TH];
            // device-coherent loads, not an agent-scope acquire and plain loads: the acquire's cache invalidation
            // costs about a microsecond and drops what has been requested for the next layer
            if constexpr (TH == 4) {
                f32x4 f[4], g[4];
                const f32x4* pf[4];
                const f32x4* pg[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    pf[t] = reinterpret_cast<const f32x4*>(yfold + (size_t)(t0 + t) * D) + k4c;
                    pg[t] = reinterpret_cast<const f32x4*>(yfix + (size_t)(t0 + t) * D) + k4c;
                }
                // (one statement for the loads and their wait: the compiler does not know the registers are in flight)
                asm volatile(
                    "global_load_dwordx4 %0, %8, off sc1\n\t"
                    "global_load_dwordx4 %1, %9, off sc1\n\t"
                    "global_load_dwordx4 %2, %10, off sc1\n\t"
                    "global_load_dwordx4 %3, %11, off sc1\n\t"
                    "global_load_dwordx4 %4, %12, off sc1\n\t"
                    "global_load_dwordx4 %5, %13, off sc1\n\t"
                    "global_load_dwordx4 %6, %14, off sc1\n\t"
                    "global_load_dwordx4 %7, %15, off sc1\n\t"
                    "s_waitcnt vmcnt(0)"
                    : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(g[0]), "=&v"(g[1]), "=&v"(g[2]), "=&v"(g[3])
                    : "v"(pf[0]), "v"(pf[1]), "v"(pf[2]), "v"(pf[3]), "v"(pg[0]), "v"(pg[1]), "v"(pg[2]), "v"(pg[3])
                    : "memory");
#pragma unroll
                for (int t = 0; t < 4; ++t)          // (FX: the parked rows are complete and the accumulators re-armed already)
                    v[t] = ((live && t0 + t < n_act) ? f[t] : zero4) + ((live && !FX) ? g[t] : zero4);
            } else {
#pragma unroll
                for (int t = 0; t < TH; ++t) {
                    const f32x4 f = (live && t0 + t < n_act) ? load_coherent4(yfold + (size_t)(t0 + t) * D + 4 * k4c) : zero4;
                    const f32x4 g = (live && !FX) ? load_coherent4(yfix + (size_t)(t0 + t) * D + 4 * k4c) : zero4;
                    v[t] = f + g;
                }
            }
            if (live && !FX) {
#pragma unroll
                for (int t = 0; t < TH; ++t) reinterpret_cast<f32x4*>(yfix + (size_t)(t0 + t) * D)[k4] = zero4;
            }
            float scale[TH];
#pragma unroll
            for (int t = 0; t < TH; ++t) scale[t] = 1.0f;
            if (norm_out) {   // whole rows are needed: the host only asks for it when d <= 4096 (one pass)
                __syncthreads();
#pragma unroll
                for (int t = 0; t < TH; ++t) {
                    const float ss =
                        td_wave_sum(v[t].x * v[t].x + v[t].y * v[t].y + v[t].z * v[t].z + v[t].w * v[t].w);
                    if (lane == 0) redt[wave * TH + t] = ss;
                }
                __syncthreads();
#pragma unroll
                for (int t = 0; t < TH; ++t) {
                    float tot = 0.0f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) tot += redt[w * TH + t];
                    scale[t] = 1.0f / sqrtf(tot / (float)D + eps);
                }
            }
            if (live) {
#pragma unroll
                for (int t = 0; t < TH; ++t) {
                    if (t0 + t >= n_act) continue;   // a slot that repeats the last real token
                    const f32x4 o4 = v[t] * scale[t];
                    uint2 o;
                    o.x = (uint32_t)td_f32_to_bf16(o4.x) | ((uint32_t)td_f32_to_bf16(o4.y) << 16);
                    o.y = (uint32_t)td_f32_to_bf16(o4.z) | ((uint32_t)td_f32_to_bf16(o4.w) << 16);
                    reinterpret_cast<uint2*>(y + (size_t)(t0 + t) * D)[k4] = o;
                }
            }
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

// union over the n tokens of a call: the neurons flagged by at least one of them (mask words and
// their number); one block, no atomics
__global__ void __launch_bounds__(256)
mask_union_kernel(const uint32_t* __restrict__ mask, int words, int n, uint32_t* __restrict__ union_mask,
                  int32_t* __restrict__ union_count) {
    __shared__ int wave_tot[4];
    int mine = 0;
    for (int w = threadIdx.x; w < words; w += 256) {
        uint32_t bits = 0u;
        for (int t = 0; t < n; ++t) bits |= mask[(size_t)t * words + w];
        if (union_mask) union_mask[w] = bits;
        mine += __popc(bits);
    }
    mine = td_wave_sum_i(mine);
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0 && union_count) *union_count = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
}

constexpr int kFxExpAt = 40;   // where, among the 64 counters of a call's working memory, the tokens' fixed-point exponents sit

template <int D, int BLOCK, int TB, int SK, bool DEFER, int NG, bool FX, bool WP8 = false>
tardis_status_t launch_decode_impl(tardis_layer_s* L, const DecodeScratch& ws, const void* x, void* y, float* yfold,
                                   uint32_t* mask, int n_act, int norm_out, hipStream_t s) {
    constexpr int RQ = 4;
    if (n_act < 1 || n_act > TB || (!DEFER && n_act != TB)) return TARDIS_ERR_INVALID_ARG;
    const int G = L->dec_blocks;
    const int h = (int)L->h;
    int npb = (h + G - 1) / G;
    npb = (npb + 31) / 32 * 32;
    const int rpb = (D + G - 1) / G;
    const int8_t* codes = SK == 8 ? L->Q : reinterpret_cast<const int8_t*>(L->Q4);
    const bool static_tokens = !DEFER && (size_t)TB * D * 3 <= 56 * 1024;    // as in the kernel
    const size_t lds = static_tokens ? 0
                       : TB == 16    ? (size_t)TB * (D + 8) * 2      // the int8 codes share the tokens' place
                                     : (size_t)TB * (DEFER ? D + 8 : D) * 2 + (size_t)TB * (NG > 0 ? D + 16 : D);
    auto kernel = decode_fused_kernel<D, BLOCK, RQ, TB, SK, DEFER, NG, FX, WP8>;
    if (FX && (rpb > 64 || G > 65535)) return TARDIS_ERR_SHAPE;   // own-column staging, 16-bit contribution count
    const DeferOut rec{ws.rec_count, ws.rec_jb, ws.rec_tb, ws.rec_delta, npb};
    // the layer that runs next, if the caller said so and it has this layer's geometry
    const unsigned char* pf_rows = nullptr;
    const tardis_layer_s* nx = L->next_layer;
    if (nx && L->prefetch_bytes > 0 && td_layer_is_live(nx) && nx->d == L->d && nx->h == L->h && nx->dec_blocks == G &&
        nx->dtype == L->dtype)
        pf_rows = reinterpret_cast<const unsigned char*>(SK == 8 ? static_cast<const void*>(nx->Q)
                                                                 : static_cast<const void*>(nx->Q4));
    hipLaunchKernelGGL(kernel, dim3(G), dim3(BLOCK), lds, s,
                       static_cast<const bf16_t*>(L->Wp), L->bp, codes, L->M4, L->tlo, L->thi,
                       static_cast<const bf16_t*>(L->W1),
                       static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h), static_cast<const bf16_t*>(L->W2T),
                       L->a, L->c, static_cast<const bf16_t*>(x), static_cast<bf16_t*>(y), yfold, ws.yfix,
                       L->dec_copies, mask, (int)L->mask_words, ws.sync, h, npb, rpb, (int)L->act, norm_out, kRmsEps,
                       rec, n_act, DEFER ? nullptr : pf_rows, (int)L->prefetch_bytes, L->fx_bound, ws.sync + kFxExpAt, (int)L->strict_release, (int)L->prefetch_shape,
                       L->Wp8, L->wp8_scale);
    TD_HIP(hipGetLastError());
    if (DEFER) {
        constexpr int SL = TB >= 16 ? 128 : 256;     // slice width: 16 wavefronts x TB x SL floats of LDS
        constexpr size_t lds2 = (size_t)16 * TB * SL * sizeof(float);
        auto k2 = down_project_kernel<TB, SL, FX>;
        const int nslices = D / SL;
        const int ngroups = nslices >= 256 ? 1 : 256 / nslices;          // about one block per CU
        const int pbw = (G + 16 * ngroups - 1) / (16 * ngroups);         // predictor blocks per wavefront
        hipLaunchKernelGGL(k2, dim3(nslices * ngroups), dim3(1024), lds2, s, static_cast<const bf16_t*>(L->W2T), rec,
                           G, pbw, yfold, ws.yfix, static_cast<bf16_t*>(y), ws.sync, D, nslices, norm_out, kRmsEps, n_act,
                           TB >= 16 ? nullptr : pf_rows,   // (sixteen tokens: its blocks end too close together for the warming to pay)
                           (int)L->prefetch_bytes, SK == 8 ? D : D / 2, npb, h, ws.sync + kFxExpAt, (int)L->prefetch_shape);
        TD_HIP(hipGetLastError());
    }
    return TARDIS_OK;
}

template <int D, int BLOCK, int TB, int SK, bool DEFER, int NG = 0>
tardis_status_t launch_decode(tardis_layer_s* L, const DecodeScratch& ws, const void* x, void* y, float* yfold,
                              uint32_t* mask, int n_act, int norm_out, hipStream_t s) {
    if constexpr (BLOCK == 1024) {   // (the 512-thread variant keeps fp32 accumulators)
        if (L->fx) return launch_decode_impl<D, BLOCK, TB, SK, DEFER, NG, true>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
        if constexpr (!DEFER && TB <= 2 && D >= 2048) {   // the compact 8-bit rows of W' where the layer keeps them
            if (L->Wp8)
                return launch_decode_impl<D, BLOCK, TB, SK, DEFER, NG, false, true>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
        }
    }
    return launch_decode_impl<D, BLOCK, TB, SK, DEFER, NG, false>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
}

// `tokens` = group size (1, 2, 4, 8, 16), `n_act` of them real (fewer only on the two-kernel path)
template <int D, int BLOCK, int SK>
tardis_status_t launch_tb(tardis_layer_s* L, const DecodeScratch& ws, const void* x, void* y, float* yfold,
                          uint32_t* mask, int tokens, int n_act, int norm_out, hipStream_t s) {
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    bf16_t* yb = static_cast<bf16_t*>(y);
    // two kernels: records, then the column-sliced pass (the block's W' rows must fit one 16-row tile)
    if (BLOCK == 1024 && L->defer_min_tokens <= tokens && (D + L->dec_blocks - 1) / L->dec_blocks <= 16) {
        if (tokens == 4) return launch_decode<D, 1024, 4, SK, true>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
        // eight and sixteen tokens need one-byte codes and 32 or 64 neurons per block (the matrix-core
        // tiling); otherwise they run as two groups of half the size
        const int npb = (((int)L->h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
        if (tokens == 16 || tokens == 8) {
            if constexpr (SK == 8) {
                if (npb == 64 && tokens == 16)
                    return launch_decode<D, 1024, 16, 8, true, 4>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
                if (npb == 32 && tokens == 16)
                    return launch_decode<D, 1024, 16, 8, true, 2>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
                if (npb == 64 && tokens == 8)
                    return launch_decode<D, 1024, 8, 8, true, 4>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
                if (npb == 32 && tokens == 8)
                    return launch_decode<D, 1024, 8, 8, true, 2>(L, ws, x, y, yfold, mask, n_act, norm_out, s);
            }
            const int half = tokens / 2;
            TD_TRY((launch_tb<D, BLOCK, SK>(L, ws, x, y, yfold, mask, half, n_act < half ? n_act : half, norm_out, s)));
            if (n_act <= half) return TARDIS_OK;
            return launch_tb<D, BLOCK, SK>(L, ws, xb + half * (size_t)D, yb + half * (size_t)D, yfold + half * (size_t)D,
                                           mask + half * L->mask_words, half, n_act - half, norm_out, s);
        }
    }
    if (n_act != tokens) return TARDIS_ERR_INVALID_ARG;      // the one-kernel form has no empty slots
    switch (tokens) {
        case 1: return launch_decode<D, BLOCK, 1, SK, false>(L, ws, x, y, yfold, mask, 1, norm_out, s);
        case 2: return launch_decode<D, BLOCK, 2, SK, false>(L, ws, x, y, yfold, mask, 2, norm_out, s);
        case 4: return launch_decode<D, BLOCK, 4, SK, false>(L, ws, x, y, yfold, mask, 4, norm_out, s);
    }
    return TARDIS_ERR_INVALID_ARG;
}

template <typename K> hipError_t allow_lds(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

}  // namespace

// Kernels whose dynamic LDS exceeds the default limit are enabled once, when the first layer is
// folded (not at launch: a launch may be under stream capture).
tardis_status_t td_decode_init() {
    static td_once once;
    return once.run([]() -> tardis_status_t {
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 8, 8, true, 4, false, false>, (size_t)8 * 4096 * 3 + 256)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 8, 8, true, 2, false, false>, (size_t)8 * 4096 * 3 + 256)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 16, 8, true, 4, false, false>, (size_t)16 * (4096 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 16, 8, true, 2, false, false>, (size_t)16 * (4096 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<2048, 1024, 4, 16, 8, true, 4, false, false>, (size_t)16 * (2048 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<2048, 1024, 4, 16, 8, true, 2, false, false>, (size_t)16 * (2048 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 8, 8, true, 4, true, false>, (size_t)8 * 4096 * 3 + 256)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 8, 8, true, 2, true, false>, (size_t)8 * 4096 * 3 + 256)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 16, 8, true, 4, true, false>, (size_t)16 * (4096 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<4096, 1024, 4, 16, 8, true, 2, true, false>, (size_t)16 * (4096 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<2048, 1024, 4, 16, 8, true, 4, true, false>, (size_t)16 * (2048 + 8) * 2)));
        TD_HIP((allow_lds(decode_fused_kernel<2048, 1024, 4, 16, 8, true, 2, true, false>, (size_t)16 * (2048 + 8) * 2)));
        TD_HIP((allow_lds((down_project_kernel<4, 256, false>), (size_t)16 * 4 * 256 * sizeof(float))));
        TD_HIP((allow_lds((down_project_kernel<8, 256, false>), (size_t)16 * 8 * 256 * sizeof(float))));
        TD_HIP((allow_lds((down_project_kernel<16, 128, false>), (size_t)16 * 16 * 128 * sizeof(float))));
        TD_HIP((allow_lds((down_project_kernel<4, 256, true>), (size_t)16 * 4 * 256 * sizeof(float))));
        TD_HIP((allow_lds((down_project_kernel<8, 256, true>), (size_t)16 * 8 * 256 * sizeof(float))));
        TD_HIP((allow_lds((down_project_kernel<16, 128, true>), (size_t)16 * 16 * 128 * sizeof(float))));
        return TARDIS_OK;
    });
}

bool td_decode_fused_supported(const tardis_layer_s* L) {
    if (L->dtype != TARDIS_BF16) return false;
    if (!(L->d == 1024 || L->d == 2048 || L->d == 4096)) return false;   // wider rows exceed the register file
    const int G = L->dec_blocks;
    if (G < 1) return false;
    int64_t npb = (L->h + G - 1) / G;
    npb = (npb + 31) / 32 * 32;
    return npb <= kMaxNeuronsPerBlock;
}

namespace {

// one group of `tokens` (1, 2, 4, 8, 16) slots, n_act of them real, with working memory `ws`
tardis_status_t decode_group(tardis_layer_s* L, const DecodeScratch& ws, const void* x, void* y, float* yfold,
                             uint32_t* mask, int tokens, int n_act, int norm_out, hipStream_t s) {
    // packed 4-bit sketch (d = 2048 or 4096 only).  Groups of 8 and 16 tokens need one-byte codes
    // (the matrix-core predictor), and with 4 tokens the unpacking already costs more vector ALU
    // time than the halved stream saves (49 against 41 us at d = 4096, h = 16384): where the layer
    // keeps one-byte codes as well - the same integers by definition - groups of 4 and more read those
    if (L->Q4 && !(tokens >= 4 && L->Q && L->dec_threads == 1024)) {
        if (L->dec_threads == 512) {
            if (L->d == 2048) return launch_tb<2048, 512, 4>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
            if (L->d == 4096) return launch_tb<4096, 512, 4>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
        } else {
            if (L->d == 2048) return launch_tb<2048, 1024, 4>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
            if (L->d == 4096) return launch_tb<4096, 1024, 4>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
        }
        return TARDIS_ERR_SHAPE;
    }
    if (L->dec_threads == 512) {
        switch (L->d) {
            case 1024: return launch_tb<1024, 512, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
            case 2048: return launch_tb<2048, 512, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
            case 4096: return launch_tb<4096, 512, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
        }
    }
    switch (L->d) {
        case 1024: return launch_tb<1024, 1024, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
        case 2048: return launch_tb<2048, 1024, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
        case 4096: return launch_tb<4096, 1024, 8>(L, ws, x, y, yfold, mask, tokens, n_act, norm_out, s);
    }
    return TARDIS_ERR_SHAPE;
}

// n tokens as groups of 16, 8, 4, 2, 1 that share one pass over the weights each; yfold: n + 16
// rows of d floats, mask: n + 16 rows of mask words (a partly filled group may touch the slack)
tardis_status_t decode_tokens(tardis_layer_s* L, const DecodeScratch& ws, const bf16_t* x, int64_t n, bf16_t* y,
                              float* yfold, uint32_t* mask, int norm_out, hipStream_t s) {
    const int d = (int)L->d;
    const bool two4 = L->dec_threads == 1024 && L->defer_min_tokens <= 4 &&
                      (d + L->dec_blocks - 1) / L->dec_blocks <= 16;   // two-kernel groups of 4 exist
    const bool wide = two4 || (L->dec_threads == 1024 && L->defer_min_tokens <= 8 &&
                               (d + L->dec_blocks - 1) / L->dec_blocks <= 16);   // ... of 8 and 16
    for (int64_t t = 0; t < n;) {
        const int64_t left = n - t;
        // a two-kernel group may be partly empty: 3 tokens cost less as a group of 4 than as 2 + 1,
        // 5-7 less as a group of 8, 9-15 less as a group of 16
        // (only where every two-kernel group size exists, so that a split group stays on that path)
        int g, act;
        if (wide && (left >= 16 || (two4 && left >= 9))) { g = 16; act = left >= 16 ? 16 : (int)left; }
        else if (wide && (left >= 8 || (two4 && left >= 5))) { g = 8; act = left >= 8 ? 8 : (int)left; }
        else if (left >= 4 || (two4 && left == 3)) { g = 4; act = left >= 4 ? 4 : 3; }
        else { g = left >= 2 ? 2 : 1; act = g; }
        TD_TRY(decode_group(L, ws, x + t * d, y + t * d, yfold + t * d, mask + t * L->mask_words, g, act, norm_out, s));
        t += act;
    }
    return TARDIS_OK;
}

}  // namespace

tardis_status_t td_decode_fused(tardis_layer_s* L, const void* x, int64_t n, void* y, int norm_out, hipStream_t s) {
    const DecodeScratch ws{L->yfix, L->sync, L->rec_count, L->rec_jb, L->rec_tb, L->rec_delta};
    return decode_tokens(L, ws, static_cast<const bf16_t*>(x), n, static_cast<bf16_t*>(y), L->yacc, L->mask, norm_out, s);
}

// ---------------------------------------------------------------------------------------------
// Static working memory: the decode path for callers that cannot allocate (HIP graph capture,
// serving loops, harnesses that forbid hipMalloc).  One array per GPU, part of the code object,
// held until the process ends; every call on a GPU shares it.
namespace {

constexpr int kStaticMaxD = 4096;            // widest layer the static working memory serves
constexpr int kStaticMaxH = 16384;           // most neurons (mask words, records)
constexpr int kStaticMaxBlocks = 4096;       // largest decode grid
constexpr int kStaticMaxRecords = 32768;     // decode blocks x neurons per block
constexpr size_t kStSync = 0;                                                               // 64 counters
constexpr size_t kStYfix = 256;                                                             // 4 x 16 x d floats
constexpr size_t kStYfold = kStYfix + (size_t)kMaxCopies * kDecodeMaxTokens * kStaticMaxD * 4;   // 32 x d floats
constexpr size_t kStMask = kStYfold + (size_t)2 * kDecodeMaxTokens * kStaticMaxD * 4;            // 32 x h/32 words
constexpr size_t kStCount = kStMask + (size_t)2 * kDecodeMaxTokens * (kStaticMaxH / 32) * 4;
constexpr size_t kStJb = kStCount + (size_t)kStaticMaxBlocks * 4;
constexpr size_t kStTb = kStJb + (size_t)kStaticMaxRecords * 4;
constexpr size_t kStDelta = kStTb + (size_t)kStaticMaxRecords * 4;
constexpr size_t kStaticScratchBytes = kStDelta + (size_t)kStaticMaxRecords * kDecodeMaxTokens * 4;   // about 3.9 MiB
static_assert(kStYfix % 256 == 0 && kStYfold % 256 == 0 && kStMask % 256 == 0 && kStCount % 256 == 0 &&
                  kStJb % 256 == 0 && kStTb % 256 == 0 && kStDelta % 256 == 0,
              "every part starts on a 256-byte boundary");

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
unsigned char* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (the array's name is not one)

// the current device's copy of the array (looked up once per device)
tardis_status_t static_scratch(unsigned char** out) {
    int dev = -1;
    TD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TARDIS_ERR_STATE;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        unsigned char* p = nullptr;
        TD_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
        if (!p) return TARDIS_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TARDIS_OK;
}

// what a call needs to find zero: the completion counters and the repair accumulators it will use
__global__ void __launch_bounds__(256) clear_static_kernel(int32_t* __restrict__ sync, float* __restrict__ yfix, int n) {
    const int i = (int)blockIdx.x * 256 + threadIdx.x;
    if (i < 64) sync[i] = 0;
    if (i < n) yfix[i] = 0.0f;
}

}  // namespace

tardis_status_t td_static_scratch_setup() {
    unsigned char* p = nullptr;
    return static_scratch(&p);
}

extern "C" tardis_status_t tardis_ffn_forward_static(tardis_handle_t L, const void* x, int64_t n, void* y,
                                                      uint32_t* mask_out, void* stream) {
    if (!L || !td_layer_is_live(L) || L->poisoned) return TARDIS_ERR_STATE;
    if (!x || !y || x == y) return TARDIS_ERR_INVALID_ARG;
    if (n < 1 || n > kDecodeMaxTokens) return TARDIS_ERR_SHAPE;
    if (!L->use_fused || L->dtype != TARDIS_BF16) return TARDIS_ERR_STATE;
    const int64_t npb = ((L->h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
    if (L->d > kStaticMaxD || L->h > kStaticMaxH || L->dec_blocks > kStaticMaxBlocks ||
        (int64_t)L->dec_blocks * npb > kStaticMaxRecords || L->dec_copies > kMaxCopies)
        return TARDIS_ERR_SHAPE;   // beyond what the static working memory holds
    unsigned char* base = nullptr;
    TD_TRY(static_scratch(&base));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const DecodeScratch ws{reinterpret_cast<float*>(base + kStYfix),    reinterpret_cast<int32_t*>(base + kStSync),
                           reinterpret_cast<int32_t*>(base + kStCount), reinterpret_cast<uint32_t*>(base + kStJb),
                           reinterpret_cast<uint32_t*>(base + kStTb),   reinterpret_cast<float*>(base + kStDelta)};
    // the array keeps the last call's contents (and an interrupted call's): clear what must start at
    // zero, with a kernel (a memset node in a captured graph is not safe to replay here)
    const int nfix = (L->dec_copies < 2 ? 2 : L->dec_copies) * kDecodeMaxTokens * (int)L->d;   // (8-byte fixed-point words fit too)
    hipLaunchKernelGGL(clear_static_kernel, dim3((nfix + 255) / 256), dim3(256), 0, s, ws.sync, ws.yfix, nfix);
    TD_HIP(hipGetLastError());
    // mask words: the caller's buffer when given and no group can be partly empty past its end
    // (a partly filled group only writes the rows of its real tokens), else the static one
    uint32_t* mask = mask_out ? mask_out : reinterpret_cast<uint32_t*>(base + kStMask);
    return decode_tokens(L, ws, static_cast<const bf16_t*>(x), n, static_cast<bf16_t*>(y),
                         reinterpret_cast<float*>(base + kStYfold), mask, 0, s);
}

tardis_status_t td_mask_union(const tardis_layer_s* L, int64_t n, uint32_t* union_mask, int32_t* union_count,
                              hipStream_t s) {
    hipLaunchKernelGGL(mask_union_kernel, dim3(1), dim3(256), 0, s, L->mask, (int)L->mask_words, (int)n, union_mask,
                       union_count);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

tardis_status_t td_mask_to_list(const tardis_layer_s* L, int64_t n, int32_t* counts, int32_t* list, hipStream_t s) {
    hipLaunchKernelGGL(mask_to_list_kernel, dim3((unsigned)n), dim3(256), 0, s, L->mask, (int)L->mask_words,
                       (int)L->h, counts, list);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
