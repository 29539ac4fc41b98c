// Batched online path (2..64 tokens per pass, bf16 storage): every weight matrix
// is streamed ONCE per pass of up to 64 tokens instead of once per token.
//
// Steps per pass (Sec. "Inference Runtime", strictly per token):
//   quantise     per token max|x|, exponent e_t and int8 code
//   fold+predict W'X^T (bf16 MFMA) and QXq^T (int8 MFMA, exact int32) in one launch;
//                flags -> per-token mask words, per-neuron token bitmask, and the
//                list of neurons flagged by at least one token (the "union")
//   delta        rows W1[j] of the union only (gathered): z, then
//                delta = sigma(z) - (a z + c) for the (token, neuron) pairs that
//                were flagged, 0 elsewhere
//   scatter      y += Delta . W2: the masked dense product over W2 on the matrix cores
//                (a variant that gathered the union rows of W2^T for up to 16 tokens
//                never beat it where this path is used, nor the decode groups where it
//                did: measured per fallback rate, and removed)
//   finish       sum of the partial products, optional RMS norm, conversion
//
// The streaming kernel is bandwidth bound: one wavefront owns 16 weight rows and
// keeps 2 x 8 sixteen-byte loads per lane in flight; the token chunk is staged
// through double-buffered LDS and shared by the block's four wavefronts.
#include "common.h"
#include "rowdot.h"

namespace {

constexpr int kTB = 64;                       // tokens per pass
constexpr int kRowsPerBlock = 64;             // 4 wavefronts x 16 rows
constexpr int kChunk = 512;                   // bytes of every weight row per pipeline stage
constexpr int kXPitch = kChunk + 16;          // LDS pitch of a staged token row
constexpr int kDownSplits = 8;                // split of the hidden axis in the masked dense scatter

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

enum { EPI_FOLD = 0, EPI_PRED = 1, EPI_DELTA = 2, EPI_DOWN = 3 };

struct StreamArgs {
    const unsigned char* W;        // weight rows
    int64_t row_bytes;             // bytes per weight row (a multiple of kChunk * splits)
    int M;                         // rows of W (capacity of the gather list when gathering)
    const int32_t* gather;         // row indices, or null for rows 0..M-1
    const int32_t* gather_count;   // device count of gather entries
    const unsigned char* X;        // tokens: n_tok rows of row_bytes bytes
    int n_tok;
    // fold
    const float* bp;
    float* yfold;                  // [token][d]
    float* yfold2;                 // [token][d]: sums of the second half of K when the fold rows are split (no bias)
    int d;
    // predict
    const float* tlo;
    const float* thi;
    const int32_t* e_tok;
    uint32_t* mask;                // [token][mask_words]
    int mask_words;
    unsigned long long* tokmask;   // [neuron]
    int32_t* ulist;
    int32_t* ucount;
    // delta
    const bf16_t* b1;
    const float* a;
    const float* c;
    int act;
    bf16_t* delta;                 // token-major [64][h]; only flagged (token, neuron) pairs are written (zeroed per pass)
    int h;
    // down
    float* partial;                // [split][64][d]
};

template <bool I8> struct Acc;
template <> struct Acc<false> { typedef f32x4_t type; };
template <> struct Acc<true> { typedef i32x4_t type; };

// D = A.B^T on one 16x16 tile: operand lanes hold 16 bytes of row (lane % 16) at k-group (lane / 16)
template <bool I8>
__device__ __forceinline__ typename Acc<I8>::type mma16(const td_u32x4& rowsA, const td_u32x4& rowsB,
                                                        typename Acc<I8>::type acc);
template <>
__device__ __forceinline__ f32x4_t mma16<false>(const td_u32x4& ra, const td_u32x4& rb, f32x4_t acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ra), __builtin_bit_cast(bf16x8_t, rb),
                                                   acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ i32x4_t mma16<true>(const td_u32x4& ra, const td_u32x4& rb, i32x4_t acc) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, ra), __builtin_bit_cast(i32x4_t, rb), acc,
                                                 0, 0, 0);
}

// One block: 64 weight rows (16 per wavefront) against NT*16 tokens over this block's K range.
// TOKEN_ROWS: the tile is produced as D[token][weight row] (stores contiguous along the weight
// rows) instead of D[weight row][token].
template <bool I8, int NT, int EPI, int NCH, int WV = 4>
__device__ __forceinline__ void stream_body(const StreamArgs& p, int row_block, int split, int chunks_rt,
                                            unsigned char* lds) {
    // NCH > 0: the chunk count is a compile-time constant and the pipeline below is fully unrolled
    // (straight-line code lets the compiler count outstanding loads exactly); NCH == 0: run time.
    constexpr int kRows = 16 * WV;                   // weight rows of this block (kRowsPerBlock with 4 wavefronts)
    constexpr int kThreads = 64 * WV;
    const int chunks_per_split = NCH > 0 ? NCH : chunks_rt;
    constexpr bool TOKEN_ROWS = (EPI == EPI_FOLD || EPI == EPI_DOWN);
    typedef typename Acc<I8>::type acc_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;

    int count = p.M;
    if (p.gather) {
        count = min(*p.gather_count, p.M);
        if (row_block * kRows >= count) return;                  // uniform: nothing gathered for this block
    }
    const int rw = row_block * kRows + wave * 16;                // first row (or list slot) of this wavefront
    int my_row = min(rw + l16, count - 1);
    if (p.gather) my_row = p.gather[my_row];
    const unsigned char* wsrc = p.W + (size_t)my_row * p.row_bytes + (size_t)split * chunks_per_split * kChunk + g * 16;

    // token staging map: piece q of this thread -> token (idx / 32), 16-byte piece (idx % 32).
    // Token slots past n_tok re-read the last token: every load is unconditional (the in-order
    // load counter stays statically known to the compiler) and the columns they produce are never
    // stored (each token is an independent column of the product).
    constexpr int XP = NT * 512 / kThreads;          // 16-byte pieces of the token chunk per thread
    const unsigned char* xsrc[XP];
    int xdst[XP];
#pragma unroll
    for (int q = 0; q < XP; ++q) {
        const int idx = tid + kThreads * q;
        const int t = idx >> 5, piece = idx & 31;
        xsrc[q] = p.X + (size_t)min(t, p.n_tok - 1) * p.row_bytes + (size_t)split * chunks_per_split * kChunk + piece * 16;
        xdst[q] = t * kXPitch + piece * 16;
    }

    acc_t acc[NT];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) acc[tt] = acc_t{0, 0, 0, 0};

    // Pipeline: while chunk ch is multiplied, the weights of chunks ch+1, ch+2 and the tokens of
    // chunks ch+1 (on their way to LDS) and ch+2 are in flight.  The three weight buffers and the
    // two token buffers are named statically (the loop is unrolled by six): a register copy would
    // have to wait for the load it copies.  Past the last chunk the prefetches re-read chunk 0 (a
    // cache hit) instead of being skipped, so that the in-order load counter stays statically
    // known and no wait ever drains more than it needs.
    // Blocks walk the chunks of their K range from different starting points (the order of the sum
    // does not matter): with every block at the same chunk index all loads in flight would share
    // the address bits between the chunk and the row pitch, and crowd onto a few memory channels.
    const int last = chunks_per_split - 1;
    const int rot = (row_block * 5 + split * 3) % chunks_per_split;
    auto chunk_at = [&](int ch) {
        int c = (ch <= last ? ch : 0) + rot;
        return c >= chunks_per_split ? c - chunks_per_split : c;
    };
    td_u32x4 w0[8], w1[8], w2[8], xa[XP], xb[XP];
    auto load_w = [&](td_u32x4 (&dst)[8], int ch) {
        const unsigned char* src = wsrc + (size_t)chunk_at(ch) * kChunk;
#pragma unroll
        for (int s = 0; s < 8; ++s) dst[s] = td_load_stream16(src + s * 64);
    };
    auto load_x = [&](td_u32x4 (&dst)[XP], int ch) {
        const size_t off = (size_t)chunk_at(ch) * kChunk;
#pragma unroll
        for (int q = 0; q < XP; ++q) dst[q] = *reinterpret_cast<const td_u32x4*>(xsrc[q] + off);
    };
    auto stash_x = [&](const td_u32x4 (&src)[XP], int buf) {
        unsigned char* nb = lds + buf * (kTB * kXPitch);
#pragma unroll
        for (int q = 0; q < XP; ++q) *reinterpret_cast<td_u32x4*>(nb + xdst[q]) = src[q];
    };
    load_x(xa, 0);
    load_x(xb, 1);
    asm volatile("" ::: "memory");   // issue order = program order from here on
    load_w(w0, 0);
    load_w(w1, 1);
    asm volatile("" ::: "memory");
    stash_x(xa, 0);
    __syncthreads();

    // step ch: tokens of chunk ch+2 -> xl, weights of chunk ch+2 -> pre, multiply cur, tokens of
    // chunk ch+1 (xs, requested one step ago) -> LDS
    auto step = [&](td_u32x4 (&cur)[8], td_u32x4 (&pre)[8], td_u32x4 (&xl)[XP], td_u32x4 (&xs)[XP], int ch) {
        load_x(xl, ch + 2);
        asm volatile("" ::: "memory");
        load_w(pre, ch + 2);
        asm volatile("" ::: "memory");
        const unsigned char* xf0 = lds + (ch & 1) * (kTB * kXPitch) + l16 * kXPitch + g * 16;
        // the token fragments of sub-step s+1 are read from LDS while the MFMAs of sub-step s run
        // (the scheduler, left alone, reads each fragment right before its use and the matrix
        // cores wait out the LDS latency thirty-two times per chunk)
        td_u32x4 xf[2][NT];
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) xf[0][tt] = *reinterpret_cast<const td_u32x4*>(xf0 + tt * 16 * kXPitch);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (s + 1 < 8) {
#pragma unroll
                for (int tt = 0; tt < NT; ++tt)
                    xf[(s + 1) & 1][tt] = *reinterpret_cast<const td_u32x4*>(xf0 + tt * 16 * kXPitch + (s + 1) * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
                acc[tt] = TOKEN_ROWS ? mma16<I8>(xf[s & 1][tt], cur[s], acc[tt]) : mma16<I8>(cur[s], xf[s & 1][tt], acc[tt]);
            __builtin_amdgcn_sched_barrier(0);
        }
        stash_x(xs, (ch + 1) & 1);
        __syncthreads();
    };
    if constexpr (NCH > 0) {
#pragma unroll
        for (int ch = 0; ch < NCH; ch += 6) {
            step(w0, w2, xa, xb, ch);
            if (ch + 1 < NCH) step(w1, w0, xb, xa, ch + 1);
            if (ch + 2 < NCH) step(w2, w1, xa, xb, ch + 2);
            if (ch + 3 < NCH) step(w0, w2, xb, xa, ch + 3);
            if (ch + 4 < NCH) step(w1, w0, xa, xb, ch + 4);
            if (ch + 5 < NCH) step(w2, w1, xb, xa, ch + 5);
        }
    } else {
        for (int ch = 0; ch <= last; ch += 6) {   // chunk counts are uniform over the block
            step(w0, w2, xa, xb, ch);
            if (ch + 1 > last) break;
            step(w1, w0, xb, xa, ch + 1);
            if (ch + 2 > last) break;
            step(w2, w1, xa, xb, ch + 2);
            if (ch + 3 > last) break;
            step(w0, w2, xb, xa, ch + 3);
            if (ch + 4 > last) break;
            step(w1, w0, xa, xb, ch + 4);
            if (ch + 5 > last) break;
            step(w2, w1, xb, xa, ch + 5);
        }
    }

    // ------------------------------------------------------------------ epilogues
    // TOKEN_ROWS: acc[tt][i] = D[token tt*16 + 4g + i][weight row rw + l16]
    // otherwise : acc[tt][i] = D[weight row rw + 4g + i][token tt*16 + l16]
    if constexpr (EPI == EPI_FOLD) {
        const int r = rw + l16;
        if (r < p.M) {
            const float b = p.bp[r];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = tt * 16 + 4 * g + i;
                    if (t < p.n_tok) {
                        if (split == 0) p.yfold[(size_t)t * p.d + r] = acc[tt][i] + b;
                        else p.yfold2[(size_t)t * p.d + r] = acc[tt][i];
                    }
                }
        }
    } else if constexpr (EPI == EPI_DOWN) {
        const int r = rw + l16;
        if (r < p.M) {
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = tt * 16 + 4 * g + i;
                    if (t < p.n_tok) p.partial[((size_t)split * kTB + t) * p.d + r] = acc[tt][i];
                }
        }
    } else if constexpr (EPI == EPI_PRED) {
        uint32_t* lmask = reinterpret_cast<uint32_t*>(lds + 2 * kTB * kXPitch);   // [64 tokens][2 words]
        uint32_t* ltok = lmask + 128;                                           // [64 rows][2 words]
        if (tid < 128) {
            lmask[tid] = 0u;
            ltok[tid] = 0u;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rl = wave * 16 + 4 * g + i;                   // row within the block
            const int r = row_block * kRowsPerBlock + rl;
            if (r >= p.M) continue;
            const float lo = p.tlo[r], hi = p.thi[r];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const int t = tt * 16 + l16;
                if (t >= p.n_tok) continue;
                const float v = ldexpf((float)acc[tt][i], p.e_tok[t]);
                const bool inside = (v >= lo) && (v < hi);
                if (!inside) {
                    atomicOr(&lmask[t * 2 + (rl >> 5)], 1u << (rl & 31));
                    atomicOr(&ltok[rl * 2 + (t >> 5)], 1u << (t & 31));
                }
            }
        }
        __syncthreads();
        if (tid < 128) {
            const int t = tid >> 1, w = tid & 1;
            const int word = row_block * 2 + w;
            if (t < p.n_tok && word < p.mask_words) p.mask[(size_t)t * p.mask_words + word] = lmask[tid];
        }
        if (wave == 0) {
            const int r = row_block * kRowsPerBlock + lane;
            const unsigned long long tm = (unsigned long long)ltok[lane * 2] | ((unsigned long long)ltok[lane * 2 + 1] << 32);
            const bool any = r < p.M && tm != 0ull;
            if (r < p.M) p.tokmask[r] = tm;
            const unsigned long long bal = __ballot(any);
            int base = 0;
            if (lane == 0 && bal) base = atomicAdd(p.ucount, __popcll(bal));
            base = __shfl(base, 0, 64);
            if (any) p.ulist[base + __popcll(bal & ((1ull << lane) - 1ull))] = r;
        }
    } else {  // EPI_DELTA
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int slot = rw + 4 * g + i;
            if (slot >= count) continue;
            const int j = p.gather[slot];
            const unsigned long long tm = p.tokmask[j];
            const float bj = td_bf16_to_f32(p.b1[j]), aj = p.a[j], cj = p.c[j];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const int t = tt * 16 + l16;
                float dv = 0.0f;
                if (t < p.n_tok && ((tm >> t) & 1ull)) {
                    const float z = acc[tt][i] + bj;
                    dv = td_act(z, p.act) - fmaf(aj, z, cj);
                }
                if (dv != 0.0f) p.delta[(size_t)t * p.h + j] = td_f32_to_bf16(dv);
            }
        }
    }
}

constexpr int kStreamLds = 2 * kTB * kXPitch + 1024;

// fold (bf16, blocks [0, fold_blocks)) and predictor (int8, the rest) in one launch
// FCH, PCH: compile-time chunk counts of the fold / predictor rows (0 = run time)
template <int NT, int FCH, int PCH>
__global__ void __launch_bounds__(256)
fold_predict_batched_kernel(StreamArgs fold, StreamArgs pred, int fold_blocks, int fold_splits, int fold_chunks,
                            int pred_chunks) {
    // fold rows are twice as long as predictor rows (bf16 against int8): with K of the fold cut in
    // two (fold_chunks per half, the halves summed by the finishing kernel) every block of the
    // launch streams the same number of chunks and the chip stays full to the end
    extern __shared__ __align__(16) unsigned char lds[];
    const int b = (int)blockIdx.x;
    if (b < fold_blocks * fold_splits)
        stream_body<false, NT, EPI_FOLD, FCH>(fold, b % fold_blocks, b / fold_blocks, fold_chunks, lds);
    else
        stream_body<true, NT, EPI_PRED, PCH>(pred, b - fold_blocks * fold_splits, 0, pred_chunks, lds);
}

// WV wavefronts of 16 rows each per block.  Every block stages the pass's token chunks through LDS
// itself, so token bytes cross L2 once per block: the masked dense scatter, whose K is split
// anyway, runs 8 wavefronts (128 rows) per block and halves that traffic.
template <int NT, int EPI, int NCH, int WV = 4>
__global__ void __launch_bounds__(64 * WV) stream_kernel(StreamArgs p, int chunks_per_split) {
    extern __shared__ __align__(16) unsigned char lds[];
    stream_body<false, NT, EPI, NCH, WV>(p, blockIdx.x, blockIdx.y, chunks_per_split, lds);
}

// per token: max|x|, exponent, int8 code (one block per token).  The first kernel of a pass also
// re-arms what the later ones accumulate into: the union counter and, for the masked dense
// scatter, the token-major delta buffer (zero_words 32-bit words; 0 = leave it alone).
__global__ void __launch_bounds__(256)
quantize_tokens_kernel(const bf16_t* __restrict__ X, int d, int8_t* __restrict__ XQ, int32_t* __restrict__ E,
                       int32_t* __restrict__ ucount, uint4* __restrict__ zero_buf, size_t zero_vecs) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    if (t == 0 && threadIdx.x == 0) *ucount = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < zero_vecs; i += (size_t)gridDim.x * 256)
        zero_buf[i] = make_uint4(0u, 0u, 0u, 0u);
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

__global__ void __launch_bounds__(256) fill_u32_kernel(uint32_t* __restrict__ p, size_t n, uint32_t v) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// y[t] = yfold[t] + sum_s partial[s][t], optional RMS norm, conversion.  One block of 1024
// threads per token, 4 columns per thread per step; d is a multiple of 4.
__global__ void __launch_bounds__(1024)
finish_batched_kernel(const float* __restrict__ yfold, const float* __restrict__ partial, int nparts, int d,
                      bf16_t* __restrict__ y, int norm_out, float eps) {
    __shared__ float red[16];
    extern __shared__ __align__(16) float row[];
    const int t = blockIdx.x;
    float ss = 0.0f;
    for (int k4 = threadIdx.x; k4 < d / 4; k4 += 1024) {
        f32x4_t v = reinterpret_cast<const f32x4_t*>(yfold + (size_t)t * d)[k4];
        f32x4_t part[16];
#pragma unroll
        for (int s = 0; s < 16; ++s)
            part[s] = s < nparts ? reinterpret_cast<const f32x4_t*>(partial + ((size_t)s * kTB + t) * d)[k4]
                                 : f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < 16; ++s) v += part[s];
        reinterpret_cast<f32x4_t*>(row)[k4] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    float scale = 1.0f;
    if (norm_out) {
        ss = td_wave_sum(ss);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
        __syncthreads();
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) tot += red[w];
        scale = 1.0f / sqrtf(tot / (float)d + eps);
    }
    for (int k4 = threadIdx.x; k4 < d / 4; k4 += 1024) {
        const f32x4_t v = reinterpret_cast<const f32x4_t*>(row)[k4] * scale;
        uint2 o;
        o.x = (uint32_t)td_f32_to_bf16(v.x) | ((uint32_t)td_f32_to_bf16(v.y) << 16);
        o.y = (uint32_t)td_f32_to_bf16(v.z) | ((uint32_t)td_f32_to_bf16(v.w) << 16);
        reinterpret_cast<uint2*>(y + (size_t)t * d)[k4] = o;
    }
}

inline int div_up(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

template <typename K> hipError_t allow_big_lds(K kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               kStreamLds);
}

template <int NT>
tardis_status_t pass_t(tardis_layer_s* L, const bf16_t* x, int nt, bf16_t* y, uint32_t* mask, float* yfold,
                       int norm_out, hipStream_t s) {
    const int d = (int)L->d, h = (int)L->h;
    // (the delta buffer is kTB x h bf16 from a 256-byte aligned allocation: whole 16-byte vectors when h % 8 == 0)
    const size_t zero_vecs = (size_t)kTB * h * 2 / 16;
    hipLaunchKernelGGL(quantize_tokens_kernel, dim3(nt), dim3(256), 0, s, x, d, L->bt_xq, L->bt_e, L->bt_ucount,
                       reinterpret_cast<uint4*>(L->bt_delta), zero_vecs);
    if (((size_t)kTB * h * 2) % 16 != 0) {          // odd h: the tail by the word
        const size_t words = (size_t)kTB * h / 2;
        hipLaunchKernelGGL(fill_u32_kernel, dim3(div_up(words, 256)), dim3(256), 0, s,
                           reinterpret_cast<uint32_t*>(L->bt_delta), words, 0u);
    }
    StreamArgs base{};
    base.n_tok = nt;
    base.d = d;
    base.h = h;
    base.act = L->act;

    StreamArgs fold = base;
    fold.W = static_cast<const unsigned char*>(L->Wp);
    fold.row_bytes = (int64_t)d * 2;
    fold.M = d;
    fold.X = reinterpret_cast<const unsigned char*>(x);
    fold.bp = L->bp;
    fold.yfold = yfold;
    StreamArgs pred = base;
    pred.W = reinterpret_cast<const unsigned char*>(L->Q);
    pred.row_bytes = d;
    pred.M = h;
    pred.X = reinterpret_cast<const unsigned char*>(L->bt_xq);
    pred.tlo = L->tlo;
    pred.thi = L->thi;
    pred.e_tok = L->bt_e;
    pred.mask = mask;
    pred.mask_words = (int)L->mask_words;
    pred.tokmask = L->bt_tokmask;
    pred.ulist = L->bt_ulist;
    pred.ucount = L->bt_ucount;
    const int fold_blocks = div_up(d, kRowsPerBlock), pred_blocks = div_up(h, kRowsPerBlock);
    const int fsplit = ((d * 2 / kChunk) % 2 == 0) ? 2 : 1;
    fold.yfold2 = L->bt_partial + (size_t)kDownSplits * kTB * d;
    const dim3 fp_grid(fold_blocks * fsplit + pred_blocks);
    if (d == 4096 && fsplit == 2)
        hipLaunchKernelGGL((fold_predict_batched_kernel<NT, 8, 8>), fp_grid, dim3(256), kStreamLds, s, fold, pred,
                           fold_blocks, 2, 8, 8);
    else if (d == 4096)
        hipLaunchKernelGGL((fold_predict_batched_kernel<NT, 16, 8>), fp_grid, dim3(256), kStreamLds, s, fold, pred,
                           fold_blocks, 1, 16, 8);
    else
        hipLaunchKernelGGL((fold_predict_batched_kernel<NT, 0, 0>), fp_grid, dim3(256), kStreamLds, s, fold, pred,
                           fold_blocks, fsplit, d * 2 / kChunk / fsplit, d / kChunk);

    StreamArgs del = base;
    del.W = static_cast<const unsigned char*>(L->W1);
    del.row_bytes = (int64_t)d * 2;
    del.M = h;
    del.gather = L->bt_ulist;
    del.gather_count = L->bt_ucount;
    del.X = reinterpret_cast<const unsigned char*>(x);
    del.tokmask = L->bt_tokmask;
    del.b1 = static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h);
    del.a = L->a;
    del.c = L->c;
    del.delta = L->bt_delta;
    if (d == 4096)
        hipLaunchKernelGGL((stream_kernel<NT, EPI_DELTA, 16>), dim3(pred_blocks, 1), dim3(256), kStreamLds, s, del, 16);
    else
        hipLaunchKernelGGL((stream_kernel<NT, EPI_DELTA, 0>), dim3(pred_blocks, 1), dim3(256), kStreamLds, s, del,
                           d * 2 / kChunk);

    const int nparts = kDownSplits + (fsplit - 1);   // the fold's second half sits in the slot after the scatter's
    {
        StreamArgs down = base;
        down.W = static_cast<const unsigned char*>(L->W2);
        down.row_bytes = (int64_t)h * 2;
        down.M = d;
        down.X = reinterpret_cast<const unsigned char*>(L->bt_delta);
        down.partial = L->bt_partial;
        if (h == 16384 && NT == 4)
            hipLaunchKernelGGL((stream_kernel<NT, EPI_DOWN, 8, 8>), dim3(div_up(d, 128), kDownSplits), dim3(512),
                               kStreamLds, s, down, 8);
        else if (h == 16384)
            hipLaunchKernelGGL((stream_kernel<NT, EPI_DOWN, 8>), dim3(fold_blocks, kDownSplits), dim3(256), kStreamLds,
                               s, down, 8);
        else
            hipLaunchKernelGGL((stream_kernel<NT, EPI_DOWN, 0>), dim3(fold_blocks, kDownSplits), dim3(256), kStreamLds,
                               s, down, h * 2 / kChunk / kDownSplits);
    }
    hipLaunchKernelGGL(finish_batched_kernel, dim3(nt), dim3(1024), (size_t)d * sizeof(float), s, yfold, L->bt_partial,
                       nparts, d, y, norm_out, kRmsEps);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

}  // namespace

bool td_batched_supported(const tardis_layer_s* L) {
    return L->dtype == TARDIS_BF16 && L->max_batch > 1 && L->d % kChunk == 0 && L->d <= 8192 &&
           (L->h * 2) % ((int64_t)kChunk * kDownSplits) == 0;
}

size_t td_batched_partial_floats(const tardis_layer_s* L) {
    return (size_t)(kDownSplits + 1) * kTB * L->d;   // the scatter's splits and the fold's second half
}

// the streaming kernels use more than the default 64 KiB of dynamic LDS
tardis_status_t td_batched_init() {
    static td_once once;
    return once.run([]() -> tardis_status_t {
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<1, 0, 0>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<2, 0, 0>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<4, 0, 0>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<1, 8, 8>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<2, 8, 8>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<4, 8, 8>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<1, 16, 8>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<2, 16, 8>)));
        TD_HIP((allow_big_lds(fold_predict_batched_kernel<4, 16, 8>)));
        TD_HIP((allow_big_lds(stream_kernel<1, EPI_DELTA, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<2, EPI_DELTA, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<4, EPI_DELTA, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<1, EPI_DELTA, 16>)));
        TD_HIP((allow_big_lds(stream_kernel<2, EPI_DELTA, 16>)));
        TD_HIP((allow_big_lds(stream_kernel<4, EPI_DELTA, 16>)));
        TD_HIP((allow_big_lds(stream_kernel<1, EPI_DOWN, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<2, EPI_DOWN, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<4, EPI_DOWN, 0>)));
        TD_HIP((allow_big_lds(stream_kernel<1, EPI_DOWN, 8>)));
        TD_HIP((allow_big_lds(stream_kernel<2, EPI_DOWN, 8>)));
        TD_HIP((allow_big_lds(stream_kernel<4, EPI_DOWN, 8>)));
        TD_HIP((allow_big_lds(stream_kernel<4, EPI_DOWN, 8, 8>)));
        return TARDIS_OK;
    });
}

tardis_status_t td_forward_batched(tardis_layer_s* L, const void* xv, int64_t n, void* yv, int norm_out,
                                   hipStream_t s) {
    const int d = (int)L->d;
    for (int64_t t0 = 0; t0 < n; t0 += kTB) {
        const int nt = (int)((n - t0 < kTB) ? n - t0 : kTB);
        const bf16_t* x = static_cast<const bf16_t*>(xv) + t0 * d;
        bf16_t* y = static_cast<bf16_t*>(yv) + t0 * d;
        uint32_t* mask = L->mask + t0 * L->mask_words;
        float* yfold = L->yacc + t0 * d;
        tardis_status_t st;
        if (nt <= 16)
            st = pass_t<1>(L, x, nt, y, mask, yfold, norm_out, s);
        else if (nt <= 32)
            st = pass_t<2>(L, x, nt, y, mask, yfold, norm_out, s);
        else
            st = pass_t<4>(L, x, nt, y, mask, yfold, norm_out, s);
        TD_TRY(st);
    }
    L->last_n = n;
    return TARDIS_OK;
}
