// One token through a whole stack of folded layers in ONE launch (the FFN stack of chained layers
// with RMS-norm glue; per layer the online step of Sec. "Inference Runtime": speculative product,
// predictor, mask, result fixing).
//
// A launch per layer pays, per layer, the launch itself (about 2.5 us back to back) and the tail of
// the single-token kernel - atomics acknowledged, completion counter, the last block's assembly -
// during which the memory system idles.  Here the grid stays resident (a cooperative launch: all
// blocks are guaranteed to run at once, so waiting for one another cannot deadlock) and no block has
// a special role: every layer owns its accumulators and its counter (those of its handle), a block
// adds its repair vectors AND its rows of W'x + b' to the layer's accumulators, counts itself done,
// requests the first predictor rows of the next layer into its REGISTERS and waits for the counter
// to reach the grid size.  Then every block reads the accumulators itself (16 KiB per copy, out of
// its XCD's L2 after the first reader), normalises, and goes on: per layer one round of atomics, one
// counter, one read - no assembly by a single block, no publication step.  Buffers that belong to a
// layer are written and read once per launch, so no cache can hold an older version of them and no
// invalidation is needed; a small kernel behind the launch re-arms them (and turns the output into
// NaNs should a bounded wait ever have run out).
//
// Work split per layer as in the single-token kernel: block b owns neurons [b*npb, (b+1)*npb)
// (predictor rows, repair of the flagged ones) and rows [b*rpb, (b+1)*rpb) of W'; contributions go
// to two accumulator copies with coalesced fp32 atomics.
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <vector>

#include "common.h"
#include "rowdot.h"

namespace {

constexpr int kMaxStackLayers = 64;          // layers per launch (a longer stack runs layer by layer)
constexpr int kStackNpbMax = 64;             // neurons per block: one pass of 16 wavefronts x 4 rows
constexpr int kStackCopies = 2;               // accumulator copies per layer (blocks alternate between them)
constexpr int kErrAt = 48;                   // counter index (first layer's) set if a bounded wait ran out

struct StackArgs {
    const td_stack_layer_dev* layer[kMaxStackLayers];
    int n_layers;
    const bf16_t* x;      // d values
    bf16_t* y;            // d values: the last layer's (un-normalised) output
    int32_t* err;
    float eps;
    int spin_limit;
#ifdef TD_STACK_TRACE
    unsigned long long* trace;   // [layer][block][8] time stamps (100 MHz), a debugging build only
#endif
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void wait_memory_acks() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Pointers that reach the kernel through a layer's descriptor (loaded from memory, not kernel
// arguments) are generic to the compiler: it would use flat loads, which also wait on the LDS
// counter.  They all point to device memory; say so.  Values that are constant once a layer is
// folded and the same for a whole wavefront (thresholds of a row) go through the constant address
// space: scalar loads, scalar registers, and not in the queue of vector loads.
#define TD_GLOBAL __attribute__((address_space(1)))
#define TD_CONST __attribute__((address_space(4)))
template <typename T> __device__ __forceinline__ const TD_GLOBAL T* gptr(const T* p) { return (const TD_GLOBAL T*)p; }
template <typename T> __device__ __forceinline__ TD_GLOBAL T* gptr(T* p) { return (TD_GLOBAL T*)p; }
template <typename T> __device__ __forceinline__ const TD_CONST T* cptr(const T* p) { return (const TD_CONST T*)p; }

// Wavefront reductions by lane-crossing moves with fixed patterns (no index registers, which the
// compiler would keep alive across the whole layer loop); the result is the same in every lane.
template <typename Op>
__device__ __forceinline__ int wave_reduce_bits(int v, Op op) {
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));    // lanes 1 apart (quad_perm 1,0,3,2)
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));    // 2 apart (quad_perm 2,3,0,1)
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));   // the other quad of each 8 (row_half_mirror)
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));   // the other 8 of each 16 (row_mirror)
    v = op(v, __builtin_amdgcn_ds_swizzle(v, 0x401F));                      // 16 apart
    return op(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 32));
}
__device__ __forceinline__ float wave_sum_f(float v) {
    return __int_as_float(wave_reduce_bits(__float_as_int(v), [](int a, int b) { return __float_as_int(__int_as_float(a) + __int_as_float(b)); }));
}
__device__ __forceinline__ float wave_max_f(float v) {
    return __int_as_float(wave_reduce_bits(__float_as_int(v), [](int a, int b) { return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b))); }));
}
__device__ __forceinline__ int wave_sum_i(int v) {
    return wave_reduce_bits(v, [](int a, int b) { return a + b; });
}

#ifdef TD_STACK_TRACE
#define TD_MARK(k) do { if (tid == 0) A.trace[((size_t)l * G + blk) * 8 + (k)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define TD_MARK(k) do { } while (0)
#endif

template <int N>
__device__ __forceinline__ void load_row16(td_u32x4 (&dst)[N], const void* row, int lane) {
    const TD_GLOBAL td_u32x4* p = gptr(static_cast<const td_u32x4*>(row)) + lane;
#pragma unroll
    for (int it = 0; it < N; ++it) dst[it] = __builtin_nontemporal_load(p + it * TD_WAVE);
}

template <int D>
__global__ void __launch_bounds__(1024) stack_decode_kernel(StackArgs A) {
    constexpr int BLOCK = 1024, NW = BLOCK / TD_WAVE, RQ = 4;
    constexpr int NVW = D / 8;                       // 16-byte vectors of a bf16 row
    constexpr int IQ = D / 16 / TD_WAVE;             // per-lane vectors of a predictor row
    constexpr int IW = NVW / TD_WAVE;                // per-lane vectors of a bf16 row
    constexpr int IWA = IW / 2;                      // vectors of the W' row requested before the flags are known
    constexpr int CPT = D / BLOCK;                   // output columns per thread
    constexpr int KPRE = RQ / 2;                     // predictor rows of the next layer requested before the wait for this one
    constexpr int NLIVE = D / 4;                     // threads that hold four values of the token
    static_assert(D % 1024 == 0 && D <= 4096, "four values of the token per thread");
    static_assert(kStackNpbMax == NW * RQ, "one predictor pass per layer");

    extern __shared__ __align__(16) bf16_t w2s[];     // NW rows of W2^T (the repair's staging)
    __shared__ __align__(16) bf16_t xs[D];
    __shared__ __align__(16) int8_t xq[D];
    __shared__ float dl[NW];
    __shared__ float red_s[NW], red_m[NW];
    __shared__ int flist[kStackNpbMax];
    __shared__ uint32_t words[kStackNpbMax / 32];
    __shared__ int nflag, bail;

    const int tid = threadIdx.x, lane = tid & (TD_WAVE - 1), blk = blockIdx.x;
    // (wave-uniform values are made known as such: row addresses then are scalar bases plus one lane offset,
    //  instead of a 64-bit address pair per load held in vector registers across the layer loop)
    const int wave = __builtin_amdgcn_readfirstlane(tid / TD_WAVE);
    const int G = (int)gridDim.x;
    const int rpb = (D + G - 1) / G;
    const int r0 = blk * rpb, rn = min(rpb, D - r0);          // W' rows owned (at most one per wavefront)
    const int ctid = (tid + TD_WAVE * (blk >> 3)) & (BLOCK - 1);   // rotated column ownership (see decode kernel)
    const bool live = tid < NLIVE;

    td_u32x4 q[RQ][IQ];
    float tl[RQ], th[RQ];
    auto load_rows = [&](auto L, auto first, auto last) {      // predictor rows [first, last) of this wavefront
#pragma unroll
        for (int i = decltype(first)::value; i < decltype(last)::value; ++i) {
            const int j = min(blk * L->npb + wave * RQ + i, L->h - 1);
            load_row16<IQ>(q[i], L->Q + (size_t)j * D, lane);
            tl[i] = cptr(L->tlo)[j];
            th[i] = cptr(L->thi)[j];
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using IK = std::integral_constant<int, KPRE>;
    using IR = std::integral_constant<int, RQ>;

    // a layer's descriptor is constant once the layer is folded: it is read through the constant address
    // space, field by field where needed, so that the values arrive by scalar loads into scalar registers
    typedef const TD_CONST td_stack_layer_dev* desc_t;
    auto descriptor = [&](int l) -> desc_t { return (desc_t)A.layer[l]; };
    load_rows(descriptor(0), I0{}, IK{});

    const float* acc_prev = nullptr;      // the previous layer's accumulators, counter and hand-over buffer
    const int32_t* cnt_prev = nullptr;
    bf16_t* hand_prev = nullptr;

#pragma unroll 1
    for (int l = 0;; ++l) {
        // (per-lane offsets are re-derived in every layer from values the compiler cannot see through: hoisted out
        //  of the layer loop they would occupy vector registers for the whole launch and end up spilled)
        int lane_v = lane, ctid_v = ctid, wave_s = wave, tid_v = tid;
        asm volatile("" : "+v"(lane_v), "+v"(ctid_v), "+s"(wave_s), "+v"(tid_v));

        // ---- this layer's token: the caller's (first layer), else the previous layer's output, complete once
        //      every block has counted itself done there (bounded wait)
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (l < A.n_layers) TD_MARK(0);
        if (l == 0) {
            if (live) {
                const u32x2 raw = reinterpret_cast<const u32x2*>(A.x)[tid_v];
                v.x = __uint_as_float(raw.x << 16);
                v.y = __uint_as_float(raw.x & 0xFFFF0000u);
                v.z = __uint_as_float(raw.y << 16);
                v.w = __uint_as_float(raw.y & 0xFFFF0000u);
            }
        } else {
            if (tid == 0) {
                int spins = 0;
                while (__hip_atomic_load(gptr(cnt_prev), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < G && ++spins < A.spin_limit)
                    __builtin_amdgcn_s_sleep(4);
                bail = spins >= A.spin_limit;
            }
            __syncthreads();
            if (__builtin_amdgcn_readfirstlane(bail) != 0) {
                // the wait ran out (the grid is resident as a whole, so this needs a fault elsewhere): leave, loudly -
                // the error word makes the kernel behind this launch turn y into NaNs; the other blocks run out too
                if (tid == 0) __hip_atomic_store(A.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
            asm volatile("" ::: "memory");
            if (live) {     // (both copies requested before either is used)
                const f32x4 c0 = gptr(reinterpret_cast<const f32x4*>(acc_prev))[tid_v];
                const f32x4 c1 = gptr(reinterpret_cast<const f32x4*>(acc_prev + D))[tid_v];
                v = c0 + c1;
            }
        }
        if (l == A.n_layers) {      // (only the first block comes here) the stack's output, not normalised
            if (live) {
                const u32x2 o = u32x2{(uint32_t)td_f32_to_bf16(v.x) | ((uint32_t)td_f32_to_bf16(v.y) << 16),
                                           (uint32_t)td_f32_to_bf16(v.z) | ((uint32_t)td_f32_to_bf16(v.w) << 16)};
                reinterpret_cast<u32x2*>(A.y)[tid_v] = o;
            }
            return;
        }
        TD_MARK(1);
        const desc_t Lc = descriptor(l);
        asm volatile("" ::: "memory");
        load_rows(Lc, IK{}, IR{});          // behind the token's own loads; the first rows were requested a layer ago

        const int h = Lc->h, npb = Lc->npb;
        const int j0 = blk * npb, jn = min(npb, h - j0);
        const float bias_out = cptr(Lc->bp)[min(r0 + wave, D - 1)];

        // ---- normalise (x_l = y_{l-1} / sqrt(mean(y_{l-1}^2) + eps)), round to bf16, int8 code: one pass over the
        //      block for the sum of squares and the largest magnitude (scaling and rounding keep the order of
        //      magnitudes, so the largest rounded value is the rounded largest)
        {
            const float ss = wave_sum_f(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
            const float mm = wave_max_f(fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            if (lane == 0) {
                red_s[wave] = ss;
                red_m[wave] = mm;
            }
            if (tid < kStackNpbMax / 32) words[tid] = 0u;
            if (tid == 0) nflag = 0;
        }
        __syncthreads();
        TD_MARK(6);
        {
            float tot = 0.0f, big = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                tot += red_s[w];
                big = fmaxf(big, red_m[w]);
            }
            const float scale = l == 0 ? 1.0f : 1.0f / sqrtf(tot / (float)D + A.eps);
            const int ex = token_exponent(td_bf16_to_f32(td_f32_to_bf16(big * scale)));
            if (live) {
                const bf16_t b0 = td_f32_to_bf16(v.x * scale), b1 = td_f32_to_bf16(v.y * scale);
                const bf16_t b2 = td_f32_to_bf16(v.z * scale), b3 = td_f32_to_bf16(v.w * scale);
                const u32x2 o = u32x2{(uint32_t)b0 | ((uint32_t)b1 << 16), (uint32_t)b2 | ((uint32_t)b3 << 16)};
                reinterpret_cast<u32x2*>(xs)[tid_v] = o;
                if (l > 0 && blk == 0) gptr(reinterpret_cast<u32x2*>(hand_prev))[tid_v] = o;     // the hand-over, for the caller
                const uint32_t code = (uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(b0), ex) |
                                      ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(b1), ex) << 8) |
                                      ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(b2), ex) << 16) |
                                      ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(b3), ex) << 24);
                reinterpret_cast<uint32_t*>(xq)[tid_v] = code;
            }
            __syncthreads();
            TD_MARK(2);

            // ---- predictor rows: exact int32 dot products, range test, block-local flagged list
            const td_u32x4* xq4 = reinterpret_cast<const td_u32x4*>(xq) + lane_v;
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
                const int total = wave_sum_i(acc[i]);
                const float z8 = ldexpf((float)total, ex);
                const bool inside = (z8 >= tl[i]) && (z8 < th[i]);
                const int jl = wave_s * RQ + i;
                if (!inside && jl < jn && lane == 0) {
                    atomicOr(&words[jl >> 5], 1u << (jl & 31));
                    flist[atomicAdd(&nflag, 1)] = j0 + jl;
                }
            }
        }
        // ---- this wavefront's row of W': first half now, second half behind the repair's loads
        td_u32x4 wp[IW];
        const TD_GLOBAL td_u32x4* wp_row = gptr(reinterpret_cast<const td_u32x4*>(Lc->Wp + (size_t)min(r0 + wave, D - 1) * D)) + lane_v;
#pragma unroll
        for (int it = 0; it < IWA; ++it) wp[it] = __builtin_nontemporal_load(wp_row + it * TD_WAVE);

        __syncthreads();
        if (jn > 0 && tid < (jn + 31) / 32) gptr(Lc->mask)[(j0 >> 5) + tid] = words[tid];
        const int nf = __builtin_amdgcn_readfirstlane(nflag);
        TD_MARK(3);
#ifdef TD_STACK_TRACE
        if (tid == 0) A.trace[((size_t)l * G + blk) * 8 + 7] = (unsigned long long)nf;
#endif

        // ---- result fixing: one wavefront per flagged neuron computes z and delta from W1[j] (registers); the
        //      rows W2^T[j] go straight from memory into LDS (no registers in between), so one round trip serves
        //      up to 16 flagged neurons - a block with many of them would otherwise hold up the whole grid.
        //      Every thread then adds delta * W2^T[j][its columns] for the block's neurons: repair vector in registers.
        float yacc[CPT];
#pragma unroll
        for (int u = 0; u < CPT; ++u) yacc[u] = 0.0f;
        auto xsv = [&](int it) -> td_u32x4 { return reinterpret_cast<const td_u32x4*>(xs)[it * TD_WAVE + lane_v]; };
        auto repair_pass = [&](auto first_tag, const int f0) {
            constexpr bool kFirst = decltype(first_tag)::value;
            constexpr int CH = D * 2 / (TD_WAVE * 16);       // 1 KiB pieces of a row of W2^T
            asm volatile("" ::: "memory");
            const int cnt = min(NW, nf - f0);
            const bool fixer = wave < cnt;
            td_u32x4 w1[IW];
            float aj = 0.0f, cj = 0.0f;
            uint32_t bj_raw = 0;
            if (fixer) {
                const int jz = __builtin_amdgcn_readfirstlane(flist[f0 + wave]);
                load_row16<IW>(w1, Lc->W1 + (size_t)jz * D, lane_v);
                aj = gptr(Lc->a)[jz];
                cj = gptr(Lc->c)[jz];
                bj_raw = gptr(Lc->b1)[jz];
            }
            for (int piece = wave; piece < cnt * CH; piece += NW) {
                const int i = piece / CH, k = piece - i * CH;
                const int j = __builtin_amdgcn_readfirstlane(flist[f0 + i]);
                const TD_GLOBAL td_u32x4* src = gptr(reinterpret_cast<const td_u32x4*>(Lc->W2T + (size_t)j * D)) + k * TD_WAVE + lane_v;
                __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void*)(w2s + (size_t)i * D + k * (TD_WAVE * 8)), 16, 0, 0);
            }
            if (kFirst) {
                asm volatile("" ::: "memory");
#pragma unroll
                for (int it = IWA; it < IW; ++it) wp[it] = __builtin_nontemporal_load(wp_row + it * TD_WAVE);
            }
            asm volatile("" : "+v"(bj_raw), "+v"(aj), "+v"(cj));
            if (fixer) {
                float z = 0.0f;
#pragma unroll
                for (int it = 0; it < IW; ++it) z = RowVec<bf16_t>::dot(w1[it], xsv(it), z);
                z = wave_sum_f(z) + td_bf16_to_f32((bf16_t)bj_raw);
                if (lane == 0) dl[wave] = td_act(z, Lc->act) - fmaf(aj, z, cj);
            }
            wait_memory_acks();          // this wavefront's pieces are in LDS
            __syncthreads();
            for (int i = 0; i < cnt; ++i) {
                const float delta = dl[i];
                const bf16_t* row = w2s + (size_t)i * D + ctid_v;
#pragma unroll
                for (int u = 0; u < CPT; ++u) yacc[u] = fmaf(delta, td_bf16_to_f32(row[u * BLOCK]), yacc[u]);
            }
            if (f0 + NW < nf) __syncthreads();     // (another pass would overwrite the rows)
        };
        if (nf == 0) {
#pragma unroll
            for (int it = IWA; it < IW; ++it) wp[it] = __builtin_nontemporal_load(wp_row + it * TD_WAVE);
        } else {
            repair_pass(std::true_type{}, 0);
            for (int f0 = NW; f0 < nf; f0 += NW) repair_pass(std::false_type{}, f0);
        }
        TD_GLOBAL float* const acc_mine = gptr(Lc->yfix) + (size_t)(blk % kStackCopies) * D;     // this block's accumulator copy
        if (nf > 0) {
            TD_GLOBAL float* dst = acc_mine + ctid_v;
#pragma unroll
            for (int u = 0; u < CPT; ++u)
                __hip_atomic_fetch_add(dst + u * BLOCK, yacc[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- speculative row: into the accumulators as well (one more addend for its column)
        if (wave < rn) {
            float sp = 0.0f;
#pragma unroll
            for (int it = 0; it < IW; ++it) sp = RowVec<bf16_t>::dot(wp[it], xsv(it), sp);
            sp = wave_sum_f(sp);
            if (lane == 0)
                __hip_atomic_fetch_add(acc_mine + r0 + wave, sp + bias_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- count this block done for the layer (every wavefront's atomics acknowledged first)
        TD_MARK(4);
        wait_memory_acks();
        __syncthreads();
        TD_MARK(5);
        if (tid == 0) __hip_atomic_fetch_add(gptr(Lc->sync), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool final_layer = l == A.n_layers - 1;
        if (final_layer && blk != 0) return;
        acc_prev = Lc->yfix;
        cnt_prev = Lc->sync;
        hand_prev = Lc->xnext;
        asm volatile("" ::: "memory");
        // the first predictor rows of the next layer travel while this layer drains (the poll of the wait above
        // comes back behind them: vector loads return in order - but they were requested a whole tail earlier)
        // (unconditional - a request that may or may not happen would keep the old rows alive through the whole
        //  layer; the one block that goes on after the final layer asks for that layer's rows once more)
        load_rows(descriptor(min(l + 1, A.n_layers - 1)), I0{}, IK{});
    }
}

// Behind the launch: every layer's accumulators and counter back to zero; if a wait ran out, NaNs for y.
__global__ void __launch_bounds__(256) stack_rearm_kernel(StackArgs A, int D) {
    const td_stack_layer_dev* L = A.layer[blockIdx.x];
    for (int i = threadIdx.x; i < kStackCopies * D; i += 256) L->yfix[i] = 0.0f;
    if (threadIdx.x == 0) L->sync[0] = 0;
    if (blockIdx.x == 0 && *A.err != 0) {
        for (int i = threadIdx.x; i < D; i += 256) A.y[i] = (bf16_t)0x7FC0;
        __syncthreads();
        if (threadIdx.x == 0) *A.err = 0;
    }
}

constexpr size_t stack_lds_bytes(int D) { return (size_t)16 * D * 2; }   // the repair's staging: 16 rows of W2^T

template <int D>
tardis_status_t launch_stack(const StackArgs& A, int G, hipStream_t s) {
    StackArgs args = A;
    void* params[] = {&args};
    TD_HIP(hipLaunchCooperativeKernel(reinterpret_cast<const void*>(stack_decode_kernel<D>), dim3(G), dim3(1024), params, (unsigned)stack_lds_bytes(D), s));
    hipLaunchKernelGGL(stack_rearm_kernel, dim3(A.n_layers), dim3(256), 0, s, A, D);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

// whether a grid of G blocks is resident as a whole on the current device (asked once per row length)
template <int D>
bool grid_fits(int G) {
    static int capacity = -1;   // blocks the device holds at once (benign race: every caller computes the same value)
    if (capacity < 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stack_decode_kernel<D>, 1024, stack_lds_bytes(D)) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        capacity = cus * per_cu;
    }
    return G <= capacity;
}

}  // namespace

// The staging rows exceed the default limit of dynamic LDS: enabled once, when the first layer is folded
// (not at launch: a launch may come while some stream is being captured).
tardis_status_t td_stack_init() {
    static td_once once;
    return once.run([]() -> tardis_status_t {
        TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(stack_decode_kernel<1024>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stack_lds_bytes(1024)));
        TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(stack_decode_kernel<2048>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stack_lds_bytes(2048)));
        TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(stack_decode_kernel<4096>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)stack_lds_bytes(4096)));
        return TARDIS_OK;
    });
}

// whether `L` can be a member of a single-launch stack (one token)
bool td_stack_decode_supported(const tardis_layer_s* L) {
    if (!L->use_fused || !L->stack_desc || L->dtype != TARDIS_BF16 || !L->Q || L->fx || L->dec_threads != 1024 || L->dec_copies < kStackCopies) return false;
    if (!(L->d == 1024 || L->d == 2048 || L->d == 4096)) return false;
    const int64_t npb = ((L->h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
    if (npb > kStackNpbMax || (L->d + L->dec_blocks - 1) / L->dec_blocks > 16) return false;
    const int G = (int)L->dec_blocks;
    return L->d == 1024 ? grid_fits<1024>(G) : L->d == 2048 ? grid_fits<2048>(G) : grid_fits<4096>(G);
}

// x (d values) through layers[0..n): the handed-over activations land in every layer's xnext, the masks in
// every layer's own mask words, y receives the last layer's output.  Working memory: every layer's own
// accumulators and counter (left zero again by the kernel behind the launch); the error word is layers[0]'s.
tardis_status_t td_stack_decode(tardis_layer_s* const* layers, int n_layers, const void* x, void* y, hipStream_t s) {
    if (n_layers < 1 || n_layers > kMaxStackLayers) return TARDIS_ERR_SHAPE;
    tardis_layer_s* L0 = layers[0];
    StackArgs A{};
    for (int i = 0; i < n_layers; ++i) A.layer[i] = layers[i]->stack_desc;
    A.n_layers = n_layers;
    A.x = static_cast<const bf16_t*>(x);
    A.y = static_cast<bf16_t*>(y);
    A.err = L0->sync + kErrAt;
    A.eps = kRmsEps;
    A.spin_limit = L0->stack_spin_limit;
#ifdef TD_STACK_TRACE
    static unsigned long long* trace_dev = nullptr;
    const size_t trace_n = (size_t)kMaxStackLayers * 1024 * 8;
    if (!trace_dev) TD_HIP(hipMalloc(&trace_dev, trace_n * 8));
    A.trace = trace_dev;
    if (L0->d == 4096) {
        TD_TRY(launch_stack<4096>(A, L0->dec_blocks, s));
        if (const char* path = getenv("TARDIS_STACK_TRACE_FILE")) {
            TD_HIP(hipStreamSynchronize(s));
            std::vector<unsigned long long> host(trace_n);
            TD_HIP(hipMemcpy(host.data(), trace_dev, trace_n * 8, hipMemcpyDeviceToHost));
            if (FILE* f = fopen(path, "wb")) {
                const int hdr[4] = {n_layers, (int)L0->dec_blocks, 8, 0};
                fwrite(hdr, sizeof(hdr), 1, f);
                fwrite(host.data(), 8, (size_t)n_layers * L0->dec_blocks * 8, f);
                fclose(f);
            }
        }
        return TARDIS_OK;
    }
#endif
    switch (L0->d) {
        case 1024: return launch_stack<1024>(A, L0->dec_blocks, s);
        case 2048: return launch_stack<2048>(A, L0->dec_blocks, s);
        case 4096: return launch_stack<4096>(A, L0->dec_blocks, s);
    }
    return TARDIS_ERR_SHAPE;
}
