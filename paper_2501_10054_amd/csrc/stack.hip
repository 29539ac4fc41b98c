// One token through a whole stack of folded layers in ONE launch (the FFN stack of chained layers
// with RMS-norm glue; per layer the online step of Sec. "Inference Runtime": speculative product,
// predictor, mask, result fixing).
//
// A launch per layer pays, per layer, the launch itself (about 2.5 us back to back) and the tail of
// the single-token kernel - atomics acknowledged, completion counter, the last block's assembly -
// during which the memory system idles.  Here the grid stays resident (a cooperative launch: all
// blocks are guaranteed to run at once, so waiting for one another cannot deadlock): a block that
// has signalled completion of layer l requests the first predictor rows of layer l+1 into its
// REGISTERS and only then waits for the layer's result; the block that finishes layer l last
// assembles and normalises it, publishes it and releases the others.  The stream of layer l+1 is
// under way while layer l drains.
//
// Work split per layer as in the single-token kernel: block b owns neurons [b*npb, (b+1)*npb)
// (predictor rows, repair of the flagged ones) and rows [b*rpb, (b+1)*rpb) of W'; repair vectors go
// to two accumulator copies with coalesced fp32 atomics.
#include <type_traits>

#include "common.h"
#include "rowdot.h"

namespace {

constexpr int kMaxStackLayers = 64;          // layers per launch (a longer stack runs layer by layer)
constexpr int kStackNpbMax = 64;             // neurons per block: one pass of 16 wavefronts x 4 rows
constexpr int kFlagAt = 32;                  // counter index of the "layers finished" word (its own 128-byte line)
constexpr int kErrAt = 48;                   // set if a bounded wait ran out

struct StackArgs {
    const td_stack_layer_dev* layer[kMaxStackLayers];
    int n_layers;
    const bf16_t* x;      // d values
    bf16_t* y;            // d values: the last layer's (un-normalised) output
    float* yfold;         // d floats
    float* yfix;          // copies x d floats, zero between launches
    int32_t* sync;        // 64 counters, zero between launches
    int copies;
    float eps;
    int spin_limit;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void wait_memory_acks() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Pointers that reach the kernel through a layer's descriptor (loaded from memory, not kernel
// arguments) are generic to the compiler: it would use flat loads, which also wait on the LDS
// counter.  They all point to device memory; say so.
#define TD_GLOBAL __attribute__((address_space(1)))
template <typename T> __device__ __forceinline__ const TD_GLOBAL T* gptr(const T* p) { return (const TD_GLOBAL T*)p; }
template <typename T> __device__ __forceinline__ TD_GLOBAL T* gptr(T* p) { return (TD_GLOBAL T*)p; }

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
    constexpr int IWA = IW / 2;
    constexpr int CPT = D / BLOCK;                   // output columns per thread
    constexpr int FCH = (16 / CPT) < NW ? (16 / CPT) : NW;   // flagged neurons per repair pass (register budget)
    constexpr int KPRE = RQ / 2;                     // predictor rows of the next layer requested before the layer barrier
    static_assert(D % 1024 == 0 && D <= 4096, "one 16-byte vector of the token and four of the result per thread");
    static_assert(kStackNpbMax == NW * RQ, "one predictor pass per layer");

    __shared__ __align__(16) bf16_t xs[D];
    __shared__ __align__(16) int8_t xq[D];
    __shared__ float dl[NW];
    __shared__ float redt[NW];
    __shared__ int flist[kStackNpbMax];
    __shared__ uint32_t words[kStackNpbMax / 32];
    __shared__ int tmax, nflag, is_last, bail;

    const int tid = threadIdx.x, lane = tid & (TD_WAVE - 1), blk = blockIdx.x;
    // (wave-uniform values are made known as such: row addresses then are scalar bases plus one lane offset,
    //  instead of a 64-bit address pair per load held in vector registers across the layer loop)
    const int wave = __builtin_amdgcn_readfirstlane(tid / TD_WAVE);
    const int G = (int)gridDim.x;
    const int rpb = (D + G - 1) / G;
    const int r0 = blk * rpb, rn = min(rpb, D - r0);          // W' rows owned (at most one per wavefront)
    int32_t* done = A.sync;
    int32_t* flag = A.sync + kFlagAt;
    const int ctid = (tid + TD_WAVE * (blk >> 3)) & (BLOCK - 1);   // rotated column ownership (see decode kernel)
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    td_u32x4 q[RQ][IQ];
    float tl[RQ], th[RQ];
    auto load_rows_a = [&](auto L) {      // rows 0 .. KPRE-1 of this wavefront
#pragma unroll
        for (int i = 0; i < KPRE; ++i) {
            const int j = min(blk * L->npb + wave * RQ + i, L->h - 1);
            load_row16<IQ>(q[i], L->Q + (size_t)j * D, lane);
            tl[i] = gptr(L->tlo)[j];
            th[i] = gptr(L->thi)[j];
        }
    };
    auto load_rows_b = [&](auto L) {      // rows KPRE .. RQ-1
#pragma unroll
        for (int i = KPRE; i < RQ; ++i) {
            const int j = min(blk * L->npb + wave * RQ + i, L->h - 1);
            load_row16<IQ>(q[i], L->Q + (size_t)j * D, lane);
            tl[i] = gptr(L->tlo)[j];
            th[i] = gptr(L->thi)[j];
        }
    };

    // a layer's descriptor is constant once the layer is folded: it is read through the constant address
    // space, field by field where needed, so that the values arrive by scalar loads into scalar registers
    typedef const __attribute__((address_space(4))) td_stack_layer_dev* desc_t;
    auto descriptor = [&](int l) -> desc_t { return (desc_t)A.layer[l]; };
    desc_t Lc = descriptor(0);
    td_u32x4 xv = reinterpret_cast<const td_u32x4*>(A.x)[min(tid, NVW - 1)];
    asm volatile("" ::: "memory");
    load_rows_a(Lc);
    load_rows_b(Lc);

#pragma unroll 1
    for (int l = 0;; ++l) {
        // (per-lane offsets are re-derived in every layer from values the compiler cannot see through: hoisted out
        //  of the layer loop they would occupy vector registers for the whole launch and end up spilled)
        int lane_v = lane, ctid_v = ctid, wave_s = wave;
        asm volatile("" : "+v"(lane_v), "+v"(ctid_v), "+s"(wave_s));
        const int h = Lc->h, npb = Lc->npb;
        const int j0 = blk * npb, jn = min(npb, h - j0);
        const float bias_out = gptr(Lc->bp)[min(r0 + wave, D - 1)];

        // ---- stage the token: maximum, int8 code
        if (tid < kStackNpbMax / 32) words[tid] = 0u;
        if (tid == 0) {
            tmax = 0;
            nflag = 0;
        }
        __syncthreads();
        if (tid < NVW) {
            reinterpret_cast<td_u32x4*>(xs)[tid] = xv;
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv);
            float m = 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(td_bf16_to_f32(e8[u])));
            m = td_wave_max(m);
            if (lane == 0) atomicMax(&tmax, __float_as_int(m));
        }
        __syncthreads();
        const int ex = token_exponent(__int_as_float(tmax));
        if (tid < NVW) {
            const bf16_t* e8 = reinterpret_cast<const bf16_t*>(&xv);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u]), ex)) << (8 * u);
                hi |= ((uint32_t)(uint8_t)quantize_value(td_bf16_to_f32(e8[u + 4]), ex)) << (8 * u);
            }
            reinterpret_cast<uint2*>(xq)[tid] = make_uint2(lo, hi);
        }
        __syncthreads();

        // ---- predictor rows: exact int32 dot products, range test, block-local flagged list
        {
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
                const int total = td_wave_sum_i(acc[i]);
                const float v = ldexpf((float)total, ex);
                const bool inside = (v >= tl[i]) && (v < th[i]);
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

        // ---- result fixing (as in the single-token kernel: one wavefront per flagged neuron computes z
        //      and delta, every thread fetches its output columns of W2^T[j], repair vector in registers)
        float yacc[CPT];
#pragma unroll
        for (int u = 0; u < CPT; ++u) yacc[u] = 0.0f;
        auto xsv = [&](int it) -> td_u32x4 { return reinterpret_cast<const td_u32x4*>(xs)[it * TD_WAVE + lane_v]; };
        auto repair_pass = [&](auto first_tag, const int f0) {
            constexpr bool kFirst = decltype(first_tag)::value;
            asm volatile("" ::: "memory");
            const int fi = f0 + wave;
            const bool fixer = wave < FCH && fi < nf;
            td_u32x4 w1[IW];
            float aj = 0.0f, cj = 0.0f;
            uint32_t bj_raw = 0;
            if (fixer) {
                const int jz = __builtin_amdgcn_readfirstlane(flist[fi]);
                load_row16<IW>(w1, Lc->W1 + (size_t)jz * D, lane_v);
                aj = gptr(Lc->a)[jz];
                cj = gptr(Lc->c)[jz];
                bj_raw = gptr(Lc->b1)[jz];
            }
            uint16_t w2[FCH][CPT];
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                const int j = __builtin_amdgcn_readfirstlane(flist[min(f0 + i, nf - 1)]);
                const TD_GLOBAL bf16_t* row = gptr(Lc->W2T + (size_t)j * D) + ctid_v;
#pragma unroll
                for (int u = 0; u < CPT; ++u) w2[i][u] = __builtin_nontemporal_load(row + u * BLOCK);
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
                z = td_wave_sum(z) + td_bf16_to_f32((bf16_t)bj_raw);
                if (lane == 0) dl[wave] = td_act(z, Lc->act) - fmaf(aj, z, cj);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                if (f0 + i < nf) {
                    const float delta = dl[i];
#pragma unroll
                    for (int u = 0; u < CPT; ++u) yacc[u] = fmaf(delta, td_bf16_to_f32(w2[i][u]), yacc[u]);
                }
            }
            __syncthreads();
        };
        if (nf == 0) {
#pragma unroll
            for (int it = IWA; it < IW; ++it) wp[it] = __builtin_nontemporal_load(wp_row + it * TD_WAVE);
        } else {
            repair_pass(std::true_type{}, 0);
            for (int f0 = FCH; f0 < nf; f0 += FCH) repair_pass(std::false_type{}, f0);
        }
        if (nf > 0) {
            float* dst = A.yfix + (size_t)(blk % A.copies) * D + ctid_v;
#pragma unroll
            for (int u = 0; u < CPT; ++u)
                __hip_atomic_fetch_add(dst + u * BLOCK, yacc[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- speculative row
        if (wave < rn) {
            float sp = 0.0f;
#pragma unroll
            for (int it = 0; it < IW; ++it) sp = RowVec<bf16_t>::dot(wp[it], xsv(it), sp);
            sp = td_wave_sum(sp);
            if (lane == 0)
                __hip_atomic_store(A.yfold + r0 + wave, sp + bias_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // ---- signal completion of this layer (every wavefront's stores and atomics acknowledged first)
        wait_memory_acks();
        __syncthreads();
        if (tid == 0) is_last = (__hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == G - 1);
        __syncthreads();
        const bool final_layer = l == A.n_layers - 1;
        const bool last_block = __builtin_amdgcn_readfirstlane(is_last) != 0;   // (uniform, and known to be)
        if (final_layer && !last_block) return;

        bf16_t* const handover = Lc->xnext;           // where this layer's normalised output goes
        if (!final_layer) Lc = descriptor(l + 1);    // from here on Lc is the NEXT layer
        if (!last_block) {
            // the first predictor rows of the next layer travel while this layer drains (unconditionally in
            // every wavefront: a conditional request into loop-carried registers makes the compiler wait for
            // and spill each vector.  Vector loads return in order, so the polling wavefront's first poll comes
            // back behind its own rows - they were requested a whole tail earlier)
            load_rows_a(Lc);
        } else {
            // ---- the last block to finish assembles the layer's output and re-arms the accumulators
            // (read past this XCD's L2 and cleared through it: within one launch the L2 of the XCD that assembled an
            //  earlier layer may still hold these lines, and the other XCDs' atomics act on memory)
            const bool live = tid < D / 4;
            auto ld2 = [&](const float* p) -> f32x4 {
                const unsigned long long* q8 = reinterpret_cast<const unsigned long long*>(p);
                const unsigned long long lo = __hip_atomic_load(q8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned long long hi = __hip_atomic_load(q8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                f32x4 r;
                r.x = __uint_as_float((uint32_t)lo);
                r.y = __uint_as_float((uint32_t)(lo >> 32));
                r.z = __uint_as_float((uint32_t)hi);
                r.w = __uint_as_float((uint32_t)(hi >> 32));
                return r;
            };
            f32x4 v = live ? ld2(A.yfold + 4 * tid) : zero4;
            for (int cidx = 0; cidx < A.copies; ++cidx) {
                if (live) {
                    float* p = A.yfix + (size_t)cidx * D + 4 * tid;
                    v += ld2(p);
                    unsigned long long* q8 = reinterpret_cast<unsigned long long*>(p);
                    __hip_atomic_store(q8, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(q8 + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            float scale = 1.0f;
            if (!final_layer) {   // x_{l+1} = y_l / sqrt(mean(y_l^2) + eps)
                const float ss = td_wave_sum(v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w);
                if (lane == 0) redt[wave] = ss;
                __syncthreads();
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) tot += redt[w];
                scale = 1.0f / sqrtf(tot / (float)D + A.eps);
            }
            if (live) {
                const f32x4 o4 = v * scale;
                const unsigned long long o =
                    (unsigned long long)((uint32_t)td_f32_to_bf16(o4.x) | ((uint32_t)td_f32_to_bf16(o4.y) << 16)) |
                    ((unsigned long long)((uint32_t)td_f32_to_bf16(o4.z) | ((uint32_t)td_f32_to_bf16(o4.w) << 16)) << 32);
                unsigned long long* out = reinterpret_cast<unsigned long long*>(final_layer ? A.y : handover) + tid;
                // written through: every block of the grid, on any XCD, reads it next
                __hip_atomic_store(out, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (tid == 0) __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            wait_memory_acks();
            __syncthreads();
            if (tid == 0)
                __hip_atomic_store(flag, final_layer ? 0 : l + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (final_layer) return;
            load_rows_a(Lc);
        }

        // ---- layer barrier: wait (bounded) until layer l's output has been published
        if (tid == 0) {
            int spins = 0;
            while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < l + 1 && ++spins < A.spin_limit)
                __builtin_amdgcn_s_sleep(4);
            bail = spins >= A.spin_limit;
        }
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(bail) != 0) {
            // the wait ran out (the grid is resident as a whole, so this needs a fault elsewhere): leave, loudly -
            // this block's share of y becomes NaN and the error word is set; the other blocks run out the same way
            if (tid < rn) A.y[r0 + tid] = (bf16_t)0x7FC0;
            if (tid == 0) __hip_atomic_store(A.sync + kErrAt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        // No cache invalidation here, on purpose: every layer has a hand-over buffer of its own (whole cache lines),
        // nobody reads it in this launch before its publication, and the launch itself starts with clean caches -
        // so neither this CU nor this XCD can hold a stale line of it.  (An agent-scope acquire would drop the
        // XCD's whole L2, per wavefront and layer, and send every block's read of these 8 KiB to memory.)
        asm volatile("" ::: "memory");
        xv = gptr(reinterpret_cast<const td_u32x4*>(handover))[min(tid, NVW - 1)];
        asm volatile("" ::: "memory");
        load_rows_b(Lc);
    }
}

template <int D>
tardis_status_t launch_stack(const StackArgs& A, int G, hipStream_t s) {
    StackArgs args = A;
    void* params[] = {&args};
    TD_HIP(hipLaunchCooperativeKernel(reinterpret_cast<const void*>(stack_decode_kernel<D>), dim3(G), dim3(1024), params, 0, s));
    return TARDIS_OK;
}

// whether a grid of G blocks is resident as a whole on the current device (asked once per row length)
template <int D>
bool grid_fits(int G) {
    static int capacity = -1;   // blocks the device holds at once (benign race: every caller computes the same value)
    if (capacity < 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stack_decode_kernel<D>, 1024, 0) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
        capacity = cus * per_cu;
    }
    return G <= capacity;
}

}  // namespace

// whether `L` can be a member of a single-launch stack (one token)
bool td_stack_decode_supported(const tardis_layer_s* L) {
    if (!L->use_fused || !L->stack_desc || L->dtype != TARDIS_BF16 || !L->Q || L->fx || L->dec_threads != 1024) return false;
    if (!(L->d == 1024 || L->d == 2048 || L->d == 4096)) return false;
    const int64_t npb = ((L->h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
    if (npb > kStackNpbMax || (L->d + L->dec_blocks - 1) / L->dec_blocks > 16) return false;
    const int G = (int)L->dec_blocks;
    return L->d == 1024 ? grid_fits<1024>(G) : L->d == 2048 ? grid_fits<2048>(G) : grid_fits<4096>(G);
}

// x (d values) through layers[0..n): the handed-over activations land in every layer's xnext, the masks in
// every layer's own mask words, y receives the last layer's output.  Working memory: layers[0]'s.
tardis_status_t td_stack_decode(tardis_layer_s* const* layers, int n_layers, const void* x, void* y, hipStream_t s) {
    if (n_layers < 1 || n_layers > kMaxStackLayers) return TARDIS_ERR_SHAPE;
    tardis_layer_s* L0 = layers[0];
    StackArgs A{};
    for (int i = 0; i < n_layers; ++i) A.layer[i] = layers[i]->stack_desc;
    A.n_layers = n_layers;
    A.x = static_cast<const bf16_t*>(x);
    A.y = static_cast<bf16_t*>(y);
    A.yfold = L0->yacc;
    A.yfix = L0->yfix;
    A.sync = L0->sync;
    A.copies = L0->dec_copies;
    A.eps = kRmsEps;
    A.spin_limit = 1 << 22;
    switch (L0->d) {
        case 1024: return launch_stack<1024>(A, L0->dec_blocks, s);
        case 2048: return launch_stack<2048>(A, L0->dec_blocks, s);
        case 4096: return launch_stack<4096>(A, L0->dec_blocks, s);
    }
    return TARDIS_ERR_SHAPE;
}
