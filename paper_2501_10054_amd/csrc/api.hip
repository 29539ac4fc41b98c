// C-ABI entry points of libtardis: argument validation, handle lifetime and
// dispatch.  No kernel lives here.
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>
#include <unordered_set>

#include "common.h"

namespace {

constexpr int64_t kMaxD = 32768;          // token + its int8 code must fit in LDS
constexpr int64_t kMaxH = 1 << 22;
constexpr int64_t kMaxCal = 32768;        // one neuron's samples are sorted in LDS
constexpr int64_t kMaxSearchCal = 8192;   // range search also keeps sigma of every sample there, in fp64
constexpr int64_t kMaxBatch = 4096;
constexpr size_t kTokenLdsCap = 60 * 1024;

// Live handles: a layer may name the layer that runs after it (a hint for cache warming); before
// that pointer is used it is looked up here, so that a hint to a destroyed layer is ignored.
std::mutex g_live_lock;
std::unordered_set<const tardis_layer_s*> g_live;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

tardis_status_t check_desc(const tardis_ffn_desc* desc) {
    if (!desc || !desc->W1 || !desc->W2) return TARDIS_ERR_INVALID_ARG;
    if (desc->dtype != TARDIS_F32 && desc->dtype != TARDIS_BF16) return TARDIS_ERR_DTYPE;
    if (desc->act < TARDIS_ACT_GELU_ERF || desc->act > TARDIS_ACT_IDENTITY) return TARDIS_ERR_INVALID_ARG;
    if (desc->d < 1 || desc->h < 1 || desc->d > kMaxD || desc->h > kMaxH) return TARDIS_ERR_SHAPE;
    if (!aligned16(desc->W1) || !aligned16(desc->W2)) return TARDIS_ERR_INVALID_ARG;
    const size_t es = td_elem_size(desc->dtype);
    if ((size_t)desc->d * (es + 1) + 16 > kTokenLdsCap) return TARDIS_ERR_SHAPE;
    return TARDIS_OK;
}

template <typename P> tardis_status_t dev_alloc(P** p, size_t bytes) {
    void* v = nullptr;
    hipError_t e = hipMalloc(&v, bytes ? bytes : 16);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        return e == hipErrorOutOfMemory ? TARDIS_ERR_OOM : TARDIS_ERR_HIP;
    }
    *p = static_cast<P*>(v);
    return TARDIS_OK;
}

// integer tuning knob from the environment (read when a layer is folded)
int env_int(const char* name, int fallback, int lo, int hi) {
    const char* v = std::getenv(name);
    if (!v || !*v) return fallback;
    const long x = std::strtol(v, nullptr, 10);
    return (x < lo || x > hi) ? fallback : (int)x;
}

void free_layer(tardis_layer_s* L) {
    if (!L) return;
    void* owned[] = {L->W2T, L->W2, L->Wp, L->Wp8, L->wp8_scale, L->bp, L->Q, L->Q4, L->M4, L->tlo, L->thi, L->a, L->c,
                     L->yacc, L->mask, L->counts, L->list, L->hidden, L->sync, L->yfix, L->fx_bound, L->stack_desc, L->zeros_h, L->xnext, L->rec_count, L->rec_jb, L->rec_tb, L->rec_delta, L->pf_scratch,
                     L->bt_xq, L->bt_e, L->bt_tokmask, L->bt_ulist, L->bt_ucount, L->bt_delta, L->bt_partial};
    for (void* p : owned)
        if (p) (void)hipFree(p);
    delete L;
}

tardis_status_t fold_impl(const tardis_ffn_desc* desc, const float* lo, const float* hi, const float* a,
                          const float* c, const tardis_fold_opts* opts, hipStream_t s, tardis_layer_s* L) {
    const int64_t d = desc->d, h = desc->h;
    const size_t es = td_elem_size(desc->dtype);
    L->d = d;
    L->h = h;
    L->dtype = desc->dtype;
    L->act = desc->act;
    L->max_batch = opts ? opts->max_batch : 1;
    L->sketch_bits = opts ? opts->sketch_bits : 8;
    L->margin = opts ? opts->margin : 0.0f;
    L->mask_words = (h + 31) / 32;
    L->W1 = desc->W1;
    L->b1 = desc->b1;
    L->b2 = desc->b2;
    L->last_n = 0;
    const size_t nb = (size_t)L->max_batch;
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->W2T), (size_t)h * d * es));
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->W2), (size_t)h * d * es));
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->Wp), (size_t)d * d * es));
    TD_TRY(dev_alloc(&L->bp, (size_t)d * 4));
    TD_TRY(dev_alloc(&L->tlo, (size_t)h * 4));
    TD_TRY(dev_alloc(&L->thi, (size_t)h * 4));
    TD_TRY(dev_alloc(&L->a, (size_t)h * 4));
    TD_TRY(dev_alloc(&L->c, (size_t)h * 4));
    // (16 rows of slack: a partially filled group of tokens writes its empty slots there)
    TD_TRY(dev_alloc(&L->yacc, (nb + kDecodeMaxTokens) * d * 4));
    TD_TRY(dev_alloc(&L->mask, (nb + kDecodeMaxTokens) * L->mask_words * 4));
    TD_TRY(dev_alloc(&L->counts, nb * 4));
    TD_TRY(dev_alloc(&L->list, nb * h * 4));
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->hidden), nb * h * es));
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->zeros_h), (size_t)h * es));
    TD_HIP(hipMemsetAsync(L->zeros_h, 0, (size_t)h * es, s));
    TD_TRY(dev_alloc(reinterpret_cast<char**>(&L->xnext), nb * d * es));
    TD_TRY(dev_alloc(&L->sync, 256));
    TD_HIP(hipMemsetAsync(L->sync, 0, 256, s));
    L->dec_threads = env_int("TARDIS_DECODE_THREADS", 1024, 512, 1024) == 512 ? 512 : 1024;
    L->dec_blocks = env_int("TARDIS_DECODE_BLOCKS", L->dec_threads == 512 ? 512 : 256, 1, 4096);
    L->dec_copies = env_int("TARDIS_DECODE_COPIES", 2, 1, 4);
    L->prefetch_bytes = env_int("TARDIS_PREFETCH_KB", 96, 0, 256) * 1024;
    L->strict_release = env_int("TARDIS_STRICT_RELEASE", 0, 0, 1);
    // what a finished block of the single-token kernel requests of the next layer, in sixteenths of prefetch_bytes:
    // the first block to finish / the last one (linear in between)
    L->prefetch_shape = env_int("TARDIS_PREFETCH_FIRST16", 32, 0, 255) | (env_int("TARDIS_PREFETCH_LAST16", 0, 0, 255) << 8);
    // (at least two copies' worth: the fixed-point accumulators are 8 bytes per token and column)
    const size_t yfix_bytes = (size_t)(L->dec_copies < 2 ? 2 : L->dec_copies) * kDecodeMaxTokens * d * 4;
    TD_TRY(dev_alloc(&L->yfix, yfix_bytes));
    TD_HIP(hipMemsetAsync(L->yfix, 0, yfix_bytes, s));
    L->use_fused = env_int("TARDIS_DECODE_FUSED", 1, 0, 1) && td_decode_fused_supported(L);
    L->defer_min_tokens = env_int("TARDIS_DEFER_MIN", 4, 4, 99);
    if (L->use_fused) {
        TD_TRY(td_decode_init());
        TD_TRY(td_static_scratch_setup());   // for tardis_ffn_forward_static on this device
        const int64_t npb = ((h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
        TD_TRY(dev_alloc(&L->rec_count, (size_t)L->dec_blocks * 4));
        TD_TRY(dev_alloc(&L->rec_jb, (size_t)L->dec_blocks * npb * 4));
        TD_TRY(dev_alloc(&L->rec_tb, (size_t)L->dec_blocks * npb * 4));
        TD_TRY(dev_alloc(&L->rec_delta, (size_t)L->dec_blocks * npb * kDecodeMaxTokens * 4));
    }
    // counted fixed-point repair accumulators: asked for by opts->deterministic, or by the knob
    L->deterministic = opts ? opts->deterministic : 0;
    L->fx = (L->deterministic || env_int("TARDIS_FIXED_POINT", 0, 0, 1)) && L->use_fused && L->dec_threads == 1024 &&
            (d + L->dec_blocks - 1) / L->dec_blocks <= 64 && L->dec_blocks <= 65535;
    if (L->deterministic && !L->fx) return TARDIS_ERR_SHAPE;   // only the fused decode kernels have the ordered path
    L->use_batched = env_int("TARDIS_BATCHED", 1, 0, 1) && td_batched_supported(L);
    L->batched_min_tokens = env_int("TARDIS_BATCHED_MIN", L->use_fused ? 17 : 1, 1, 64);
    // 4-bit sketch: the decode kernel reads the packed form (d = 2048, 4096); every other path
    // reads one-byte effective codes, kept only where such a path can run
    const bool packed4 = L->sketch_bits < 8 && L->use_fused && (d == 2048 || d == 4096);
    const bool byte_codes = !packed4 || (L->use_batched && L->max_batch > L->batched_min_tokens);
    if (byte_codes) TD_TRY(dev_alloc(&L->Q, (size_t)h * d));
    if (packed4) TD_TRY(dev_alloc(&L->Q4, (size_t)h * d / 2));
    if (L->sketch_bits < 8) TD_TRY(dev_alloc(&L->M4, (size_t)h * ((d + 31) / 32)));
    L->prefill_min_tokens = env_int("TARDIS_PREFILL_MIN", 65, 33, 1 << 20);
    if (L->max_batch >= L->prefill_min_tokens && td_prefill_supported(L)) {
        char* scratch = nullptr;
        L->prefill_chunk = env_int("TARDIS_PREFILL_CHUNK", 16384, 64, 32768);
        if (L->prefill_chunk > L->max_batch) L->prefill_chunk = (int32_t)L->max_batch;
        TD_TRY(dev_alloc(&scratch, td_prefill_scratch_bytes(L, L->prefill_chunk)));
        L->pf_scratch = scratch;
    }
    if (L->use_batched) {
        TD_TRY(td_batched_init());
        TD_TRY(dev_alloc(&L->bt_xq, (size_t)64 * d));
        TD_TRY(dev_alloc(&L->bt_e, 64 * 4));
        TD_TRY(dev_alloc(&L->bt_tokmask, (size_t)h * 8));
        TD_TRY(dev_alloc(&L->bt_ulist, (size_t)h * 4));
        TD_TRY(dev_alloc(&L->bt_ucount, 16));
        TD_TRY(dev_alloc(&L->bt_delta, (size_t)64 * h * 2));
        TD_TRY(dev_alloc(&L->bt_partial, td_batched_partial_floats(L) * 4));
        TD_HIP(hipMemsetAsync(L->bt_delta, 0, (size_t)64 * h * 2, s));
        TD_HIP(hipMemsetAsync(L->bt_ucount, 0, 16, s));
    }
    TD_HIP(hipMemsetAsync(L->counts, 0, nb * 4, s));
    TD_HIP(hipMemsetAsync(L->mask, 0, nb * L->mask_words * 4, s));
    TD_HIP(hipMemsetAsync(L->yacc, 0, nb * d * 4, s));
    TD_HIP(hipMemcpyAsync(L->a, a, (size_t)h * 4, hipMemcpyDeviceToDevice, s));
    TD_HIP(hipMemcpyAsync(L->c, c, (size_t)h * 4, hipMemcpyDeviceToDevice, s));
    TD_HIP(hipMemcpyAsync(L->W2, desc->W2, (size_t)h * d * es, hipMemcpyDeviceToDevice, s));
    TD_TRY(td_transpose(desc->W2, L->W2T, d, h, desc->dtype, s));
    TD_TRY(td_build_sketch(desc->W1, desc->b1, lo, hi, h, d, desc->dtype, L->sketch_bits, L->margin, L->Q, L->Q4, L->M4, L->tlo,
                           L->thi, s));
    if (opts && opts->folded_dtype == TARDIS_FP8_E4M3) {
        TD_TRY(dev_alloc(&L->Wp8, (size_t)d * d));
        TD_TRY(dev_alloc(&L->wp8_scale, (size_t)d * 4));
    }
    TD_TRY(td_fold(desc, L->a, L->c, L->Wp, L->bp, L->Wp8, L->wp8_scale, s));
    L->stack_fused = env_int("TARDIS_STACK_FUSED", 0, 0, 2);   // 2: refuse a one-token stack the single launch cannot serve
    L->stack_spin_limit = env_int("TARDIS_STACK_SPIN_LIMIT", 1 << 22, 1, 1 << 30);
    if (L->use_fused && L->dtype == TARDIS_BF16 && L->Q) {   // this layer's entry for the single-launch stack kernel
        const int64_t npb = ((h + L->dec_blocks - 1) / L->dec_blocks + 31) / 32 * 32;
        const td_stack_layer_dev hd{static_cast<const bf16_t*>(L->Wp), L->bp, L->Q, L->tlo, L->thi,
                                    static_cast<const bf16_t*>(L->W1),
                                    static_cast<const bf16_t*>(L->b1 ? L->b1 : L->zeros_h),
                                    static_cast<const bf16_t*>(L->W2T), L->a, L->c, L->mask,
                                    static_cast<bf16_t*>(L->xnext), L->yfix, L->sync, (int32_t)h, (int32_t)npb, L->act, 0};
        TD_TRY(td_stack_init());
        TD_TRY(dev_alloc(&L->stack_desc, sizeof(hd)));
        TD_HIP(hipMemcpyAsync(L->stack_desc, &hd, sizeof(hd), hipMemcpyHostToDevice, s));
        TD_HIP(hipStreamSynchronize(s));   // (hd lives on this stack frame)
    }
    if (L->fx) {
        TD_TRY(dev_alloc(&L->fx_bound, 8));
        TD_TRY(td_fx_bounds(L, L->fx_bound, s));
    }
    TD_HIP(hipStreamSynchronize(s));
    return TARDIS_OK;
}

}  // namespace

bool td_layer_is_live(const tardis_layer_s* L) {
    std::lock_guard<std::mutex> guard(g_live_lock);
    return g_live.count(L) != 0;
}

namespace {

// a handle this library made and has not destroyed, and whose working memory is in a known state
tardis_status_t check_handle(const tardis_layer_s* L) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    return L->poisoned ? TARDIS_ERR_STATE : TARDIS_OK;
}

// An online call that fails after its first launch may leave completion counters and accumulators
// armed; every later call on the handle would then assemble garbage without saying so.  Such a
// handle is marked and refuses further online calls (destroy and fold again).
tardis_status_t online_result(tardis_layer_s* L, tardis_status_t st) {
    if (st == TARDIS_ERR_HIP) L->poisoned = 1;
    return st;
}

}  // namespace

extern "C" {

tardis_status_t tardis_calibrate(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal, float coverage,
                                 const float* coverage_per_neuron, float* lo, float* hi, float* a, float* c,
                                 void* stream) {
    TD_TRY(check_desc(desc));
    if (!X_cal || !lo || !hi || !a || !c) return TARDIS_ERR_INVALID_ARG;
    if (!aligned16(X_cal)) return TARDIS_ERR_INVALID_ARG;
    if (n_cal < 1 || n_cal > kMaxCal) return TARDIS_ERR_SHAPE;
    if (!coverage_per_neuron && !(coverage > 0.0f && coverage <= 1.0f)) return TARDIS_ERR_INVALID_ARG;
    return td_calibrate(desc, X_cal, n_cal, coverage, coverage_per_neuron, 0.0f, lo, hi, a, c,
                        static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_calibrate_search(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal,
                                        float coverage, const float* coverage_per_neuron, float step, float* lo,
                                        float* hi, float* a, float* c, void* stream) {
    TD_TRY(check_desc(desc));
    if (!X_cal || !lo || !hi || !a || !c) return TARDIS_ERR_INVALID_ARG;
    if (!aligned16(X_cal)) return TARDIS_ERR_INVALID_ARG;
    if (n_cal < 1 || n_cal > kMaxSearchCal) return TARDIS_ERR_SHAPE;
    if (!coverage_per_neuron && !(coverage > 0.0f && coverage <= 1.0f)) return TARDIS_ERR_INVALID_ARG;
    if (!(step > 0.0f) || !(step < INFINITY)) return TARDIS_ERR_INVALID_ARG;
    return td_calibrate(desc, X_cal, n_cal, coverage, coverage_per_neuron, step, lo, hi, a, c,
                        static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_estimate_errors(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal, const float* lo,
                                       const float* hi, const float* a, const float* c, float* err_neurons,
                                       float* err_layer, void* stream) {
    TD_TRY(check_desc(desc));
    if (!X_cal || !lo || !hi || !a || !c || !err_neurons) return TARDIS_ERR_INVALID_ARG;
    if (!aligned16(X_cal)) return TARDIS_ERR_INVALID_ARG;
    if (n_cal < 1 || n_cal > kMaxCal) return TARDIS_ERR_SHAPE;
    return td_estimate_errors(desc, X_cal, n_cal, lo, hi, a, c, err_neurons, err_layer, static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_assign_thresholds(const float* err, int64_t n, float t, float t_min, float t_max, float* t_out,
                                         void* stream) {
    if (!err || !t_out) return TARDIS_ERR_INVALID_ARG;
    if (n < 1 || n > kMaxH) return TARDIS_ERR_SHAPE;
    if (!(t_min >= 0.0f) || !(t_max <= 1.0f) || !(t_min <= t) || !(t <= t_max)) return TARDIS_ERR_INVALID_ARG;
    return td_assign_thresholds(err, n, t, t_min, t_max, t_out, static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_fold(const tardis_ffn_desc* desc, const float* lo, const float* hi, const float* a,
                            const float* c, const tardis_fold_opts* opts, void* stream, tardis_handle_t* out) {
    if (!out) return TARDIS_ERR_INVALID_ARG;
    *out = nullptr;
    TD_TRY(check_desc(desc));
    if (!lo || !hi || !a || !c) return TARDIS_ERR_INVALID_ARG;
    if (opts) {
        if (opts->sketch_bits != 8 && opts->sketch_bits != 4 && opts->sketch_bits != 3 && opts->sketch_bits != 2)
            return TARDIS_ERR_INVALID_ARG;
        if (!(opts->margin >= 0.0f) || !(opts->margin < 0.5f)) return TARDIS_ERR_INVALID_ARG;
        if (opts->folded_dtype != desc->dtype &&
            !(opts->folded_dtype == TARDIS_FP8_E4M3 && desc->dtype == TARDIS_BF16))
            return TARDIS_ERR_DTYPE;
        if (opts->max_batch < 1 || opts->max_batch > kMaxBatch) return TARDIS_ERR_SHAPE;
        if (opts->deterministic != 0 && opts->deterministic != 1) return TARDIS_ERR_INVALID_ARG;
    }
    tardis_layer_s* L = new (std::nothrow) tardis_layer_s();
    if (!L) return TARDIS_ERR_OOM;
    tardis_status_t st = fold_impl(desc, lo, hi, a, c, opts, static_cast<hipStream_t>(stream), L);
    if (st != TARDIS_OK) {
        (void)hipDeviceSynchronize();
        free_layer(L);
        return st;
    }
    {
        std::lock_guard<std::mutex> guard(g_live_lock);
        g_live.insert(L);
    }
    *out = L;
    return TARDIS_OK;
}

tardis_status_t tardis_set_next_layer(tardis_handle_t L, tardis_handle_t next) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    if (next && !td_layer_is_live(next)) return TARDIS_ERR_STATE;
    L->next_layer = next;
    return TARDIS_OK;
}

tardis_status_t tardis_ffn_forward(tardis_handle_t L, const void* x, void* y, void* stream) {
    return tardis_ffn_forward_batched(L, x, 1, y, stream);
}

tardis_status_t tardis_ffn_forward_batched(tardis_handle_t L, const void* x, int64_t n, void* y, void* stream) {
    TD_TRY(check_handle(L));
    if (!x || !y || x == y) return TARDIS_ERR_INVALID_ARG;
    if (n < 1 || n > L->max_batch) return TARDIS_ERR_SHAPE;
    return online_result(L, td_forward(L, x, n, y, 0, static_cast<hipStream_t>(stream)));
}

tardis_status_t tardis_stack_forward(const tardis_handle_t* layers, int32_t n_layers, const void* x, int64_t n,
                                     void* y, void* stream) {
    if (!layers || n_layers < 1 || n_layers > 4096) return TARDIS_ERR_INVALID_ARG;
    if (!x || !y || x == y) return TARDIS_ERR_INVALID_ARG;
    for (int32_t l = 0; l < n_layers; ++l) {
        TD_TRY(check_handle(layers[l]));
        if (layers[l]->d != layers[0]->d || layers[l]->dtype != layers[0]->dtype) return TARDIS_ERR_SHAPE;
        if (n < 1 || n > layers[l]->max_batch) return TARDIS_ERR_SHAPE;
        for (int32_t m = 0; m < l; ++m)
            if (layers[m] == layers[l]) return TARDIS_ERR_INVALID_ARG;   // each handle owns its hand-over buffer
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // one token through layers the single-token kernel serves: the whole stack in ONE launch whose grid
    // stays resident (not while the stream is being captured: a captured graph keeps the per-layer launches)
    if (n == 1 && n_layers >= 2 && n_layers <= 64 && layers[0]->stack_fused) {
        bool ok = true;
        for (int32_t l = 0; l < n_layers && ok; ++l)
            ok = td_stack_decode_supported(layers[l]) && layers[l]->dec_blocks == layers[0]->dec_blocks &&
                 layers[l]->deterministic == 0;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (ok && hipStreamIsCapturing(s, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) {
            const tardis_status_t st = online_result(layers[0], td_stack_decode(layers, n_layers, x, y, s));
            if (st == TARDIS_OK)
                for (int32_t l = 0; l < n_layers; ++l) layers[l]->last_n = 1;
            return st;
        }
        if (layers[0]->stack_fused == 2) return TARDIS_ERR_SHAPE;
    }
    const void* cur = x;
    for (int32_t l = 0; l < n_layers; ++l) {
        const bool last = l == n_layers - 1;
        void* out = last ? y : layers[l]->xnext;
        const tardis_layer_s* keep = layers[l]->next_layer;
        if (!last) layers[l]->next_layer = layers[l + 1];        // the stack knows what runs next
        const tardis_status_t st = online_result(layers[l], td_forward(layers[l], cur, n, out, last ? 0 : 1, s));
        layers[l]->next_layer = keep;
        TD_TRY(st);
        cur = out;
    }
    return TARDIS_OK;
}

tardis_status_t tardis_dense_forward(tardis_handle_t L, const void* x, int64_t n, void* y, void* stream) {
    TD_TRY(check_handle(L));
    if (!x || !y || x == y) return TARDIS_ERR_INVALID_ARG;
    if (n < 1 || n > L->max_batch) return TARDIS_ERR_SHAPE;
    return td_dense_forward(L, x, n, y, static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_get_folded(tardis_handle_t L, void* Wp, float* bp, void* stream) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (Wp) TD_HIP(hipMemcpyAsync(Wp, L->Wp, (size_t)L->d * L->d * td_elem_size(L->dtype), hipMemcpyDeviceToDevice, s));
    if (bp) TD_HIP(hipMemcpyAsync(bp, L->bp, (size_t)L->d * 4, hipMemcpyDeviceToDevice, s));
    return TARDIS_OK;
}

tardis_status_t tardis_get_predictor_state(tardis_handle_t L, int8_t* Q, float* tlo, float* thi, void* stream) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (Q) {
        if (L->Q)
            TD_HIP(hipMemcpyAsync(Q, L->Q, (size_t)L->h * L->d, hipMemcpyDeviceToDevice, s));
        else
            TD_TRY(td_unpack_sketch4(L->Q4, L->M4, L->h, L->d, Q, s));
    }
    if (tlo) TD_HIP(hipMemcpyAsync(tlo, L->tlo, (size_t)L->h * 4, hipMemcpyDeviceToDevice, s));
    if (thi) TD_HIP(hipMemcpyAsync(thi, L->thi, (size_t)L->h * 4, hipMemcpyDeviceToDevice, s));
    return TARDIS_OK;
}

tardis_status_t tardis_get_sketch_groups(tardis_handle_t L, uint8_t* M, void* stream) {
    if (!L || !td_layer_is_live(L) || L->sketch_bits >= 8) return TARDIS_ERR_STATE;
    if (!M) return TARDIS_ERR_INVALID_ARG;
    TD_HIP(hipMemcpyAsync(M, L->M4, (size_t)L->h * ((L->d + 31) / 32), hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(stream)));
    return TARDIS_OK;
}

tardis_status_t tardis_get_last_outliers(tardis_handle_t L, int64_t n, uint32_t* mask, int32_t* counts,
                                         int32_t* list, void* stream) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    if (n < 1 || n != L->last_n) return TARDIS_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t nn = (size_t)n;
    if (mask) TD_HIP(hipMemcpyAsync(mask, L->mask, nn * L->mask_words * 4, hipMemcpyDeviceToDevice, s));
    if (counts || list) TD_TRY(td_mask_to_list(L, n, counts, list, s));   // derived from the mask words
    return TARDIS_OK;
}

tardis_status_t tardis_get_last_union(tardis_handle_t L, int64_t n, uint32_t* union_mask, int32_t* union_count,
                                      void* stream) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    if (n < 1 || n != L->last_n) return TARDIS_ERR_STATE;
    if (!union_mask && !union_count) return TARDIS_OK;
    return td_mask_union(L, n, union_mask, union_count, static_cast<hipStream_t>(stream));
}

tardis_status_t tardis_get_handover(tardis_handle_t L, int64_t n, void* out, void* stream) {
    if (!L || !td_layer_is_live(L)) return TARDIS_ERR_STATE;
    if (!out) return TARDIS_ERR_INVALID_ARG;
    if (n < 1 || n > L->max_batch) return TARDIS_ERR_SHAPE;
    TD_HIP(hipMemcpyAsync(out, L->xnext, (size_t)n * L->d * td_elem_size(L->dtype), hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(stream)));
    return TARDIS_OK;
}

tardis_status_t tardis_destroy(tardis_handle_t L) {
    if (!L) return TARDIS_OK;
    {
        std::lock_guard<std::mutex> guard(g_live_lock);
        if (g_live.erase(L) == 0) return TARDIS_ERR_STATE;   // not a handle of this library, or destroyed already
    }
    free_layer(L);
    return TARDIS_OK;
}

const char* tardis_status_string(tardis_status_t s) {
    switch (s) {
        case TARDIS_OK: return "ok";
        case TARDIS_ERR_INVALID_ARG: return "invalid argument";
        case TARDIS_ERR_SHAPE: return "unsupported shape or size";
        case TARDIS_ERR_DTYPE: return "unsupported dtype";
        case TARDIS_ERR_STATE: return "handle not usable for this call";
        case TARDIS_ERR_OOM: return "device out of memory";
        case TARDIS_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int32_t tardis_version(void) { return TARDIS_VERSION; }

}  // extern "C"
