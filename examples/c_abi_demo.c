/* Plain C against the C ABI of libtardis (no Python, no C++): builds a small fp32 layer from a
 * counter-based generator, folds it twice with hand-made ranges and checks two identities that
 * need no reference implementation (Sec. "Overview" of the paper: the folded result plus the
 * repair of the flagged neurons):
 *   1. empty ranges (lo = hi): every neuron is flagged and repaired exactly, so the folded path
 *      must reproduce the unmodified FFN whatever lines (a, c) were folded in;
 *   2. identity activation with a = 1, c = 0 and unbounded ranges: nothing is flagged and the
 *      folded product alone is the unmodified FFN.
 * Exit status 0 and a last line "c_abi_demo: OK" on success.
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude examples/c_abi_demo.c \
 *       -o examples/c_abi_demo paper_2501_10054_amd/libtardis.so -L/opt/rocm/lib -lamdhip64 -lm
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "tardis.h"

#define D 64
#define H 256
#define NTOK 5

#define HIP_OK(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__);           \
            return 2;                                                                  \
        }                                                                              \
    } while (0)
#define TD_OK(call)                                                                    \
    do {                                                                               \
        tardis_status_t s_ = (call);                                                   \
        if (s_ != TARDIS_OK) {                                                         \
            fprintf(stderr, "%s at line %d\n", tardis_status_string(s_), __LINE__);    \
            return 3;                                                                  \
        }                                                                              \
    } while (0)

/* splitmix64 -> uniform in (-1, 1) */
static uint64_t g_state = 20250110u;
static float next_uniform(void) {
    uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (float)((double)(z >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static void* to_device(const void* host, size_t bytes) {
    void* p = NULL;
    if (hipMalloc(&p, bytes) != hipSuccess) return NULL;
    if (hipMemcpy(p, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return p;
}

static double rel_l2(const float* a, const float* b, int n) {
    double num = 0.0, den = 0.0;
    for (int i = 0; i < n; ++i) {
        num += ((double)a[i] - b[i]) * ((double)a[i] - b[i]);
        den += (double)b[i] * b[i];
    }
    return sqrt(num / (den > 0.0 ? den : 1.0));
}

int main(void) {
    static float W1[H * D], W2[D * H], b1[H], b2[D], X[NTOK * D];
    static float lo[H], hi[H], a[H], c[H], y[NTOK * D], yd[NTOK * D];
    for (int i = 0; i < H * D; ++i) W1[i] = 0.3f * next_uniform();
    for (int i = 0; i < D * H; ++i) W2[i] = 0.1f * next_uniform();
    for (int i = 0; i < H; ++i) b1[i] = 0.1f * next_uniform();
    for (int i = 0; i < D; ++i) b2[i] = 0.1f * next_uniform();
    for (int i = 0; i < NTOK * D; ++i) X[i] = 2.0f * next_uniform();

    void *dW1 = to_device(W1, sizeof W1), *dW2 = to_device(W2, sizeof W2), *db1 = to_device(b1, sizeof b1),
         *db2 = to_device(b2, sizeof b2), *dX = to_device(X, sizeof X);
    float *dlo, *dhi, *da, *dc;
    void *dy, *dyd;
    int32_t* dcounts;
    uint32_t* dmask;
    HIP_OK(hipMalloc((void**)&dlo, sizeof lo));
    HIP_OK(hipMalloc((void**)&dhi, sizeof hi));
    HIP_OK(hipMalloc((void**)&da, sizeof a));
    HIP_OK(hipMalloc((void**)&dc, sizeof c));
    HIP_OK(hipMalloc(&dy, sizeof y));
    HIP_OK(hipMalloc(&dyd, sizeof yd));
    HIP_OK(hipMalloc((void**)&dcounts, NTOK * sizeof(int32_t)));
    HIP_OK(hipMalloc((void**)&dmask, NTOK * (H / 32) * sizeof(uint32_t)));
    if (!dW1 || !dW2 || !db1 || !db2 || !dX) return 2;

    tardis_fold_opts opts = {8, TARDIS_F32, NTOK, 0, 0};
    int failures = 0;
    for (int variant = 0; variant < 2; ++variant) {
        tardis_ffn_desc desc = {D, H, TARDIS_F32, variant == 0 ? TARDIS_ACT_GELU_ERF : TARDIS_ACT_IDENTITY,
                                dW1, db1, dW2, db2};
        for (int j = 0; j < H; ++j) {
            if (variant == 0) {            /* empty ranges, arbitrary lines */
                lo[j] = hi[j] = 0.0f;
                a[j] = next_uniform();
                c[j] = next_uniform();
            } else {                       /* everything in range, the exact line of the identity */
                lo[j] = -1e30f;
                hi[j] = 1e30f;
                a[j] = 1.0f;
                c[j] = 0.0f;
            }
        }
        HIP_OK(hipMemcpy(dlo, lo, sizeof lo, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(dhi, hi, sizeof hi, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(da, a, sizeof a, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(dc, c, sizeof c, hipMemcpyHostToDevice));
        tardis_handle_t L = NULL;
        TD_OK(tardis_fold(&desc, dlo, dhi, da, dc, &opts, NULL, &L));
        TD_OK(tardis_ffn_forward_batched(L, dX, NTOK, dy, NULL));
        TD_OK(tardis_get_last_outliers(L, NTOK, dmask, dcounts, NULL, NULL));
        TD_OK(tardis_dense_forward(L, dX, NTOK, dyd, NULL));
        HIP_OK(hipDeviceSynchronize());
        int32_t counts[NTOK];
        HIP_OK(hipMemcpy(y, dy, sizeof y, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(yd, dyd, sizeof yd, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(counts, dcounts, sizeof counts, hipMemcpyDeviceToHost));
        const double err = rel_l2(y, yd, NTOK * D);
        const int want = variant == 0 ? H : 0;
        int counts_ok = 1;
        for (int t = 0; t < NTOK; ++t) counts_ok &= counts[t] == want;
        printf("variant %d: flagged per token %d (expected %d), folded path against the unmodified FFN: rel-L2 %.2e\n",
               variant, (int)counts[0], want, err);
        if (!counts_ok || !(err < 1e-4)) ++failures;
        TD_OK(tardis_destroy(L));
    }
    if (failures) {
        printf("c_abi_demo: FAILED (%d)\n", failures);
        return 1;
    }
    printf("c_abi_demo: OK\n");
    return 0;
}
