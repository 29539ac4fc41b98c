// C[m][n] = sum_k A[m][k] * B[n][k]  -- both operands K-contiguous ("NT"), C fp32.
//
// Used offline: the fold  W' = W2 . (diag(a) W1)  (Sec. "Constant Folded Matrix
// Generation") with A = W2 (d x h) and B = (diag(a) W1)^T (d x h), and the
// calibration pre-activations Z^T = W1 . X_cal^T (Sec. "Non-linear Function
// Approximation", step 2) with A = W1 (h x d) and B = X_cal (n x d).
#include <cstdlib>

#include "common.h"

namespace {

// ------------------------------------------------------------------ any shape
// 64x64 output tile, 16-deep K slices through LDS, 4x4 outputs per thread.
// Works for any M, N, K and for fp32 or bf16 operands (fp32 arithmetic).
constexpr int GT = 64, GK = 16;

template <typename T>
__global__ void __launch_bounds__(256)
gemm_nt_generic_kernel(const T* __restrict__ A, const T* __restrict__ B, float* __restrict__ C, int64_t M,
                       int64_t N, int64_t K, int accumulate, const T* __restrict__ row_bias) {
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int64_t m0 = (int64_t)blockIdx.y * GT, n0 = (int64_t)blockIdx.x * GT;
    const int tx = tid % 16, ty = tid / 16;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    // each thread stages 4 consecutive k of one row of A and of B per slice
    const int lr = tid / 4, lk = (tid % 4) * 4;
    for (int64_t k0 = 0; k0 < K; k0 += GK) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t k = k0 + lk + u;
            const int64_t am = m0 + lr, bn = n0 + lr;
            As[lk + u][lr] = (am < M && k < K) ? td_load<T>(A + am * K + k) : 0.0f;
            Bs[lk + u][lr] = (bn < N && k < K) ? td_load<T>(B + bn * K + k) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
        const float rb = row_bias ? td_load<T>(row_bias + m) : 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j] + rb;
            if (accumulate) v += C[m * N + n];
            C[m * N + n] = v;
        }
    }
}


// ------------------------------------------------------------------ bf16 MFMA
// 256x256 output tile per block of 4 wavefronts (2x2, 128x128 each = 4x4 MFMA
// 32x32x16 tiles, 256 fp32 accumulators per lane), K in slices of 64 staged
// through double-buffered LDS (rows padded to 144 bytes), next slice prefetched
// global -> registers while the current one feeds the matrix cores.  Blocks are
// numbered so that each XCD (blocks b, b+8, b+16, ...) works on a contiguous band
// of tile rows and re-uses its slice of A from its own L2.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int MT = 256, MK = 64;
constexpr int MSTRIDE = MK * 2 + 16;                 // bytes per staged row
constexpr int MSTAGE = 2 * MT * MSTRIDE;             // A tile + B tile
constexpr int MLDS = 2 * MSTAGE;

__device__ __forceinline__ td_u32x4 load_chunk(const bf16_t* base, int64_t row, int64_t rows, int64_t k,
                                               int64_t K) {
    if (row < rows && k + 8 <= K) return *reinterpret_cast<const td_u32x4*>(base + row * K + k);
    td_u32x4 z = {0, 0, 0, 0};
    if (row < rows && k < K) {                       // ragged K tail: element by element
        bf16_t* e = reinterpret_cast<bf16_t*>(&z);
        for (int u = 0; u < 8 && k + u < K; ++u) e[u] = base[row * K + k + u];
    }
    return z;
}

__global__ void __launch_bounds__(256)
gemm_nt_mfma_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, float* __restrict__ C,
                         int64_t M, int64_t N, int64_t K, int accumulate, const bf16_t* __restrict__ row_bias,
                         int tiles_m, int tiles_n) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order
    const int T = tiles_m * tiles_n;
    const int per_xcd = (T + 7) / 8;
    const int tile = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (tile >= T) return;
    const int64_t m0 = (int64_t)(tile / tiles_n) * MT, n0 = (int64_t)(tile % tiles_n) * MT;

    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // staging map: chunk c = tid + 256*i, i = 0..7 -> row c/8, 16-byte piece c%8
    td_u32x4 ra[8], rb[8];
    const int srow = tid >> 3, spiece = tid & 7;
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            ra[i] = load_chunk(A, m0 + srow + 32 * i, M, k0 + spiece * 8, K);
            rb[i] = load_chunk(B, n0 + srow + 32 * i, N, k0 + spiece * 8, K);
        }
    };
    auto stash = [&](int stage) {
        unsigned char* as = lds + stage * MSTAGE;
        unsigned char* bs = as + MT * MSTRIDE;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<td_u32x4*>(as + (srow + 32 * i) * MSTRIDE + spiece * 16) = ra[i];
            *reinterpret_cast<td_u32x4*>(bs + (srow + 32 * i) * MSTRIDE + spiece * 16) = rb[i];
        }
    };

    const int nk = (int)((K + MK - 1) / MK);
    fetch(0);
    stash(0);
    __syncthreads();
    const int frow = lane & 31, fk = (lane >> 5) * 16;  // fragment row and byte offset of its 8 k values
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) fetch((int64_t)(kt + 1) * MK);
        const unsigned char* as = lds + (kt & 1) * MSTAGE + (wm * 128 + frow) * MSTRIDE + fk;
        const unsigned char* bs = lds + (kt & 1) * MSTAGE + MT * MSTRIDE + (wn * 128 + frow) * MSTRIDE + fk;
        // fragments of slice ks+1 are read from LDS while the 16 MFMAs of slice ks run
        bf16x8_t fa[2][4], fb[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[0][i] = *reinterpret_cast<const bf16x8_t*>(as + i * 32 * MSTRIDE);
            fb[0][i] = *reinterpret_cast<const bf16x8_t*>(bs + i * 32 * MSTRIDE);
        }
#pragma unroll
        for (int ks = 0; ks < MK / 16; ++ks) {
            if (ks + 1 < MK / 16) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    fa[(ks + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(as + i * 32 * MSTRIDE + (ks + 1) * 32);
                    fb[(ks + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(bs + i * 32 * MSTRIDE + (ks + 1) * 32);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) stash((kt + 1) & 1);
        __syncthreads();
    }

    // D layout of the 32x32 tile: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m >= M) continue;
            const float rbias = row_bias ? td_bf16_to_f32(row_bias[m]) : 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
                if (n >= N) continue;
                float v = acc[i][j][r] + rbias;
                if (accumulate) v += C[m * N + n];
                C[m * N + n] = v;
            }
        }
    }
}

template <typename T>
void launch_generic(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K, int accumulate,
                    const void* row_bias, hipStream_t s) {
    dim3 grid((unsigned)((N + GT - 1) / GT), (unsigned)((M + GT - 1) / GT));
    hipLaunchKernelGGL(gemm_nt_generic_kernel<T>, grid, dim3(256), 0, s, static_cast<const T*>(A),
                       static_cast<const T*>(B), C, M, N, K, accumulate, static_cast<const T*>(row_bias));
}

bool gemm_force_generic() {
    const char* v = std::getenv("TARDIS_GEMM_GENERIC");
    return v && v[0] == '1';
}

}  // namespace

tardis_status_t td_gemm_nt(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K, int32_t dtype,
                           int accumulate, const void* row_bias, hipStream_t s) {
    if (M <= 0 || N <= 0 || K <= 0) return TARDIS_ERR_SHAPE;
    if ((M + GT - 1) / GT > 65535) return TARDIS_ERR_SHAPE;
    if (dtype == TARDIS_BF16 && M >= 128 && N >= 128 && K >= 64 &&
        (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0 && K % 8 == 0 &&
        !gemm_force_generic()) {
        const int tiles_m = (int)((M + MT - 1) / MT), tiles_n = (int)((N + MT - 1) / MT);
        const int T = tiles_m * tiles_n;
        const int grid = ((T + 7) / 8) * 8;
        static bool attr_set = false;
        if (!attr_set) {
            TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt_mfma_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, MLDS));
            attr_set = true;
        }
        hipLaunchKernelGGL(gemm_nt_mfma_bf16_kernel, dim3(grid), dim3(256), MLDS, s, static_cast<const bf16_t*>(A),
                           static_cast<const bf16_t*>(B), C, M, N, K, accumulate,
                           static_cast<const bf16_t*>(row_bias), tiles_m, tiles_n);
    } else if (dtype == TARDIS_BF16)
        launch_generic<bf16_t>(A, B, C, M, N, K, accumulate, row_bias, s);
    else
        launch_generic<float>(A, B, C, M, N, K, accumulate, row_bias, s);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
