// C[m][n] = sum_k A[m][k] * B[n][k]  -- both operands K-contiguous ("NT"); C fp32 (bf16 or fp32
// operands) or exact int32 (int8 operands).
//
// Used offline: the fold  W' = W2 . (diag(a) W1)  (Sec. "Constant Folded Matrix
// Generation") with A = W2 (d x h) and B = (diag(a) W1)^T (d x h), and the
// calibration pre-activations Z^T = W1 . X_cal^T (Sec. "Non-linear Function
// Approximation", step 2) with A = W1 (h x d) and B = X_cal (n x d).  Used online for calls with
// many tokens (prompts), where every step of the method is a product of the token matrix with a
// weight matrix: predictor sums Xq . Q^T (int8), pre-activations X . W1^T, folded product X . W'^T
// and the down projection of the masked delta.
#include <cstdlib>
#include <type_traits>

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


// ------------------------------------------------------------------ MFMA (bf16 or int8)
// 256x256 output tile per block of 4 wavefronts (2x2, 128x128 each = 4x4 MFMA 32x32 tiles, 256
// accumulators per lane), K in slices of 128 bytes per row (64 bf16 or 128 int8: the byte
// geometry of the two is the same, 16 bytes per lane and MFMA) staged through two LDS stages
// (rows padded to 144 bytes) and two register sets.
//
// Schedule of one slice (four steps of 16 MFMAs each).  A wavefront issues in order and each SIMD
// holds one wavefront here, so whatever is not an MFMA is placed BETWEEN the MFMAs of a step, a
// few instructions after each, instead of after them where the matrix cores would idle:
//   step 1-2 the register set that holds slice kt+1 -> the other LDS stage
//   barrier
//   step 3   reads the first fragments of that stage; loads of slice kt+3 -> the set just freed
//            (they are written to LDS six steps later)
// and every step reads the LDS fragments of the next one.  On MI355X this runs the fold at about
// 1 PFLOP/s; what remains is the LDS traffic (each staged byte is written once and read by two
// wavefronts: 1536 LDS cycles against 2048 MFMA cycles per slice) and the global-load path.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));

constexpr int MT = 256;
constexpr int MKB = 128;                             // bytes of one staged row slice
constexpr int MSTRIDE = MKB + 16;                    // bytes per staged row (padded)
constexpr int mfma_stage_bytes(int im) { return (64 * im + MT) * MSTRIDE; }   // A tile (64*im rows) + B tile
constexpr int mfma_lds_bytes(int im) { return 2 * mfma_stage_bytes(im); }

// Which block computes which tile.  Blocks b, b+8, b+16, ... run on one XCD and share its L2, so
// each XCD gets a rectangle of rm x rn tiles (the 8 XCDs form a gm x gn grid over the tile grid,
// times `splits` ranges of K), and inside the rectangle consecutive blocks walk `group` tile rows
// column by column: the 32 blocks an XCD runs at once then cover a compact patch and re-use each
// other's slices of A and B from L2 instead of fetching them from HBM again.
struct TileMap {
    int tiles_m, tiles_n;      // tile grid of C
    int splits;                // K ranges (1, 2, 4 or 8); more than one: results are added atomically into C
    int gn;                    // XCD grid columns (rows = 8 / splits / gn)
    int rm, rn;                // tiles per XCD rectangle
    int group;                 // tile rows walked together
    int slices;                // K slices per range
};

TileMap make_tile_map(int64_t M, int64_t N, int64_t K, int es, int splits, int tile_rows) {
    TileMap t;
    t.tiles_m = (int)((M + tile_rows - 1) / tile_rows);
    t.tiles_n = (int)((N + 255) / 256);
    t.splits = splits;
    const int nx = 8 / splits;
    int best = 1 << 30, gm = nx;
    for (int cand = 1; cand <= nx; cand *= 2) {            // cand = XCD grid rows
        const int rm = (t.tiles_m + cand - 1) / cand, rn = (t.tiles_n + nx / cand - 1) / (nx / cand);
        if (rm + rn < best) { best = rm + rn; gm = cand; }
    }
    t.gn = nx / gm;
    t.rm = (t.tiles_m + gm - 1) / gm;
    t.rn = (t.tiles_n + t.gn - 1) / t.gn;
    t.group = t.rm < 8 ? t.rm : 8;
    const int nk = (int)((K * es + 127) / 128);
    t.slices = (nk + splits - 1) / splits;
    return t;
}

// RAGGED: K is not a multiple of the slice; the last slice is then moved back to end at K and the
// pieces it shares with the slice before it are zeroed on their way to LDS (costs four selects
// per LDS write, so it is a variant of its own).
// IM: 32-row MFMA tiles per wavefront along M - the output tile is (64*IM) x 256.  IM = 4 is the
// square tile for large products; IM = 2 and 1 serve products with at most 128 / 64 rows (a few
// dozen tokens against a weight matrix), which are bound by the stream of B, not by the MFMAs.
template <bool I8, bool ATOMIC, bool RAGGED, int IM>
__global__ void __launch_bounds__(256)
gemm_nt_mfma_kernel(const unsigned char* __restrict__ A0, const unsigned char* __restrict__ B0, void* __restrict__ Cv,
                    int64_t M, int64_t N, int64_t K0, int accumulate, const bf16_t* __restrict__ row_bias,
                    TileMap tm) {
    constexpr int ES = I8 ? 1 : 2;                   // bytes per element
    constexpr int MK = MKB / ES;                     // elements per K slice
    constexpr int PER = 16 / ES;                     // elements per 16-byte chunk
    constexpr int MTA = 64 * IM;                     // rows of the A tile
    constexpr int NLA = 2 * IM;                      // loads per thread and slice for A (8 for B)
    constexpr int MSTAGE = mfma_stage_bytes(IM);
    typedef typename std::conditional<I8, i32x16_t, f32x16_t>::type acc_t;
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const int xcd = (int)blockIdx.x & 7, local = (int)blockIdx.x >> 3;
    const int ks = xcd % tm.splits, xg = xcd / tm.splits;
    const int per_group = tm.group * tm.rn;
    const int g = local / per_group, r = local % per_group;
    const int gsz = min(tm.group, tm.rm - g * tm.group);
    const int tile_m = (xg / tm.gn) * tm.rm + g * tm.group + r % gsz;
    const int tile_n = (xg % tm.gn) * tm.rn + r / gsz;
    if (tile_m >= tm.tiles_m || tile_n >= tm.tiles_n) return;
    const int64_t m0 = (int64_t)tile_m * MTA, n0 = (int64_t)tile_n * MT;
    // this block's range of K: operands advanced to its start, K = what remains from there
    const int64_t kskip = (int64_t)ks * tm.slices * MK;
    if (kskip >= K0) return;
    const int64_t K = K0 - kskip;
    const int nk = min((int)((K + MK - 1) / MK), tm.slices);

    acc_t acc[IM][4];
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // staging map: chunk c = tid + 256*i, i = 0..7 -> row c/8, 16-byte piece c%8.  The address of
    // a load is a wave-uniform base (tile start + slice) plus one of eight lane offsets, the same
    // for both operands (same row pitch).  Rows past the matrix read row 0 of the tile instead;
    // they are not zeroed: they only reach output rows and columns that are never stored.
    td_u32x4 ra0[NLA], rb0[8], ra1[NLA], rb1[8];
    const int srow = tid >> 3, spiece = tid & 7;
    unsigned offa[NLA], offb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned off = (unsigned)(((32 * i + srow) * K0 + spiece * PER) * ES);
        if (i < NLA) offa[i] = m0 + 32 * i + srow < M ? off : 0u;
        offb[i] = n0 + 32 * i + srow < N ? off : 0u;
    }
    const unsigned char* tileA = A0 + (m0 * K0 + kskip) * ES;
    const unsigned char* tileB = B0 + (n0 * K0 + kskip) * ES;
    // slices past the last one re-read slice 0 (never multiplied): every load below is issued
    // unconditionally, so the number of loads in flight at each wait is known statically
    auto fetch = [&](td_u32x4 (&ra)[NLA], td_u32x4 (&rb)[8], unsigned& keep, int kt) {
        const int64_t k0 = (int64_t)kt * MK;
        int64_t kb = kt < nk ? k0 : 0;
        keep = 1u;
        if constexpr (RAGGED) {
            if (kt < nk && k0 + MK > K) kb = K - MK;                  // the last slice, moved back
            keep = kb + spiece * PER >= k0 ? 1u : 0u;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i < NLA) ra[i] = *reinterpret_cast<const td_u32x4*>(tileA + kb * ES + offa[i]);
            rb[i] = *reinterpret_cast<const td_u32x4*>(tileB + kb * ES + offb[i]);
        }
    };
    auto stash_rows = [&](auto& rr, unsigned keep, unsigned char* dst) {     // rr: NLA or 8 row groups
        const td_u32x4 zero = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < (int)(sizeof(rr) / sizeof(rr[0])); ++i)
            *reinterpret_cast<td_u32x4*>(dst + 32 * i * MSTRIDE) = (!RAGGED || keep) ? rr[i] : zero;
    };
    auto stash_a = [&](const td_u32x4 (&rr)[NLA], unsigned keep, int stage) {
        stash_rows(rr, keep, lds + stage * MSTAGE + srow * MSTRIDE + spiece * 16);
    };
    auto stash_b = [&](const td_u32x4 (&rr)[8], unsigned keep, int stage) {
        stash_rows(rr, keep, lds + stage * MSTAGE + MTA * MSTRIDE + srow * MSTRIDE + spiece * 16);
    };
    const int frow = lane & 31, fk = (lane >> 5) * 16;  // fragment row and byte offset of its 16 bytes of k
    td_u32x4 fa[2][IM], fb[2][4];
    auto read_frags = [&](td_u32x4 (&da)[IM], td_u32x4 (&db)[4], int stage, int kstep) {
        const unsigned char* as = lds + stage * MSTAGE + (wm * 32 * IM + frow) * MSTRIDE + fk + kstep * 32;
        const unsigned char* bs = lds + stage * MSTAGE + MTA * MSTRIDE + (wn * 128 + frow) * MSTRIDE + fk + kstep * 32;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i < IM) da[i] = *reinterpret_cast<const td_u32x4*>(as + i * 32 * MSTRIDE);
            db[i] = *reinterpret_cast<const td_u32x4*>(bs + i * 32 * MSTRIDE);
        }
    };
    auto mfma16 = [&](const td_u32x4 (&ua)[IM], const td_u32x4 (&ub)[4]) {   // 4 * IM MFMAs
#pragma unroll
        for (int i = 0; i < IM; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (I8)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4_t, ua[i]),
                                                                      __builtin_bit_cast(i32x4_t, ub[j]), acc[i][j], 0, 0, 0);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ua[i]),
                                                                        __builtin_bit_cast(bf16x8_t, ub[j]), acc[i][j], 0, 0, 0);
            }
    };
    // the scheduler is told the order inside a step of the square tile: one MFMA, `alu` VALU/SALU
    // instructions, and after every `every`-th MFMA one memory instruction of class `cls` (0x020
    // load, 0x200 LDS write).  The short tiles have 4 or 8 MFMAs per step and are bound by the
    // stream of B: the compiler's own order serves them.
#define TD_GEMM_INTERLEAVE(alu, cls, every)                                          \
    _Pragma("unroll") for (int q = 0; q < 16; ++q) {                                 \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                           \
        __builtin_amdgcn_sched_group_barrier(0x006, alu, 0);                         \
        if (q % every == every - 1) __builtin_amdgcn_sched_group_barrier(cls, 1, 0); \
    }
    // `sa`/`sb` (holding slice kt+1) go to the other LDS stage in steps 1-2 and are reloaded with
    // slice kt+3 in step 3; the other register set (slice kt+2) stays in flight through the phase
    auto phase = [&](int stage, td_u32x4 (&sa)[NLA], td_u32x4 (&sb)[8], unsigned& skeep, int lkt) {
        read_frags(fa[1], fb[1], stage, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma16(fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa[0], fb[0], stage, 2);
        __builtin_amdgcn_sched_barrier(0);
        mfma16(fa[1], fb[1]);
        stash_b(sb, skeep, stage ^ 1);
        if constexpr (IM == 4) { TD_GEMM_INTERLEAVE(RAGGED ? 3 : 1, 0x200, 2) }
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa[1], fb[1], stage, 3);
        __builtin_amdgcn_sched_barrier(0);
        mfma16(fa[0], fb[0]);
        stash_a(sa, skeep, stage ^ 1);
        if constexpr (IM == 4) { TD_GEMM_INTERLEAVE(RAGGED ? 3 : 1, 0x200, 2) }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        read_frags(fa[0], fb[0], stage ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma16(fa[1], fb[1]);
        fetch(sa, sb, skeep, lkt);
        if constexpr (IM == 4) { TD_GEMM_INTERLEAVE(2, 0x020, 1) }
        __builtin_amdgcn_sched_barrier(0);
    };
#undef TD_GEMM_INTERLEAVE

    unsigned keep0 = 1u, keep1 = 1u;
    fetch(ra0, rb0, keep0, 0);
    fetch(ra1, rb1, keep1, 1);
    stash_a(ra0, keep0, 0);
    stash_b(rb0, keep0, 0);
    fetch(ra0, rb0, keep0, 2);
    __syncthreads();
    read_frags(fa[0], fb[0], 0, 0);
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        phase(0, ra1, rb1, keep1, kt + 3);           // multiplies slice kt, stages slice kt+1
        phase(1, ra0, rb0, keep0, kt + 4);           // multiplies slice kt+1, stages slice kt+2
    }
    if (kt < nk) phase(0, ra1, rb1, keep1, kt + 3);  // odd count: the last slice

    // D layout of the 32x32 tile: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
    for (int i = 0; i < IM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t m = m0 + wm * 32 * IM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + wn * 128 + j * 32 + (lane & 31);
                if (n >= N) continue;
                if constexpr (I8) {
                    int32_t* C = static_cast<int32_t*>(Cv);
                    if constexpr (ATOMIC)
                        __hip_atomic_fetch_add(C + m * N + n, acc[i][j][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    else
                        C[m * N + n] = acc[i][j][r];
                } else {
                    float* C = static_cast<float*>(Cv);
                    float v = acc[i][j][r] + ((row_bias && ks == 0) ? td_bf16_to_f32(row_bias[m]) : 0.0f);
                    if constexpr (ATOMIC) {
                        __hip_atomic_fetch_add(C + m * N + n, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        if (accumulate) v += C[m * N + n];
                        C[m * N + n] = v;
                    }
                }
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

__global__ void __launch_bounds__(256) gemm_zero_kernel(uint32_t* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

// The kernels that add atomically (K cut into ranges, and every short-tile variant) need C to
// hold the value they add onto: zeros unless the caller accumulates.
void zero_result(void* C, int64_t M, int64_t N, hipStream_t s) {
    const size_t n = (size_t)M * (size_t)N;
    const unsigned blocks = (unsigned)((n / 4 + 255) / 256 < 4096 ? (n / 4 + 255) / 256 + 1 : 4096);
    hipLaunchKernelGGL(gemm_zero_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint32_t*>(C), n);
}

template <bool I8, bool ATOMIC, bool RAGGED, int IM>
void launch_mfma(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int accumulate,
                 const void* row_bias, const TileMap& tm, hipStream_t s) {
    hipLaunchKernelGGL((gemm_nt_mfma_kernel<I8, ATOMIC, RAGGED, IM>), dim3(8 * tm.rm * tm.rn), dim3(256),
                       mfma_lds_bytes(IM), s, static_cast<const unsigned char*>(A),
                       static_cast<const unsigned char*>(B), C, M, N, K, accumulate,
                       static_cast<const bf16_t*>(row_bias), tm);
}

bool gemm_force_generic() {
    const char* v = std::getenv("TARDIS_GEMM_GENERIC");
    return v && v[0] == '1';
}

}  // namespace

// the matrix-core kernels use more LDS than the default limit; raised once, outside any stream capture
tardis_status_t td_gemm_init() {
    static td_once once;
    return once.run([]() -> tardis_status_t {
        struct { const void* fn; int lds; } kernels[] = {
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<false, false, false, 4>), mfma_lds_bytes(4)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<false, false, true, 4>), mfma_lds_bytes(4)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<false, true, false, 4>), mfma_lds_bytes(4)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<true, false, false, 4>), mfma_lds_bytes(4)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<true, true, false, 4>), mfma_lds_bytes(4)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<false, true, false, 2>), mfma_lds_bytes(2)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<true, true, false, 2>), mfma_lds_bytes(2)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<false, true, false, 1>), mfma_lds_bytes(1)},
            {reinterpret_cast<const void*>(gemm_nt_mfma_kernel<true, true, false, 1>), mfma_lds_bytes(1)}};
        for (const auto& k : kernels)
            TD_HIP(hipFuncSetAttribute(k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, k.lds));
        return TARDIS_OK;
    });
}

// rows of the output tile the matrix-core kernel uses for a product with M rows
int td_gemm_tile_rows(int64_t M) { return M <= 64 ? 64 : (M <= 128 ? 128 : 256); }

tardis_status_t td_gemm_nt(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K, int32_t dtype,
                           int accumulate, const void* row_bias, hipStream_t s) {
    return td_gemm_nt_split(A, B, C, M, N, K, dtype, accumulate, row_bias, 1, s);
}

// the same with K cut into `splits` ranges (1, 2, 4, 8) that run as separate blocks - for products
// whose tile grid alone would leave most of the chip idle.  The ranges add their partial sums into C
// atomically (C is zeroed first unless `accumulate`); so do the short-tile variants (M <= 128).
tardis_status_t td_gemm_nt_split(const void* A, const void* B, float* C, int64_t M, int64_t N, int64_t K,
                                 int32_t dtype, int accumulate, const void* row_bias, int splits, hipStream_t s) {
    if (M <= 0 || N <= 0 || K <= 0) return TARDIS_ERR_SHAPE;
    if ((M + GT - 1) / GT > 65535) return TARDIS_ERR_SHAPE;
    if (splits != 1 && splits != 2 && splits != 4 && splits != 8) return TARDIS_ERR_INVALID_ARG;
    // (any M, N work on the matrix cores; small products are not worth it)
    if (dtype == TARDIS_BF16 && M >= 32 && N >= 32 && M * N >= 128 * 128 && K >= 64 &&
        (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0 && K % 8 == 0 &&
        !gemm_force_generic()) {
        TD_TRY(td_gemm_init());
        if (K % 64 != 0) {       // a ragged K runs unsplit on the square tile: plain stores
            launch_mfma<false, false, true, 4>(A, B, C, M, N, K, accumulate, row_bias, make_tile_map(M, N, K, 2, 1, 256), s);
        } else {
            const int rows = td_gemm_tile_rows(M);
            const TileMap tm = make_tile_map(M, N, K, 2, splits, rows);
            const bool atomic = splits > 1 || rows < 256;
            if (atomic && !accumulate) zero_result(C, M, N, s);
            if (rows == 64) launch_mfma<false, true, false, 1>(A, B, C, M, N, K, 1, row_bias, tm, s);
            else if (rows == 128) launch_mfma<false, true, false, 2>(A, B, C, M, N, K, 1, row_bias, tm, s);
            else if (atomic) launch_mfma<false, true, false, 4>(A, B, C, M, N, K, 1, row_bias, tm, s);
            else launch_mfma<false, false, false, 4>(A, B, C, M, N, K, accumulate, row_bias, tm, s);
        }
    } else if (dtype == TARDIS_BF16)
        launch_generic<bf16_t>(A, B, C, M, N, K, accumulate, row_bias, s);
    else
        launch_generic<float>(A, B, C, M, N, K, accumulate, row_bias, s);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

// C (int32, M x N) = A (int8, M x K) . B (int8, N x K)^T, exact.  16-byte aligned operands, K % 128 == 0.
// splits: K ranges as above (integer adds, so the result is the same exact sum).
tardis_status_t td_gemm_nt_i8(const int8_t* A, const int8_t* B, int32_t* C, int64_t M, int64_t N, int64_t K,
                              int splits, hipStream_t s) {
    if (M <= 0 || N <= 0 || K <= 0 || K % 128 != 0) return TARDIS_ERR_SHAPE;
    if (splits != 1 && splits != 2 && splits != 4 && splits != 8) return TARDIS_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(A) & 15) || (reinterpret_cast<uintptr_t>(B) & 15)) return TARDIS_ERR_INVALID_ARG;
    TD_TRY(td_gemm_init());
    const int rows = td_gemm_tile_rows(M);
    const TileMap tm = make_tile_map(M, N, K, 1, splits, rows);
    const bool atomic = splits > 1 || rows < 256;
    if (atomic) zero_result(C, M, N, s);
    if (rows == 64) launch_mfma<true, true, false, 1>(A, B, C, M, N, K, 0, nullptr, tm, s);
    else if (rows == 128) launch_mfma<true, true, false, 2>(A, B, C, M, N, K, 0, nullptr, tm, s);
    else if (atomic) launch_mfma<true, true, false, 4>(A, B, C, M, N, K, 0, nullptr, tm, s);
    else launch_mfma<true, false, false, 4>(A, B, C, M, N, K, 0, nullptr, tm, s);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}
