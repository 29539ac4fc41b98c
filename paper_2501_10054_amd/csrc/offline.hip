// Offline steps: range selection and line fit (calibrate), constant folding,
// predictor construction, and the layout copies the online path needs.
#include "common.h"

namespace {

constexpr int kBlock = 256;

// ------------------------------------------------------------------ transpose
// dst[c][r] = src[r][c], element size 2 or 4 bytes.
template <typename E>
__global__ void __launch_bounds__(256)
transpose_kernel(const E* __restrict__ src, E* __restrict__ dst, int64_t rows, int64_t cols) {
    __shared__ E tile[32][33];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
    const int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t r = r0 + ty + i, c = c0 + tx;
        if (r < rows && c < cols) tile[ty + i][tx] = src[r * cols + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t c = c0 + ty + i, r = r0 + tx;
        if (r < rows && c < cols) dst[c * rows + r] = tile[tx][ty + i];
    }
}

// ------------------------------------------------------- scaled transpose (fold)
// P = diag(a) W1 (h x d) written transposed (d x h).  For bf16 storage the fp32
// product is split into a bf16 head and a bf16 remainder so that the folded
// matrix is accumulated from ~16 significant bits instead of 8 (the paper's
// Sec. "Precision Effects on Reordering FFN" finds bf16 intermediates visibly
// worse than fp32).
__global__ void __launch_bounds__(256)
scale_transpose_bf16_kernel(const bf16_t* __restrict__ W1, const float* __restrict__ a, bf16_t* __restrict__ Phi,
                            bf16_t* __restrict__ Plo, int64_t h, int64_t d) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    const int64_t k0 = (int64_t)blockIdx.x * 32, j0 = (int64_t)blockIdx.y * 32;
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t j = j0 + ty + i, k = k0 + tx;
        if (j < h && k < d) tile[ty + i][tx] = a[j] * td_bf16_to_f32(W1[j * d + k]);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t k = k0 + ty + i, j = j0 + tx;
        if (j < h && k < d) {
            const float p = tile[tx][ty + i];
            const bf16_t hi = td_f32_to_bf16(p);
            Phi[k * h + j] = hi;
            Plo[k * h + j] = td_f32_to_bf16(p - td_bf16_to_f32(hi));
        }
    }
}

__global__ void __launch_bounds__(256)
scale_transpose_f32_kernel(const float* __restrict__ W1, const float* __restrict__ a, float* __restrict__ P,
                           int64_t h, int64_t d) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    const int64_t k0 = (int64_t)blockIdx.x * 32, j0 = (int64_t)blockIdx.y * 32;
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t j = j0 + ty + i, k = k0 + tx;
        if (j < h && k < d) tile[ty + i][tx] = a[j] * W1[j * d + k];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; i += 8) {
        const int64_t k = k0 + ty + i, j = j0 + tx;
        if (j < h && k < d) P[k * h + j] = tile[tx][ty + i];
    }
}

__global__ void __launch_bounds__(256)
f32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = td_f32_to_bf16(src[i]);
}

// b'[r] = sum_j W2[r][j] * (c_j + a_j b1_j) + b2[r]; one block per output row,
// fp64 accumulation.
template <typename T>
__global__ void __launch_bounds__(kBlock)
fold_bias_kernel(const T* __restrict__ W2, const T* __restrict__ b1, const T* __restrict__ b2,
                 const float* __restrict__ a, const float* __restrict__ c, float* __restrict__ bp, int64_t d,
                 int64_t h) {
    __shared__ double red[kBlock / TD_WAVE];
    const int64_t r = blockIdx.x;
    double acc = 0.0;
    for (int64_t j = threadIdx.x; j < h; j += kBlock) {
        double kj = (double)c[j];
        if (b1) kj += (double)a[j] * (double)td_load<T>(b1 + j);
        acc += (double)td_load<T>(W2 + r * h + j) * kj;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kBlock / TD_WAVE; ++w) t += red[w];
        if (b2) t += (double)td_load<T>(b2 + r);
        bp[r] = (float)t;
    }
}

// ---------------------------------------------------------------- predictor
// One block per neuron row: s = max|w| / 127 (fp64), q = rint(w / s) clamped,
// bounds in code units.  All arithmetic is IEEE fp64 so the codes are a pure
// function of the inputs.
// The range the predictor tests against: the neuron's range with the fraction `margin` of its
// width taken off at either end (margin = 0: the range itself).  A narrower test flags more
// neurons - flagged neurons are repaired exactly, so this trades time for recall of a coarse sketch.
__device__ __forceinline__ void predictor_range(double lo, double hi, double margin, double& rl, double& rh) {
    rl = lo;
    rh = hi;
    const double w = hi - lo;
    if (margin > 0.0 && w > 0.0 && w < INFINITY) {
        rl = lo + margin * w;
        rh = hi - margin * w;
    }
}

template <typename T>
__global__ void __launch_bounds__(kBlock)
sketch_kernel(const T* __restrict__ W1, const T* __restrict__ b1, const float* __restrict__ lo,
              const float* __restrict__ hi, int64_t d, int8_t* __restrict__ Q, float* __restrict__ tlo,
              float* __restrict__ thi, float margin) {
    __shared__ float red[kBlock / TD_WAVE];
    const int64_t j = blockIdx.x;
    const T* row = W1 + j * d;
    float m = 0.0f;
    for (int64_t k = threadIdx.x; k < d; k += kBlock) m = fmaxf(m, fabsf(td_load<T>(row + k)));
    m = td_wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / TD_WAVE; ++w) m = fmaxf(m, red[w]);
    const double s = (double)m / 127.0;
    const double bj = b1 ? (double)td_load<T>(b1 + j) : 0.0;
    double rl, rh;
    predictor_range((double)lo[j], (double)hi[j], (double)margin, rl, rh);
    if (m > 0.0f) {
        for (int64_t k = threadIdx.x; k < d; k += kBlock) {
            double q = rint((double)td_load<T>(row + k) / s);
            q = fmin(fmax(q, -127.0), 127.0);
            Q[j * d + k] = (int8_t)(int)q;
        }
        if (threadIdx.x == 0) {
            tlo[j] = (float)((rl - bj) / s);
            thi[j] = (float)((rh - bj) / s);
        }
    } else {
        for (int64_t k = threadIdx.x; k < d; k += kBlock) Q[j * d + k] = 0;
        if (threadIdx.x == 0) {
            const bool inside = (rl <= bj) && (bj < rh);
            tlo[j] = inside ? -INFINITY : INFINITY;
            thi[j] = INFINITY;
        }
    }
}

// Grouped low-bit sketch (groups of 32 consecutive columns), codes of 4, 3 or 2 bits with the
// largest code qmax = 7, 3 or 1: group maxima g, row maximum r,
// s = r / (qmax*15), multiplier m = ceil(g / (qmax s)) in [1, 15], code q = rint(w / (m s)) in [-qmax, qmax];
// all in fp64, each step one IEEE operation, so every output is a function of the inputs.
// Outputs: M4 (one byte per group); Q (optional) the effective one-byte code m*q; Q4 (optional,
// d % 32 == 0) the packed form read by the decode kernel: group G is the 16-byte vector G of the
// row, byte b of its dword w holds column 4w+b in the low nibble and column 16+4w+b in the high one.
template <typename T>
__global__ void __launch_bounds__(kBlock)
sketch4_kernel(const T* __restrict__ W1, const T* __restrict__ b1, const float* __restrict__ lo,
               const float* __restrict__ hi, int64_t d, int ng, int8_t* __restrict__ Q, uint8_t* __restrict__ Q4,
               uint8_t* __restrict__ M4, float* __restrict__ tlo, float* __restrict__ thi, int qmax, float margin) {
    extern __shared__ int gval[];                    // group maxima (bit patterns), then multipliers
    __shared__ float red[kBlock / TD_WAVE];
    const int64_t j = blockIdx.x;
    const T* row = W1 + j * d;
    for (int g = threadIdx.x; g < ng; g += kBlock) gval[g] = 0;
    __syncthreads();
    for (int64_t k = threadIdx.x; k < d; k += kBlock)   // non-negative floats order like their bit patterns
        atomicMax(&gval[k >> 5], __float_as_int(fabsf(td_load<T>(row + k))));
    __syncthreads();
    float r = 0.0f;
    for (int g = threadIdx.x; g < ng; g += kBlock) r = fmaxf(r, __int_as_float(gval[g]));
    r = td_wave_max(r);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = r;
    __syncthreads();
    r = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / TD_WAVE; ++w) r = fmaxf(r, red[w]);
    const double s = (double)r / (double)(qmax * 15);   // (4 bits: 7 * 15)
    const double bj = b1 ? (double)td_load<T>(b1 + j) : 0.0;
    const bool live = r > 0.0f;
    for (int g = threadIdx.x; g < ng; g += kBlock) {
        int m = 1;
        if (live) {
            const double t = ceil((double)__int_as_float(gval[g]) / ((double)qmax * s));
            m = (int)fmin(fmax(t, 1.0), 15.0);
        }
        gval[g] = m;
        M4[j * ng + g] = (uint8_t)m;
    }
    __syncthreads();
    auto code = [&](int64_t k) -> int {              // 4-bit code of column k
        if (!live) return 0;
        const double q = rint((double)td_load<T>(row + k) / ((double)gval[k >> 5] * s));
        return (int)fmin(fmax(q, -(double)qmax), (double)qmax);
    };
    if (Q4) {   // d is a multiple of 32 here
        uint32_t* out = reinterpret_cast<uint32_t*>(Q4 + j * (d / 2));
        for (int64_t idx = threadIdx.x; idx < d / 8; idx += kBlock) {
            const int64_t g = idx >> 2, w = idx & 3;
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int64_t klo = 32 * g + 4 * w + b, khi = klo + 16;
                const int qlo = code(klo), qhi = code(khi);
                word |= (uint32_t)((qlo & 0xF) | ((qhi & 0xF) << 4)) << (8 * b);
                if (Q) {
                    Q[j * d + klo] = (int8_t)(gval[g] * qlo);
                    Q[j * d + khi] = (int8_t)(gval[g] * qhi);
                }
            }
            out[idx] = word;
        }
    } else if (Q) {
        for (int64_t k = threadIdx.x; k < d; k += kBlock) Q[j * d + k] = (int8_t)(gval[k >> 5] * code(k));
    }
    if (threadIdx.x == 0) {
        double rl, rh;
        predictor_range((double)lo[j], (double)hi[j], (double)margin, rl, rh);
        if (live) {
            tlo[j] = (float)((rl - bj) / s);
            thi[j] = (float)((rh - bj) / s);
        } else {
            const bool inside = (rl <= bj) && (bj < rh);
            tlo[j] = inside ? -INFINITY : INFINITY;
            thi[j] = INFINITY;
        }
    }
}

__global__ void __launch_bounds__(kBlock)
unpack_sketch4_kernel(const uint8_t* __restrict__ Q4, const uint8_t* __restrict__ M4, int64_t d,
                      int8_t* __restrict__ Q) {
    const int64_t j = blockIdx.x;
    const uint32_t* in = reinterpret_cast<const uint32_t*>(Q4 + j * (d / 2));
    for (int64_t idx = threadIdx.x; idx < d / 8; idx += kBlock) {
        const int64_t g = idx >> 2, w = idx & 3;
        const int m = M4[j * (d / 32) + g];
        const uint32_t word = in[idx];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int byte = (int)((word >> (8 * b)) & 0xFFu);
            const int qlo = ((byte & 0xF) ^ 8) - 8, qhi = ((byte >> 4) ^ 8) - 8;   // sign-extend 4 bits
            Q[j * d + 32 * g + 4 * w + b] = (int8_t)(m * qlo);
            Q[j * d + 32 * g + 16 + 4 * w + b] = (int8_t)(m * qhi);
        }
    }
}

// -------------------------------------------------------------- calibration
// One block per neuron.  zt: that neuron's n calibration pre-activations.
// Sort in LDS (bitonic, padded with +inf), read the two quantiles by linear
// interpolation at q*(n-1), then fit sigma(z) ~ a z + c over lo <= z < hi.
__device__ __forceinline__ double block_sum(double v, double* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kBlock / TD_WAVE; ++w) t += red[w];
    return t;
}

__device__ __forceinline__ double quantile_sorted(const float* v, int n, double q) {
    const double pos = q * (double)(n - 1);
    int i = (int)floor(pos);
    i = min(max(i, 0), n - 1);
    const double g = pos - (double)i;
    const int i1 = min(i + 1, n - 1);
    return (double)v[i] + g * ((double)v[i1] - (double)v[i]);
}

// sorts vals[0..npad) ascending (npad a power of two, padded with +inf)
__device__ __forceinline__ void sort_lds(float* vals, int npad) {
    for (int k = 2; k <= npad; k <<= 1) {
        for (int s = k >> 1; s > 0; s >>= 1) {
            for (int t = threadIdx.x; t < npad / 2; t += kBlock) {
                const int i = 2 * t - (t & (s - 1));  // index with bit `s` clear
                const int p = i + s;
                const bool up = (i & k) == 0;
                const float x0 = vals[i], x1 = vals[p];
                if ((x0 > x1) == up) {
                    vals[i] = x1;
                    vals[p] = x0;
                }
            }
            __syncthreads();
        }
    }
}

// least-squares line of sigma(z) on z over the samples with lo32 <= z < hi32, and the four outputs
__device__ __forceinline__ void fit_and_store(const float* vals, int n, float lo32, float hi32, int act, double* red,
                                              int64_t j, float* lo, float* hi, float* a, float* c) {
    double cnt = 0.0, sz = 0.0, sg = 0.0;
    for (int i = threadIdx.x; i < n; i += kBlock) {
        const float v = vals[i];
        if (v >= lo32 && v < hi32) {
            cnt += 1.0;
            sz += (double)v;
            sg += td_act_f64((double)v, act);
        }
    }
    cnt = block_sum(cnt, red);
    sz = block_sum(sz, red);
    sg = block_sum(sg, red);
    float aj, cj;
    if (cnt < 0.5) {
        aj = 0.0f;
        cj = (float)td_act_f64((double)lo32, act);
    } else {
        const double zbar = sz / cnt, gbar = sg / cnt;
        double var = 0.0, cov = 0.0;
        for (int i = threadIdx.x; i < n; i += kBlock) {
            const float v = vals[i];
            if (v >= lo32 && v < hi32) {
                const double dz = (double)v - zbar;
                var += dz * dz;
                cov += dz * (td_act_f64((double)v, act) - gbar);
            }
        }
        var = block_sum(var, red);
        cov = block_sum(cov, red);
        if (cnt < 1.5 || !(var > 0.0)) {
            aj = 0.0f;
            cj = (float)gbar;
        } else {
            const double slope = cov / var;
            aj = (float)slope;
            cj = (float)(gbar - slope * zbar);
        }
    }
    if (threadIdx.x == 0) {
        lo[j] = lo32;
        hi[j] = hi32;
        a[j] = aj;
        c[j] = cj;
    }
}

__global__ void __launch_bounds__(kBlock)
calibrate_neuron_kernel(const float* __restrict__ Zt, int n, int npad, float coverage,
                        const float* __restrict__ cov_pn, int act, float* __restrict__ lo, float* __restrict__ hi,
                        float* __restrict__ a, float* __restrict__ c) {
    extern __shared__ float vals[];
    __shared__ double red[kBlock / TD_WAVE];
    const int64_t j = blockIdx.x;
    const float* z = Zt + j * (int64_t)n;
    for (int i = threadIdx.x; i < npad; i += kBlock) vals[i] = i < n ? z[i] : INFINITY;
    __syncthreads();
    sort_lds(vals, npad);
    const double t = cov_pn ? (double)cov_pn[j] : (double)coverage;
    const float lo32 = (float)quantile_sorted(vals, n, (1.0 - t) / 2.0);
    const float hi32 = (float)quantile_sorted(vals, n, (1.0 + t) / 2.0);
    fit_and_store(vals, n, lo32, hi32, act, red, j, lo, hi, a, c);
}

// ------------------------------------------------------------- range search
// Greedy range of Algorithm 1 (inner loop), one block per neuron: centroid = mode of a Gaussian
// kernel density estimate on a grid of 256 points (bandwidth 1.06 std n^-1/5), then the range
// grows by `step` to the left or to the right, whichever candidate's least-squares line leaves
// the smaller sum of |sigma(z) - (a z + c)| over its samples (right on equality), until it holds
// the portion t of the samples.  A side whose end lies beyond every sample is not offered again,
// so the loop ends after at most (max z - min z) / step + 2 steps; kSearchMaxSteps is a guard on
// the run time of one block, and a neuron that hits it makes the whole call fail.
constexpr int kKdeGrid = 256;
constexpr int kSearchMaxSteps = 4096;
static_assert(kKdeGrid == kBlock, "one grid point per thread");

// four block-wide sums at once
__device__ __forceinline__ void block_sum4(double (&v)[4], double (*red4)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[q] += __shfl_xor(v[q], o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) red4[threadIdx.x / 64][q] = v[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / TD_WAVE; ++w) t += red4[w][q];
        v[q] = t;
    }
}

// first index i in [0, n) with vals[i] >= x (n if none)
__device__ __forceinline__ int lower_bound_lds(const float* vals, int n, double x) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((double)vals[mid] >= x) hi = mid; else lo = mid + 1;
    }
    return lo;
}

__global__ void __launch_bounds__(kBlock)
range_search_kernel(const float* __restrict__ Zt, int n, int npad, float coverage, const float* __restrict__ cov_pn,
                    float step32, int act, float* __restrict__ lo, float* __restrict__ hi, float* __restrict__ a,
                    float* __restrict__ c, int* __restrict__ n_capped) {
    extern __shared__ double gv[];                   // sigma of the sorted samples, then the samples
    float* vals = reinterpret_cast<float*>(gv + ((n + 1) & ~1));
    __shared__ double red[kBlock / TD_WAVE];
    __shared__ double red4[kBlock / TD_WAVE][4];
    __shared__ double dens[kKdeGrid];
    const int64_t j = blockIdx.x;
    const float* z = Zt + j * (int64_t)n;
    for (int i = threadIdx.x; i < npad; i += kBlock) vals[i] = i < n ? z[i] : INFINITY;
    __syncthreads();
    sort_lds(vals, npad);
    for (int i = threadIdx.x; i < n; i += kBlock) gv[i] = td_act_f64((double)vals[i], act);
    const double zmin = (double)vals[0], zmax = (double)vals[n - 1];
    const double t = cov_pn ? (double)cov_pn[j] : (double)coverage;
    const double step = (double)step32;

    // ---- centroid
    double cen = zmin;
    if (n >= 2 && zmax > zmin) {
        double sz = 0.0;
        for (int i = threadIdx.x; i < n; i += kBlock) sz += (double)vals[i];
        const double mean = block_sum(sz, red) / (double)n;
        double sv = 0.0;
        for (int i = threadIdx.x; i < n; i += kBlock) {
            const double dz = (double)vals[i] - mean;
            sv += dz * dz;
        }
        const double sd = sqrt(block_sum(sv, red) / (double)(n - 1));
        const double bw = 1.06 * sd * pow((double)n, -0.2);
        const double delta = (zmax - zmin) / (double)(kKdeGrid - 1);
        const double u = zmin + (double)threadIdx.x * delta;
        double dsum = 0.0;
        for (int k = 0; k < n; ++k) {
            const double q = (u - (double)vals[k]) / bw;
            dsum += exp(-0.5 * q * q);
        }
        dens[threadIdx.x] = dsum;
        __syncthreads();
        int best = 0;
        double best_d = dens[0];
        for (int g = 1; g < kKdeGrid; ++g)           // the leftmost among equal maxima
            if (dens[g] > best_d) {
                best_d = dens[g];
                best = g;
            }
        cen = zmin + (double)best * delta;
    }
    __syncthreads();

    // ---- growth (every thread carries the same scalars)
    double rlo = cen, rhi = cen;
    bool done = false;
    for (int it = 0; it < kSearchMaxSteps && !done; ++it) {
        const int il = lower_bound_lds(vals, n, rlo), ih = lower_bound_lds(vals, n, rhi);
        if ((double)(ih - il) / (double)n >= t) {
            done = true;
            break;
        }
        const bool left_open = rlo > zmin, right_open = !(rhi > zmax);
        if (!left_open && !right_open) {
            done = true;
            break;
        }
        bool go_left = left_open;
        if (left_open && right_open) {
            // candidate 0: [rlo - step, rhi) = samples [cl, ih); candidate 1: [rlo, rhi + step) = samples [il, ch)
            const int cl = lower_bound_lds(vals, n, rlo - step), ch = lower_bound_lds(vals, n, rhi + step);
            const int n0 = ih - cl, n1 = ch - il;
            double sums[4] = {0.0, 0.0, 0.0, 0.0};   // sum z, sum g of both candidates
            for (int i = cl + (int)threadIdx.x; i < ch; i += kBlock) {
                const double zi = (double)vals[i], gi = gv[i];
                if (i < ih) { sums[0] += zi; sums[1] += gi; }
                if (i >= il) { sums[2] += zi; sums[3] += gi; }
            }
            block_sum4(sums, red4);
            const double zb0 = n0 ? sums[0] / n0 : 0.0, gb0 = n0 ? sums[1] / n0 : 0.0;
            const double zb1 = n1 ? sums[2] / n1 : 0.0, gb1 = n1 ? sums[3] / n1 : 0.0;
            double vc[4] = {0.0, 0.0, 0.0, 0.0};     // var, cov of both candidates
            for (int i = cl + (int)threadIdx.x; i < ch; i += kBlock) {
                const double zi = (double)vals[i], gi = gv[i];
                if (i < ih) { vc[0] += (zi - zb0) * (zi - zb0); vc[1] += (zi - zb0) * (gi - gb0); }
                if (i >= il) { vc[2] += (zi - zb1) * (zi - zb1); vc[3] += (zi - zb1) * (gi - gb1); }
            }
            block_sum4(vc, red4);
            double a0 = 0.0, c0 = gb0, a1 = 0.0, c1 = gb1;
            if (n0 >= 2 && vc[0] > 0.0) { a0 = vc[1] / vc[0]; c0 = gb0 - a0 * zb0; }
            if (n1 >= 2 && vc[2] > 0.0) { a1 = vc[3] / vc[2]; c1 = gb1 - a1 * zb1; }
            double er[4] = {0.0, 0.0, 0.0, 0.0};
            for (int i = cl + (int)threadIdx.x; i < ch; i += kBlock) {
                const double zi = (double)vals[i], gi = gv[i];
                if (i < ih) er[0] += fabs(gi - (a0 * zi + c0));
                if (i >= il) er[1] += fabs(gi - (a1 * zi + c1));
            }
            block_sum4(er, red4);
            go_left = er[0] < er[1];
        }
        if (go_left) rlo = rlo - step; else rhi = rhi + step;
    }
    if (!done) {   // the run-time guard on the number of steps was hit (a step far below the samples'
                   // spread): reported to the host, which fails the call; the whole sample range is
                   // stored so that the outputs are at least well defined
        if (threadIdx.x == 0) atomicAdd(n_capped, 1);
        rlo = zmin;
        rhi = nextafter(zmax, INFINITY);
    }
    __syncthreads();
    fit_and_store(vals, n, (float)rlo, (float)rhi, act, red, j, lo, hi, a, c);
}

// ------------------------------------------------- 8-bit floating-point storage of W'
// Nearest e4m3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest
// value 448) of v, ties to the even mantissa, magnitudes above 448 saturate.
__device__ __forceinline__ uint32_t f32_to_e4m3(float v) {
    const uint32_t sign = (__float_as_uint(v) >> 24) & 0x80u;
    float m = fminf(fabsf(v), 448.0f);
    if (!(m == m)) return sign | 0x7Fu;
    uint32_t code;
    if (m < 0.015625f) {                              // below 2^-6: multiples of 2^-9 (8 is the first normal code)
        code = (uint32_t)rintf(m * 512.0f);
    } else {
        uint32_t u = __float_as_uint(m);
        u += 0x7FFFFu + ((u >> 20) & 1u);            // round the mantissa to 3 bits, ties to even (may carry into the exponent)
        u &= 0xFFF00000u;
        const uint32_t e = (u >> 23) - 127u + 7u;
        code = (e << 3) | ((u >> 20) & 7u);
        if (code > 0x7Eu) code = 0x7Eu;
    }
    return sign | code;
}

__device__ __forceinline__ float e4m3_to_f32(uint32_t code) {
    const uint32_t e = (code >> 3) & 15u, m = code & 7u;
    const float mag = e ? ldexpf(1.0f + (float)m * 0.125f, (int)e - 7) : (float)m * 0.001953125f;
    return (code & 0x80u) ? -mag : mag;
}

// One block per row of the fp32 folded matrix: the smallest power of two 2^e with max|row| / 2^e <= 448,
// the row's e4m3 codes in that scale, and the stored values code * 2^e as bf16 (exactly representable)
__global__ void __launch_bounds__(kBlock)
wp_to_fp8_kernel(const float* __restrict__ acc, int64_t d, uint8_t* __restrict__ codes, float* __restrict__ scale,
                 bf16_t* __restrict__ Wp) {
    __shared__ float red[kBlock / TD_WAVE];
    const int64_t i = blockIdx.x;
    const float* row = acc + i * d;
    float m = 0.0f;
    for (int64_t k = threadIdx.x; k < d; k += kBlock) m = fmaxf(m, fabsf(row[k]));
    m = td_wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = m;
    __syncthreads();
    m = red[0];
#pragma unroll
    for (int w = 1; w < kBlock / TD_WAVE; ++w) m = fmaxf(m, red[w]);
    int e = 0;
    if (m > 0.0f && m < INFINITY) {
        int k;
        const float f = frexpf(m, &k);               // m = f 2^k, 0.5 <= f < 1; 448 = 0.875 * 2^9
        e = f <= 0.875f ? k - 9 : k - 8;
    }
    if (threadIdx.x == 0) scale[i] = ldexpf(1.0f, e);
    for (int64_t k = threadIdx.x; k < d; k += kBlock) {
        const uint32_t cde = f32_to_e4m3(ldexpf(row[k], -e));
        codes[i * d + k] = (uint8_t)cde;
        Wp[i * d + k] = td_f32_to_bf16(ldexpf(e4m3_to_f32(cde), e));
    }
}

// ------------------------------------------------- adaptive thresholding (Algorithm 1, outer loops)
// E_n = ||W2[:, n]||_2 * sum over the calibration inputs with lo_n <= z < hi_n of |sigma(z) - (a_n z + c_n)|:
// the section's per-neuron error metric err_n summed over the calibration set (outside the range
// the approximated activation equals the exact one).  One block per neuron, fp64 sums.
__global__ void __launch_bounds__(kBlock)
neuron_error_kernel(const float* __restrict__ Zt, int n, const float* __restrict__ lo, const float* __restrict__ hi,
                    const float* __restrict__ a, const float* __restrict__ c, const float* __restrict__ colnorm, int act,
                    float* __restrict__ err) {
    __shared__ double red[kBlock / TD_WAVE];
    const int64_t j = blockIdx.x;
    const float* z = Zt + j * (int64_t)n;
    const double l = (double)lo[j], r = (double)hi[j], aj = (double)a[j], cj = (double)c[j];
    double sum = 0.0;
    for (int i = threadIdx.x; i < n; i += kBlock) {
        const double zi = (double)z[i];
        if (zi >= l && zi < r) sum += fabs(td_act_f64(zi, act) - (aj * zi + cj));
    }
    sum = block_sum(sum, red);
    if (threadIdx.x == 0) err[j] = (float)(sum * (double)colnorm[j]);
}

// colnorm[j] = ||W2[:, j]||_2 for W2 stored d x h (thread per column, rows walked in order)
template <typename T>
__global__ void __launch_bounds__(kBlock)
col_norm_kernel(const T* __restrict__ W2, int64_t d, int64_t h, float* __restrict__ colnorm) {
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j >= h) return;
    double ss = 0.0;
    for (int64_t i = 0; i < d; ++i) {
        const double w = (double)td_load<T>(W2 + i * h + j);
        ss += w * w;
    }
    colnorm[j] = (float)sqrt(ss);
}

// out[0] = sum of v[0..n) in a fixed order (one block)
__global__ void __launch_bounds__(kBlock) sum_fixed_kernel(const float* __restrict__ v, int64_t n, float* __restrict__ out) {
    __shared__ double red[kBlock / TD_WAVE];
    double sum = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += kBlock) sum += (double)v[i];
    sum = block_sum(sum, red);
    if (threadIdx.x == 0) out[0] = (float)sum;
}

// Solution of   minimise sum E_i t_i,  sum t_i = t n,  t_min <= t_i <= t_max :
// the k = floor((n t_max - t n) / (t_max - t_min)) items of largest error (equal errors: lower index
// first) get t_min, the next one t_max minus the rest of the excess, all others t_max.  Thread i
// finds its own rank by counting (tiles of the errors staged in LDS).
__global__ void __launch_bounds__(kBlock)
assign_thresholds_kernel(const float* __restrict__ E, int64_t n, double t, double t_min, double t_max,
                         float* __restrict__ out) {
    __shared__ float tile[kBlock];
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const float mine = i < n ? E[i] : 0.0f;
    int64_t rank = 0;
    for (int64_t j0 = 0; j0 < n; j0 += kBlock) {
        __syncthreads();
        tile[threadIdx.x] = j0 + threadIdx.x < n ? E[j0 + threadIdx.x] : 0.0f;
        __syncthreads();
        const int lim = (int)(n - j0 < kBlock ? n - j0 : kBlock);
        for (int u = 0; u < lim; ++u) {
            const float other = tile[u];
            rank += (other > mine || (other == mine && j0 + u < i)) ? 1 : 0;
        }
    }
    if (i >= n) return;
    double v = t_max;
    if (t_max > t_min) {
        const double width = t_max - t_min;
        const double excess = (double)n * t_max - t * (double)n;
        double k = floor(excess / width);
        if (k > (double)n) k = (double)n;
        if ((double)rank < k) v = t_min;
        else if ((double)rank == k) v = t_max - (excess - k * width);
    }
    out[i] = (float)v;
}

// ------------------------------------------------- bound for the fixed-point repair accumulators
// For a token x and any set F of neurons, every partial sum of the terms that make up output i,
//     W'[i,:] x + b'_i      and      delta_j W2[i,j]  (j in F),
// is bounded in magnitude by  K1 max|x| + K2  with
//     K1 = max_i ( sum_k |W'_ik| + sum_j |W2_ij| (1 + |a_j|) ||W1_j||_1 )
//     K2 = max_i ( |b'_i|        + sum_j |W2_ij| ((1 + |a_j|) |b1_j| + |c_j|) )
// because |delta_j| = |sigma(z_j) - (a_j z_j + c_j)| <= (1 + |a_j|) |z_j| + |c_j| for every supported
// activation (|sigma(z)| <= |z|) and |z_j| <= ||W1_j||_1 max|x| + |b1_j|.
template <typename T>
__global__ void __launch_bounds__(kBlock)
fx_row_terms_kernel(const T* __restrict__ W1, const T* __restrict__ b1, const float* __restrict__ a,
                    const float* __restrict__ c, int64_t d, float* __restrict__ g, float* __restrict__ kk) {
    __shared__ float red[kBlock / TD_WAVE];
    const int64_t j = blockIdx.x;
    float sabs = 0.0f;
    for (int64_t k = threadIdx.x; k < d; k += kBlock) sabs += fabsf(td_load<T>(W1 + j * d + k));
    sabs = td_wave_sum(sabs);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sabs;
    __syncthreads();
    if (threadIdx.x == 0) {
        float tot = 0.0f;
        for (int w = 0; w < kBlock / TD_WAVE; ++w) tot += red[w];
        const float aj = 1.0f + fabsf(a[j]);
        g[j] = aj * tot;
        kk[j] = aj * (b1 ? fabsf(td_load<T>(b1 + j)) : 0.0f) + fabsf(c[j]);
    }
}

// P[(chunk * 2 + q) * d + i] = sum over the chunk's neurons j of |W2T[j][i]| * (q == 0 ? g_j : kk_j)
template <typename T>
__global__ void __launch_bounds__(kBlock)
fx_col_terms_kernel(const T* __restrict__ W2T, int64_t h, int64_t d, const float* __restrict__ g,
                    const float* __restrict__ kk, int64_t rows_per_chunk, float* __restrict__ P) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t ch = blockIdx.y;
    if (i >= d) return;
    const int64_t j0 = ch * rows_per_chunk, j1 = j0 + rows_per_chunk < h ? j0 + rows_per_chunk : h;
    float s1 = 0.0f, s2 = 0.0f;
    for (int64_t j = j0; j < j1; ++j) {
        const float w = fabsf(td_load<T>(W2T + j * d + i));
        s1 = fmaf(w, g[j], s1);
        s2 = fmaf(w, kk[j], s2);
    }
    P[(ch * 2 + 0) * d + i] = s1;
    P[(ch * 2 + 1) * d + i] = s2;
}

// out[0] = K1, out[1] = K2 (maxima over the outputs; non-negative floats order like their bit patterns)
template <typename T>
__global__ void __launch_bounds__(kBlock)
fx_bound_kernel(const T* __restrict__ Wp, const float* __restrict__ bp, int64_t d, const float* __restrict__ P,
                int chunks, float* __restrict__ out) {
    __shared__ float red[kBlock / TD_WAVE];
    const int64_t i = blockIdx.x;
    float sabs = 0.0f;
    for (int64_t k = threadIdx.x; k < d; k += kBlock) sabs += fabsf(td_load<T>(Wp + i * d + k));
    sabs = td_wave_sum(sabs);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sabs;
    __syncthreads();
    if (threadIdx.x == 0) {
        float k1 = 0.0f, k2 = fabsf(bp[i]);
        for (int w = 0; w < kBlock / TD_WAVE; ++w) k1 += red[w];
        for (int ch = 0; ch < chunks; ++ch) {
            k1 += P[((int64_t)ch * 2 + 0) * d + i];
            k2 += P[((int64_t)ch * 2 + 1) * d + i];
        }
        // a little above the fp32 value of the sums, so that their own rounding cannot undercut the bound
        atomicMax(reinterpret_cast<int*>(out), __float_as_int(k1 * 1.01f));
        atomicMax(reinterpret_cast<int*>(out) + 1, __float_as_int(k2 * 1.01f));
    }
}

struct DevBuf {  // frees on scope exit
    void* p = nullptr;
    ~DevBuf() {
        if (p) (void)hipFree(p);
    }
    tardis_status_t alloc(size_t bytes) {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
        if (e != hipSuccess) {
            p = nullptr;
            (void)hipGetLastError();
            return e == hipErrorOutOfMemory ? TARDIS_ERR_OOM : TARDIS_ERR_HIP;
        }
        return TARDIS_OK;
    }
};

dim3 tile_grid(int64_t cols, int64_t rows) { return dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)); }

}  // namespace

template <typename T>
static tardis_status_t fx_bounds_t(const tardis_layer_s* L, float* out2, hipStream_t s) {
    const int64_t d = L->d, h = L->h;
    const int chunks = 32;
    const int64_t rpc = (h + chunks - 1) / chunks;
    DevBuf g, kk, P;
    TD_TRY(g.alloc((size_t)h * 4));
    TD_TRY(kk.alloc((size_t)h * 4));
    TD_TRY(P.alloc((size_t)chunks * 2 * d * 4));
    TD_HIP(hipMemsetAsync(out2, 0, 8, s));
    hipLaunchKernelGGL(fx_row_terms_kernel<T>, dim3((unsigned)h), dim3(kBlock), 0, s, static_cast<const T*>(L->W1),
                       static_cast<const T*>(L->b1), L->a, L->c, d, static_cast<float*>(g.p), static_cast<float*>(kk.p));
    hipLaunchKernelGGL(fx_col_terms_kernel<T>, dim3((unsigned)((d + kBlock - 1) / kBlock), chunks), dim3(kBlock), 0, s,
                       static_cast<const T*>(L->W2T), h, d, static_cast<const float*>(g.p),
                       static_cast<const float*>(kk.p), rpc, static_cast<float*>(P.p));
    hipLaunchKernelGGL(fx_bound_kernel<T>, dim3((unsigned)d), dim3(kBlock), 0, s, static_cast<const T*>(L->Wp), L->bp, d,
                       static_cast<const float*>(P.p), chunks, out2);
    TD_HIP(hipGetLastError());
    TD_HIP(hipStreamSynchronize(s));   // the temporaries go out of scope
    return TARDIS_OK;
}

tardis_status_t td_estimate_errors(const tardis_ffn_desc* desc, const void* X, int64_t n, const float* lo,
                                   const float* hi, const float* a, const float* c, float* err, float* err_layer,
                                   hipStream_t s) {
    const int64_t d = desc->d, h = desc->h;
    DevBuf zt, cn;
    TD_TRY(zt.alloc((size_t)h * n * 4));
    TD_TRY(cn.alloc((size_t)h * 4));
    TD_TRY(td_gemm_nt(desc->W1, X, static_cast<float*>(zt.p), h, n, d, desc->dtype, 0, desc->b1, s));
    const dim3 cgrid((unsigned)((h + kBlock - 1) / kBlock));
    if (desc->dtype == TARDIS_BF16)
        hipLaunchKernelGGL(col_norm_kernel<bf16_t>, cgrid, dim3(kBlock), 0, s, static_cast<const bf16_t*>(desc->W2), d, h,
                           static_cast<float*>(cn.p));
    else
        hipLaunchKernelGGL(col_norm_kernel<float>, cgrid, dim3(kBlock), 0, s, static_cast<const float*>(desc->W2), d, h,
                           static_cast<float*>(cn.p));
    hipLaunchKernelGGL(neuron_error_kernel, dim3((unsigned)h), dim3(kBlock), 0, s, static_cast<const float*>(zt.p), (int)n,
                       lo, hi, a, c, static_cast<const float*>(cn.p), (int)desc->act, err);
    if (err_layer) hipLaunchKernelGGL(sum_fixed_kernel, dim3(1), dim3(kBlock), 0, s, err, h, err_layer);
    TD_HIP(hipGetLastError());
    TD_HIP(hipStreamSynchronize(s));
    return TARDIS_OK;
}

tardis_status_t td_assign_thresholds(const float* err, int64_t n, float t, float t_min, float t_max, float* out,
                                     hipStream_t s) {
    hipLaunchKernelGGL(assign_thresholds_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, err, n,
                       (double)t, (double)t_min, (double)t_max, out);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

// K1, K2 of the fixed-point accumulators' magnitude bound into out2[0..1] (device); needs W2T, W', b', a, c
tardis_status_t td_fx_bounds(const tardis_layer_s* L, float* out2, hipStream_t s) {
    return L->dtype == TARDIS_BF16 ? fx_bounds_t<bf16_t>(L, out2, s) : fx_bounds_t<float>(L, out2, s);
}

tardis_status_t td_transpose(const void* src, void* dst, int64_t rows, int64_t cols, int32_t dtype, hipStream_t s) {
    if ((rows + 31) / 32 > 65535) return TARDIS_ERR_SHAPE;
    if (dtype == TARDIS_BF16)
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, tile_grid(cols, rows), dim3(256), 0, s,
                           static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), rows, cols);
    else
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, tile_grid(cols, rows), dim3(256), 0, s,
                           static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst), rows, cols);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

tardis_status_t td_build_sketch(const void* W1, const void* b1, const float* lo, const float* hi, int64_t h,
                                int64_t d, int32_t dtype, int32_t bits, float margin, int8_t* Q, uint8_t* Q4,
                                uint8_t* M4, float* tlo, float* thi, hipStream_t s) {
    if (bits == 4 || bits == 3 || bits == 2) {
        const int qmax = (1 << (bits - 1)) - 1;
        const int64_t ng = (d + 31) / 32;
        if (!M4 || (Q4 && d % 32 != 0) || ng * 4 > 64 * 1024) return TARDIS_ERR_SHAPE;
        if (dtype == TARDIS_BF16)
            hipLaunchKernelGGL(sketch4_kernel<bf16_t>, dim3((unsigned)h), dim3(kBlock), (size_t)ng * 4, s,
                               static_cast<const bf16_t*>(W1), static_cast<const bf16_t*>(b1), lo, hi, d, (int)ng,
                               Q, Q4, M4, tlo, thi, qmax, margin);
        else
            hipLaunchKernelGGL(sketch4_kernel<float>, dim3((unsigned)h), dim3(kBlock), (size_t)ng * 4, s,
                               static_cast<const float*>(W1), static_cast<const float*>(b1), lo, hi, d, (int)ng,
                               Q, Q4, M4, tlo, thi, qmax, margin);
        TD_HIP(hipGetLastError());
        return TARDIS_OK;
    }
    if (bits != 8 || !Q) return TARDIS_ERR_INVALID_ARG;
    if (dtype == TARDIS_BF16)
        hipLaunchKernelGGL(sketch_kernel<bf16_t>, dim3((unsigned)h), dim3(kBlock), 0, s,
                           static_cast<const bf16_t*>(W1), static_cast<const bf16_t*>(b1), lo, hi, d, Q, tlo, thi, margin);
    else
        hipLaunchKernelGGL(sketch_kernel<float>, dim3((unsigned)h), dim3(kBlock), 0, s,
                           static_cast<const float*>(W1), static_cast<const float*>(b1), lo, hi, d, Q, tlo, thi, margin);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

tardis_status_t td_unpack_sketch4(const uint8_t* Q4, const uint8_t* M4, int64_t h, int64_t d, int8_t* Q,
                                  hipStream_t s) {
    hipLaunchKernelGGL(unpack_sketch4_kernel, dim3((unsigned)h), dim3(kBlock), 0, s, Q4, M4, d, Q);
    TD_HIP(hipGetLastError());
    return TARDIS_OK;
}

tardis_status_t td_fold(const tardis_ffn_desc* desc, const float* a, const float* c, void* Wp, float* bp,
                        uint8_t* Wp8, float* wp8_scale, hipStream_t s) {
    if (Wp8 && desc->dtype != TARDIS_BF16) return TARDIS_ERR_DTYPE;
    const int64_t d = desc->d, h = desc->h;
    if ((h + 31) / 32 > 65535 || (d + 31) / 32 > 65535) return TARDIS_ERR_SHAPE;
    if (desc->dtype == TARDIS_BF16) {
        DevBuf phi, plo, acc;
        TD_TRY(phi.alloc((size_t)d * h * 2));
        TD_TRY(plo.alloc((size_t)d * h * 2));
        TD_TRY(acc.alloc((size_t)d * d * 4));
        hipLaunchKernelGGL(scale_transpose_bf16_kernel, tile_grid(d, h), dim3(256), 0, s,
                           static_cast<const bf16_t*>(desc->W1), a, static_cast<bf16_t*>(phi.p),
                           static_cast<bf16_t*>(plo.p), h, d);
        TD_TRY(td_gemm_nt(desc->W2, phi.p, static_cast<float*>(acc.p), d, d, h, TARDIS_BF16, 0, nullptr, s));
        TD_TRY(td_gemm_nt(desc->W2, plo.p, static_cast<float*>(acc.p), d, d, h, TARDIS_BF16, 1, nullptr, s));
        const int64_t n = d * d;
        if (Wp8)
            hipLaunchKernelGGL(wp_to_fp8_kernel, dim3((unsigned)d), dim3(kBlock), 0, s, static_cast<const float*>(acc.p),
                               d, Wp8, wp8_scale, static_cast<bf16_t*>(Wp));
        else
            hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                               static_cast<const float*>(acc.p), static_cast<bf16_t*>(Wp), n);
        hipLaunchKernelGGL(fold_bias_kernel<bf16_t>, dim3((unsigned)d), dim3(kBlock), 0, s,
                           static_cast<const bf16_t*>(desc->W2), static_cast<const bf16_t*>(desc->b1),
                           static_cast<const bf16_t*>(desc->b2), a, c, bp, d, h);
        TD_HIP(hipGetLastError());
        TD_HIP(hipStreamSynchronize(s));  // temporaries are freed on return
    } else {
        DevBuf p;
        TD_TRY(p.alloc((size_t)d * h * 4));
        hipLaunchKernelGGL(scale_transpose_f32_kernel, tile_grid(d, h), dim3(256), 0, s,
                           static_cast<const float*>(desc->W1), a, static_cast<float*>(p.p), h, d);
        TD_TRY(td_gemm_nt(desc->W2, p.p, static_cast<float*>(Wp), d, d, h, TARDIS_F32, 0, nullptr, s));
        hipLaunchKernelGGL(fold_bias_kernel<float>, dim3((unsigned)d), dim3(kBlock), 0, s,
                           static_cast<const float*>(desc->W2), static_cast<const float*>(desc->b1),
                           static_cast<const float*>(desc->b2), a, c, bp, d, h);
        TD_HIP(hipGetLastError());
        TD_HIP(hipStreamSynchronize(s));
    }
    return TARDIS_OK;
}

tardis_status_t td_calibrate(const tardis_ffn_desc* desc, const void* X, int64_t n, float coverage,
                             const float* cov_pn, float step, float* lo, float* hi, float* a, float* c,
                             hipStream_t s) {
    const int64_t d = desc->d, h = desc->h;
    DevBuf zt;
    TD_TRY(zt.alloc((size_t)h * n * 4));
    TD_TRY(td_gemm_nt(desc->W1, X, static_cast<float*>(zt.p), h, n, d, desc->dtype, 0, desc->b1, s));
    int npad = 2;
    while (npad < n) npad <<= 1;
    if (step > 0.0f) {   // greedy range search instead of central quantiles
        const size_t lds = (size_t)((n + 1) & ~(int64_t)1) * sizeof(double) + (size_t)npad * sizeof(float);
        if (lds > 48 * 1024)
            TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(range_search_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        DevBuf capped;
        TD_TRY(capped.alloc(sizeof(int)));
        TD_HIP(hipMemsetAsync(capped.p, 0, sizeof(int), s));
        hipLaunchKernelGGL(range_search_kernel, dim3((unsigned)h), dim3(kBlock), lds, s,
                           static_cast<const float*>(zt.p), (int)n, npad, coverage, cov_pn, step, (int)desc->act, lo,
                           hi, a, c, static_cast<int*>(capped.p));
        TD_HIP(hipGetLastError());
        int n_capped = 0;
        TD_HIP(hipMemcpyAsync(&n_capped, capped.p, sizeof(int), hipMemcpyDeviceToHost, s));
        TD_HIP(hipStreamSynchronize(s));
        // Algorithm 1 has no limit on the number of growth steps; the kernel's guard (4096) is only
        // reached when `step` is absurdly small against a neuron's spread of inputs: refuse, do not
        // substitute another range
        return n_capped > 0 ? TARDIS_ERR_INVALID_ARG : TARDIS_OK;
    }
    const size_t lds = (size_t)npad * sizeof(float);
    if (lds > 48 * 1024)
        TD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(calibrate_neuron_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(calibrate_neuron_kernel, dim3((unsigned)h), dim3(kBlock), lds, s,
                       static_cast<const float*>(zt.p), (int)n, npad, coverage, cov_pn, (int)desc->act, lo, hi, a, c);
    TD_HIP(hipGetLastError());
    TD_HIP(hipStreamSynchronize(s));
    return TARDIS_OK;
}
