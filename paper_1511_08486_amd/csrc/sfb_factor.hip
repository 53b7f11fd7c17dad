// Factor u of Section 2.1: u_i = d f_i(z_i) / d z_i, one row of scores at a time.
//
// The scores arrive as split-K partial sums; this kernel adds the slices in slice order,
// keeps the row in registers, and makes a single pass over memory:
//   MLR    row max, row sum of exp (wavefront / workgroup reductions), u = softmax - e_y,
//          f = logsumexp(z) - z_y
//   DML    row sum of squares q, u = c z with c = 2 (similar) or -2 [q < 1] (dissimilar),
//          f = q or max(0, 1 - q)                         (Section 2, DML paragraph)
//   L2SVM  t_j = +-1, h = max(0, 1 - t_j z_j), u_j = -2 t_j h, f = sum_j h^2
// Memory-bound: reads split_k * J and writes J floats per row.
//
// SDCA (Section 2.1, "Stochastic DCA") on the logistic loss reuses the MLR row: with
// r = softmax - e_y (so that -r is the dual vector that is optimal for these scores) and the
// sample's dual vector u, the factor that is broadcast is delta u = s (u + r), the dual
// vector becomes u - delta u, and f*(-u) = sum_j p_j log p_j with p = e_y - u.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kFactorThreads = 256;

// GROUP threads cooperate on one row (64 = one wavefront, 256 = the workgroup).
template <int GROUP>
__device__ __forceinline__ float group_sum(float v, float* red) {
    v = wave_sum(v);
    if (GROUP == 64) return v;
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}
template <int GROUP>
__device__ __forceinline__ float group_max(float v, float* red) {
    v = wave_max(v);
    if (GROUP == 64) return v;
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ f32x4 load4_guarded(const float* row, int col, int ncols, bool vec) {
    if (vec && col + 3 < ncols) return *reinterpret_cast<const f32x4*>(row + col);
    f32x4 v{0.f, 0.f, 0.f, 0.f};
    if (col + 0 < ncols) v.x = row[col + 0];
    if (col + 1 < ncols) v.y = row[col + 1];
    if (col + 2 < ncols) v.z = row[col + 2];
    if (col + 3 < ncols) v.w = row[col + 3];
    return v;
}

// R = 128-bit items per thread held in registers: covers J <= GROUP * 4 * R.
template <int MODEL, int GROUP, int R, bool SDCA>
__global__ __launch_bounds__(kFactorThreads) void factor_u_kernel(
    const float* __restrict__ Zp, int64_t ldz, int64_t zstride, int split_k, const int32_t* __restrict__ y,
    float* __restrict__ U, int64_t ldu, float* __restrict__ loss, int n_rows, int J, bool vec_u, SdcaDev sd) {
    static_assert(!SDCA || MODEL == kMLR, "the dual update is defined for the logistic loss only");
    __shared__ float red[4];
    constexpr int ROWS = kFactorThreads / GROUP;
    const int t = threadIdx.x % GROUP;
    // GROUP == 256: the whole workgroup shares `row`, so the barriers inside the
    // reductions are reached by all threads or by none.
    const int row = blockIdx.x * ROWS + threadIdx.x / GROUP;
    const bool live = row < n_rows;
    const int rr = live ? row : 0;
    const int label = y[rr];

    // Sum the split-K slices in slice order.  The slice loop is outermost and unrolled so
    // that several independent loads are in flight per thread; out-of-range items are
    // clamped to column 0 (always valid) and discarded.
    f32x4 z[R];
#pragma unroll
    for (int r = 0; r < R; ++r) z[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float* zrow = Zp + (int64_t)rr * ldz;       // ldz is a multiple of 4, base 16-byte aligned
#pragma unroll 4
    for (int k = 0; k < split_k; ++k) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int col = 4 * (t + GROUP * r);
            // a row of the workspace is padded to a multiple of 4 floats, so the whole
            // 128-bit item is in bounds; elements at or beyond J are garbage and every
            // use below masks them
            const f32x4 v = ldg4(zrow + (int64_t)k * zstride + (col < J ? col : 0));
            z[r] += (col < J) ? v : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    if (!live) {
#pragma unroll
        for (int r = 0; r < R; ++r) z[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    float f = 0.f;
    if (MODEL == kMLR) {
        float m = -INFINITY;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * (t + GROUP * r) + e < J) m = fmaxf(m, z[r][e]);
        m = group_max<GROUP>(m, red);
        float sum = 0.f, zy = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = 4 * (t + GROUP * r) + e;
                if (col == label) zy = z[r][e];
                const float ex = col < J ? __expf(z[r][e] - m) : 0.f;
                z[r][e] = ex;
                sum += ex;
            }
        sum = group_sum<GROUP>(sum, red);
        zy = group_sum<GROUP>(zy, red);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = 4 * (t + GROUP * r) + e;
                z[r][e] = z[r][e] * inv - (col == label ? 1.0f : 0.0f);
            }
        f = m + __logf(sum) - zy;
        if (SDCA) {
            const int si = live ? sd.sample[row] : 0;
            float* drow = sd.dual + (int64_t)si * sd.ldd;
            float cj = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int col = 4 * (t + GROUP * r);
                f32x4 dv = load4_guarded(drow, col < J ? col : 0, J, sd.vec);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float du = sd.frac * (dv[e] + z[r][e]);
                    dv[e] -= du;
                    z[r][e] = du;
                    const float pj = ((col + e == label) ? 1.0f : 0.0f) - dv[e];
                    cj += (col + e < J && pj > 0.f) ? pj * __logf(pj) : 0.f;
                }
                if (live && col < J) store4(drow, col, J, sd.vec, dv);
            }
            cj = group_sum<GROUP>(cj, red);
            if (live && sd.conj != nullptr && t == 0) sd.conj[si] = cj;
        }
    } else if (MODEL == kDML) {
        float q = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) q += (4 * (t + GROUP * r) + e < J) ? z[r][e] * z[r][e] : 0.f;
        q = group_sum<GROUP>(q, red);
        const float c = (label != 0) ? 2.0f : (q < 1.0f ? -2.0f : 0.0f);
#pragma unroll
        for (int r = 0; r < R; ++r) z[r] *= c;
        f = (label != 0) ? q : fmaxf(0.f, 1.0f - q);
    } else {
        float hs = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = 4 * (t + GROUP * r) + e;
                const float tj = (col == label) ? 1.0f : -1.0f;
                const float h = col < J ? fmaxf(0.f, 1.0f - tj * z[r][e]) : 0.f;
                z[r][e] = -2.0f * tj * h;
                hs += h * h;
            }
        f = group_sum<GROUP>(hs, red);
    }

    if (live) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int col = 4 * (t + GROUP * r);
            if (col < J) store4(U + (int64_t)row * ldu, col, J, vec_u, z[r]);
        }
        if (loss != nullptr && t == 0) loss[row] = f;
    }
}

// Any J: three passes over the row's partial sums (they sit in L2 after the contraction).
template <int MODEL, bool SDCA>
__global__ __launch_bounds__(kFactorThreads) void factor_u_long_kernel(
    const float* __restrict__ Zp, int64_t ldz, int64_t zstride, int split_k, const int32_t* __restrict__ y,
    float* __restrict__ U, int64_t ldu, float* __restrict__ loss, int n_rows, int J, SdcaDev sd) {
    static_assert(!SDCA || MODEL == kMLR, "the dual update is defined for the logistic loss only");
    __shared__ float red[4];
    const int row = blockIdx.x;      // grid = n_rows exactly
    const int t = threadIdx.x;
    const int label = y[row];
    const float* p = Zp + (int64_t)row * ldz;
    auto zval = [&](int col) {
        float s = 0.f;
        for (int k = 0; k < split_k; ++k) s += p[(int64_t)k * zstride + col];
        return s;
    };
    float f = 0.f;
    if (MODEL == kMLR) {
        float m = -INFINITY;
        for (int col = t; col < J; col += kFactorThreads) m = fmaxf(m, zval(col));
        m = group_max<256>(m, red);
        float sum = 0.f;
        for (int col = t; col < J; col += kFactorThreads) sum += __expf(zval(col) - m);
        sum = group_sum<256>(sum, red);
        const float inv = 1.0f / sum;
        float zy = 0.f, cj = 0.f;
        const int si = SDCA ? sd.sample[row] : 0;
        for (int col = t; col < J; col += kFactorThreads) {
            const float zc = zval(col);
            if (col == label) zy = zc;
            float r = __expf(zc - m) * inv - (col == label ? 1.0f : 0.0f);
            if (SDCA) {
                float* d = sd.dual + (int64_t)si * sd.ldd + col;
                const float dv = *d;
                r = sd.frac * (dv + r);
                *d = dv - r;
                const float pj = (col == label ? 1.0f : 0.0f) - (dv - r);
                cj += pj > 0.f ? pj * __logf(pj) : 0.f;
            }
            U[(int64_t)row * ldu + col] = r;
        }
        zy = group_sum<256>(zy, red);
        f = m + __logf(sum) - zy;
        if (SDCA) {
            cj = group_sum<256>(cj, red);
            if (sd.conj != nullptr && t == 0) sd.conj[si] = cj;
        }
    } else if (MODEL == kDML) {
        float q = 0.f;
        for (int col = t; col < J; col += kFactorThreads) {
            const float zc = zval(col);
            q += zc * zc;
        }
        q = group_sum<256>(q, red);
        const float c = (label != 0) ? 2.0f : (q < 1.0f ? -2.0f : 0.0f);
        for (int col = t; col < J; col += kFactorThreads) U[(int64_t)row * ldu + col] = c * zval(col);
        f = (label != 0) ? q : fmaxf(0.f, 1.0f - q);
    } else {
        float hs = 0.f;
        for (int col = t; col < J; col += kFactorThreads) {
            const float tj = (col == label) ? 1.0f : -1.0f;
            const float h = fmaxf(0.f, 1.0f - tj * zval(col));
            U[(int64_t)row * ldu + col] = -2.0f * tj * h;
            hs += h * h;
        }
        f = group_sum<256>(hs, red);
    }
    if (loss != nullptr && t == 0) loss[row] = f;
}

template <int MODEL, bool SDCA>
static hipError_t launch_factor_m(const FactorArgs& a, hipStream_t s) {
    const bool vec_u = ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0;
#define SFB_FACTOR_LAUNCH(GROUP, R)                                                                     \
    SFB_LAUNCH((factor_u_kernel<MODEL, GROUP, R, SDCA>),                                                \
                       dim3((a.n_rows + (kFactorThreads / GROUP) - 1) / (kFactorThreads / GROUP)),      \
                       dim3(kFactorThreads), 0, s, a.zp, a.ldz, a.zstride, a.split_k, a.y, a.u, a.ldu,  \
                       a.loss, a.n_rows, a.J, vec_u, a.sdca)
    if (a.J <= 64 * 4 * 1) SFB_FACTOR_LAUNCH(64, 1);
    else if (a.J <= 256 * 4 * 1) SFB_FACTOR_LAUNCH(256, 1);
    else if (a.J <= 256 * 4 * 4) SFB_FACTOR_LAUNCH(256, 4);
    else if (a.J <= 256 * 4 * 12) SFB_FACTOR_LAUNCH(256, 12);
    else
        SFB_LAUNCH((factor_u_long_kernel<MODEL, SDCA>), dim3(a.n_rows), dim3(kFactorThreads), 0, s, a.zp,
                           a.ldz, a.zstride, a.split_k, a.y, a.u, a.ldu, a.loss, a.n_rows, a.J, a.sdca);
#undef SFB_FACTOR_LAUNCH
    return hipGetLastError();
}

hipError_t launch_factor(const FactorArgs& a, hipStream_t s) {
    if (a.sdca.dual != nullptr) return a.model == kMLR ? launch_factor_m<kMLR, true>(a, s) : hipErrorInvalidValue;
    switch (a.model) {
        case kMLR: return launch_factor_m<kMLR, false>(a, s);
        case kDML: return launch_factor_m<kDML, false>(a, s);
        case kL2SVM: return launch_factor_m<kL2SVM, false>(a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sfb
