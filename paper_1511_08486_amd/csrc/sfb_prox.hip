// The proximal step of proximal SGD (Section 2.1): after W <- W - eta dW the operator
// prox_{eta h} is applied to W.  The regularisers of Section 2 with an entrywise or columnwise
// closed form:
//   squared l2   h = lam/2 ||W||_F^2                 W <- W / (1 + eta lam)
//   l1           h = lam ||W||_1                     W <- sign(w) max(|w| - eta lam, 0)
//   column ball  h = indicator{||W_k||_2 <= r}       W_k <- W_k min(1, r / ||W_k||_2)
//                (sparse coding, Section 2: every column of the dictionary inside the ball)
// All of it is HBM-bound streaming over W: one read and one write of J*D floats for the
// entrywise ones; the column projection reads W once for the column sums of squares and, only
// for the columns that are outside the ball, once more to rescale them.
//
// A workgroup owns kProxCols consecutive columns (one 128-bit item per thread, so a wavefront
// reads whole 1 KB row segments) and a chunk of rows; the column sums of squares go to
// partial[chunk][column] and are added up in a fixed order by a second kernel, so the result
// does not depend on the order workgroups happen to run in.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kProxThreads = 256;
constexpr int kProxCols = kProxThreads * 4;

// Rows per workgroup: enough workgroups to fill the part several times over, at most 256 row
// chunks (which bounds the partial sums at 256 rows of D floats).
int prox_rows_per_chunk(int64_t J, int64_t D) {
    const int64_t col_blocks = (D + kProxCols - 1) / kProxCols;
    int64_t rc = J * col_blocks / 2048;
    if (rc < 4) rc = 4;
    const int64_t floor_rc = (J + 255) / 256;
    if (rc < floor_rc) rc = floor_rc;
    return (int)rc;
}

size_t prox_workspace(int64_t J, int64_t D) {
    const int64_t rc = prox_rows_per_chunk(J, D);
    const int64_t chunks = (J + rc - 1) / rc;
    const int64_t ldp = (D + 3) / 4 * 4;
    return (size_t)(chunks + 1) * ldp * sizeof(float);     // partial sums, then one row of scale factors
}

__device__ __forceinline__ f32x4 prox_load(const float* row, int col, int D, bool vec) {
    if (vec && col + 3 < D) return *reinterpret_cast<const f32x4*>(row + col);
    f32x4 v{0.f, 0.f, 0.f, 0.f};
    if (col + 0 < D) v.x = row[col + 0];
    if (col + 1 < D) v.y = row[col + 1];
    if (col + 2 < D) v.z = row[col + 2];
    if (col + 3 < D) v.w = row[col + 3];
    return v;
}

// KIND 1: w * a (a = 1 / (1 + eta lam));  KIND 2: soft threshold at a = eta lam
template <int KIND>
__global__ __launch_bounds__(kProxThreads) void prox_entry_kernel(float* __restrict__ W, int64_t ldw, int J, int D,
                                                                  int rows_per_chunk, float a, bool vec) {
    const int col = blockIdx.x * kProxCols + threadIdx.x * 4;
    if (col >= D) return;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(J, r0 + rows_per_chunk);
    constexpr int UN = 4;                                  // rows in flight per thread
    for (int r = r0; r < r1; r += UN) {
        f32x4 v[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) v[i] = prox_load(W + (int64_t)min(r + i, r1 - 1) * ldw, col, D, vec);
#pragma unroll
        for (int i = 0; i < UN; ++i) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[i][e] = prox_entry(v[i][e], KIND, a);
            }
            if (r + i < r1) store4(W + (int64_t)(r + i) * ldw, col, D, vec, v[i]);
        }
    }
}

__global__ __launch_bounds__(kProxThreads) void column_sumsq_kernel(const float* __restrict__ W, int64_t ldw, int J,
                                                                    int D, int rows_per_chunk,
                                                                    float* __restrict__ partial, int64_t ldp, bool vec) {
    const int col = blockIdx.x * kProxCols + threadIdx.x * 4;
    if (col >= D) return;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(J, r0 + rows_per_chunk);
    constexpr int UN = 4;
    f32x4 acc{0.f, 0.f, 0.f, 0.f};
    for (int r = r0; r < r1; r += UN) {
        f32x4 v[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) v[i] = prox_load(W + (int64_t)min(r + i, r1 - 1) * ldw, col, D, vec);
#pragma unroll
        for (int i = 0; i < UN; ++i)
            if (r + i < r1) acc += v[i] * v[i];
    }
    // ldp is a multiple of 4 and the base is 16-byte aligned: the item is always in bounds
    *reinterpret_cast<f32x4*>(partial + (int64_t)blockIdx.y * ldp + col) = acc;
}

// scale[k] = min(1, r / ||W_k||).  64 columns per workgroup; wavefront g adds the chunks
// g, g + 4, g + 8, ... in that order (independent loads, several in flight), and the four sums
// are combined as (s0 + s1) + (s2 + s3): a fixed order, whatever the launch does.
__global__ __launch_bounds__(kProxThreads) void column_scale_kernel(const float* __restrict__ partial, int64_t ldp,
                                                                    int chunks, int D, float radius,
                                                                    float* __restrict__ scale) {
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + lane;
    const int kk = k < D ? k : D - 1;
    float s = 0.f;
#pragma unroll 8
    for (int c = g; c < chunks; c += 4) s += partial[(int64_t)c * ldp + kk];
    part[g][lane] = s;
    __syncthreads();
    if (g == 0 && k < D) {
        const float sum = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
        const float norm = sqrtf(sum);
        scale[k] = norm > radius ? radius / norm : 1.0f;
    }
}

__global__ __launch_bounds__(kProxThreads) void column_rescale_kernel(float* __restrict__ W, int64_t ldw, int J, int D,
                                                                      int rows_per_chunk,
                                                                      const float* __restrict__ scale, bool vec) {
    const int col = blockIdx.x * kProxCols + threadIdx.x * 4;
    if (col >= D) return;
    // the scale row is padded to a multiple of 4 floats; entries at or beyond D are never used
    const f32x4 s = *reinterpret_cast<const f32x4*>(scale + col);
    const bool inside = (s.x == 1.0f || col + 0 >= D) && (s.y == 1.0f || col + 1 >= D) &&
                        (s.z == 1.0f || col + 2 >= D) && (s.w == 1.0f || col + 3 >= D);
    if (inside) return;                                   // nothing to do for columns inside the ball
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(J, r0 + rows_per_chunk);
    constexpr int UN = 4;
    for (int r = r0; r < r1; r += UN) {
        f32x4 v[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) v[i] = prox_load(W + (int64_t)min(r + i, r1 - 1) * ldw, col, D, vec);
#pragma unroll
        for (int i = 0; i < UN; ++i)
            if (r + i < r1) store4(W + (int64_t)(r + i) * ldw, col, D, vec, v[i] * s);
    }
}

hipError_t launch_prox(const ProxArgs& a, void* workspace, hipStream_t s) {
    const int rc = prox_rows_per_chunk(a.J, a.D);
    const int chunks = (a.J + rc - 1) / rc;
    const dim3 grid((a.D + kProxCols - 1) / kProxCols, chunks);
    const bool vec = ((uintptr_t)a.w % 16) == 0 && (a.ldw % 4) == 0;
    switch (a.kind) {
        case 0: return hipSuccess;
        case 1:
            SFB_LAUNCH(prox_entry_kernel<1>, grid, dim3(kProxThreads), 0, s, a.w, a.ldw, a.J, a.D, rc,
                       1.0f / (1.0f + a.eta * a.param), vec);
            return hipGetLastError();
        case 2:
            SFB_LAUNCH(prox_entry_kernel<2>, grid, dim3(kProxThreads), 0, s, a.w, a.ldw, a.J, a.D, rc, a.eta * a.param,
                       vec);
            return hipGetLastError();
        case 3: {
            const int64_t ldp = ((int64_t)a.D + 3) / 4 * 4;
            float* partial = (float*)workspace;
            float* scale = partial + (int64_t)chunks * ldp;
            // the timed kernel of this family: it always makes its full pass over W
            SFB_LAUNCH(column_sumsq_kernel, grid, dim3(kProxThreads), 0, s, (const float*)a.w, a.ldw, a.J, a.D, rc,
                       partial, ldp, vec);
            hipLaunchKernelGGL(column_scale_kernel, dim3((a.D + 63) / 64), dim3(kProxThreads), 0,
                               s, (const float*)partial, ldp, chunks, a.D, a.param, scale);
            hipLaunchKernelGGL(column_rescale_kernel, grid, dim3(kProxThreads), 0, s, a.w, a.ldw, a.J, a.D, rc,
                               (const float*)scale, vec);
            return hipGetLastError();
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace sfb
