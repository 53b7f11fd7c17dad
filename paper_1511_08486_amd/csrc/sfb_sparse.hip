// Sparse-feature helpers for the L2-SVM workload (the paper exploits sparse features to
// cut computation, Section 6): v_i = a_i is delivered as the dense row of the CSR matrix,
// because the reconstruction consumes V as a dense [N][D] operand.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kDensifyThreads = 256;

// One workgroup per sample: zero the row with wide stores, then scatter the stored
// entries.  The barrier orders the two phases inside the workgroup, and no other
// workgroup touches this row.
__global__ __launch_bounds__(kDensifyThreads) void csr_densify_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ col, const float* __restrict__ val,
    float* __restrict__ V, int64_t ldv, int D, int64_t nnz, bool vec_v) {
    const int row = blockIdx.x;
    float* out = V + (int64_t)row * ldv;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int c = 4 * threadIdx.x; c < D; c += 4 * kDensifyThreads) store4(out, c, D, vec_v, zero);
    __syncthreads();
    // a row pointer outside [0, nnz] is a caller error; clamp so that no access leaves the arrays
    const int64_t beg = max(0, rowptr[row]);
    const int64_t end = min((int64_t)rowptr[row + 1], nnz);
    for (int64_t n = beg + threadIdx.x; n < end; n += kDensifyThreads) {
        const int c = col[n];
        if (c >= 0 && c < D) out[c] = val[n];
    }
}

hipError_t launch_csr_densify(const DensifyArgs& a, hipStream_t s) {
    const bool vec_v = ((uintptr_t)a.v % 16) == 0 && (a.ldv % 4) == 0;
    hipLaunchKernelGGL(csr_densify_kernel, dim3(a.n_rows), dim3(kDensifyThreads), 0, s, a.rowptr, a.col,
                       a.val, a.v, a.ldv, a.D, a.nnz, vec_v);
    return hipGetLastError();
}

}  // namespace sfb

namespace sfb {

// Plain streaming copy: the yardstick for "what does a kernel that only moves bytes reach
// on this part", and the known-size kernel the HBM traffic counters are calibrated on.
__global__ __launch_bounds__(256) void stream_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                          int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_copy(const void* src, void* dst, int64_t bytes, hipStream_t s) {
    const int64_t n16 = bytes / 16;
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const f32x4*)src, (f32x4*)dst,
                       n16);
    return hipGetLastError();
}

}  // namespace sfb
