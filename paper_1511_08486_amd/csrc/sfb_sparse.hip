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
    SFB_LAUNCH(csr_densify_kernel, dim3(a.n_rows), dim3(kDensifyThreads), 0, s, a.rowptr, a.col,
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
    SFB_LAUNCH(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const f32x4*)src, (f32x4*)dst,
                       n16);
    return hipGetLastError();
}

}  // namespace sfb

namespace sfb {

// ---------------------------------------------------------------------------------------
// Scores for CSR features: z_i[j] = sum over the stored entries (c, v) of sample i of
// v * W[j][c]  (problem (P) with sparse a_i; the paper's implementation exploits feature
// sparsity the same way, Section 6).  W is row-major, so one sample touches a strided
// column of every W row; instead of gathering from HBM, a workgroup parks four W rows in
// LDS, interleaved as [column][4 rows], and streams every sample of the batch past them:
// one 128-bit LDS read per stored entry yields the four products' operands.  Lanes run
// over the entries of one sample (coalesced col/val reads); the four partial sums are
// reduced across the wavefront with a halving butterfly (7 shuffles instead of 24).
// Work: 2 * nnz * J flops; W is read once from HBM, the CSR arrays J/4 times from L2.
// ---------------------------------------------------------------------------------------
constexpr int kSpRows = 4;
constexpr int kSpThreads = 1024;   // 16 wavefronts share the parked rows: 4 per SIMD hide L2 latency
constexpr int kSpBatch = 4;        // consecutive samples a wavefront has in flight at once
constexpr int kSpPre = 3;          // 64-entry slabs per sample whose loads are issued up front

__global__ __launch_bounds__(kSpThreads) void csr_scores_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ col, const float* __restrict__ val, int64_t nnz,
    const float* __restrict__ W, int64_t ldw, float* __restrict__ Z, int64_t ldz, int n_rows, int J, int D,
    bool vec_w) {
    extern __shared__ __attribute__((aligned(16))) float wcols[];   // [D][4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = kSpThreads / 64;
    const int j0 = blockIdx.x * kSpRows;
    if (nnz <= 0) {   // nothing stored: every score is 0 (and col / val may be null)
        for (int i = tid; i < n_rows * kSpRows; i += kSpThreads) {
            const int r = i % kSpRows;
            if (j0 + r < J) Z[(int64_t)(i / kSpRows) * ldz + j0 + r] = 0.f;
        }
        return;
    }

    for (int c4 = tid; 4 * c4 < D; c4 += kSpThreads) {
        f32x4 w[kSpRows];
#pragma unroll
        for (int r = 0; r < kSpRows; ++r) {
            const float* row = W + (int64_t)min(j0 + r, J - 1) * ldw;
            // aligned rows and a whole quad inside the row: one unguarded 128-bit load
            // (uniform per quad except at the ragged end, so the loads stay back to back)
            w[r] = (vec_w && 4 * c4 + 3 < D) ? ldg4(row + 4 * c4) : load4(row, 4 * c4, D, false);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (4 * c4 + q < D)
                *reinterpret_cast<f32x4*>(&wcols[(4 * c4 + q) * 4]) = f32x4{w[0][q], w[1][q], w[2][q], w[3][q]};
    }
    __syncthreads();

    // row pointers of a batch of consecutive samples (clamped into the batch: a row pointer
    // outside [0, nnz] is a caller error and must not carry an access out of the arrays)
    auto load_ptrs = [&](int n, int64_t (&p)[kSpBatch + 1]) {
#pragma unroll
        for (int s = 0; s <= kSpBatch; ++s) {
            const int64_t v = rowptr[min(n + s, n_rows)];
            p[s] = v < 0 ? 0 : (v > nnz ? nnz : v);
        }
    };
    int64_t ptr[kSpBatch + 1], next_ptr[kSpBatch + 1];
    int n = wave * kSpBatch;
    if (n < n_rows) load_ptrs(n, ptr);
    for (; n < n_rows; n += NW * kSpBatch) {
        const int n_next = n + NW * kSpBatch;
        if (n_next < n_rows) load_ptrs(n_next, next_ptr);   // one batch ahead
        // issue every load of the batch's first slabs before using any of them
        int cc[kSpBatch][kSpPre];
        float vv[kSpBatch][kSpPre];
#pragma unroll
        for (int s = 0; s < kSpBatch; ++s)
#pragma unroll
            for (int it = 0; it < kSpPre; ++it) {
                // always a valid address (clamped), the select discards what is out of the row:
                // no branch sits between the loads, so all of them are in flight together
                const int64_t e = ptr[s] + it * 64 + lane;
                const int64_t ec = e < nnz ? e : nnz - 1;
                const int cl = col[ec];
                vv[s][it] = val[ec];
                cc[s][it] = e < ptr[s + 1] ? cl : -1;
            }
        f32x4 acc[kSpBatch];
#pragma unroll
        for (int s = 0; s < kSpBatch; ++s) {
            acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int it = 0; it < kSpPre; ++it) {
                const int c = cc[s][it];
                if (c >= 0 && c < D) acc[s] += vv[s][it] * *reinterpret_cast<const f32x4*>(&wcols[c * 4]);
            }
            // rows longer than the prefetched slabs
            for (int64_t e = ptr[s] + kSpPre * 64 + lane; e < ptr[s + 1]; e += 64) {
                const int c = col[e];
                const float v = val[e];
                if (c >= 0 && c < D) acc[s] += v * *reinterpret_cast<const f32x4*>(&wcols[c * 4]);
            }
        }
        // halving butterfly per sample: after two exchanges each lane carries one class
#pragma unroll
        for (int s = 0; s < kSpBatch; ++s) {
            const bool hi = lane & 32;
            const float g0 = hi ? acc[s].x : acc[s].z, g1 = hi ? acc[s].y : acc[s].w;   // what I give away
            const float k0 = hi ? acc[s].z : acc[s].x, k1 = hi ? acc[s].w : acc[s].y;   // what I keep
            const float a0 = k0 + __shfl_xor(g0, 32, 64), a1 = k1 + __shfl_xor(g1, 32, 64);
            const bool hi2 = lane & 16;
            const float give = hi2 ? a0 : a1, keep = hi2 ? a1 : a0;
            float t = keep + __shfl_xor(give, 16, 64);
            t += __shfl_xor(t, 8, 64);
            t += __shfl_xor(t, 4, 64);
            t += __shfl_xor(t, 2, 64);
            t += __shfl_xor(t, 1, 64);
            // lanes 0..15 hold class 0, 16..31 class 1, 32..47 class 2, 48..63 class 3
            const int r = lane >> 4;
            if ((lane & 15) == 0 && n + s < n_rows && j0 + r < J) Z[(int64_t)(n + s) * ldz + j0 + r] = t;
        }
#pragma unroll
        for (int s = 0; s <= kSpBatch; ++s) ptr[s] = next_ptr[s];
    }
}

bool csr_scores_ok(int D) { return (size_t)D * kSpRows * sizeof(float) <= 160 * 1024 - 1024; }

hipError_t launch_csr_scores(const DensifyArgs& a, const float* W, int64_t ldw, float* Z, int64_t ldz, int J,
                             hipStream_t s) {
    const size_t lds_bytes = (size_t)a.D * kSpRows * sizeof(float);
    static size_t raised = 0;   // largest LDS size opted in to so far
    if (lds_bytes > 64 * 1024 && lds_bytes > raised) {
        hipError_t e = hipFuncSetAttribute((const void*)csr_scores_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = lds_bytes;
    }
    const bool vec_w = ((uintptr_t)W % 16) == 0 && (ldw % 4) == 0;
    SFB_LAUNCH(csr_scores_kernel, dim3((J + kSpRows - 1) / kSpRows), dim3(kSpThreads), lds_bytes, s,
                       a.rowptr, a.col, a.val, a.nnz, W, ldw, Z, ldz, a.n_rows, J, a.D, vec_w);
    return hipGetLastError();
}

}  // namespace sfb
