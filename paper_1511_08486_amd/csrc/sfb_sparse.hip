// Sparse-feature helpers for the L2-SVM workload (the paper exploits sparse features to
// cut computation, Section 6): v_i = a_i is delivered as the dense row of the CSR matrix,
// because the reconstruction consumes V as a dense [N][D] operand.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kDensifyThreads = 256;

// One workgroup per sample.  Entries are ADDED into a zeroed row, so a column that appears more than
// once in a row contributes the sum of its values, exactly as it does in the scores computed from the
// stored entries; a column that appears once lands bit for bit (0 + v = v).  With three or more
// repeats the order of the additions is not fixed.
//   IN_LDS: the row is built in LDS (zero, barrier, LDS atomic adds, barrier) and written out once
//           with wide coalesced stores: one pass over the row in memory, no atomics on memory.
//   else:   rows longer than the LDS holds are zeroed in memory with wide stores and the entries
//           added with fp32 atomics on memory (the barrier orders the two phases inside the
//           workgroup, and no other workgroup touches this row).
template <bool IN_LDS>
__global__ __launch_bounds__(kDensifyThreads) void csr_densify_kernel(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ col, const float* __restrict__ val,
    float* __restrict__ V, int64_t ldv, int D, int64_t nnz, bool vec_v) {
    extern __shared__ __attribute__((aligned(16))) float dense_row[];   // [round_up4(D)] when IN_LDS
    const int row = blockIdx.x;
    float* out = V + (int64_t)row * ldv;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int c = 4 * threadIdx.x; c < D; c += 4 * kDensifyThreads) {
        if (IN_LDS) *reinterpret_cast<f32x4*>(&dense_row[c]) = zero;
        else store4(out, c, D, vec_v, zero);
    }
    __syncthreads();
    // a row pointer outside [0, nnz] is a caller error; clamp so that no access leaves the arrays
    const int64_t beg = max(0, rowptr[row]);
    const int64_t end = min((int64_t)rowptr[row + 1], nnz);
    for (int64_t n = beg + threadIdx.x; n < end; n += kDensifyThreads) {
        const int c = col[n];
        if (c >= 0 && c < D) {
            if (IN_LDS) atomicAdd(&dense_row[c], val[n]);
            else unsafeAtomicAdd(out + c, val[n]);
        }
    }
    if (IN_LDS) {
        __syncthreads();
        for (int c = 4 * threadIdx.x; c < D; c += 4 * kDensifyThreads)
            store4(out, c, D, vec_v, *reinterpret_cast<const f32x4*>(&dense_row[c]));
    }
}

hipError_t launch_csr_densify(const DensifyArgs& a, hipStream_t s) {
    const bool vec_v = ((uintptr_t)a.v % 16) == 0 && (a.ldv % 4) == 0;
    const size_t lds_bytes = ((size_t)a.D + 3) / 4 * 16;
    if (lds_bytes <= 64 * 1024) {
        SFB_LAUNCH(csr_densify_kernel<true>, dim3(a.n_rows), dim3(kDensifyThreads), lds_bytes, s, a.rowptr, a.col,
                   a.val, a.v, a.ldv, a.D, a.nnz, vec_v);
    } else {
        SFB_LAUNCH(csr_densify_kernel<false>, dim3(a.n_rows), dim3(kDensifyThreads), 0, s, a.rowptr, a.col,
                   a.val, a.v, a.ldv, a.D, a.nnz, vec_v);
    }
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

    // The kernel is bound by the number of vector instructions per stored entry, not by memory, so the
    // per-entry bookkeeping is kept off the vector unit:
    //  * col and val are read through buffer descriptors: the address is (one 32-bit byte offset per sample
    //    and lane) + an immediate per slab, and an offset beyond the array returns 0 by hardware, so there
    //    is no 64-bit address arithmetic and no clamp (the host checks nnz <= 2^30 - 1024: the byte range of
    //    a descriptor and the offsets are 32-bit);
    //  * the wavefront number is made scalar, so row pointers are scalar loads and their clamps scalar
    //    arithmetic;
    //  * a lane past the end of its row gets value 0 (one compare + one select per slab); its column is
    //    whatever the array holds there (an entry of a later row, or 0 past the end): a valid place in the
    //    parked rows, multiplied by zero.
    const __amdgpu_buffer_rsrc_t col_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)col, (short)0, (int)((uint32_t)nnz * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)val, (short)0, (int)((uint32_t)nnz * 4u), 0x00020000);
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t dmax = (uint32_t)(D - 1);
    // row pointers of a batch of consecutive samples (clamped into [0, nnz]: a row pointer
    // outside is a caller error and must not carry an access out of the arrays)
    auto load_ptrs = [&](int n, int (&p)[kSpBatch + 1]) {
#pragma unroll
        for (int s = 0; s <= kSpBatch; ++s) p[s] = min(max(rowptr[min(n + s, n_rows)], 0), (int)nnz);
    };
    // the first slabs of a batch: every load is issued before any is used, no branch in between
    auto load_entries = [&](const int (&p)[kSpBatch + 1], uint32_t (&c)[kSpBatch][kSpPre], float (&v)[kSpBatch][kSpPre]) {
#pragma unroll
        for (int s = 0; s < kSpBatch; ++s) {
            const int off = (int)((uint32_t)(p[s] + lane) * 4u);   // byte offset of this lane's entry of slab 0
            const int left = p[s + 1] - p[s] - lane;         // > 64 * it: the lane's entry of slab it belongs to the row
#pragma unroll
            for (int it = 0; it < kSpPre; ++it) {
                const uint32_t cl = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(col_rsrc, off + it * 256, 0, 0);
                const float vl = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(val_rsrc, off + it * 256, 0, 0));
                v[s][it] = left > it * 64 ? vl : 0.f;
                c[s][it] = min(cl, dmax);                    // a column outside [0, D) is a caller error: stay inside the LDS tile
            }
        }
    };
    // Three batches are in flight per wavefront: the one being multiplied (its entries were requested a
    // round ago), the next (row pointers here, entries requested now) and the one after (row pointers
    // requested now), so that the trips to L2 for the CSR arrays run under the LDS gathers of the round
    // before instead of in front of every round.
    int ptr[kSpBatch + 1], next_ptr[kSpBatch + 1], after_ptr[kSpBatch + 1];
    uint32_t cc0[kSpBatch][kSpPre], cc1[kSpBatch][kSpPre];
    float vv0[kSpBatch][kSpPre], vv1[kSpBatch][kSpPre];
    constexpr int STRIDE = NW * kSpBatch;
    int n = wave_s * kSpBatch;
    if (n < n_rows) {
        load_ptrs(n, ptr);
        load_entries(ptr, cc0, vv0);
    }
    if (n + STRIDE < n_rows) load_ptrs(n + STRIDE, next_ptr);
    // one round: request the next batch's entries into (ncc, nvv), multiply the batch held in (cc, vv)
    auto round = [&](uint32_t (&cc)[kSpBatch][kSpPre], float (&vv)[kSpBatch][kSpPre], uint32_t (&ncc)[kSpBatch][kSpPre],
                     float (&nvv)[kSpBatch][kSpPre]) {
        if (n + 2 * STRIDE < n_rows) load_ptrs(n + 2 * STRIDE, after_ptr);
        if (n + STRIDE < n_rows) load_entries(next_ptr, ncc, nvv);
        float acc[kSpBatch * kSpRows];                      // [sample][class]
#pragma unroll
        for (int s = 0; s < kSpBatch; ++s) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int it = 0; it < kSpPre; ++it) a += vv[s][it] * *reinterpret_cast<const f32x4*>(&wcols[cc[s][it] * 4]);
            // rows longer than the prefetched slabs (uniform trip count per wavefront)
            for (int e0 = ptr[s] + kSpPre * 64; e0 < ptr[s + 1]; e0 += 64) {
                const int off = (int)((uint32_t)(e0 + lane) * 4u);
                const uint32_t cl = min((uint32_t)__builtin_amdgcn_raw_buffer_load_b32(col_rsrc, off, 0, 0), dmax);
                const float vl = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(val_rsrc, off, 0, 0));
                a += (e0 + lane < ptr[s + 1] ? vl : 0.f) * *reinterpret_cast<const f32x4*>(&wcols[cl * 4]);
            }
#pragma unroll
            for (int r = 0; r < kSpRows; ++r) acc[s * kSpRows + r] = a[r];
        }
        // Halving butterfly over all 16 sums of the batch at once: at every exchange a lane
        // gives away half of what it still holds and adds what it receives to the other half,
        // 8 + 4 + 2 + 1 exchanges; then two more for the last factor four.  Lane l ends up with
        // value index (l >> 2) & 15 summed over all 64 lanes (17 exchanges instead of 96).  The exchanges
        // over 32 and 16 lanes are one swap instruction each: v_permlane32_swap trades the upper half of
        // its first operand for the lower half of its second (v_permlane16_swap: the odd rows of 16 lanes
        // for the even rows), after which "kept + received" is the sum of the two registers.
        static_assert(kSpBatch * kSpRows == 16, "butterfly below is written for 16 values");
        // (written as instructions: the compiler's own form of these two returned one register twice in the
        // sums below; the waits before and after cover the instruction's issue rules for operands that a
        // vector instruction has just written or is about to read)
        float v8[8], v4[4], v2[2], v1;
        asm volatile("s_nop 1");
#pragma unroll
        for (int k = 0; k < 8; ++k) asm volatile("v_permlane32_swap_b32 %0, %1" : "+v"(acc[k]), "+v"(acc[k + 8]));
        asm volatile("s_nop 1");
#pragma unroll
        for (int k = 0; k < 8; ++k) v8[k] = acc[k] + acc[k + 8];       // lanes < 32 now hold values 0..7, the rest 8..15
        asm volatile("s_nop 1");
#pragma unroll
        for (int k = 0; k < 4; ++k) asm volatile("v_permlane16_swap_b32 %0, %1" : "+v"(v8[k]), "+v"(v8[k + 4]));
        asm volatile("s_nop 1");
#pragma unroll
        for (int k = 0; k < 4; ++k) v4[k] = v8[k] + v8[k + 4];         // bit 4 of the lane clear: value k, set: k + 4
        {
            const bool hi = lane & 8;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float give = hi ? v4[k] : v4[k + 2], keep = hi ? v4[k + 2] : v4[k];
                v2[k] = keep + __shfl_xor(give, 8, 64);
            }
        }
        {
            const bool hi = lane & 4;
            const float give = hi ? v2[0] : v2[1], keep = hi ? v2[1] : v2[0];
            v1 = keep + __shfl_xor(give, 4, 64);
        }
        v1 += __shfl_xor(v1, 2, 64);
        v1 += __shfl_xor(v1, 1, 64);
        // value index = 8*(lane bit 5) + 4*(bit 4) + 2*(bit 3) + (bit 2) = (lane >> 2) & 15 = sample * 4 + class
        {
            const int idx = (lane >> 2) & 15, sm = idx >> 2, r = idx & 3;
            if ((lane & 3) == 0 && n + sm < n_rows && j0 + r < J) Z[(int64_t)(n + sm) * ldz + j0 + r] = v1;
        }
#pragma unroll
        for (int s = 0; s <= kSpBatch; ++s) {
            ptr[s] = next_ptr[s];
            next_ptr[s] = after_ptr[s];
        }
        n += STRIDE;
    };
    // the two register sets trade places every round (no copies)
    while (n < n_rows) {
        round(cc0, vv0, cc1, vv1);
        if (n < n_rows) round(cc1, vv1, cc0, vv0);
    }
}

bool csr_scores_ok(int D) { return (size_t)D * kSpRows * sizeof(float) <= 160 * 1024 - 1024; }
// (the caller also needs nnz <= 2^30 - 1024: the kernel reads the CSR arrays through 32-bit byte offsets)

// Which score pass is cheaper for this batch, in microseconds fitted to one MI355X (N = 256 and 1024, J = 16 to
// 5000, D = 1024 to 10000, 2 % and 20 % stored).  From the entries: J / 4 workgroups, one per compute unit at a time,
// each walks every row; a row costs about 20 ns plus 2 ns per 64-entry slab up to the three the kernel keeps in
// flight and 19 ns per slab beyond, counted from 3.5 (long rows wait for their own loads and gathers).  Dense, on the densified
// rows: the fp32 contraction at about 110 TFLOP/s on at least one 64-class block, and no faster than its walk
// through D.  The entries win at the
// benchmark's 2 % of 8192 columns with 2000 classes (66 against 283 us) and lose with few classes (J = 64: 30
// against 13 us), short rows (D = 1024) or dense ones (20 %: 962 against 280 us).
bool csr_scores_wins(int64_t n_rows, int64_t J, int64_t D, int64_t nnz) {
    if (n_rows <= 0) return true;
    double slabs = (double)((nnz / n_rows + 63) / 64);
    if (slabs < 1.0) slabs = 1.0;
    const double per_row = 0.020 + 0.0019 * (slabs < 3.0 ? slabs : 3.0) + 0.019 * (slabs > 3.5 ? slabs - 3.5 : 0.0);
    const double rounds = (double)(((J + kSpRows - 1) / kSpRows + 255) / 256);
    const double from_entries = 1.1 * rounds * (4.0 + (double)n_rows * per_row);
    const double flops_us = 2.0 * (double)n_rows * (double)(J > 64 ? J : 64) * (double)D / 1.1e8;
    const double walk_us = 0.0012 * (double)D;               // a small grid still walks its slices of D stage by stage
    const double dense = 4.0 + (flops_us > walk_us ? flops_us : walk_us);
    return from_entries < dense;
}

hipError_t launch_csr_scores(const DensifyArgs& a, const float* W, int64_t ldw, float* Z, int64_t ldz, int J,
                             hipStream_t s) {
    const size_t lds_bytes = (size_t)a.D * kSpRows * sizeof(float);
    static std::atomic<size_t> raised{0};   // largest LDS size opted in to so far
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
