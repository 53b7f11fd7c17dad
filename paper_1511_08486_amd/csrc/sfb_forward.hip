// Scores of problem (P), Section 2: z_i = W a_i for all samples of the step, as one
// contraction Z[n][j] = sum_d A[n][d] * W[j][d] on the fp32 matrix cores.
//
// Both operands are contiguous along the contraction (D), the output is small
// (n_rows x J) and D is long, so the grid is tiles x split-K: every workgroup owns a
// BM x BN output tile over one slice of D and writes a partial sum; the factor kernel
// adds the slices in a fixed order (deterministic, no atomics, no zero fill).
//
// The workgroups with class-block 0 also write v_i = a_i (DML: x_i - y_i) into V:
// the features pass through registers here anyway, so the "write_v" copy of
// Section 4.2 costs no extra read.
//
// MFMA: v_mfma_f32_32x32x2_f32.  Lane l supplies A[l%32][l/32] and B[l/32][l%32] and
// holds C[8*(i/4) + 4*(l/32) + i%4][l%32] in accumulator element i.  The contraction
// index is a dummy, so each lane reads four consecutive d with one 128-bit LDS read
// and feeds them to four successive MFMAs (both operands use the same permutation).
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kFwdBK = 32;                 // columns of D per LDS stage
constexpr int kFwdLds = kFwdBK + 4;        // padded row: conflict-free 128-bit reads
constexpr int kFwdThreads = 256;

template <int BM, int BN, typename TIn, bool DIFF>
__global__ __launch_bounds__(kFwdThreads) void fwd_scores_kernel(
    const TIn* __restrict__ A, const TIn* __restrict__ A2, int64_t lda, const float* __restrict__ W,
    int64_t ldw, float* __restrict__ Zp, int64_t ldz, int64_t zstride, TIn* __restrict__ V, int64_t ldv,
    int n_rows, int J, int D, int k_slice, int n_nb, int n_jb, int total, bool vec_a, bool vec_w,
    bool vec_v) {
    constexpr int BK = kFwdBK, LS = kFwdLds;
    constexpr int WM = BM / 2, WN = BN / 2;       // 2 x 2 waves
    constexpr int MT = WM / 32, NT = WN / 32;
    constexpr int A_LD = BM * BK / 4 / kFwdThreads;  // 128-bit loads per thread per stage
    constexpr int B_LD = BN * BK / 4 / kFwdThreads;
    static_assert(MT >= 1 && NT >= 1 && A_LD >= 1 && B_LD >= 1, "tile too small");

    __shared__ float As[BM * LS];
    __shared__ float Bs[BN * LS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // tile id: sample block fastest, so the workgroups that share a W block are
    // neighbours inside one die's contiguous range.
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int nb = id % n_nb;
    id /= n_nb;
    const int jb = id % n_jb;
    const int ks = id / n_jb;
    const int n0 = nb * BM, j0 = jb * BN;
    const int k_begin = ks * k_slice;
    const int k_end = min(D, k_begin + k_slice);
    const int n_chunks = (k_end - k_begin + BK - 1) / BK;
    const bool write_v = (V != nullptr) && (jb == 0);

    f32x4 ra[A_LD], rb[B_LD];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int r = idx / (BK / 4), c = (idx % (BK / 4)) * 4;
            const int row = n0 + r;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (row < n_rows) {
                // columns at or beyond k_end belong to the next slice: read them as 0
                v = load4(A + (int64_t)row * lda, k0 + c, k_end, vec_a);
                if (DIFF) v -= load4(A2 + (int64_t)row * lda, k0 + c, k_end, vec_a);
                if (write_v) store4(V + (int64_t)row * ldv, k0 + c, k_end, vec_v, v);
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int r = idx / (BK / 4), c = (idx % (BK / 4)) * 4;
            const int row = j0 + r;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (row < J) v = load4(W + (int64_t)row * ldw, k0 + c, k_end, vec_w);
            rb[i] = v;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int r = idx / (BK / 4), c = (idx % (BK / 4)) * 4;
            *reinterpret_cast<f32x4*>(&As[r * LS + c]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int r = idx / (BK / 4), c = (idx % (BK / 4)) * 4;
            *reinterpret_cast<f32x4*>(&Bs[r * LS + c]) = rb[i];
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    if (n_chunks > 0) fetch(k_begin);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();  // everyone has finished reading the previous stage
        stage();
        __syncthreads();
        if (c + 1 < n_chunks) fetch(k_begin + (c + 1) * BK);
#pragma unroll
        for (int q = 0; q < BK / 8; ++q) {
            f32x4 a[MT], b[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                a[i] = *reinterpret_cast<const f32x4*>(&As[(wm * WM + i * 32 + l32) * LS + q * 8 + half * 4]);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                b[j] = *reinterpret_cast<const f32x4*>(&Bs[(wn * WN + j * 32 + l32) * LS + q * 8 + half * 4]);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][r], b[j][r], acc[i][j], 0, 0, 0);
        }
    }

    float* zout = Zp + (int64_t)ks * zstride;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int col = j0 + wn * WN + j * 32 + l32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = n0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                if (row < n_rows && col < J) zout[(int64_t)row * ldz + col] = acc[i][j][e];
            }
        }
}

FwdPlan plan_forward(int64_t n_rows, int64_t J, int64_t D) {
    FwdPlan p;
    p.bm = 128;
    p.bn = 128;
    if (n_rows <= 64) p.bm = 64;
    if (J <= 64) p.bn = 64;
    const int64_t tiles = ((n_rows + p.bm - 1) / p.bm) * ((J + p.bn - 1) / p.bn);
    const int64_t chunks = (D + kFwdBK - 1) / kFwdBK;
    // enough workgroups for two per compute unit, but never slices shorter than 4 chunks
    int64_t s = (512 + tiles - 1) / tiles;
    int64_t s_max = chunks / 4 > 0 ? chunks / 4 : 1;
    if (s > s_max) s = s_max;
    if (s > 16) s = 16;
    p.split_k = (int)s;
    finish_forward_plan(&p, n_rows, J, D);
    return p;
}

void finish_forward_plan(FwdPlan* p, int64_t n_rows, int64_t J, int64_t D) {
    const int64_t tiles = ((n_rows + p->bm - 1) / p->bm) * ((J + p->bn - 1) / p->bn);
    const int64_t chunks = (D + kFwdBK - 1) / kFwdBK;
    int64_t s = p->split_k < 1 ? 1 : p->split_k;
    if (s > chunks) s = chunks;
    const int64_t per = (chunks + s - 1) / s;     // chunks per slice
    s = (chunks + per - 1) / per;                 // drop empty slices
    p->split_k = (int)s;
    p->k_slice = (int)(per * kFwdBK);
    p->grid = (int)(tiles * s);
}

template <int BM, int BN, typename TIn, bool DIFF>
static hipError_t launch_fwd_t(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    const int n_nb = (a.n_rows + BM - 1) / BM, n_jb = (a.J + BN - 1) / BN;
    const int total = n_nb * n_jb * p.split_k;
    const int esz = (int)sizeof(TIn);
    auto aligned = [&](const void* ptr, int64_t ld, int bytes) {
        return ptr == nullptr || (((uintptr_t)ptr % bytes) == 0 && (ld % 4) == 0);
    };
    const bool vec_a = aligned(a.a, a.lda, 4 * esz) && aligned(a.a2, a.lda, 4 * esz);
    const bool vec_w = aligned(a.w, a.ldw, 16);
    const bool vec_v = aligned(a.v, a.ldv, 4 * esz);
    hipLaunchKernelGGL((fwd_scores_kernel<BM, BN, TIn, DIFF>), dim3(total), dim3(kFwdThreads), 0, s,
                       (const TIn*)a.a, (const TIn*)a.a2, a.lda, a.w, a.ldw, a.zp, a.ldz, a.zstride,
                       (TIn*)a.v, a.ldv, a.n_rows, a.J, a.D, p.k_slice, n_nb, n_jb, total, vec_a, vec_w,
                       vec_v);
    return hipGetLastError();
}

template <typename TIn, bool DIFF>
static hipError_t launch_fwd_tile(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    if (p.bm == 128 && p.bn == 128) return launch_fwd_t<128, 128, TIn, DIFF>(a, p, s);
    if (p.bm == 128 && p.bn == 64) return launch_fwd_t<128, 64, TIn, DIFF>(a, p, s);
    if (p.bm == 64 && p.bn == 128) return launch_fwd_t<64, 128, TIn, DIFF>(a, p, s);
    if (p.bm == 64 && p.bn == 64) return launch_fwd_t<64, 64, TIn, DIFF>(a, p, s);
    return hipErrorInvalidValue;
}

hipError_t launch_forward(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    if (a.bf16) {
        if (a.diff) return hipErrorInvalidValue;
        return launch_fwd_tile<bf16_t, false>(a, p, s);
    }
    return a.diff ? launch_fwd_tile<float, true>(a, p, s) : launch_fwd_tile<float, false>(a, p, s);
}

}  // namespace sfb
