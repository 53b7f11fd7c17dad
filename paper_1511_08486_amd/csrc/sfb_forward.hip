// Scores of problem (P), Section 2: z_i = W a_i for all samples of the step, as one
// contraction Z[n][j] = sum_d A[n][d] * W[j][d] on the fp32 matrix cores.
//
// Both operands are contiguous along the contraction (D), the output is small
// (n_rows x J) and D is long, so the grid is tiles x split-K: every workgroup owns a
// BM x BN output tile over one slice of D and writes a partial sum; the factor kernel
// adds the slices in a fixed order (deterministic, no atomics, no zero fill).
//
// The workgroups also write v_i = a_i (DML: x_i - y_i) into V, each class block its share of
// the chunks of D (one block doing all of it would be the straggler every other workgroup
// waits for): the features pass through the compute unit anyway, so the "write_v" copy of
// Section 4.2 costs no extra read.
//
// MFMA: v_mfma_f32_32x32x2_f32.  Lane l supplies A[l%32][l/32] and B[l/32][l%32] and
// holds C[8*(i/4) + 4*(l/32) + i%4][l%32] in accumulator element i.  The contraction
// index is a dummy, so each lane reads four consecutive d with one 128-bit LDS read
// and feeds them to four successive MFMAs (both operands use the same permutation).
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kFwdBK = 32;                 // columns of D per LDS stage
constexpr int kFwdLds = kFwdBK + 4;        // padded row: conflict-free 128-bit reads
constexpr int kFwdThreads = 256;

// Pipeline (one or two wavefronts per SIMD, so latency is hidden in the instruction
// stream): features and W rows are fetched two stages ahead into registers as raw words,
// converted / subtracted on the way into a double-buffered LDS tile (one barrier per
// stage), and the operand fragments of the next 8 columns are read from LDS while the
// MFMAs of the current 8 execute.  FAST: aligned pointers, D a multiple of 4 -- no branch
// around any load (rows and columns are clamped into the matrix and zeroed by a select).
template <int BM, int BN, typename TIn, bool DIFF, bool FAST>
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
    constexpr int NQ = BK / 8;                       // fragment groups per stage
    static_assert(MT >= 1 && NT >= 1 && A_LD >= 1 && B_LD >= 1, "tile too small");

    // two stages of the feature tile [BM][LS], then two stages of the W tile [BN][LS]
    extern __shared__ __attribute__((aligned(16))) float fwd_lds[];
    float* const As = fwd_lds;
    float* const Bs = fwd_lds + 2 * BM * LS;

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
    const bool write_v = V != nullptr;   // shared by the class blocks: block jb takes the chunks c with c % n_jb == jb

    // FAST: one wide load per item; otherwise four clamped scalar loads per item, kept as loaded
    // (what lies outside the matrix or the slice is zeroed when the stage is written to LDS).
    using RawA = typename RawOf<TIn>::type;
    using RawSlow = typename std::conditional<std::is_same<TIn, float>::value, f32x4, u32x4>::type;
    using RawS = typename std::conditional<FAST, RawA, RawSlow>::type;
    struct Stage { RawS a[A_LD]; RawS a2[DIFF ? A_LD : 1]; f32x4 b[B_LD]; };
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    // Raw words only: nothing may depend on a load before the stage that consumes it.
    auto fetch = [&](Stage& r, int k0) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int row = n0 + idx / (BK / 4), col = k0 + (idx % (BK / 4)) * 4;
            if constexpr (FAST) {
                const int64_t off = (int64_t)min(row, n_rows - 1) * lda + min(col, D - 4);
                r.a[i] = ldraw4(A + off);
                if (DIFF) r.a2[i] = ldraw4(A2 + off);
            } else {
                // columns at or beyond k_end belong to the next slice: the stage zeroes them
                r.a[i] = load4_clamped_raw(A, row, lda, n_rows, col, k_end);
                if (DIFF) r.a2[i] = load4_clamped_raw(A2, row, lda, n_rows, col, k_end);
            }
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int row = j0 + idx / (BK / 4), col = k0 + (idx % (BK / 4)) * 4;
            if constexpr (FAST) {
                r.b[i] = ldg4(W + (int64_t)min(row, J - 1) * ldw + min(col, D - 4));
            } else {
                r.b[i] = load4_clamped_raw(W, row, ldw, J, col, k_end);
            }
        }
    };
    // widen / subtract / zero out-of-range elements on the way into LDS; v_i is delivered here too
    auto stage = [&](const Stage& r, int buf, int k0) {
        const bool my_v = write_v && (((k0 - k_begin) / BK) % n_jb) == jb;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int rr = idx / (BK / 4), cc = (idx % (BK / 4)) * 4;
            const int row = n0 + rr, col = k0 + cc;
            f32x4 v = widen4(r.a[i]);
            if (DIFF) v -= widen4(r.a2[i]);
            const bool in = row < n_rows && col < k_end;   // FAST: k_end is a multiple of 4
            if constexpr (FAST) v = in ? v : zero4;
            else v = in_matrix4(v, row < n_rows, col, k_end);
            *reinterpret_cast<f32x4*>(&As[buf * BM * LS + rr * LS + cc]) = v;
            if (my_v && in) {
                if constexpr (FAST) *reinterpret_cast<RawA*>(V + (int64_t)row * ldv + col) = to_raw<TIn>(v);
                else store4(V + (int64_t)row * ldv, col, k_end, vec_v, v);
            }
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int idx = tid + i * kFwdThreads;
            const int rr = idx / (BK / 4), cc = (idx % (BK / 4)) * 4;
            f32x4 v = r.b[i];
            if constexpr (FAST) v = (j0 + rr < J && k0 + cc < k_end) ? v : zero4;
            else v = in_matrix4(v, j0 + rr < J, k0 + cc, k_end);
            *reinterpret_cast<f32x4*>(&Bs[buf * BN * LS + rr * LS + cc]) = v;
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
    struct Frag { f32x4 a[MT], b[NT]; };
    auto read_frag = [&](Frag& f, int buf, int q) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
            f.a[i] = *reinterpret_cast<const f32x4*>(
                &As[buf * BM * LS + (wm * WM + i * 32 + l32) * LS + q * 8 + half * 4]);
#pragma unroll
        for (int j = 0; j < NT; ++j)
            f.b[j] = *reinterpret_cast<const f32x4*>(
                &Bs[buf * BN * LS + (wn * WN + j * 32 + l32) * LS + q * 8 + half * 4]);
    };
    auto mma_frag = [&](const Frag& f) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[i][r], f.b[j][r], acc[i][j], 0, 0, 0);
    };
    auto compute = [&](int buf) {
        Frag f0, f1;
        read_frag(f0, buf, 0);
#pragma unroll
        for (int q = 0; q < NQ; q += 2) {
            if (q + 1 < NQ) read_frag(f1, buf, q + 1);
            __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs they do not feed
            mma_frag(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (q + 1 < NQ) {
                if (q + 2 < NQ) read_frag(f0, buf, q + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma_frag(f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    Stage r0, r1;
    fetch(r0, k_begin);
    fetch(r1, k_begin + BK);
    stage(r0, 0, k_begin);
    __syncthreads();
    // Pair of steps (c, c+1): LDS stage 0 holds chunk c, r1 holds chunk c+1, r0 is free.
    // One straight-line block per pair keeps every fetch two stages ahead of its use.
    int c = 0;
    for (; c + 1 < n_chunks; c += 2) {
        fetch(r0, k_begin + (c + 2) * BK);
        compute(0);
        stage(r1, 1, k_begin + (c + 1) * BK);
        __syncthreads();
        fetch(r1, k_begin + (c + 3) * BK);
        compute(1);
        stage(r0, 0, k_begin + (c + 2) * BK);
        __syncthreads();
    }
    if (c < n_chunks) compute(0);   // odd count: the last chunk is already staged

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

// ---------------------------------------------------------------------------------------
// LDS-DMA variant (fp32 features, no pair difference, aligned pointers, D a multiple of
// the stage depth): feature and W tiles go from HBM/L2 straight into LDS, three stages
// deep, with completion tracked by hand (see lds_dma16).  A tile row is 32 floats = eight
// 16-byte items and the DMA fills LDS linearly, so the bank-conflict padding of the
// register-staged kernel is replaced by a swizzle on the *source* side: the lane that
// fills item slot (r, p) fetches logical item p ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 1),
// and the fragment reads apply the same XOR.  Sixteen consecutive rows then hit sixteen
// different 16-byte bank groups.
// The workgroups of class block 0 copy the staged feature tile on to V.
// ---------------------------------------------------------------------------------------
constexpr int kFwdDmaStages = 3;

__device__ __forceinline__ int fwd_swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// DIFF (pair models, Section 2 DML): the second point of each pair is staged next to the
// first and a = x - y is formed when a fragment (or the V copy) is read from LDS.
template <int BM, int BN, bool DIFF>
__global__ __launch_bounds__(kFwdThreads) void fwd_scores_dma_kernel(
    const float* __restrict__ A, const float* __restrict__ A2, int64_t lda, const float* __restrict__ W, int64_t ldw, float* __restrict__ Zp,
    int64_t ldz, int64_t zstride, float* __restrict__ V, int64_t ldv, int n_rows, int J, int D, int k_slice,
    int n_nb, int n_jb, int total) {
    constexpr int BK = kFwdBK, NST = kFwdDmaStages;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int MT = WM / 32, NT = WN / 32;
    constexpr int A_LD = BM * BK / 4 / kFwdThreads;
    constexpr int B_LD = BN * BK / 4 / kFwdThreads;
    constexpr int NQ = BK / 8;
    constexpr int A2_FLOATS = DIFF ? BM * BK : 0;      // second-point tile sits after the W tile
    constexpr int STAGE_FLOATS = (BM + BN) * BK + A2_FLOATS;
    static_assert(MT >= 1 && NT >= 1 && A_LD >= 1 && B_LD >= 1, "tile too small");

    extern __shared__ __attribute__((aligned(16))) float fwd_lds[];   // NST x (A tile, W tile[, A2 tile])

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int nb = id % n_nb;
    id /= n_nb;
    const int jb = id % n_jb;
    const int ks = id / n_jb;
    const int n0 = nb * BM, j0 = jb * BN;
    const int k_begin = ks * k_slice;
    const int n_chunks = (min(D, k_begin + k_slice) - k_begin) / BK;   // host: D % BK == 0
    // v_i = a_i is written once: the class blocks share the job, block jb takes the chunks c with c % n_jb == jb
    const bool write_v = V != nullptr;

    // slot s = tid + i*256 of a tile holds row s/8, physical item s%8 = logical item ^ f(row)
    const float* pa[A_LD];
    int64_t a2_delta = 0;                 // A2 - A in elements: the two points share lda
    if (DIFF) a2_delta = A2 - A;
    const float* pb[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int s = tid + i * kFwdThreads, r = s >> 3, c = (s & 7) ^ fwd_swz(r);
        pa[i] = A + (int64_t)min(n0 + r, n_rows - 1) * lda + k_begin + 4 * c;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int s = tid + i * kFwdThreads, r = s >> 3, c = (s & 7) ^ fwd_swz(r);
        pb[i] = W + (int64_t)min(j0 + r, J - 1) * ldw + k_begin + 4 * c;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)fwd_lds;
    auto issue = [&](int chunk, int st) {
        const uint32_t abase =
            __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_FLOATS + wave * 64 * 4) * 4u);
        const uint32_t bbase = abase + (uint32_t)(BM * BK) * 4u;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) lds_dma16(pa[i] + chunk * BK, abase + (uint32_t)(i * kFwdThreads * 16));
#pragma unroll
        for (int i = 0; i < B_LD; ++i) lds_dma16(pb[i] + chunk * BK, bbase + (uint32_t)(i * kFwdThreads * 16));
        if (DIFF) {
            const uint32_t a2base = bbase + (uint32_t)(BN * BK) * 4u;
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                lds_dma16(pa[i] + a2_delta + chunk * BK, a2base + (uint32_t)(i * kFwdThreads * 16));
        }
    };
    constexpr int DMAS = A_LD + B_LD + (DIFF ? A_LD : 0);   // per thread per stage

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    // float offsets of this lane's item for each of the NQ fragment groups (row base excluded);
    // all of this lane's rows are congruent to l32 mod 32, so one swizzle value serves them
    int qoff[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) qoff[q] = 4 * ((2 * q + half) ^ fwd_swz(l32));

    struct Frag { f32x4 a[MT], b[NT]; };
    auto read_frag = [&](Frag& f, int st, int q) {
        const float* as = &fwd_lds[st * STAGE_FLOATS + (wm * WM + l32) * BK + qoff[q]];
        const float* bs = &fwd_lds[st * STAGE_FLOATS + BM * BK + (wn * WN + l32) * BK + qoff[q]];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            f.a[i] = *reinterpret_cast<const f32x4*>(as + i * 32 * BK);
            if (DIFF) f.a[i] -= *reinterpret_cast<const f32x4*>(as + (BM + BN) * BK + i * 32 * BK);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) f.b[j] = *reinterpret_cast<const f32x4*>(bs + j * 32 * BK);
    };
    auto mma_frag = [&](const Frag& f) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[i][r], f.b[j][r], acc[i][j], 0, 0, 0);
    };
    auto compute = [&](int st) {
        Frag f0, f1;
        read_frag(f0, st, 0);
#pragma unroll
        for (int q = 0; q < NQ; q += 2) {
            if (q + 1 < NQ) read_frag(f1, st, q + 1);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (q + 1 < NQ) {
                if (q + 2 < NQ) read_frag(f0, st, q + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma_frag(f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // v_i = a_i: pass the staged feature items on to V
    auto copy_v = [&](int chunk, int st) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int s = tid + i * kFwdThreads, r = s >> 3, c = (s & 7) ^ fwd_swz(r);
            f32x4 v = *reinterpret_cast<const f32x4*>(&fwd_lds[st * STAGE_FLOATS + 4 * s]);
            if (DIFF) v -= *reinterpret_cast<const f32x4*>(&fwd_lds[st * STAGE_FLOATS + (BM + BN) * BK + 4 * s]);
            if (n0 + r < n_rows)
                *reinterpret_cast<f32x4*>(V + (int64_t)(n0 + r) * ldv + k_begin + chunk * BK + 4 * c) = v;
        }
    };

    if (n_chunks > 0) issue(0, 0);
    if (n_chunks > 1) issue(1, 1);
    auto step = [&](int c, int st) {
        if (c + 1 < n_chunks) wait_vmcnt<DMAS>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (c + 2 < n_chunks) issue(c + 2, (st + 2) % NST);
        if (write_v && (c % n_jb) == jb) copy_v(c, st);
        compute(st);
    };
    int c = 0;
    for (; c + 2 < n_chunks; c += 3) {
        step(c, 0);
        step(c + 1, 1);
        step(c + 2, 2);
    }
    if (c < n_chunks) step(c, 0);
    if (c + 1 < n_chunks) step(c + 1, 1);

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

template <int BM, int BN, bool DIFF>
static hipError_t launch_fwd_dma(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    const int n_nb = (a.n_rows + BM - 1) / BM, n_jb = (a.J + BN - 1) / BN;
    const int total = n_nb * n_jb * p.split_k;
    constexpr size_t lds_bytes = kFwdDmaStages * (BM + BN + (DIFF ? BM : 0)) * kFwdBK * sizeof(float);
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd_scores_dma_kernel<BM, BN, DIFF>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    SFB_LAUNCH((fwd_scores_dma_kernel<BM, BN, DIFF>), dim3(total), dim3(kFwdThreads), lds_bytes, s,
                       (const float*)a.a, (const float*)a.a2, a.lda, a.w, a.ldw, a.zp, a.ldz, a.zstride, (float*)a.v, a.ldv, a.n_rows,
                       a.J, a.D, p.k_slice, n_nb, n_jb, total);
    return hipGetLastError();
}

// Shapes the DMA kernel accepts; everything else runs the register-staged kernel.
static bool fwd_dma_ok(const FwdArgs& a) {
    auto al = [](const void* ptr, int64_t ld) { return ((uintptr_t)ptr % 16) == 0 && (ld % 4) == 0; };
    return !a.bf16 && al(a.a, a.lda) && (!a.diff || al(a.a2, a.lda)) && al(a.w, a.ldw) &&
           (a.v == nullptr || al(a.v, a.ldv)) && (a.D % kFwdBK) == 0 && a.D >= kFwdBK;
}

FwdPlan plan_forward(int64_t n_rows, int64_t J, int64_t D) {
    FwdPlan p;
    p.dma = true;
    const int64_t chunks = (D + kFwdBK - 1) / kFwdBK;
    // Small cost model, in microseconds.  A compute unit multiplies at a fixed rate whatever
    // the number of resident workgroups, so the contraction takes
    //     rounds-of-256-workgroups x (flops of one workgroup) / (rate of one compute unit),
    // smaller tiles pay a little more LDS traffic per flop, and every slice of D costs one
    // write and one read of a partial Z through the workspace.
    const int cand[4][2] = {{128, 128}, {64, 128}, {128, 64}, {64, 64}};
    const double tile_penalty[4] = {1.00, 1.03, 1.08, 1.12};
    const double cu_flops_per_us = 0.65 * 256.0 * 2400.0;              // ~65 % of 256 flop/clk at 2.4 GHz
    const double partial_us = (double)n_rows * (double)J * 8.0 / 3.0e6; // 8 bytes per score at ~3 TB/s
    const int64_t s_max = chunks / 4 > 0 ? (chunks / 4 < 16 ? chunks / 4 : 16) : 1;
    double best = 1e300;
    p.bm = 64; p.bn = 64; p.split_k = 1;
    for (int i = 0; i < 4; ++i) {
        const int bm = cand[i][0], bn = cand[i][1];
        if ((n_rows <= 64 && bm > 64) || (J <= 64 && bn > 64)) continue;
        const int64_t tiles = ((n_rows + bm - 1) / bm) * ((J + bn - 1) / bn);
        for (int64_t s = 1; s <= s_max; ++s) {
            const double rounds = (double)((tiles * s + 255) / 256);
            const double wg_flops = 2.0 * bm * bn * (double)((chunks + s - 1) / s * kFwdBK);
            const double us = tile_penalty[i] * rounds * wg_flops / cu_flops_per_us + partial_us * (double)s;
            if (us < best * (1.0 - 1e-9)) { best = us; p.bm = bm; p.bn = bn; p.split_k = (int)s; }
        }
    }
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

template <int BM, int BN, typename TIn, bool DIFF, bool FAST>
static hipError_t launch_fwd_f(const FwdArgs& a, const FwdPlan& p, hipStream_t s, bool vec_a, bool vec_w,
                               bool vec_v) {
    const int n_nb = (a.n_rows + BM - 1) / BM, n_jb = (a.J + BN - 1) / BN;
    const int total = n_nb * n_jb * p.split_k;
    constexpr size_t lds_bytes = 2 * (BM + BN) * kFwdLds * sizeof(float);
    static std::atomic<bool> raised{false};   // opt in once to more than 64 KB of LDS per workgroup
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)fwd_scores_kernel<BM, BN, TIn, DIFF, FAST>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    SFB_LAUNCH((fwd_scores_kernel<BM, BN, TIn, DIFF, FAST>), dim3(total), dim3(kFwdThreads), lds_bytes,
                       s, (const TIn*)a.a, (const TIn*)a.a2, a.lda, a.w, a.ldw, a.zp, a.ldz, a.zstride,
                       (TIn*)a.v, a.ldv, a.n_rows, a.J, a.D, p.k_slice, n_nb, n_jb, total, vec_a, vec_w, vec_v);
    return hipGetLastError();
}

template <int BM, int BN, typename TIn, bool DIFF>
static hipError_t launch_fwd_t(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    const int esz = (int)sizeof(TIn);
    auto aligned = [&](const void* ptr, int64_t ld, int bytes) {
        return ptr == nullptr || (((uintptr_t)ptr % bytes) == 0 && (ld % 4) == 0);
    };
    const bool vec_a = aligned(a.a, a.lda, 4 * esz) && aligned(a.a2, a.lda, 4 * esz);
    const bool vec_w = aligned(a.w, a.ldw, 16);
    const bool vec_v = aligned(a.v, a.ldv, 4 * esz);
    const bool fast = vec_a && vec_w && vec_v && (a.D % 4) == 0 && a.D >= 4;
    if (fast) return launch_fwd_f<BM, BN, TIn, DIFF, true>(a, p, s, vec_a, vec_w, vec_v);
    return launch_fwd_f<BM, BN, TIn, DIFF, false>(a, p, s, vec_a, vec_w, vec_v);
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
    if (p.dma && fwd_dma_ok(a)) {
        if (a.diff) {   // 128 x 128 with a second feature tile would not leave room for three stages
            if (p.bm == 64 && p.bn == 128) return launch_fwd_dma<64, 128, true>(a, p, s);
            if (p.bm == 128 && p.bn == 64) return launch_fwd_dma<128, 64, true>(a, p, s);
            if (p.bm == 64 && p.bn == 64) return launch_fwd_dma<64, 64, true>(a, p, s);
        } else {
            if (p.bm == 128 && p.bn == 128) return launch_fwd_dma<128, 128, false>(a, p, s);
            if (p.bm == 128 && p.bn == 64) return launch_fwd_dma<128, 64, false>(a, p, s);
            if (p.bm == 64 && p.bn == 128) return launch_fwd_dma<64, 128, false>(a, p, s);
            if (p.bm == 64 && p.bn == 64) return launch_fwd_dma<64, 64, false>(a, p, s);
        }
    }
    if (a.bf16) {
        if (a.diff) return hipErrorInvalidValue;
        return launch_fwd_tile<bf16_t, false>(a, p, s);
    }
    return a.diff ? launch_fwd_tile<float, true>(a, p, s) : launch_fwd_tile<float, false>(a, p, s);
}

}  // namespace sfb
