// Scores (Section 2, z = W a) for fp32 features, computed on the bf16 matrix cores at fp32
// accuracy.
//
// gfx950 multiplies bf16 sixteen times faster than fp32 on its matrix cores.  Every fp32
// operand is split exactly into three bf16 terms, x = h + m + l (h = bf16(x), m = bf16(x - h),
// l = bf16(x - h - m): 3 x 8 significand bits cover fp32's 24, and both differences are exact
// in fp32), and a product a * b is taken as the six term products whose weight is at least
// 2^-16 of the leading one:
//     a_h b_h  +  (a_h b_m + a_m b_h)  +  (a_h b_l + a_l b_h + a_m b_m).
// What is dropped (a_m b_l, a_l b_m, a_l b_l) is below 2^-24 of |a b|: the same size as one
// fp32 rounding.  Each term product is exact in the fp32 accumulator's input (8 x 8 bits), the
// leading products and the corrections are accumulated separately and added once at the end.
// Six bf16 MFMAs replace one fp32 MFMA of the same shape at 1/16 of the time each.
//
// Both operands are contiguous along k.  A lane keeps PF chunks of raw fp32 words in flight
// in registers (the prefetch), splits a chunk once on its way into LDS (three bf16 planes per
// operand, swizzled rows of 64 bytes), and two LDS stages alternate with one barrier per chunk.
// 64 samples x 128 classes per workgroup, 2 x 2 wavefronts, D cut into slices (partial sums
// go to the workspace as in the fp32 kernels).  DIFF: the operand is x_i - y_i (metric learning).
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

typedef __bf16 sbf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t su32x4 __attribute__((ext_vector_type(4)));

constexpr int kSsThreads = 256, kSsBM = 64, kSsBN = 128, kSsBK = 32;
constexpr int kSsRowB = kSsBK * 2;                                   // bytes per row of one bf16 plane
constexpr int kSsPlaneA = kSsBM * kSsRowB, kSsPlaneB = kSsBN * kSsRowB;
constexpr int kSsStageBytes = 3 * (kSsPlaneA + kSsPlaneB);

__device__ __forceinline__ int ss_swz(int r) { return (r >> 2) & 3; }   // 16-byte item c of row r sits at c ^ ss_swz(r)

__device__ __forceinline__ void ss_barrier() {
    // LDS writes of this wavefront visible, then the workgroup barrier; the prefetch loads stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// four consecutive k of one row -> 8 bytes per plane
__device__ __forceinline__ void split3_x4(f32x4 x, uint2& h, uint2& m, uint2& l) {
    split3_pair(x[0], x[1], h.x, m.x, l.x);
    split3_pair(x[2], x[3], h.y, m.y, l.y);
}

template <bool DIFF>
__global__ __launch_bounds__(kSsThreads) void scores_split_kernel(
    const float* __restrict__ A, const float* __restrict__ A2, int64_t lda, const float* __restrict__ W, int64_t ldw,
    float* __restrict__ Z, int64_t ldz, int64_t zstride, float* __restrict__ Vout, int64_t ldv, int M, int N, int K,
    int k_slice, int n_mb, int n_nb, int total) {
    constexpr int BM = kSsBM, BN = kSsBN, BK = kSsBK, ROWB = kSsRowB;
    constexpr int WGN = 2, WM = 32, WN = 64, NT = 2;
    constexpr int A_LD = BM * 8 / kSsThreads, W_LD = BN * 8 / kSsThreads;   // 16-byte pieces (4 fp32) per lane
    constexpr int ROW_STEP = kSsThreads / 8;                                 // rows between a lane's pieces
    extern __shared__ __attribute__((aligned(16))) unsigned char ss_lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, half = lane >> 5;

    // consecutive ids share the class block (its W rows then sit in one die's L2)
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int mb = id % n_mb;
    id /= n_mb;
    const int nb = id % n_nb, ks = id / n_nb;
    const int m0 = mb * BM, n0 = nb * BN;
    const int k_begin = ks * k_slice;
    const int n_chunks = (min(K, k_begin + k_slice) - k_begin) / BK;   // host: K % BK == 0

    // eight lanes per row: one wavefront instruction reads eight whole 128-byte lines.
    // Addresses = uniform base + 32-bit lane offset, rows clamped into the matrix.
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(A + (int64_t)m0 * lda + k_begin);
    const unsigned char* a2_base = DIFF ? reinterpret_cast<const unsigned char*>(A2 + (int64_t)m0 * lda + k_begin) : nullptr;
    const unsigned char* w_base = reinterpret_cast<const unsigned char*>(W + (int64_t)n0 * ldw + k_begin);
    const int r0 = tid >> 3, c0 = tid & 7;
    uint32_t a_off[A_LD], w_off[W_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
        a_off[i] = (uint32_t)min(r0 + i * ROW_STEP, M - 1 - m0) * (uint32_t)lda * 4u + 16u * c0;
#pragma unroll
    for (int i = 0; i < W_LD; ++i)
        w_off[i] = (uint32_t)min(r0 + i * ROW_STEP, N - 1 - n0) * (uint32_t)ldw * 4u + 16u * c0;
    // where a lane's four values land inside a plane (piece i: ROW_STEP rows further down, same swizzle)
    const int lds_piece = r0 * ROWB + 16 * ((c0 >> 1) ^ ss_swz(r0)) + 8 * (c0 & 1);
    // the class blocks share the copy: block nb takes the chunks c with c % n_nb == nb
    const bool write_v = Vout != nullptr;

    struct Chunk { f32x4 a[A_LD]; f32x4 a2[DIFF ? A_LD : 1]; f32x4 w[W_LD]; };
    auto fetch = [&](Chunk& r, int chunk) {
        const int cc = min(chunk, n_chunks - 1);       // past the end: a harmless repeat, never staged
        const int64_t kb = (int64_t)cc * (BK * 4);
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            r.a[i] = *reinterpret_cast<const f32x4*>(a_base + kb + a_off[i]);
            if (DIFF) r.a2[i] = *reinterpret_cast<const f32x4*>(a2_base + kb + a_off[i]);
        }
#pragma unroll
        for (int i = 0; i < W_LD; ++i) r.w[i] = *reinterpret_cast<const f32x4*>(w_base + kb + w_off[i]);
    };
    auto stage = [&](const Chunk& r, int st, int chunk) {
        unsigned char* sa = ss_lds + st * kSsStageBytes + lds_piece;
        unsigned char* sb = sa + 3 * kSsPlaneA;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            f32x4 x = r.a[i];
            if (DIFF) x -= r.a2[i];
            uint2 h, m, l;
            split3_x4(x, h, m, l);
            *reinterpret_cast<uint2*>(sa + i * ROW_STEP * ROWB) = h;
            *reinterpret_cast<uint2*>(sa + kSsPlaneA + i * ROW_STEP * ROWB) = m;
            *reinterpret_cast<uint2*>(sa + 2 * kSsPlaneA + i * ROW_STEP * ROWB) = l;
            if (write_v && (chunk % n_nb) == nb) {        // v_i = a_i (or x_i - y_i)
                const int row = m0 + r0 + i * ROW_STEP;
                if (row < M)
                    *reinterpret_cast<f32x4*>(Vout + (int64_t)row * ldv + k_begin + chunk * BK + 4 * c0) = x;
            }
        }
#pragma unroll
        for (int i = 0; i < W_LD; ++i) {
            uint2 h, m, l;
            split3_x4(r.w[i], h, m, l);
            *reinterpret_cast<uint2*>(sb + i * ROW_STEP * ROWB) = h;
            *reinterpret_cast<uint2*>(sb + kSsPlaneB + i * ROW_STEP * ROWB) = m;
            *reinterpret_cast<uint2*>(sb + 2 * kSsPlaneB + i * ROW_STEP * ROWB) = l;
        }
    };

    f32x16 lead[NT], corr[NT];      // leading products and corrections, added once at the end
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            lead[j][e] = 0.f;
            corr[j][e] = 0.f;
        }

    // every row a lane reads is congruent to l32 modulo 32: the swizzle is a lane constant
    const int frag_row = l32 * ROWB;
    const int frag_item[2] = {16 * ((0 + half) ^ ss_swz(l32)), 16 * ((2 + half) ^ ss_swz(l32))};
    auto mfma = [](su32x4 a, su32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sbf16x8, a), __builtin_bit_cast(sbf16x8, b), c,
                                                       0, 0, 0);
    };
    auto compute = [&](int st) {
        const unsigned char* as = ss_lds + st * kSsStageBytes + wm * WM * ROWB + frag_row;
        const unsigned char* bs = ss_lds + st * kSsStageBytes + 3 * kSsPlaneA + wn * WN * ROWB + frag_row;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            su32x4 fa[3], fb[3][NT];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                fa[p] = *reinterpret_cast<const su32x4*>(as + p * kSsPlaneA + frag_item[s]);
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    fb[p][j] = *reinterpret_cast<const su32x4*>(bs + p * kSsPlaneB + j * 32 * ROWB + frag_item[s]);
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                lead[j] = mfma(fa[0], fb[0][j], lead[j]);            // h h
                corr[j] = mfma(fa[0], fb[2][j], corr[j]);            // h l
                corr[j] = mfma(fa[2], fb[0][j], corr[j]);            // l h
                corr[j] = mfma(fa[1], fb[1][j], corr[j]);            // m m
                corr[j] = mfma(fa[0], fb[1][j], corr[j]);            // h m
                corr[j] = mfma(fa[1], fb[0][j], corr[j]);            // m h
            }
        }
    };

    // Chunk c waits in register slot c % 3 until it is staged, one step before it is
    // multiplied; the slot is then reloaded with chunk c + 3.  Straight-line groups of three
    // steps keep the slot indices static and every load three chunks ahead of its use.
    Chunk q0, q1, q2;
    fetch(q0, 0);
    fetch(q1, 1);
    fetch(q2, 2);
    stage(q0, 0, 0);
    ss_barrier();
    int c = 0;
    for (; c + 3 <= n_chunks; c += 3) {
        fetch(q0, c + 3);
        __builtin_amdgcn_sched_barrier(0);   // the loads go out before anything waits on older ones
        compute(c & 1);
        stage(q1, (c + 1) & 1, c + 1);
        ss_barrier();
        fetch(q1, c + 4);
        __builtin_amdgcn_sched_barrier(0);
        compute((c + 1) & 1);
        stage(q2, (c + 2) & 1, c + 2);
        ss_barrier();
        fetch(q2, c + 5);
        __builtin_amdgcn_sched_barrier(0);
        compute((c + 2) & 1);
        if (c + 3 < n_chunks) stage(q0, (c + 3) & 1, c + 3);
        ss_barrier();
    }
    // at most two chunks left; chunk c is staged, c + 1 sits in q1
    if (c < n_chunks) {
        compute(c & 1);
        if (c + 1 < n_chunks) {
            stage(q1, (c + 1) & 1, c + 1);
            ss_barrier();
            compute((c + 1) & 1);
        }
    }

    float* zout = Z + (int64_t)ks * zstride;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = n0 + wn * WN + j * 32 + l32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = m0 + wm * WM + 8 * (e / 4) + 4 * half + (e % 4);
            if (row < M && col < N) zout[(int64_t)row * ldz + col] = lead[j][e] + corr[j][e];
        }
    }
}

bool forward_split_ok(const FwdArgs& a) {
    auto al = [](const void* ptr, int64_t ld) { return ((uintptr_t)ptr % 16) == 0 && (ld % 4) == 0; };
    return !a.bf16 && al(a.a, a.lda) && (!a.diff || al(a.a2, a.lda)) && al(a.w, a.ldw) &&
           (a.v == nullptr || al(a.v, a.ldv)) && (a.D % kSsBK) == 0 && a.D >= kSsBK && a.lda < (1 << 23) &&
           a.ldw < (1 << 22);   // lane offsets (up to 64 rows of A, 128 of W, 4 bytes each) stay below 2^32
}

template <bool DIFF>
static hipError_t launch_split(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    constexpr size_t lds_bytes = 2 * (size_t)kSsStageBytes;
    static std::atomic<bool> raised{false};
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)scores_split_kernel<DIFF>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_mb = (a.n_rows + kSsBM - 1) / kSsBM, n_nb = (a.J + kSsBN - 1) / kSsBN;
    const int total = n_mb * n_nb * p.split_k;
    SFB_LAUNCH((scores_split_kernel<DIFF>), dim3(total), dim3(kSsThreads), lds_bytes, s, (const float*)a.a,
               (const float*)a.a2, a.lda, a.w, a.ldw, a.zp, a.ldz, a.zstride, (float*)a.v, a.ldv, a.n_rows, a.J, a.D,
               p.k_slice, n_mb, n_nb, total);
    return hipGetLastError();
}

// The plan must have been made for 64 x 128 tiles (p.bm, p.bn) with k_slice a multiple of 32.
hipError_t launch_forward_split(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    return a.diff ? launch_split<true>(a, p, s) : launch_split<false>(a, p, s);
}

}  // namespace sfb
