// Reconstruction + update (Section 3, Section 2.1) for fp32 factors on the bf16 matrix cores at
// fp32 accuracy:  W += alpha * U^T V  with every fp32 operand split exactly into three bf16
// terms and every product taken as its six leading term products (see sfb_forward_split.hip
// for the arithmetic and its error).
//
// The contraction runs over the factor pairs (the rows of U and V), which is the slow index of
// both operands in memory, while the bf16 MFMA wants eight consecutive k per lane.  The
// transposition happens in registers on the way into LDS: a lane loads a 4 (pairs) x 4
// (columns) block with four 16-byte loads, splits its 16 values, and writes, per plane, four
// 8-byte items "one column, four consecutive pairs".  Planes are [row = column of U or V][k]
// with rows padded to 80 bytes: the 8-byte writes of a wavefront then fall two per bank group
// (the minimum for 512 bytes) and the 16-byte fragment reads of 16 consecutive rows hit 16
// different bank groups.
// 128 x 128 tile of W, 8 wavefronts (4 x 2, two per SIMD: one splits while the other
// multiplies), three chunks of raw words prefetched in registers, two LDS stages, one barrier
// per 32 pairs.  The W tile is requested first and consumed in the epilogue.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

typedef __bf16 rbf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t ru32x4 __attribute__((ext_vector_type(4)));

constexpr int kRsThreads = 512, kRsBM = 128, kRsBN = 128, kRsBK = 32;
constexpr int kRsRowB = kRsBK * 2 + 16;                              // padded bytes per plane row
constexpr int kRsPlane = (kRsBM + kRsBN) * kRsRowB;                  // rows 0..127: U columns, 128..255: V columns
constexpr int kRsStageBytes = 3 * kRsPlane;

__device__ __forceinline__ void rs_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__global__ __launch_bounds__(kRsThreads, 2) void reconstruct_split_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a) {
    constexpr int BM = kRsBM, BN = kRsBN, BK = kRsBK, ROWB = kRsRowB;
    constexpr int WGN = 2, WM = 32, WN = 64, NT = 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char rs_lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, half = lane >> 5;
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // W tile first (clamped addresses, no branches); the loads are ordinary ones, the compiler
    // tracks them, and they have the whole contraction to arrive
    float wreg[NT][16];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = min(d0 + wn * WN + t * 32 + l32, D - 1);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = j0 + wm * WM + 8 * (e / 4) + 4 * half + (e % 4);
            wreg[t][e] = W[(int64_t)min(row, J - 1) * ldw + col];
        }
    }

    // lanes 0..255 stage U, 256..511 stage V: a 4 x 4 block (pairs 4kb.., columns 4rb..) each
    const bool is_v = tid >= 256;
    const int t8 = tid & 255, kb = t8 & 7, rb = t8 >> 3;
    const int ncols = is_v ? D : J;
    const int col0 = min((is_v ? d0 : j0) + 4 * rb, ncols - 4);       // host: J, D multiples of 4 and >= 4
    const int64_t ld = is_v ? ldv : ldu;
    const float* src = (is_v ? V : U) + col0 + (int64_t)(4 * kb) * ld;
    // first of the four rows this lane writes in a plane, at its 8-byte item
    const int lds_block = ((is_v ? BM : 0) + 4 * rb) * ROWB + 8 * kb;
    const int n_chunks = N / BK;                                       // host: N % BK == 0, N >= BK

    struct Chunk { f32x4 x[4]; };
    auto fetch = [&](Chunk& r, int chunk) {
        const float* p = src + (int64_t)min(chunk, n_chunks - 1) * BK * ld;   // past the end: a harmless repeat
#pragma unroll
        for (int i = 0; i < 4; ++i) r.x[i] = *reinterpret_cast<const f32x4*>(p + (int64_t)i * ld);
    };
    auto stage = [&](const Chunk& r, int st) {
        unsigned char* base = rs_lds + st * kRsStageBytes + lds_block;
        // per column e: the four pairs' terms as two packed words (pairs 0-1, 2-3), 8 bytes per plane
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint2 h, m, l;
            split3_pair(r.x[0][e], r.x[1][e], h.x, m.x, l.x);
            split3_pair(r.x[2][e], r.x[3][e], h.y, m.y, l.y);
            *reinterpret_cast<uint2*>(base + e * ROWB) = h;
            *reinterpret_cast<uint2*>(base + kRsPlane + e * ROWB) = m;
            *reinterpret_cast<uint2*>(base + 2 * kRsPlane + e * ROWB) = l;
        }
    };

    f32x16 lead[NT], corr[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            lead[t][e] = 0.f;
            corr[t][e] = 0.f;
        }
    auto mfma = [](ru32x4 a, ru32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(rbf16x8, a), __builtin_bit_cast(rbf16x8, b), c,
                                                       0, 0, 0);
    };
    const int a_row = (wm * WM + l32) * ROWB, b_row = (BM + wn * WN + l32) * ROWB;
    auto compute = [&](int st) {
        const unsigned char* sp = rs_lds + st * kRsStageBytes;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int item = 16 * (2 * s + half);
            ru32x4 fa[3], fb[3][NT];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                fa[p] = *reinterpret_cast<const ru32x4*>(sp + p * kRsPlane + a_row + item);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    fb[p][t] = *reinterpret_cast<const ru32x4*>(sp + p * kRsPlane + b_row + t * 32 * ROWB + item);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                lead[t] = mfma(fa[0], fb[0][t], lead[t]);            // h h
                corr[t] = mfma(fa[0], fb[2][t], corr[t]);            // h l
                corr[t] = mfma(fa[2], fb[0][t], corr[t]);            // l h
                corr[t] = mfma(fa[1], fb[1][t], corr[t]);            // m m
                corr[t] = mfma(fa[0], fb[1][t], corr[t]);            // h m
                corr[t] = mfma(fa[1], fb[0][t], corr[t]);            // m h
            }
        }
    };

    // Chunk c waits in register slot c % 3 until it is staged, one step before it is multiplied
    Chunk q0, q1, q2;
    fetch(q0, 0);
    fetch(q1, 1);
    fetch(q2, 2);
    stage(q0, 0);
    rs_barrier();
    int c = 0;
    for (; c + 3 <= n_chunks; c += 3) {
        fetch(q0, c + 3);
        __builtin_amdgcn_sched_barrier(0);   // the loads go out before anything waits on older ones
        compute(c & 1);
        stage(q1, (c + 1) & 1);
        rs_barrier();
        fetch(q1, c + 4);
        __builtin_amdgcn_sched_barrier(0);
        compute((c + 1) & 1);
        stage(q2, (c + 2) & 1);
        rs_barrier();
        fetch(q2, c + 5);
        __builtin_amdgcn_sched_barrier(0);
        compute((c + 2) & 1);
        if (c + 3 < n_chunks) stage(q0, (c + 3) & 1);
        rs_barrier();
    }
    if (c < n_chunks) {
        compute(c & 1);
        if (c + 1 < n_chunks) {
            stage(q1, (c + 1) & 1);
            rs_barrier();
            compute((c + 1) & 1);
        }
    }

    // W + alpha * (U^T V): lane l32 owns one column, 32 lanes cover a whole 128-byte line
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = d0 + wn * WN + t * 32 + l32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = j0 + wm * WM + 8 * (e / 4) + 4 * half + (e % 4);
            if (row < J && col < D) W[(int64_t)row * ldw + col] =
                    prox_entry(wreg[t][e] + alpha * (lead[t][e] + corr[t][e]), prox_kind, prox_a);
        }
    }
}

bool reconstruct_split_ok(const ReconArgs& a) {
    auto al = [](const void* ptr, int64_t ld) { return ((uintptr_t)ptr % 16) == 0 && (ld % 4) == 0; };
    return !a.bf16 && !a.use_mask && al(a.u, a.ldu) && al(a.v, a.ldv) && (a.J % 4) == 0 && a.J >= 4 &&
           (a.D % 4) == 0 && a.D >= 4 && (a.N % kRsBK) == 0 && a.N >= kRsBK;
}

hipError_t launch_reconstruct_split(const ReconArgs& a, hipStream_t s) {
    constexpr size_t lds_bytes = 2 * (size_t)kRsStageBytes;
    static std::atomic<bool> raised{false};
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_split_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_jb = (a.J + kRsBM - 1) / kRsBM, n_db = (a.D + kRsBN - 1) / kRsBN;
    const int total = n_jb * n_db;
    SFB_LAUNCH(reconstruct_split_kernel, dim3(total), dim3(kRsThreads), lds_bytes, s, a.w, a.ldw, a.u, a.ldu,
               (const float*)a.v, a.ldv, a.J, a.D, a.N, a.alpha, n_jb, total, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

}  // namespace sfb
