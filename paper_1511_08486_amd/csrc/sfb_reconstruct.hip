// Update reconstruction fused with the SGD step (Section 3 and Section 2.1):
//     W[j][d] <- W[j][d] + alpha * sum_n U[n][j] * V[n][d],   alpha = -eta * scale,
// n running over the N = P*B received factor pairs (rows of dead workers are skipped).
// This is a "TN" contraction with a short inner dimension N and a read-modify-write
// of W as its epilogue.  In the paper's cost table (Section 5.1) it is the O(P K J D)
// "W update time" of one worker.
//
// Both operands are stored n-major, so a row of the U tile (consecutive j) and a row of
// the V tile (consecutive d) are contiguous in HBM and in LDS, which is exactly the
// operand order of v_mfma_f32_32x32x2_f32: lane l supplies A[m = l%32][k = l/32] and
// B[k = l/32][n = l%32].  No transposes, no padding, conflict-free LDS reads.
//
// Tile shape.  A wavefront owns 32*MT rows x 128 columns.  Columns are interleaved by 4:
// MFMA column tile t of lane l is d0 + 4*(l%32) + t, so one 128-bit LDS read feeds the
// four column tiles and each lane ends up with four consecutive d of a W row: the W
// read-modify-write is done with 128-bit accesses, 512 contiguous bytes per half-wave.
// Rows are interleaved by MT the same way.
//
// Pipeline.  One wavefront per SIMD leaves no other wavefront to hide latency behind, so
// it is hidden in the instruction stream: factor rows are fetched from HBM/L2 two stages
// ahead into registers, staged through a double-buffered LDS tile (one barrier per
// stage), and the LDS operand fragments of the next four MFMA k-steps are read while the
// current four execute.  The FAST variant has no branch around any load: out-of-range
// rows are clamped into the matrix and zeroed by a select.
//
// alpha is folded into U while the tile is staged (one rounding per element); the sum of
// outer products is accumulated from zero and added to the prefetched W tile once, in the
// epilogue.  U = 0 leaves W bit-identical.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kReconBK = 32;   // factor pairs per LDS stage
constexpr int kReconBN = 128;  // W columns per tile
constexpr int kReconGroup = 4; // MFMA k-steps (of 2 factor pairs each) per operand fragment

// FAST: every pointer 16-byte aligned (8 for bf16 V), leading dimensions multiples of 4,
// D a multiple of 128 and J a multiple of 4 -- checked on the host.
template <int MT, int NWAVES, typename TV, bool FAST, bool MASK>
__global__ __launch_bounds__(NWAVES * 64) void reconstruct_apply_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const TV* __restrict__ V,
    int64_t ldv, int J, int D, int N, int B, float alpha, uint64_t live_mask, int n_jb, int total, bool vec_w,
    bool vec_u, bool vec_v) {
    constexpr int BK = kReconBK, BN = kReconBN, G = kReconGroup;
    constexpr int WMR = 32 * MT;            // rows per wavefront
    constexpr int BM = WMR * NWAVES;
    constexpr int THREADS = NWAVES * 64;
    constexpr int U_LD = BK * BM / 4 / THREADS;
    constexpr int V_LD = BK * BN / 4 / THREADS;
    constexpr int NGROUPS = BK / 2 / G;
    static_assert(U_LD >= 1 && V_LD >= 1, "tile too small for the thread count");
    static_assert(MT == 1 || MT == 2 || MT == 4, "row interleave must be 1, 2 or 4");
    static_assert(NGROUPS >= 1 && NGROUPS * G * 2 == BK, "stage depth must be a multiple of the fragment group");

    // two stages of the U tile [BK][BM] followed by two stages of the V tile [BK][BN]
    extern __shared__ __attribute__((aligned(16))) float recon_lds[];
    float* const Us = recon_lds;
    float* const Vs = recon_lds + 2 * BK * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;

    // consecutive ids walk down the J blocks of one column block, so the workgroups of a die
    // share a few column blocks of V and all of U in that die's L2.
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // Raw loaded words only: no arithmetic may depend on a load before the stage that
    // consumes it, or the wait for the load would move up to the load itself.
    using RawV = typename RawOf<TV>::type;
    struct Stage { f32x4 u[U_LD]; RawV v[V_LD]; };
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    auto row_live = [&](int k) {
        bool live = k < N;
        if (MASK) live = live && ((live_mask >> (min(k, N - 1) / B)) & 1ull);
        return live;
    };
    auto fetch = [&](Stage& r, int k0) {
#pragma unroll
        for (int i = 0; i < U_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BM / 4), c = j0 + (idx % (BM / 4)) * 4;
            if (FAST) {
                r.u[i] = ldg4(U + (int64_t)min(k, N - 1) * ldu + min(c, J - 4));
            } else {
                r.u[i] = k < N ? load4(U + (int64_t)k * ldu, c, J, vec_u) : zero4;
            }
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BN / 4), c = d0 + (idx % (BN / 4)) * 4;
            if (FAST) {
                r.v[i] = ldraw4(V + (int64_t)min(k, N - 1) * ldv + c);
            } else {
                r.v[i] = to_raw<TV>(k < N ? load4(V + (int64_t)k * ldv, c, D, vec_v) : zero4);
            }
        }
    };
    // alpha, the dead-row select and the bf16 widening happen here, on the way into LDS
    auto stage = [&](const Stage& r, int buf, int k0) {
#pragma unroll
        for (int i = 0; i < U_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BM / 4), c = j0 + (idx % (BM / 4)) * 4;
            const f32x4 v = (row_live(k) && c < J) ? r.u[i] * alpha : zero4;
            *reinterpret_cast<f32x4*>(&Us[buf * BK * BM + (idx / (BM / 4)) * BM + (idx % (BM / 4)) * 4]) = v;
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BN / 4);
            const f32x4 v = row_live(k) ? widen4(r.v[i]) : zero4;
            *reinterpret_cast<f32x4*>(&Vs[buf * BK * BN + (idx / (BN / 4)) * BN + (idx % (BN / 4)) * 4]) = v;
        }
    };

    f32x16 acc[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][n][e] = 0.f;

    struct Frag { float a[G][MT]; f32x4 b[G]; };
    auto read_frag = [&](Frag& f, int buf, int g) {
        const float* us = &Us[buf * BK * BM + wave * WMR + MT * l32];
        const float* vs = &Vs[buf * BK * BN + 4 * l32];
#pragma unroll
        for (int s = 0; s < G; ++s) {
            const int k = 2 * (g * G + s) + half;
            if constexpr (MT == 1) {
                f.a[s][0] = us[k * BM];
            } else if constexpr (MT == 2) {
                const float2 t2 = *reinterpret_cast<const float2*>(&us[k * BM]);
                f.a[s][0] = t2.x;
                f.a[s][1] = t2.y;
            } else {
                const f32x4 t4 = *reinterpret_cast<const f32x4*>(&us[k * BM]);
#pragma unroll
                for (int t = 0; t < MT; ++t) f.a[s][t] = t4[t];
            }
            f.b[s] = *reinterpret_cast<const f32x4*>(&vs[k * BN]);
        }
    };
    auto mma_frag = [&](const Frag& f) {
#pragma unroll
        for (int s = 0; s < G; ++s)
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int n = 0; n < 4; ++n)
                    acc[t][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[s][t], f.b[s][n], acc[t][n], 0, 0, 0);
    };
    // the LDS reads of fragment g+1 are issued before the MFMAs of fragment g
    auto compute = [&](int buf) {
        Frag f0, f1;
        read_frag(f0, buf, 0);
#pragma unroll
        for (int g = 0; g < NGROUPS; g += 2) {
            if (g + 1 < NGROUPS) read_frag(f1, buf, g + 1);
            __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the MFMAs they do not feed
            mma_frag(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 1 < NGROUPS) {
                if (g + 2 < NGROUPS) read_frag(f0, buf, g + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma_frag(f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    const int n_chunks = (N + BK - 1) / BK;
    Stage r0, r1;
    fetch(r0, 0);

    // ---- request the W tile right behind the first factor stage; it is only consumed in
    // the epilogue.  (Starting the accumulators from W instead would add every tiny
    // partial product to a large number and lose most of the update to rounding.) ----
    f32x4 wreg[MT][16];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wave * WMR + MT * m + t;
            if (FAST) {
                wreg[t][e] = ldg4(W + (int64_t)min(row, J - 1) * ldw + d0 + 4 * l32);
            } else {
                wreg[t][e] = row < J ? load4(W + (int64_t)row * ldw, d0 + 4 * l32, D, vec_w) : zero4;
            }
        }
    fetch(r1, BK);

    stage(r0, 0, 0);
    __syncthreads();
    // Invariant at the top of a pair of steps (c, c+1): LDS stage 0 holds chunk c, r1 holds
    // chunk c+1 (possibly still in flight), r0 is free.  The pair is one straight-line block
    // (no exit in the middle), so every fetch stays where it is written: two stages ahead of
    // its use.  A fetch past the last chunk reads clamped rows and stages zeros.
    int c = 0;
    for (; c + 1 < n_chunks; c += 2) {
        fetch(r0, (c + 2) * BK);
        compute(0);
        stage(r1, 1, (c + 1) * BK);
        __syncthreads();
        fetch(r1, (c + 3) * BK);
        compute(1);
        stage(r0, 0, (c + 2) * BK);
        __syncthreads();
    }
    if (c < n_chunks) compute(0);   // odd count: the last chunk is already staged

    // ---- epilogue: W <- W + acc, 128-bit stores ----
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wave * WMR + MT * m + t;
            if (row < J) {
                f32x4 w = wreg[t][e];
                w.x += acc[t][0][e];
                w.y += acc[t][1][e];
                w.z += acc[t][2][e];
                w.w += acc[t][3][e];
                if (FAST) *reinterpret_cast<f32x4*>(W + (int64_t)row * ldw + d0 + 4 * l32) = w;
                else store4(W + (int64_t)row * ldw, d0 + 4 * l32, D, vec_w, w);
            }
        }
}

struct ReconVariant { int mt, nwaves; };
static const ReconVariant kReconVariants[] = {
    {1, 4},  // 128 x 128 tile, 256 threads
    {1, 2},  // 64 x 128
    {1, 1},  // 32 x 128
    {2, 4},  // 256 x 128
};

ReconPlan plan_reconstruct(int64_t J, int64_t D, int64_t N) {
    (void)N;
    // largest tile that still gives every compute unit a workgroup; the smallest otherwise
    const int order[] = {3, 0, 1, 2};
    int variant = 2;
    for (int v : order) {
        const int64_t bm = 32 * kReconVariants[v].mt * kReconVariants[v].nwaves;
        const int64_t tiles = ((J + bm - 1) / bm) * ((D + kReconBN - 1) / kReconBN);
        if (tiles >= 256) { variant = v; break; }
    }
    if (J <= 32) variant = 2;
    return plan_reconstruct_variant(J, D, variant);
}

ReconPlan plan_reconstruct_variant(int64_t J, int64_t D, int variant) {
    ReconPlan p;
    p.variant = variant;
    p.bm = 32 * kReconVariants[variant].mt * kReconVariants[variant].nwaves;
    p.bn = kReconBN;
    p.grid = (int)(((J + p.bm - 1) / p.bm) * ((D + p.bn - 1) / p.bn));
    return p;
}

template <int MT, int NWAVES, typename TV, bool FAST, bool MASK>
static hipError_t launch_recon_f(const ReconArgs& a, hipStream_t s, bool vec_w, bool vec_u, bool vec_v) {
    constexpr int BM = 32 * MT * NWAVES;
    const int n_jb = (a.J + BM - 1) / BM, n_db = (a.D + kReconBN - 1) / kReconBN;
    const int total = n_jb * n_db;
    constexpr size_t lds_bytes = 2 * kReconBK * (BM + kReconBN) * sizeof(float);
    static bool raised = false;   // opt in once to more than 64 KB of LDS per workgroup
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_kernel<MT, NWAVES, TV, FAST, MASK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((reconstruct_apply_kernel<MT, NWAVES, TV, FAST, MASK>), dim3(total), dim3(NWAVES * 64),
                       lds_bytes, s, a.w, a.ldw, a.u, a.ldu, (const TV*)a.v, a.ldv, a.J, a.D, a.N, a.B, a.alpha,
                       a.live_mask, n_jb, total, vec_w, vec_u, vec_v);
    return hipGetLastError();
}

template <int MT, int NWAVES, typename TV>
static hipError_t launch_recon_t(const ReconArgs& a, hipStream_t s) {
    const bool vec_w = ((uintptr_t)a.w % 16) == 0 && (a.ldw % 4) == 0;
    const bool vec_u = ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0;
    const bool vec_v = ((uintptr_t)a.v % (4 * sizeof(TV))) == 0 && (a.ldv % 4) == 0;
    const bool fast = vec_w && vec_u && vec_v && (a.D % kReconBN) == 0 && (a.J % 4) == 0 && a.J >= 4;
    if (a.use_mask) {   // a worker is missing: rare, so only the generic kernel carries the mask
        return launch_recon_f<MT, NWAVES, TV, false, true>(a, s, vec_w, vec_u, vec_v);
    }
    if (fast) return launch_recon_f<MT, NWAVES, TV, true, false>(a, s, vec_w, vec_u, vec_v);
    return launch_recon_f<MT, NWAVES, TV, false, false>(a, s, vec_w, vec_u, vec_v);
}

template <typename TV>
static hipError_t launch_recon_v(const ReconArgs& a, const ReconPlan& p, hipStream_t s) {
    switch (p.variant) {
        case 0: return launch_recon_t<1, 4, TV>(a, s);
        case 1: return launch_recon_t<1, 2, TV>(a, s);
        case 2: return launch_recon_t<1, 1, TV>(a, s);
        case 3: return launch_recon_t<2, 4, TV>(a, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_reconstruct(const ReconArgs& a, const ReconPlan& p, hipStream_t s) {
    return a.bf16 ? launch_recon_v<bf16_t>(a, p, s) : launch_recon_v<float>(a, p, s);
}

}  // namespace sfb
