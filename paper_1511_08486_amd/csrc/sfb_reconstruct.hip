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
// Rows are interleaved by MT the same way.  The W tile is requested from HBM before the
// contraction starts and only consumed in the epilogue, so its latency hides under the MFMAs.
//
// alpha is folded into U while the tile is staged (one rounding per element), so the
// epilogue is a single add: W + acc.  U = 0 leaves W bit-identical.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kReconBK = 32;   // factor pairs per LDS stage
constexpr int kReconBN = 128;  // W columns per tile

template <int MT, int NWAVES, typename TV>
__global__ __launch_bounds__(NWAVES * 64) void reconstruct_apply_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const TV* __restrict__ V,
    int64_t ldv, int J, int D, int N, int B, float alpha, uint64_t live_mask, bool use_mask, int n_jb,
    int total, bool vec_w, bool vec_u, bool vec_v) {
    constexpr int BK = kReconBK, BN = kReconBN;
    constexpr int WMR = 32 * MT;            // rows per wavefront
    constexpr int BM = WMR * NWAVES;
    constexpr int THREADS = NWAVES * 64;
    constexpr int U_LD = BK * BM / 4 / THREADS;
    constexpr int V_LD = BK * BN / 4 / THREADS;
    static_assert(U_LD >= 1 && V_LD >= 1, "tile too small for the thread count");
    static_assert(MT == 1 || MT == 2 || MT == 4, "row interleave must be 1, 2 or 4");

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

    // ---- request the W tile now; it is consumed only in the epilogue ----
    f32x4 wreg[MT][16];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wave * WMR + MT * m + t;
            f32x4 w = {0.f, 0.f, 0.f, 0.f};
            if (row < J) w = load4(W + (int64_t)row * ldw, d0 + 4 * l32, D, vec_w);
            wreg[t][e] = w;
        }

    f32x4 ru[U_LD], rv[V_LD];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < U_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BM / 4), c = (idx % (BM / 4)) * 4;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (k < N && (!use_mask || ((live_mask >> (k / B)) & 1ull)))
                v = load4(U + (int64_t)k * ldu, j0 + c, J, vec_u) * alpha;
            ru[i] = v;
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BN / 4), c = (idx % (BN / 4)) * 4;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (k < N && (!use_mask || ((live_mask >> (k / B)) & 1ull)))
                v = load4(V + (int64_t)k * ldv, d0 + c, D, vec_v);
            rv[i] = v;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < U_LD; ++i) {
            const int idx = tid + i * THREADS;
            *reinterpret_cast<f32x4*>(&Us[buf * BK * BM + (idx / (BM / 4)) * BM + (idx % (BM / 4)) * 4]) = ru[i];
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            *reinterpret_cast<f32x4*>(&Vs[buf * BK * BN + (idx / (BN / 4)) * BN + (idx % (BN / 4)) * 4]) = rv[i];
        }
    };

    f32x16 acc[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][n][e] = 0.f;

    const int n_chunks = (N + BK - 1) / BK;
    fetch(0);
    stage(0);
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < n_chunks) fetch((c + 1) * BK);
        const float* us = &Us[buf * BK * BM + wave * WMR + MT * l32];
        const float* vs = &Vs[buf * BK * BN + 4 * l32];
#pragma unroll
        for (int s = 0; s < BK / 2; ++s) {
            const int k = 2 * s + half;
            float a[MT];
            if constexpr (MT == 1) {
                a[0] = us[k * BM];
            } else if constexpr (MT == 2) {
                const float2 t2 = *reinterpret_cast<const float2*>(&us[k * BM]);
                a[0] = t2.x;
                a[1] = t2.y;
            } else {
                const f32x4 t4 = *reinterpret_cast<const f32x4*>(&us[k * BM]);
#pragma unroll
                for (int t = 0; t < MT; ++t) a[t] = t4[t];
            }
            const f32x4 b = *reinterpret_cast<const f32x4*>(&vs[k * BN]);
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int n = 0; n < 4; ++n)
                    acc[t][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[n], acc[t][n], 0, 0, 0);
        }
        // the other buffer was last read before the previous barrier: safe to refill
        if (c + 1 < n_chunks) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: W <- W + acc, 128-bit read-modify-write ----
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
                store4(W + (int64_t)row * ldw, d0 + 4 * l32, D, vec_w, w);
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
    ReconPlan p;
    // largest tile that still yields at least two workgroups per compute unit; the
    // smallest tile otherwise
    const int order[] = {3, 0, 1, 2};
    p.variant = 2;
    for (int v : order) {
        const int64_t bm = 32 * kReconVariants[v].mt * kReconVariants[v].nwaves;
        const int64_t tiles = ((J + bm - 1) / bm) * ((D + kReconBN - 1) / kReconBN);
        if (tiles >= 512) { p.variant = v; break; }
    }
    if (J <= 32) p.variant = 2;
    return plan_reconstruct_variant(J, D, p.variant);
}

ReconPlan plan_reconstruct_variant(int64_t J, int64_t D, int variant) {
    ReconPlan p;
    p.variant = variant;
    p.bm = 32 * kReconVariants[variant].mt * kReconVariants[variant].nwaves;
    p.bn = kReconBN;
    p.grid = (int)(((J + p.bm - 1) / p.bm) * ((D + p.bn - 1) / p.bn));
    return p;
}

template <int MT, int NWAVES, typename TV>
static hipError_t launch_recon_t(const ReconArgs& a, hipStream_t s) {
    constexpr int BM = 32 * MT * NWAVES;
    const int n_jb = (a.J + BM - 1) / BM, n_db = (a.D + kReconBN - 1) / kReconBN;
    const int total = n_jb * n_db;
    const bool vec_w = ((uintptr_t)a.w % 16) == 0 && (a.ldw % 4) == 0;
    const bool vec_u = ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0;
    const bool vec_v = ((uintptr_t)a.v % (4 * sizeof(TV))) == 0 && (a.ldv % 4) == 0;
    constexpr size_t lds_bytes = 2 * kReconBK * (BM + kReconBN) * sizeof(float);
    static bool raised = false;   // opt in once to more than 64 KB of LDS per workgroup
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_kernel<MT, NWAVES, TV>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((reconstruct_apply_kernel<MT, NWAVES, TV>), dim3(total), dim3(NWAVES * 64), lds_bytes, s, a.w,
                       a.ldw, a.u, a.ldu, (const TV*)a.v, a.ldv, a.J, a.D, a.N, a.B, a.alpha, a.live_mask,
                       a.use_mask, n_jb, total, vec_w, vec_u, vec_v);
    return hipGetLastError();
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
