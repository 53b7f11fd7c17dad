// Reconstruction + update (Section 3, Section 2.1), fine-grained form:
//     W[j][d] <- W[j][d] + alpha * sum_n U[n][j] * V[n][d]
// with 64 x 64 tiles of W and ONE 32 x 32 MFMA block per wavefront.
//
// Why a second tile shape.  The unit of matrix-core work is a 32 x 32 block of W carried
// through all N factor pairs, and a launch is as slow as its busiest SIMD.  With the 32 x 128
// wavefront tiles of the other kernels a SIMD gets work in lumps of four blocks: J = 600,
// D = 4096 is 2432 blocks for 1024 SIMDs, 2.4 each on average, but 4 for the busiest.  Handing
// out single blocks (2560 wavefronts, two or three per SIMD) makes that 3 (measured: the time
// per factor pair drops from 4.0 to 3.5 block times, J = 600: 71 -> 64 us).  The price is less
// operand reuse: every MFMA needs its own two LDS words, and a 64 x 64 tile fetches twice the
// factor bytes per flop of a 128 x 128 one -- affordable, the factors sit in L2.  The host
// picks this kernel only where the block count says it wins.
//
// Staging is the LDS-DMA ring of the larger kernel: factor tiles [k][64] go from L2 straight
// into LDS (lds_dma16), three stages, completion tracked by hand with the in-order
// vector-memory counter; the W block is requested after the first stage (ordinary loads) and
// consumed in the epilogue.  alpha and the entrywise proximal operator are applied there.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kRsmBM = 64, kRsmBN = 64, kRsmBK = 32, kRsmStages = 3, kRsmThreads = 256;

// PARTIAL: the factor pairs are cut into slices of k_rows and the grid holds `tiles` workgroups per slice;
// the workgroup of slice s contracts only its pairs and stores the bare sums (no alpha, no W, no proximal
// operator) into plane s of W = the partial-sum planes [slice][J][ldw], which apply_partials_kernel then
// adds up in slice order into the real W.
template <bool PARTIAL>
__global__ __launch_bounds__(kRsmThreads) void reconstruct_apply_small_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a, int tiles,
    int k_rows, int64_t pstride) {
    constexpr int BM = kRsmBM, BN = kRsmBN, BK = kRsmBK, NST = kRsmStages, THREADS = kRsmThreads;
    constexpr int U_LD = BK * BM / 4 / THREADS, V_LD = BK * BN / 4 / THREADS;      // 16-byte DMAs per thread and stage
    constexpr int DMAS = U_LD + V_LD;
    constexpr int STAGE_FLOATS = BK * (BM + BN);
    constexpr int W_LOADS = PARTIAL ? 0 : 16;
    static_assert(U_LD == 2 && V_LD == 2, "tile / thread count mismatch");
    static_assert(NST == 3, "ring depth");
    static_assert(DMAS + W_LOADS <= 63, "wait count encoding");
    __shared__ __attribute__((aligned(16))) float lds[NST * STAGE_FLOATS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wr = wave >> 1, wc = wave & 1;                // this wavefront's 32 x 32 block of the tile
    int id = xcd_contiguous_id(blockIdx.x, total);
    if constexpr (PARTIAL) {
        const int slice = id / tiles;                        // a die's workgroups share a slice's rows of U and V
        id -= slice * tiles;
        U += (int64_t)slice * k_rows * ldu;
        V += (int64_t)slice * k_rows * ldv;
        W += (int64_t)slice * pstride;
        N = min(k_rows, N - slice * k_rows);                 // host: positive, a multiple of BK
    }
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // source of DMA i of a stage: item idx = tid + i * THREADS, row idx / 16 of the chunk,
    // 16-byte item idx % 16 of the 64-float row.  Columns of U beyond J rounded up to 4 are clamped
    // (host: a row of U holds that many floats): they feed rows of W that are never stored.
    const int ju = (J + 3) & ~3;
    const float* pu[U_LD];
    const float* pv[V_LD];
#pragma unroll
    for (int i = 0; i < U_LD; ++i) {
        const int idx = tid + i * THREADS;
        pu[i] = U + (int64_t)(idx / (BM / 4)) * ldu + min(j0 + (idx % (BM / 4)) * 4, ju - 4);
    }
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
        const int idx = tid + i * THREADS;
        pv[i] = V + (int64_t)(idx / (BN / 4)) * ldv + d0 + (idx % (BN / 4)) * 4;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int64_t ustep = (int64_t)BK * ldu, vstep = (int64_t)BK * ldv;
    auto issue = [&](int chunk, int st) {
        const uint32_t ubase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_FLOATS + wave * 64 * 4) * 4u);
        const uint32_t vbase = ubase + (uint32_t)(BK * BM) * 4u;
#pragma unroll
        for (int i = 0; i < U_LD; ++i) lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * THREADS * 16));
#pragma unroll
        for (int i = 0; i < V_LD; ++i) lds_dma16(pv[i] + chunk * vstep, vbase + (uint32_t)(i * THREADS * 16));
    };

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;

    // MFMA k-step kk covers pairs 2 kk and 2 kk + 1 of the chunk: lanes 0-31 carry the first
    // (row / column l32), lanes 32-63 the second.  All 32 operand words of a chunk are read
    // before its first MFMA, so that no MFMA but the first waits on LDS.
    auto compute = [&](int st) {
        const float* us = &lds[st * STAGE_FLOATS + wr * 32 + l32 + half * BM];
        const float* vs = &lds[st * STAGE_FLOATS + BK * BM + wc * 32 + l32 + half * BN];
        constexpr int KS = BK / 2;
        float a[KS], b[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            a[s] = us[2 * s * BM];
            b[s] = vs[2 * s * BN];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int n_chunks = N / BK;   // host: N % BK == 0, N >= BK
    issue(0, 0);
    if (1 < n_chunks) issue(1, 1);

    // step c: my DMAs of chunk c have landed once at most `allowed` younger operations are
    // outstanding; the barrier makes everybody's visible and says that stage (c - 1) % 3 is
    // free again, which the DMAs of chunk c + 2 then refill
    auto step = [&](int c, int st, int allowed) {
        if (allowed >= DMAS + W_LOADS) wait_vmcnt<DMAS + W_LOADS>();
        else if (allowed >= W_LOADS) wait_vmcnt<W_LOADS>();
        else if (allowed >= DMAS) wait_vmcnt<DMAS>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (c + 2 < n_chunks) issue(c + 2, st == 0 ? 2 : st - 1);
        compute(st);
    };

    step(0, 0, 1 < n_chunks ? DMAS : 0);
    // W block after the first stage: nothing competes with chunk 0 for the first MFMA, and the
    // loads have the rest of the contraction to arrive.  In counter order they sit between the
    // DMAs of chunk 2 and those of chunk 3: while chunks 1 and 2 are waited for they count as
    // younger operations, from chunk 3 on they are older and have retired.
    float wreg[16];
    const int col = d0 + wc * 32 + l32;                     // beyond D only in the last tile of padded factors
    const int colc = min(col, D - 1);
    if constexpr (!PARTIAL) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = j0 + wr * 32 + 8 * (e / 4) + 4 * half + (e % 4);
            wreg[e] = W[(int64_t)min(row, J - 1) * ldw + colc];
        }
    }
    int st = 1;
    for (int c = 1; c < n_chunks; ++c) {
        step(c, st, (c + 1 < n_chunks ? DMAS : 0) + (c <= 2 ? W_LOADS : 0));
        st = st == 2 ? 0 : st + 1;
    }

#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int row = j0 + wr * 32 + 8 * (e / 4) + 4 * half + (e % 4);
        if constexpr (PARTIAL) {
            if (row < J) W[(int64_t)row * ldw + col] = acc[e];          // a plane holds whole column tiles
        } else {
            if (row < J && col < D) W[(int64_t)row * ldw + col] = prox_entry(wreg[e] + alpha * acc[e], prox_kind, prox_a);
        }
    }
}

bool reconstruct_small_ok(const ReconArgs& a) {
    auto al = [](const void* p, int64_t ld) { return ((uintptr_t)p % 16) == 0 && (ld % 4) == 0; };
    if (a.bf16 || a.use_mask || !al(a.u, a.ldu) || !al(a.v, a.ldv) || (a.tile_cols() % kRsmBN) != 0 ||
        (a.N % kRsmBK) != 0 || a.N < kRsmBK)
        return false;
    return a.conformed || ((a.J % 4) == 0 && a.J >= 4);     // padded copies of U hold J rounded up to 4 columns
}

// 32 x 32 blocks the busiest SIMD carries when the work is handed out as `waves` wavefronts
// of `blocks_per_wave` blocks each (1024 SIMDs; the dispatcher spreads wavefronts evenly).
static int64_t busiest_simd_blocks(int64_t waves, int blocks_per_wave) {
    return (waves + 1023) / 1024 * blocks_per_wave;
}

// True when single-block wavefronts finish clearly sooner than the given larger tile would.
bool reconstruct_small_wins(int64_t J, int64_t D, int big_bm, int big_waves) {
    if ((D % kRsmBN) != 0) return false;
    const int64_t small_waves = ((J + kRsmBM - 1) / kRsmBM) * (D / kRsmBN) * 4;
    const int64_t big_tiles = ((J + big_bm - 1) / big_bm) * ((D + 127) / 128);
    const int blocks_per_big_wave = (big_bm / big_waves) / 32 * 4;
    return 10 * busiest_simd_blocks(small_waves, 1) <= 8 * busiest_simd_blocks(big_tiles * big_waves, blocks_per_big_wave);
}

hipError_t launch_reconstruct_small(const ReconArgs& a, hipStream_t s) {
    const int n_jb = (a.J + kRsmBM - 1) / kRsmBM, n_db = a.tile_cols() / kRsmBN;
    const int total = n_jb * n_db;
    SFB_LAUNCH(reconstruct_apply_small_kernel<false>, dim3(total), dim3(kRsmThreads), 0, s, a.w, a.ldw, a.u, a.ldu,
               (const float*)a.v, a.ldv, a.J, a.D, a.N, a.alpha, n_jb, total, a.prox_kind, a.prox_a, total, 0,
               (int64_t)0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Few tiles, many factor pairs (ten classes x 784 features with 12000 pairs: 14 tiles, 375 stages):
// one workgroup per tile leaves most of the chip idle for a long walk.  The pairs are cut into
// n_split slices, tiles x n_split workgroups store their slice's bare sums into planes of the
// workspace, and one streaming kernel adds the planes in slice order -- a fixed order, so results do
// not depend on timing -- scales by alpha, adds W and applies the proximal operator.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void apply_partials_kernel(float* __restrict__ W, int64_t ldw,
                                                             const float* __restrict__ P, int64_t ldp, int64_t pstride,
                                                             int n_split, int J, int D, float alpha, int n_cb,
                                                             int prox_kind, float prox_a) {
    const int row = blockIdx.x / n_cb, col = (blockIdx.x % n_cb) * 256 + threadIdx.x;
    if (row >= J || col >= D) return;
    const float* p = P + (int64_t)row * ldp + col;
    float sum = 0.f;
    for (int k = 0; k < n_split; ++k) sum += p[(int64_t)k * pstride];
    float* w = W + (int64_t)row * ldw + col;
    *w = prox_entry(*w + alpha * sum, prox_kind, prox_a);
}

// Slices of the pairs for a (J, D, N) whose plan is the single-block tile: the count that minimises, in
// microseconds, max(latency of one workgroup's walk, the busiest compute unit's share of all walks) + the
// adding-up pass.  A stage of 32 pairs takes a lone wavefront per SIMD about 0.67 us, and a compute unit
// turns over one workgroup-stage per 0.49 us when several workgroups share it.  1: do not split.
int reconstruct_small_split(int64_t J, int64_t D, int64_t N, int* k_rows) {
    *k_rows = 0;
    if ((D % kRsmBN) != 0 || (N % kRsmBK) != 0) return 1;
    const int64_t tiles = ((J + kRsmBM - 1) / kRsmBM) * (D / kRsmBN), chunks = N / kRsmBK;
    int64_t best = 1;
    double best_cost = 1e300, whole_cost = 1e300;
    for (int64_t s = 1; s <= 32 && (s == 1 || chunks / s >= 4); ++s) {
        const int64_t per = (chunks + s - 1) / s;
        if ((chunks + per - 1) / per != s) continue;                          // the same cut as a smaller count
        if (s > 1 && s * J * D * 4 > (64LL << 20)) break;                     // planes of partial sums: 64 MB at most
        const double latency = (double)per * 0.67;
        const double share = (double)((tiles * s + 255) / 256) * (double)per * 0.49;
        double cost = (latency > share ? latency : share) + 6.0;
        if (s > 1) cost += 6.0 + ((double)s * (double)J * (double)D * 4.0 + (double)J * (double)D * 8.0) / 4e6;
        if (s == 1) whole_cost = cost;
        else if (cost < best_cost * 0.95) { best_cost = cost; best = s; }     // a further slice must buy 5 %
    }
    if (best == 1 || best_cost > 0.8 * whole_cost) return 1;                  // and splitting at all 20 %
    *k_rows = (int)((chunks + best - 1) / best * kRsmBK);
    return (int)best;
}

size_t reconstruct_small_split_workspace(int n_split, int64_t J, int64_t D) {
    return n_split > 1 ? ((size_t)n_split * (size_t)J * (size_t)D * sizeof(float) + 255) / 256 * 256 : 0;
}

// a.partial: n_split planes of J x a.tile_cols() floats, 256-byte aligned.
hipError_t launch_reconstruct_small_split(const ReconArgs& a, int n_split, int k_rows, hipStream_t s) {
    const int n_jb = (a.J + kRsmBM - 1) / kRsmBM, n_db = a.tile_cols() / kRsmBN;
    const int tiles = n_jb * n_db, total = tiles * n_split;
    const int64_t ldp = a.tile_cols(), pstride = (int64_t)a.J * ldp;
    SFB_LAUNCH(reconstruct_apply_small_kernel<true>, dim3(total), dim3(kRsmThreads), 0, s, a.partial, ldp, a.u, a.ldu,
               (const float*)a.v, a.ldv, a.J, a.D, a.N, 1.0f, n_jb, total, 0, 0.f, tiles, k_rows, pstride);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n_cb = (a.D + 255) / 256;
    hipLaunchKernelGGL(apply_partials_kernel, dim3(a.J * n_cb), dim3(256), 0, s, a.w, a.ldw, a.partial, ldp, pstride,
                       n_split, a.J, a.D, a.alpha, n_cb, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

}  // namespace sfb
