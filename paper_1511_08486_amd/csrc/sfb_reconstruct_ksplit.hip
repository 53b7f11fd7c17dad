// Reconstruction + update (Section 3, Section 2.1), evenly divided form:
//     W[j][d] <- W[j][d] + alpha * sum_n U[n][j] * V[n][d]
// with tiles of 32*RB rows x 64 columns of W and four wavefronts that split BOTH the tile's
// two column blocks and every stage's factor pairs.
//
// Why a third tile shape.  A launch is as slow as its busiest SIMD.  The unit the other kernels
// hand out is a whole 32 x 32 block of W carried through all N pairs: J = 600, D = 4096 is
// 19 x 128 = 2432 blocks for 1024 SIMDs, 2.4 each on average but 3 on the busiest even with
// single-block wavefronts (and a lone wavefront in the last round hides none of its waits: 3.5
// block times measured).  Here a wavefront carries RB blocks (one column block of the tile, all
// its row blocks) through HALF of the pairs, its partner the other half; the two exchange partial
// sums through LDS once, at the end, and each finishes half of every block.  J = 600 becomes four
// row tiles of five row blocks x 64 column tiles = 256 workgroups, one per compute unit, and
// every SIMD multiplies exactly 5 blocks x N/2 pairs = 2.5 block times, 95 % of it on rows that
// exist.  The B fragment (v) of a step feeds RB matrix instructions, and four of the row blocks
// share one 16-byte LDS read (rows interleaved by four, as the columns are in the large kernel).
//
// Staging is the LDS-DMA ring of the other kernels: per stage 32 pairs of u [k][32*RB] and of
// v [k][64] go from L2 straight into LDS, four stages, completion counted by hand with the
// in-order vector-memory counter; the W entries a wavefront finishes are requested after the
// first stage and consumed in the epilogue, where alpha and the entrywise proximal operator are
// applied.  Sums are formed as (first half of every stage's pairs) + (second half), then added
// to W: one fixed order, results do not depend on timing.
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kRksBN = 64, kRksBK = 32, kRksStages = 4, kRksThreads = 256;

template <int RB>
__global__ __launch_bounds__(kRksThreads) void reconstruct_apply_ksplit_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a) {
    constexpr int BM = 32 * RB, BN = kRksBN, BK = kRksBK, NST = kRksStages, THREADS = kRksThreads;
    constexpr int U_LD = BK * BM / 4 / THREADS, V_LD = BK * BN / 4 / THREADS;      // 16-byte DMAs per thread and stage
    constexpr int DMAS = U_LD + V_LD;
    constexpr int STAGE_FLOATS = BK * (BM + BN);
    constexpr int NQD = RB / 4;                  // groups of four row blocks read with one 16-byte LDS read (rows interleaved)
    constexpr int NS = RB - 4 * NQD;             // remaining row blocks: 32 consecutive rows each
    constexpr int W_LOADS = RB * 8;              // a wavefront finishes half of each of its RB blocks
    static_assert(U_LD == RB && V_LD == 2, "tile / thread count mismatch");
    static_assert(NST == 4, "ring depth");
    static_assert(DMAS + W_LOADS <= 63, "wait count encoding");
    static_assert(4 * RB * 2 * 1024 <= NST * STAGE_FLOATS * 4, "the exchange area reuses the stage ring");
    extern __shared__ __attribute__((aligned(16))) float rks_lds[];      // NST * STAGE_FLOATS

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wc = wave & 1, kh = wave >> 1;                // column block of the tile, half of every stage's pairs
    const int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // source of DMA i of a stage: item idx = tid + i * THREADS of the [k][BM] (resp. [k][64]) tile in row-major
    // order of 16-byte items.  Columns of U beyond J are clamped (host: J % 4 == 0, J >= 4): they feed rows
    // of W that are never stored.
    const float* pu[U_LD];
    const float* pv[V_LD];
#pragma unroll
    for (int i = 0; i < U_LD; ++i) {
        const int idx = tid + i * THREADS;
        pu[i] = U + (int64_t)(idx / (BM / 4)) * ldu + min(j0 + (idx % (BM / 4)) * 4, J - 4);
    }
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
        const int idx = tid + i * THREADS;
        pv[i] = V + (int64_t)(idx / (BN / 4)) * ldv + d0 + (idx % (BN / 4)) * 4;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)rks_lds;
    const int64_t ustep = (int64_t)BK * ldu, vstep = (int64_t)BK * ldv;
    auto issue = [&](int chunk, int st) {
        const uint32_t ubase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_FLOATS + wave * 64 * 4) * 4u);
        const uint32_t vbase = ubase + (uint32_t)(BK * BM) * 4u;
#pragma unroll
        for (int i = 0; i < U_LD; ++i) lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * THREADS * 16));
#pragma unroll
        for (int i = 0; i < V_LD; ++i) lds_dma16(pv[i] + chunk * vstep, vbase + (uint32_t)(i * THREADS * 16));
    };

    // Row of the tile that accumulator entry m (0..31, the MFMA row index) of block b stands for.
    auto tile_row = [](int b, int m) { return b < 4 * NQD ? 128 * (b / 4) + 4 * m + (b % 4) : 128 * NQD + 32 * (b - 4 * NQD) + m; };

    f32x16 acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    // MFMA k-step s (0..7) of this wavefront's half covers pairs 16 kh + 2 s and + 1 of the stage: lanes 0-31
    // carry the first (row / column l32), lanes 32-63 the second.  The operand words of four k-steps form one
    // set of fragments; a stage is two sets.
    struct Frags {
        f32x4 aq[4][NQD > 0 ? NQD : 1];
        float as[4][NS > 0 ? NS : 1], bv[4];
    };
    // k-step s of half h of a stage
    auto load_step = [&](int st, int h, int s, Frags& f) {
        const float* us = &rks_lds[st * STAGE_FLOATS + (16 * kh + 8 * h + half) * BM];
        const float* vs = &rks_lds[st * STAGE_FLOATS + BK * BM + (16 * kh + 8 * h + half) * BN + wc * 32 + l32];
#pragma unroll
        for (int q = 0; q < NQD; ++q) f.aq[s][q] = *reinterpret_cast<const f32x4*>(us + 2 * s * BM + 128 * q + 4 * l32);
#pragma unroll
        for (int r = 0; r < NS; ++r) f.as[s][r] = us[2 * s * BM + 128 * NQD + 32 * r + l32];
        f.bv[s] = vs[2 * s * BN];
    };
    auto load_frags = [&](int st, int h, Frags& f) {
#pragma unroll
        for (int s = 0; s < 4; ++s) load_step(st, h, s, f);
    };
    // The matrix instructions of one set; between(s) runs after those of k-step s: whatever else has to be
    // issued (LDS reads of a later set, copies of a later chunk) goes there, one piece per k-step, so that it
    // is issued in the shadow of the matrix pipe instead of in one lump between two sets.
    auto multiply = [&](const Frags& f, auto between) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NQD; ++q)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[4 * q + t] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.aq[s][q][t], f.bv[s], acc[4 * q + t], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < NS; ++r)
                acc[4 * NQD + r] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.as[s][r], f.bv[s], acc[4 * NQD + r], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            between(s);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // copy instruction i (0 .. DMAS - 1) of a chunk
    auto issue_one = [&](int chunk, int st, int i) {
        const uint32_t ubase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_FLOATS + wave * 64 * 4) * 4u);
        if (i < U_LD) lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * THREADS * 16));
        else lds_dma16(pv[i - U_LD] + chunk * vstep, ubase + (uint32_t)(BK * BM) * 4u + (uint32_t)((i - U_LD) * THREADS * 16));
    };
    auto wait_allowing = [&](int allowed) {      // at most `allowed` younger operations may still be outstanding
        if (allowed >= DMAS + W_LOADS) wait_vmcnt<DMAS + W_LOADS>();
        else if (allowed >= W_LOADS) wait_vmcnt<W_LOADS>();
        else if (allowed >= 2 * DMAS) wait_vmcnt<2 * DMAS>();
        else if (allowed >= DMAS) wait_vmcnt<DMAS>();
        else wait_vmcnt<0>();
    };

    const int n_chunks = N / BK;   // host: N % BK == 0, N >= BK
    issue(0, 0);
    if (1 < n_chunks) issue(1, 1);
    if (2 < n_chunks) issue(2, 2);
    wait_allowing(DMAS * min(2, n_chunks - 1));
    __builtin_amdgcn_s_barrier();
    Frags fa, fb;
    load_frags(0, 0, fa);
    // The W entries this wavefront finishes (accumulator entries 8 kh .. 8 kh + 7 of every block): requested
    // once the first fragments are on their way, consumed in the epilogue.  In counter order they sit after the
    // copies of chunks 0-2 and before those of chunk 3: they count as younger operations while chunks 1 and 2
    // are waited for, from chunk 3 on they are older and have retired.
    float wreg[RB][8];
    const int col = d0 + wc * 32 + l32;                     // host: D % 64 == 0, so col < D
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int e = 8 * kh + t;
            const int row = j0 + tile_row(b, 8 * (e / 4) + 4 * half + (e % 4));
            wreg[b][t] = W[(int64_t)min(row, J - 1) * ldw + col];
        }
    // This is the only wavefront of its SIMD: nothing else hides an LDS wait or a barrier.  So the hand-over to
    // the next chunk sits in the MIDDLE of a chunk's matrix work: first half multiplied while the second half of
    // the fragments is read, then (my copies of chunk c + 1 have landed; barrier: everybody's have, and
    // everybody is past chunk c - 1, whose stage the copies of chunk c + 3 now refill), second half multiplied
    // while those copies are issued and the first fragments of chunk c + 1 are read.
    // (the last chunk is written out on its own so that the loop body is one straight line: the LDS reads of
    // the next set then need no more than the counted waits)
    for (int c = 0; c + 1 < n_chunks; ++c) {
        const int st = c & 3;
        multiply(fa, [&](int s) { load_step(st, 1, s, fb); });
        wait_allowing((c + 2 < n_chunks ? DMAS : 0) + (c <= 1 ? W_LOADS : 0));
        __builtin_amdgcn_s_barrier();
        const bool more = c + 3 < n_chunks;
        multiply(fb, [&](int s) {
            if (more) {
#pragma unroll
                for (int i = 0; i < DMAS; ++i)
                    if (i * 4 / DMAS == s) issue_one(c + 3, (c + 3) & 3, i);
            }
            load_step((c + 1) & 3, 0, s, fa);
        });
    }
    multiply(fa, [&](int s) { load_step((n_chunks - 1) & 3, 1, s, fb); });
    multiply(fb, [](int) {});

    // Exchange of partial sums: every stage has been read (barrier), the ring is free.  Slot of wavefront w,
    // block b: two 16-byte items per lane = the eight accumulator entries the PARTNER finishes.
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    f32x4* xch = reinterpret_cast<f32x4*>(rks_lds);
    auto finish = [&](auto KHc) {
        constexpr int KH = decltype(KHc)::value;
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                constexpr int e0 = 8 * (1 - KH);
                xch[((wave * RB + b) * 2 + j) * 64 + lane] =
                    f32x4{acc[b][e0 + 4 * j], acc[b][e0 + 4 * j + 1], acc[b][e0 + 4 * j + 2], acc[b][e0 + 4 * j + 3]};
            }
        __syncthreads();
        const int partner = wave ^ 2;
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const f32x4 p = xch[((partner * RB + b) * 2 + j) * 64 + lane];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int t = 4 * j + u, e = 8 * KH + t;
                    const float sum = KH == 0 ? acc[b][e] + p[u] : p[u] + acc[b][e];      // (first half) + (second half)
                    const int row = j0 + tile_row(b, 8 * (e / 4) + 4 * half + (e % 4));
                    if (row < J) W[(int64_t)row * ldw + col] = prox_entry(wreg[b][t] + alpha * sum, prox_kind, prox_a);
                }
            }
    };
    // both branches reach the same barrier inside: the condition is workgroup-wide per wavefront, not per lane
    if (kh == 0) finish(std::integral_constant<int, 0>{});
    else finish(std::integral_constant<int, 1>{});
}

// Row blocks per tile: as few row tiles as keep a tile within five row blocks.
static int ksplit_rb(int64_t J) {
    const int64_t n_rb = (J + 31) / 32;
    const int64_t tiles = (n_rb + 4) / 5;
    return (int)((n_rb + tiles - 1) / tiles);
}

bool reconstruct_ksplit_ok(const ReconArgs& a) {
    auto al = [](const void* p, int64_t ld) { return ((uintptr_t)p % 16) == 0 && (ld % 4) == 0; };
    const int rb = ksplit_rb(a.J);
    return !a.bf16 && !a.use_mask && al(a.u, a.ldu) && al(a.v, a.ldv) && (a.D % kRksBN) == 0 && (a.J % 4) == 0 &&
           a.J >= 4 && (a.N % kRksBK) == 0 && a.N >= kRksBK && rb >= 3 && rb <= 5;
}

int reconstruct_ksplit_rows(int64_t J) { return 32 * ksplit_rb(J); }

// True when splitting the pairs leaves the busiest SIMD with clearly less than `other_blocks`
// whole-block times (what the tile it would replace gives it).
bool reconstruct_ksplit_wins(int64_t J, int64_t D, int64_t other_blocks) {
    if ((D % kRksBN) != 0) return false;
    const int rb = ksplit_rb(J);
    if (rb < 3 || rb > 5) return false;
    const int64_t tiles = ((J + 32 * rb - 1) / (32 * rb)) * (D / kRksBN);
    const int64_t waves_per_simd = (tiles * 4 + 1023) / 1024;
    // rb half-blocks per wavefront: compare in half-block units
    return 10 * waves_per_simd * rb <= 9 * 2 * other_blocks;
}

template <int RB>
static hipError_t launch_ksplit(const ReconArgs& a, hipStream_t s) {
    constexpr int BM = 32 * RB;
    constexpr size_t lds_bytes = (size_t)kRksStages * kRksBK * (BM + kRksBN) * sizeof(float);
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_ksplit_kernel<RB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_jb = (a.J + BM - 1) / BM, n_db = a.D / kRksBN;
    const int total = n_jb * n_db;
    SFB_LAUNCH(reconstruct_apply_ksplit_kernel<RB>, dim3(total), dim3(kRksThreads), lds_bytes, s, a.w, a.ldw, a.u, a.ldu,
               (const float*)a.v, a.ldv, a.J, a.D, a.N, a.alpha, n_jb, total, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

hipError_t launch_reconstruct_ksplit(const ReconArgs& a, hipStream_t s) {
    switch (ksplit_rb(a.J)) {
        case 3: return launch_ksplit<3>(a, s);
        case 4: return launch_ksplit<4>(a, s);
        case 5: return launch_ksplit<5>(a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sfb
