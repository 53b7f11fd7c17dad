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
// Rows are interleaved by MT the same way.  A workgroup is NWR row groups x KS wavefronts
// that split every stage's factor pairs between them (KS = 2 puts two wavefronts on each
// SIMD, so one computes while the other stages or waits at the barrier); the KS partial
// sums are exchanged through LDS at the end and each wavefront finishes 1/KS of the rows.
//
// Pipeline.  Factor rows are fetched from HBM/L2 two stages ahead into registers as raw
// words, staged through a double-buffered LDS tile (one barrier per stage), and the LDS
// operand fragments of the next four MFMA k-steps are read while the current four
// execute.  The FAST variant has no branch around any load: out-of-range rows are
// clamped into the matrix and zeroed by a select.
//
// alpha is folded into U while the tile is staged (one rounding per element); the sum of
// outer products is accumulated from zero and added to the prefetched W tile once, in the
// epilogue.  U = 0 leaves W bit-identical.
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kReconBK = 32;   // factor pairs per LDS stage
constexpr int kReconBN = 128;  // W columns per tile
constexpr int kReconGroup = 4; // MFMA k-steps (of 2 factor pairs each) per operand fragment

// FAST: every pointer 16-byte aligned (8 for bf16 V), leading dimensions multiples of 4,
// D a multiple of 128 and J a multiple of 4 -- checked on the host.
template <int MT, int NWR, int KS, typename TV, bool FAST, bool MASK>
__global__ __launch_bounds__(NWR * KS * 64) void reconstruct_apply_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const TV* __restrict__ V,
    int64_t ldv, int J, int D, int N, int B, float alpha, uint64_t live_mask, int n_jb, int total, bool vec_w,
    bool vec_u, bool vec_v, int prox_kind, float prox_a) {
    constexpr int BK = kReconBK, BN = kReconBN, G = kReconGroup;
    constexpr int WMR = 32 * MT;            // rows per wavefront
    constexpr int BM = WMR * NWR;
    constexpr int THREADS = NWR * KS * 64;
    constexpr int U_LD = BK * BM / 4 / THREADS;
    constexpr int V_LD = BK * BN / 4 / THREADS;
    constexpr int SPW = BK / 2 / KS;        // MFMA k-steps per wavefront per stage
    constexpr int NGROUPS = SPW / G;
    constexpr int EH = 16 / KS;             // accumulator rows each wavefront finishes
    static_assert(U_LD >= 1 && V_LD >= 1, "tile too small for the thread count");
    static_assert(MT == 1 || MT == 2 || MT == 4, "row interleave must be 1, 2 or 4");
    static_assert(KS == 1 || KS == 2, "one or two wavefronts per row group");
    static_assert(NGROUPS >= 1 && NGROUPS * G * 2 * KS == BK, "stage depth must split into fragment groups");
    static_assert(KS == 1 || 2 * BK * (BM + BN) >= NWR * KS * MT * 4 * (16 - EH) * 64,
                  "LDS too small for the exchange of partial sums");

    // two stages of the U tile [BK][BM] followed by two stages of the V tile [BK][BN]
    extern __shared__ __attribute__((aligned(16))) float recon_lds[];
    float* const Us = recon_lds;
    float* const Vs = recon_lds + 2 * BK * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave % NWR, wk = wave / NWR;    // row group, share of the factor pairs
    const int l32 = lane & 31, half = lane >> 5;

    // consecutive ids walk down the J blocks of one column block, so the workgroups of a die
    // share a few column blocks of V and all of U in that die's L2.
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // Raw loaded words only: no arithmetic may depend on a load before the stage that
    // consumes it, or the wait for the load would move up to the load itself.
    // FAST: one wide load per item; otherwise four clamped scalar loads per item, kept as loaded
    // (the elements outside the matrix are zeroed when the stage is written to LDS).
    using RawFast = typename RawOf<TV>::type;
    using RawSlow = typename std::conditional<std::is_same<TV, float>::value, f32x4, u32x4>::type;
    using RawV = typename std::conditional<FAST, RawFast, RawSlow>::type;
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
            if constexpr (FAST) {
                r.u[i] = ldg4(U + (int64_t)min(k, N - 1) * ldu + min(c, J - 4));
            } else {
                r.u[i] = load4_clamped_raw(U, k, ldu, N, c, J);
            }
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BN / 4), c = d0 + (idx % (BN / 4)) * 4;
            if constexpr (FAST) {
                r.v[i] = ldraw4(V + (int64_t)min(k, N - 1) * ldv + c);
            } else {
                r.v[i] = load4_clamped_raw(V, k, ldv, N, c, D);
            }
        }
    };
    // alpha, the dead-row select and the bf16 widening happen here, on the way into LDS
    auto stage = [&](const Stage& r, int buf, int k0) {
#pragma unroll
        for (int i = 0; i < U_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BM / 4), c = j0 + (idx % (BM / 4)) * 4;
            f32x4 v;
            if constexpr (FAST) v = (row_live(k) && c < J) ? r.u[i] * alpha : zero4;
            else v = in_matrix4(r.u[i] * alpha, row_live(k), c, J);
            *reinterpret_cast<f32x4*>(&Us[buf * BK * BM + (idx / (BM / 4)) * BM + (idx % (BM / 4)) * 4]) = v;
        }
#pragma unroll
        for (int i = 0; i < V_LD; ++i) {
            const int idx = tid + i * THREADS;
            const int k = k0 + idx / (BN / 4), c = d0 + (idx % (BN / 4)) * 4;
            f32x4 v;
            if constexpr (FAST) v = row_live(k) ? widen4(r.v[i]) : zero4;
            else v = in_matrix4(widen4(r.v[i]), row_live(k), c, D);
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
        const float* us = &Us[buf * BK * BM + wr * WMR + MT * l32];
        const float* vs = &Vs[buf * BK * BN + 4 * l32];
#pragma unroll
        for (int s = 0; s < G; ++s) {
            const int k = 2 * (wk * SPW + g * G + s) + half;
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

    // ---- request this wavefront's share of the W tile right behind the first factor
    // stage; it is only consumed in the epilogue.  (Starting the accumulators from W
    // instead would add every tiny partial product to a large number and lose most of
    // the update to rounding.)  Wavefront wk finishes accumulator rows [wk*EH, wk*EH+EH).
    f32x4 wreg[MT][EH];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int x = 0; x < EH; ++x) {
            const int e = wk * EH + x;
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wr * WMR + MT * m + t;
            if (FAST) {
                wreg[t][x] = ldg4(W + (int64_t)min(row, J - 1) * ldw + d0 + 4 * l32);
            } else {
                wreg[t][x] = load4_clamped(W, row, ldw, J, d0 + 4 * l32, D);
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

    // ---- KS = 2: swap the halves of the partial sums the partner will finish ----
    if constexpr (KS == 2) {
        __syncthreads();   // every wavefront is done reading the stage buffers
        constexpr int SLOT = MT * 4 * EH * 64;                 // floats one wavefront sends
        float* const mine = recon_lds + (wr * 2 + wk) * SLOT;        // what I receive
        float* const theirs = recon_lds + (wr * 2 + (1 - wk)) * SLOT;   // what I send
        auto send = [&](auto other) {
            constexpr int O = decltype(other)::value;          // the half I give away
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int n = 0; n < 4; ++n)
#pragma unroll
                    for (int x = 0; x < EH; ++x)
                        theirs[((t * 4 + n) * EH + x) * 64 + lane] = acc[t][n][O * EH + x];
        };
        if (wk == 0) send(std::integral_constant<int, 1>{}); else send(std::integral_constant<int, 0>{});
        __syncthreads();
        auto recv = [&](auto keep) {
            constexpr int K = decltype(keep)::value;
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int n = 0; n < 4; ++n)
#pragma unroll
                    for (int x = 0; x < EH; ++x)
                        acc[t][n][K * EH + x] += mine[((t * 4 + n) * EH + x) * 64 + lane];
        };
        if (wk == 0) recv(std::integral_constant<int, 0>{}); else recv(std::integral_constant<int, 1>{});
    }

    // ---- epilogue: W <- W + acc for this wavefront's rows, 128-bit stores ----
    auto finish = [&](auto keep) {
        constexpr int K = decltype(keep)::value;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int x = 0; x < EH; ++x) {
                const int e = K * EH + x;
                const int m = 8 * (e / 4) + 4 * half + (e % 4);
                const int row = j0 + wr * WMR + MT * m + t;
                if (row < J) {
                    f32x4 w = wreg[t][x];
                    w.x += acc[t][0][K * EH + x];
                    w.y += acc[t][1][K * EH + x];
                    w.z += acc[t][2][K * EH + x];
                    w.w += acc[t][3][K * EH + x];
                    w = prox_entry4(w, prox_kind, prox_a);
                    if (FAST) *reinterpret_cast<f32x4*>(W + (int64_t)row * ldw + d0 + 4 * l32) = w;
                    else store4(W + (int64_t)row * ldw, d0 + 4 * l32, D, vec_w, w);
                }
            }
    };
    if (KS == 1 || wk == 0) finish(std::integral_constant<int, 0>{});
    else finish(std::integral_constant<int, KS - 1>{});
}

// ---------------------------------------------------------------------------------------
// LDS-DMA variant (fp32 factors, every worker live, N a multiple of the stage depth, the
// FAST alignment conditions): the factor tiles go from HBM/L2 straight into LDS with
// global_load_lds_dwordx4 -- no staging registers, no LDS stores, no VALU work per stage.
// Lane i of a wavefront-wide DMA lands at (LDS base in M0) + 16*i, which is exactly the
// row-major [k][128] tile layout the MFMA operands are read from.  Three LDS stages form
// a ring: while stage c is multiplied, the DMAs of stages c+1 and c+2 are in flight.  The
// compiler does not see the DMA (inline asm), so completion is tracked by hand: the
// vector-memory counter retires in order, `s_waitcnt vmcnt(n)` with n = the number of
// younger DMAs this wavefront has issued means "my share of stage c has landed", and the
// barrier that follows extends that to every wavefront's share.  The same barrier also
// says that everyone is done reading stage c-1, which the next DMA overwrites.
// alpha cannot be folded into U on the way in, so it is applied once in the epilogue:
// W + alpha * acc.
// ---------------------------------------------------------------------------------------

// BK factor pairs per stage, NST stages in the ring (NST - 1 of them in flight ahead).
template <int MT, int NWR, int BK, int NST, int WPS>
__global__ __launch_bounds__(NWR * 64, WPS) void reconstruct_apply_dma_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a) {
    constexpr int BN = kReconBN, G = kReconGroup;
    constexpr int WMR = 32 * MT;
    constexpr int BM = WMR * NWR;
    constexpr int THREADS = NWR * 64;
    constexpr int U_LD = BK * BM / 4 / THREADS;
    constexpr int V_LD = BK * BN / 4 / THREADS;
    constexpr int NGROUPS = BK / 2 / G;
    constexpr int STAGE_FLOATS = BK * (BM + BN);
    static_assert(U_LD >= 1 && V_LD >= 1 && NGROUPS >= 1, "tile too small");
    static_assert(U_LD + V_LD <= 32, "too many DMAs per stage for the wait encoding used");

    extern __shared__ __attribute__((aligned(16))) float recon_lds[];   // NST x (U tile, V tile)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // per-thread source pointers of stage 0; a stage is BK rows further down
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
    const uint32_t lds0 = (uint32_t)(uintptr_t)recon_lds;
    const int64_t ustep = (int64_t)BK * ldu, vstep = (int64_t)BK * ldv;

    // DMA number i (U items first, then V items) of stage `st` for chunk `chunk`
    auto issue_one = [&](int chunk, int st, int i) {
        const uint32_t ubase =
            __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_FLOATS + wave * 64 * 4) * 4u);
        if (i < U_LD) {
            lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * THREADS * 16));
        } else {
            const uint32_t vbase = ubase + (uint32_t)(BK * BM) * 4u;
            lds_dma16(pv[i - U_LD] + chunk * vstep, vbase + (uint32_t)((i - U_LD) * THREADS * 16));
        }
    };
    auto issue = [&](int chunk, int st) {
#pragma unroll
        for (int i = 0; i < U_LD + V_LD; ++i) issue_one(chunk, st, i);
    };

    f32x16 acc[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][n][e] = 0.f;

    struct Frag { float a[G][MT]; f32x4 b[G]; };
    auto read_frag = [&](Frag& f, int st, int g) {
        const float* us = &recon_lds[st * STAGE_FLOATS + wave * WMR + MT * l32];
        const float* vs = &recon_lds[st * STAGE_FLOATS + BK * BM + 4 * l32];
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
    // The same MFMAs with one DMA of a later stage slipped in after each of the first
    // U_LD + V_LD of them: the address arithmetic and the DMA issue run in the shadow of a
    // 64-cycle MFMA instead of holding up the first MFMA of the stage.
    auto mma_frag_issue = [&](const Frag& f, int chunk, int st) {
#pragma unroll
        for (int s = 0; s < G; ++s)
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    acc[t][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[s][t], f.b[s][n], acc[t][n], 0, 0, 0);
                    const int slot = (s * MT + t) * 4 + n;
                    if (slot < U_LD + V_LD) {
                        __builtin_amdgcn_sched_barrier(0);
                        issue_one(chunk, st, slot);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
    };
    static_assert(U_LD + V_LD <= G * MT * 4, "more DMAs per stage than MFMAs in the first fragment group");
    // issue_chunk >= 0: the DMAs of that chunk (into stage issue_st) ride along the first group
    auto compute = [&](int st, int issue_chunk, int issue_st) {
        Frag f0, f1;
        read_frag(f0, st, 0);
#pragma unroll
        for (int g = 0; g < NGROUPS; g += 2) {
            if (g + 1 < NGROUPS) read_frag(f1, st, g + 1);
            __builtin_amdgcn_sched_barrier(0);
            if (g == 0 && issue_chunk >= 0) mma_frag_issue(f0, issue_chunk, issue_st);
            else mma_frag(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 1 < NGROUPS) {
                if (g + 2 < NGROUPS) read_frag(f0, st, g + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma_frag(f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    const int n_chunks = N / BK;   // the host guarantees N % BK == 0 and N >= BK
#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < n_chunks) issue(p, p);

    // One step: stage `st` holds chunk c once my DMAs (all but the newest stage's) have
    // retired and everyone has passed the barrier; then refill the stage read in step c-1.
    auto step = [&](int c, int st) {
        const int younger = min(n_chunks - 1 - c, NST - 2);   // chunks issued after chunk c
        if (younger >= 1) wait_vmcnt<U_LD + V_LD>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        compute(st, c + NST - 1 < n_chunks ? c + NST - 1 : -1, (st + NST - 1) % NST);
    };
    static_assert(NST == 3, "ring depth");
    // Chunk 0 first, with nothing else competing for HBM; the W tile is requested right
    // after it (ordinary loads, consumed in the epilogue), so its read overlaps the
    // remaining stages instead of delaying the first MFMA.
    step(0, 0);
    constexpr int W_LOADS = MT * 16;
    f32x4 wreg[MT][16];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wave * WMR + MT * m + t;
            wreg[t][e] = ldg4(W + (int64_t)min(row, J - 1) * ldw + d0 + 4 * l32);
        }
    // The vector-memory counter retires in order and the W loads sit between the DMAs of
    // chunk 2 (issued during chunk 0) and those of chunk 3: the waits of chunks 1 and 2 count
    // them among the younger operations, so that neither stalls on the W tile's trip to HBM;
    // by chunk 3 (two stages later) the tile has long arrived.
    static_assert(U_LD + V_LD + W_LOADS <= 63, "wait count encoding");
    auto step_w = [&](int c, int st) {
        const bool dma_younger = (c == 1) ? (2 < n_chunks) : (3 < n_chunks);
        if (dma_younger) wait_vmcnt<U_LD + V_LD + W_LOADS>(); else wait_vmcnt<W_LOADS>();
        __builtin_amdgcn_s_barrier();
        compute(st, c + NST - 1 < n_chunks ? c + NST - 1 : -1, (st + NST - 1) % NST);
    };
    if (1 < n_chunks) step_w(1, 1);
    if (2 < n_chunks) step_w(2, 2);

    int c = 3;
    for (; c + NST - 1 < n_chunks; c += NST) {
        step(c, 0);
        step(c + 1, 1);
        step(c + 2, 2);
    }
    if (c < n_chunks) step(c, 0);
    if (c + 1 < n_chunks) step(c + 1, 1);

#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = 8 * (e / 4) + 4 * half + (e % 4);
            const int row = j0 + wave * WMR + MT * m + t;
            if (row < J) {
                f32x4 w = wreg[t][e];
                w.x += alpha * acc[t][0][e];
                w.y += alpha * acc[t][1][e];
                w.z += alpha * acc[t][2][e];
                w.w += alpha * acc[t][3][e];
                w = prox_entry4(w, prox_kind, prox_a);
                *reinterpret_cast<f32x4*>(W + (int64_t)row * ldw + d0 + 4 * l32) = w;
            }
        }
}

template <int MT, int NWR, int BK, int NST, int WPS = 1>
static hipError_t launch_recon_dma(const ReconArgs& a, hipStream_t s) {
    constexpr int BM = 32 * MT * NWR;
    const int n_jb = (a.J + BM - 1) / BM, n_db = a.D / kReconBN;
    const int total = n_jb * n_db;
    constexpr size_t lds_bytes = (size_t)NST * BK * (BM + kReconBN) * sizeof(float);
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_dma_kernel<MT, NWR, BK, NST, WPS>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    SFB_LAUNCH((reconstruct_apply_dma_kernel<MT, NWR, BK, NST, WPS>), dim3(total), dim3(NWR * 64), lds_bytes, s, a.w,
                       a.ldw, a.u, a.ldu, (const float*)a.v, a.ldv, a.J, a.D, a.N, a.alpha, n_jb, total, a.prox_kind,
                       a.prox_a);
    return hipGetLastError();
}

// Shapes the DMA kernel accepts; everything else runs the register-staged kernel.
static bool dma_ok(const ReconArgs& a, int bk) {
    return !a.bf16 && !a.use_mask && ((uintptr_t)a.w % 16) == 0 && (a.ldw % 4) == 0 &&
           ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0 && ((uintptr_t)a.v % 16) == 0 && (a.ldv % 4) == 0 &&
           (a.D % kReconBN) == 0 && (a.J % 4) == 0 && a.J >= 4 && (a.N % bk) == 0 && a.N >= bk;
}

struct ReconVariant { int mt, nwr, ks; bool dma; };
static const ReconVariant kReconVariants[] = {
    {1, 4, 1, false},  // 0: 128 x 128 tile, 4 wavefronts
    {1, 2, 1, false},  // 1: 64 x 128, 2 wavefronts
    {1, 1, 1, false},  // 2: 32 x 128, 1 wavefront
    {2, 4, 1, false},  // 3: 256 x 128, 4 wavefronts
    {1, 4, 2, false},  // 4: 128 x 128, 8 wavefronts (two per SIMD)
    {1, 2, 2, false},  // 5: 64 x 128, 4 wavefronts
    {2, 2, 2, false},  // 6: 128 x 128, 4 wavefronts of 64 rows
    {1, 4, 1, true},   // 7: 128 x 128, 4 wavefronts, LDS-DMA staging (falls back to 0)
    {1, 2, 1, true},   // 8: 64 x 128, 2 wavefronts, LDS-DMA staging (falls back to 1)
    {1, 2, 1, true},   // 9: 64 x 64, 4 wavefronts of one 32 x 32 block each, LDS-DMA staging (falls back to 8)
    {1, 4, 1, true},   // 10: as 7 with 16-pair stages and a register budget for two workgroups per compute unit
    {1, 2, 1, true},   // 11: (96..160) x 64, 8 wavefronts = 2 column blocks x 2 halves of every stage's pairs x 2 groups taking the stages in turn (falls back to 9)
    {1, 4, 1, true},   // 12: 128 x 128, 8 wavefronts = 4 strips of 32 rows x 2 groups taking the stages in turn, LDS-DMA (falls back to 7)
};
constexpr int kSmallVariant = 9, kKsplitVariant = 11, kPairVariant = 12;
constexpr int kNumReconVariants = sizeof(kReconVariants) / sizeof(kReconVariants[0]);

int num_reconstruct_variants() { return kNumReconVariants; }

ReconPlan plan_reconstruct(int64_t J, int64_t D, int64_t N) {
    // largest tile that still gives every compute unit a workgroup; the smallest otherwise.
    // 7 and 8 are the LDS-DMA forms of the 128- and 64-row tiles (they fall back to the
    // register-staged kernel by themselves when the shape does not allow DMA).
    // The 32-row tile (one wavefront per workgroup, register-staged) is a candidate only where the single-block
    // LDS-DMA tiles below cannot take over (D not in whole 64-column tiles): 256 lone wavefronts leave three
    // quarters of the SIMDs idle (J = 256, D = 4096, N = 1024: 95 us against 26 us with single blocks).
    const int order[] = {7, 8, 2};
    int variant = -1;
    for (int v : order) {
        if (v == 2 && (D % 64) == 0) continue;
        const int64_t bm = 32 * kReconVariants[v].mt * kReconVariants[v].nwr;
        const int64_t tiles = ((J + bm - 1) / bm) * ((D + kReconBN - 1) / kReconBN);
        if (tiles >= 256) { variant = v; break; }
    }
    if (variant < 0) {
        // too small to fill the chip whatever the tile, so latency decides: 64-row tiles give
        // the most workgroups that still have two wavefronts each; up to 64 rows one 128-row
        // tile is used for its four wavefronts (more lanes to fetch with; the surplus
        // wavefronts multiply clamped rows that are never stored)
        variant = J > 64 ? 8 : 7;
    }
    // 128-row tiles: eight wavefronts, two per SIMD, in two groups that take the stages in turn, so that a
    // hand-over between stages does not idle the matrix pipe (measured against the four-wavefront form:
    // mlr_medium 41.9-44.7 -> 38.4-40.9 us; J = 2000, D = 8192, N = 1024 (four tiles per compute unit), where
    // variant 10 lets two workgroups share a compute unit instead: 267-275 -> 262-263 us).
    if (variant == 7) variant = kPairVariant;
    // single-block wavefronts where the lumps of four blocks would leave the busiest SIMD with
    // clearly more than its share (e.g. J = 600: 3 blocks instead of 4)
    if (kReconVariants[variant].dma) {
        const int bm = 32 * kReconVariants[variant].mt * kReconVariants[variant].nwr;
        const int nwr = kReconVariants[variant].nwr;
        // whole 32 x 32 blocks (through all pairs) on the busiest SIMD with the choice so far
        int64_t busiest = (((J + bm - 1) / bm) * ((D + kReconBN - 1) / kReconBN) * nwr + 1023) / 1024 * 4;
        if (reconstruct_small_wins(J, D, bm, nwr)) {
            variant = kSmallVariant;
            busiest = (((J + 63) / 64) * (D / 64) * 4 + 1023) / 1024;
        }
        // splitting the pairs as well where that evens the load out further (J = 600: 2.5 instead of 3)
        if (reconstruct_ksplit_wins(J, D, busiest)) variant = kKsplitVariant;
    }
    ReconPlan p = plan_reconstruct_variant(J, D, variant);
    if (variant == kSmallVariant) {
        // few tiles and many factor pairs: slices of the pairs over workgroups as well
        p.n_split = reconstruct_small_split(J, D, N, &p.k_rows);
        p.n_rows = (int)N;
        p.grid *= p.n_split;
    }
    return p;
}

ReconPlan plan_reconstruct_variant(int64_t J, int64_t D, int variant) {
    ReconPlan p;
    p.variant = variant;
    p.bm = variant == kKsplitVariant ? reconstruct_ksplit_rows(J) : 32 * kReconVariants[variant].mt * kReconVariants[variant].nwr;
    p.bn = (variant == kSmallVariant || variant == kKsplitVariant) ? 64 : kReconBN;
    p.grid = (int)(((J + p.bm - 1) / p.bm) * ((D + p.bn - 1) / p.bn));
    return p;
}

template <int MT, int NWR, int KS, typename TV, bool FAST, bool MASK>
static hipError_t launch_recon_f(const ReconArgs& a, hipStream_t s, bool vec_w, bool vec_u, bool vec_v) {
    constexpr int BM = 32 * MT * NWR;
    const int n_jb = (a.J + BM - 1) / BM, n_db = (a.D + kReconBN - 1) / kReconBN;
    const int total = n_jb * n_db;
    constexpr size_t lds_bytes = 2 * kReconBK * (BM + kReconBN) * sizeof(float);
    static std::atomic<bool> raised{false};   // opt in once to more than 64 KB of LDS per workgroup
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_kernel<MT, NWR, KS, TV, FAST, MASK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    SFB_LAUNCH((reconstruct_apply_kernel<MT, NWR, KS, TV, FAST, MASK>), dim3(total),
                       dim3(NWR * KS * 64), lds_bytes, s, a.w, a.ldw, a.u, a.ldu, (const TV*)a.v, a.ldv, a.J, a.D,
                       a.N, a.B, a.alpha, a.live_mask, n_jb, total, vec_w, vec_u, vec_v, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

template <int MT, int NWR, int KS, typename TV>
static hipError_t launch_recon_t(const ReconArgs& a, hipStream_t s) {
    const bool vec_w = ((uintptr_t)a.w % 16) == 0 && (a.ldw % 4) == 0;
    const bool vec_u = ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0;
    const bool vec_v = ((uintptr_t)a.v % (4 * sizeof(TV))) == 0 && (a.ldv % 4) == 0;
    const bool fast = vec_w && vec_u && vec_v && (a.D % kReconBN) == 0 && (a.J % 4) == 0 && a.J >= 4;
    if (a.use_mask) {   // a worker is missing: rare, so only the generic kernel carries the mask
        return launch_recon_f<MT, NWR, KS, TV, false, true>(a, s, vec_w, vec_u, vec_v);
    }
    if (fast) return launch_recon_f<MT, NWR, KS, TV, true, false>(a, s, vec_w, vec_u, vec_v);
    return launch_recon_f<MT, NWR, KS, TV, false, false>(a, s, vec_w, vec_u, vec_v);
}

template <typename TV>
static hipError_t launch_recon_v(const ReconArgs& a, const ReconPlan& p, hipStream_t s) {
    switch (p.variant) {
        case 0: return launch_recon_t<1, 4, 1, TV>(a, s);
        case 1: return launch_recon_t<1, 2, 1, TV>(a, s);
        case 2: return launch_recon_t<1, 1, 1, TV>(a, s);
        case 3: return launch_recon_t<2, 4, 1, TV>(a, s);
        case 4: return launch_recon_t<1, 4, 2, TV>(a, s);
        case 5: return launch_recon_t<1, 2, 2, TV>(a, s);
        case 6: return launch_recon_t<2, 2, 2, TV>(a, s);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// Ragged or misaligned fp32 factors.  The LDS-DMA kernels want 16-byte aligned rows of whole
// 16-byte items, whole column tiles and whole stages; shapes such as 600 x 780 (the metric
// of Section 6 on 780 pixel features) or ten classes have none of that, and the
// register-staged kernel takes them element by element with a bounds check each, several
// times slower per factor pair.  The factors are small next to the work done with them
// (N (J + D) numbers against N J D multiply-adds), so they are copied once into padded rows
// -- J rounded up to 4 floats, D to whole 128-column tiles, N to whole stages of zero rows, a
// dead worker's rows zero (selected, not multiplied: a dead slot may hold anything) -- and
// the LDS-DMA kernels run on the copies.  W stays where it is: those kernels then take its
// entries one by one, within J x D.
// ---------------------------------------------------------------------------------------
constexpr int kConformCols = 1024;   // columns of the concatenated [Jp + Dp] row per workgroup

__global__ __launch_bounds__(256) void conform_factors_kernel(
    const float* __restrict__ U, int64_t ldu, const float* __restrict__ V, int64_t ldv, float* __restrict__ Uc, int Jp,
    float* __restrict__ Vc, int Dp, int N, int J, int D, int B, uint64_t live_mask, int use_mask) {
    const int row = blockIdx.x;                               // < N rounded up to whole stages
    bool live = row < N;
    if (live && use_mask) live = ((live_mask >> (row / B)) & 1ull) != 0;      // host: a mask means at most 64 workers
    const int c0 = blockIdx.y * kConformCols;
#pragma unroll
    for (int i = 0; i < kConformCols / 256; ++i) {
        const int c = c0 + i * 256 + threadIdx.x;             // column of the row [ u (Jp) | v (Dp) ]
        if (c < Jp) {
            Uc[(int64_t)row * Jp + c] = (live && c < J) ? U[(int64_t)row * ldu + c] : 0.f;
        } else if (c < Jp + Dp) {
            const int d = c - Jp;
            Vc[(int64_t)row * Dp + d] = (live && d < D) ? V[(int64_t)row * ldv + d] : 0.f;
        }
    }
}

int64_t conform_cols(int64_t D) { return (D + 127) / 128 * 128; }
int64_t conform_rows(int64_t N) { return (N + kReconBK - 1) / kReconBK * kReconBK; }

static size_t round_up_256(size_t x) { return (x + 255) / 256 * 256; }

size_t conform_workspace(int64_t J, int64_t D, int64_t N) {
    const size_t np = (size_t)conform_rows(N), jp = (size_t)((J + 3) / 4 * 4), dp = (size_t)conform_cols(D);
    return round_up_256(np * jp * sizeof(float)) + round_up_256(np * dp * sizeof(float));
}

// The kernel that stands in for `variant` on padded factors: the 128 x 128 and the 64-row tiles map to
// their eight-wavefront and single-block forms; 0 for the register-staged variants (no such form).
static int conformed_variant(int variant) {
    switch (variant) {
        case 7: case 10: case kPairVariant: return kPairVariant;
        case 8: case kSmallVariant: return kSmallVariant;
        case kKsplitVariant: return kKsplitVariant;
    }
    return 0;
}

bool conformed_variant_ok(int variant) { return conformed_variant(variant) != 0; }

ReconPlan plan_reconstruct_padded(int64_t J, int64_t D, int64_t N, int variant) {
    const int64_t dp = conform_cols(D);
    const ReconPlan p = variant >= 0 ? plan_reconstruct_variant(J, dp, variant) : plan_reconstruct(J, dp, conform_rows(N));
    int v = conformed_variant(p.variant);
    if (v == 0) return p;                                    // register-staged: taken as it is, on the factors as they are
    if (v == kKsplitVariant) {
        const int rows = reconstruct_ksplit_rows(J);
        if (rows < 96 || rows > 160) v = kSmallVariant;      // what launch_reconstruct_conformed falls back to
    }
    if (v == p.variant) return p;                            // (with the planner's slices of the pairs, if any)
    return plan_reconstruct_variant(J, dp, v);
}

// A dead worker in a shape the LDS-DMA kernels take as it is: only U is copied (N x J rounded up to 4
// floats, the dead workers' rows as zeros), V and W are used where they are, and the plan's kernel
// runs without a mask.  hipErrorNotSupported (nothing launched) when the same call without its mask
// would not end in an LDS-DMA kernel either.
size_t masked_workspace(int64_t J, int64_t N) { return round_up_256((size_t)N * (size_t)((J + 3) / 4 * 4) * sizeof(float)); }

hipError_t launch_reconstruct_masked(const ReconArgs& a, const ReconPlan& p, void* workspace, hipStream_t s) {
    if (!a.use_mask || a.bf16 || workspace == nullptr || ((uintptr_t)workspace % 256) != 0) return hipErrorNotSupported;
    const int jp = (a.J + 3) / 4 * 4;
    ReconArgs c = a;
    float* uc = (float*)workspace;
    c.u = uc; c.ldu = jp;
    c.use_mask = false; c.live_mask = ~0ull;
    if (!reconstruct_takes_dma(c, p)) return hipErrorNotSupported;
    hipLaunchKernelGGL(conform_factors_kernel, dim3(a.N, (jp + kConformCols - 1) / kConformCols), dim3(256), 0, s, a.u,
                       a.ldu, (const float*)a.v, a.ldv, uc, jp, (float*)nullptr, 0, a.N, a.J, a.D, a.B, a.live_mask, 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_reconstruct(c, p, s);
}

hipError_t launch_reconstruct_conformed(const ReconArgs& a, const ReconPlan& p, void* workspace, hipStream_t s) {
    static_assert(kReconBK == 32, "stage depth of the kernels that take padded factors");
    int variant = conformed_variant(p.variant);              // (plan_reconstruct_padded has already mapped it)
    if (variant == 0 || a.bf16 || workspace == nullptr || ((uintptr_t)workspace % 256) != 0) return hipErrorNotSupported;
    const int np = (int)conform_rows(a.N), jp = (a.J + 3) / 4 * 4, dp = (int)conform_cols(a.D);
    ReconArgs c = a;
    float* uc = (float*)workspace;
    float* vc = (float*)((char*)workspace + round_up_256((size_t)np * jp * sizeof(float)));
    c.u = uc; c.ldu = jp; c.v = vc; c.ldv = dp; c.N = np;
    c.use_mask = false; c.live_mask = ~0ull;
    c.conformed = true; c.Dp = dp;
    if (variant == kKsplitVariant && !reconstruct_ksplit_ok(c)) variant = kSmallVariant;
    if (variant == kPairVariant ? !reconstruct_pair_ok(c) : variant == kSmallVariant ? !reconstruct_small_ok(c) : false)
        return hipErrorNotSupported;
    hipLaunchKernelGGL(conform_factors_kernel, dim3(np, (jp + dp + kConformCols - 1) / kConformCols), dim3(256), 0, s,
                       a.u, a.ldu, (const float*)a.v, a.ldv, uc, jp, vc, dp, a.N, a.J, a.D, a.B, a.live_mask,
                       a.use_mask ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (variant == kPairVariant) return launch_reconstruct_pair(c, s);
    if (variant == kKsplitVariant) return launch_reconstruct_ksplit(c, s);
    if (p.variant == kSmallVariant && p.n_split > 1 && c.partial != nullptr && c.N == p.n_rows)
        return launch_reconstruct_small_split(c, p.n_split, p.k_rows, s);
    return launch_reconstruct_small(c, s);
}

// True when launch_reconstruct(a, p) ends in one of the LDS-DMA kernels (the same chain of
// fall-backs, without launching anything).
bool reconstruct_takes_dma(const ReconArgs& a, const ReconPlan& p) {
    int v = p.variant;
    if (a.bf16 || !kReconVariants[v].dma) return false;
    if (v == kPairVariant) {
        if (reconstruct_pair_ok(a)) return true;
        if (!a.conformed && (a.J % 4) == 0 && a.J >= 4) {     // W alone off the 16-byte grid
            ReconArgs c = a;
            c.conformed = true;
            if (reconstruct_pair_ok(c)) return true;
        }
        v = 7;
    }
    if (v == kKsplitVariant) {
        if (reconstruct_ksplit_ok(a)) return true;
        v = kSmallVariant;
    }
    if (v == kSmallVariant) {
        if (reconstruct_small_ok(a)) return true;
        v = 8;
    }
    if (v == 10 && dma_ok(a, 16)) return true;
    return dma_ok(a, kReconBK);
}

hipError_t launch_reconstruct(const ReconArgs& a, const ReconPlan& p, hipStream_t s) {
    ReconPlan q = p;
    if (p.variant == kPairVariant) {
        if (reconstruct_pair_ok(a)) return launch_reconstruct_pair(a, s);
        // whole, aligned factors and only W off the 16-byte grid (or with a leading dimension that is not a
        // multiple of 4): the same kernel in the form that takes W entry by entry
        if (!a.conformed && (a.J % 4) == 0 && a.J >= 4) {
            ReconArgs c = a;
            c.conformed = true;
            if (reconstruct_pair_ok(c)) return launch_reconstruct_pair(c, s);
        }
        q.variant = 7;
    }
    if (p.variant == kKsplitVariant) {
        if (reconstruct_ksplit_ok(a)) return launch_reconstruct_ksplit(a, s);
        q.variant = kSmallVariant;
    }
    if (q.variant == kSmallVariant) {
        if (reconstruct_small_ok(a)) {
            if (p.variant == kSmallVariant && p.n_split > 1 && a.partial != nullptr && a.N == p.n_rows)
                return launch_reconstruct_small_split(a, p.n_split, p.k_rows, s);
            return launch_reconstruct_small(a, s);
        }
        q.variant = 8;
    }
    if (kReconVariants[q.variant].dma) {
        if (q.variant == 10) {
            if (dma_ok(a, 16)) return launch_recon_dma<1, 4, 16, 3, 2>(a, s);
            q.variant = 7;
        }
        if (dma_ok(a, kReconBK)) {
            switch (q.variant) {
                case 7: return launch_recon_dma<1, 4, kReconBK, 3>(a, s);
                case 8: return launch_recon_dma<1, 2, kReconBK, 3>(a, s);
            }
        }
        q.variant = q.variant == 8 ? 1 : 0;   // same tile, register staging
    }
    return a.bf16 ? launch_recon_v<bf16_t>(a, q, s) : launch_recon_v<float>(a, q, s);
}

}  // namespace sfb
