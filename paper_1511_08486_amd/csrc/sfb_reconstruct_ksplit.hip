// Reconstruction + update (Section 3, Section 2.1), evenly divided form:
//     W[j][d] <- W[j][d] + alpha * sum_n U[n][j] * V[n][d]
// with tiles of 32*RB rows x 64 columns of W and eight wavefronts that split the tile's two
// column blocks, every chunk's factor pairs, and the chunks themselves.
//
// Why a third tile shape.  A launch is as slow as its busiest SIMD.  The unit the other kernels
// hand out is a whole 32 x 32 block of W carried through all N pairs: J = 600, D = 4096 is
// 19 x 128 = 2432 blocks for 1024 SIMDs, 2.4 each on average but 3 on the busiest even with
// single-block wavefronts (and a lone wavefront in the last round hides none of its waits: 3.5
// block times measured).  Here a wavefront carries RB blocks (one column block of the tile, all
// its row blocks) through a QUARTER of the pairs; the four wavefronts that share the blocks
// exchange partial sums through LDS once, at the end, and each finishes a quarter of every block.
// J = 600 becomes four row tiles of five row blocks x 64 column tiles = 256 workgroups, one per
// compute unit, and every SIMD multiplies exactly 5 blocks x N/2 pairs = 2.5 block times, 95 % of
// it on rows that exist.  The B fragment (v) of a step feeds RB matrix instructions, and four of the
// row blocks share one 16-byte LDS read (rows interleaved by four, as the columns are in the large
// kernel).
//
// The eight wavefronts are two per SIMD, in two groups of four that take the chunks of 32 pairs in
// turn (group 0 the even chunks, group 1 the odd ones); inside a group: 2 column blocks x 2 halves of
// the chunk's pairs.  With one wavefront per SIMD every hand-over to the next chunk (wait for the
// copies, barrier, issue the next copies, first LDS reads) is time the matrix pipe stands still (a
// four-wavefront form of this kernel lost 5.3 of its 42.6 ns per pair that way); here the other
// group's wavefront on the same SIMD is in the middle of its own chunk at that moment and keeps the
// pipe busy.  Barrier number c is the hand-over to chunk c: the group that owns chunk c reaches it
// between two chunks, the other group in the middle of chunk c - 1 (20 of its 40 matrix instructions
// issued); every wavefront executes every barrier exactly once.  A group stages its own chunks by
// LDS-DMA (32 pairs of u [k][32*RB] and of v [k][64] straight from L2, a ring of four stages, two per
// group, completion counted by hand with the in-order vector-memory counter) and only it reads them,
// so a chunk's stage is free again as soon as the group has passed its next hand-over.  The W entries
// a wavefront finishes are requested during its first chunk and consumed in the epilogue, where alpha
// and the entrywise proximal operator are applied.  Four partial sums per entry (2 halves x 2 groups)
// are added in one fixed order (quarter owners 0, 1, 2, 3), then to W: results do not depend on timing.
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kRksBN = 64, kRksBK = 32;

template <int RB>
__global__ __launch_bounds__(512) void reconstruct_apply_ksplit_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a) {
    constexpr int BM = 32 * RB, BN = kRksBN, BK = kRksBK, GT = 256;   // GT: threads of a group; ring of four stages
    constexpr int U_LD = BK * BM / 4 / GT, V_LD = BK * BN / 4 / GT;               // 16-byte DMAs per thread and chunk
    constexpr int DMAS = U_LD + V_LD;
    constexpr int STAGE_FLOATS = BK * (BM + BN);
    constexpr int NQD = RB / 4, NS = RB - 4 * NQD;
    constexpr int W_LOADS = RB * 4;              // a wavefront finishes a quarter of each of its RB blocks
    static_assert(U_LD == RB && V_LD == 2, "tile / thread count mismatch");
    static_assert(DMAS + W_LOADS <= 63, "wait count encoding");
    extern __shared__ __attribute__((aligned(16))) float rks_lds[];   // max(ring, exchange area): see the launcher

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int g = wave >> 2, gw = wave & 3, gtid = tid & (GT - 1);
    const int wc = gw & 1, kh = gw >> 1;
    const int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    const float* pu[U_LD];
    const float* pv[V_LD];
    const int ju = (J + 3) & ~3;                             // host: a row of U holds J rounded up to 4 floats
#pragma unroll
    for (int i = 0; i < U_LD; ++i) {
        const int idx = gtid + i * GT;
        pu[i] = U + (int64_t)(idx / (BM / 4)) * ldu + min(j0 + (idx % (BM / 4)) * 4, ju - 4);
    }
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
        const int idx = gtid + i * GT;
        pv[i] = V + (int64_t)(idx / (BN / 4)) * ldv + d0 + (idx % (BN / 4)) * 4;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)rks_lds;
    const int64_t ustep = (int64_t)BK * ldu, vstep = (int64_t)BK * ldv;
    auto issue_one = [&](int chunk, int i) {
        const uint32_t ubase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)((chunk & 3) * STAGE_FLOATS + gw * 64 * 4) * 4u);
        if (i < U_LD) lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * GT * 16));
        else lds_dma16(pv[i - U_LD] + chunk * vstep, ubase + (uint32_t)(BK * BM) * 4u + (uint32_t)((i - U_LD) * GT * 16));
    };
    auto tile_row = [](int b, int m) { return b < 4 * NQD ? 128 * (b / 4) + 4 * m + (b % 4) : 128 * NQD + 32 * (b - 4 * NQD) + m; };

    f32x16 acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    struct Frags {
        f32x4 aq[4][NQD > 0 ? NQD : 1];
        float as[4][NS > 0 ? NS : 1], bv[4];
    };
    auto load_step = [&](int st, int h, int s, Frags& f) {
        const float* us = &rks_lds[st * STAGE_FLOATS + (16 * kh + 8 * h + half) * BM];
        const float* vs = &rks_lds[st * STAGE_FLOATS + BK * BM + (16 * kh + 8 * h + half) * BN + wc * 32 + l32];
#pragma unroll
        for (int q = 0; q < NQD; ++q) f.aq[s][q] = *reinterpret_cast<const f32x4*>(us + 2 * s * BM + 128 * q + 4 * l32);
#pragma unroll
        for (int r = 0; r < NS; ++r) f.as[s][r] = us[2 * s * BM + 128 * NQD + 32 * r + l32];
        f.bv[s] = vs[2 * s * BN];
    };
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

    const int n_chunks = N / BK;   // host: N % BK == 0, N >= BK
    // my group's first chunk; every later one is requested right after the hand-over two chunks before it
    if (g < n_chunks) {
#pragma unroll
        for (int i = 0; i < DMAS; ++i) issue_one(g, i);
    }
    if (g == 1) __builtin_amdgcn_s_barrier();                // barrier 0 is group 0's first hand-over
    float wreg[RB][4];
    const int col = d0 + wc * 32 + l32;                      // beyond D only in the last tile of padded factors
    const int colc = min(col, D - 1);
    const int quad = 2 * kh + g;                             // accumulator entries 4 quad .. 4 quad + 3 are mine to finish
    auto load_w = [&]() {
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = j0 + tile_row(b, 8 * quad + 4 * half + t);
                wreg[b][t] = W[(int64_t)min(row, J - 1) * ldw + colc];
            }
    };
    if (g >= n_chunks) load_w();                             // a single chunk: group 1 has none, but finishes its quarter
    Frags fa, fb;
    for (int c = g; c < n_chunks; c += 2) {
        // hand-over to chunk c.  In counter order my copies of chunk c are followed by nothing but, once, the W
        // loads (requested during my first chunk, i.e. after the copies of my second one)
        if (c == g + 2) wait_vmcnt<W_LOADS>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();                        // barrier c
        const int st = c & 3;
        const bool more = c + 2 < n_chunks;
#pragma unroll
        for (int s = 0; s < 4; ++s) load_step(st, 0, s, fa);
        if (c == g) {
            // the copies of my second chunk first, then the W entries I finish: they have the whole contraction to arrive
            if (more) {
#pragma unroll
                for (int i = 0; i < DMAS; ++i) issue_one(c + 2, i);
            }
            load_w();
            multiply(fa, [&](int s) { load_step(st, 1, s, fb); });
        } else {
            multiply(fa, [&](int s) {
                if (more) {
#pragma unroll
                    for (int i = 0; i < DMAS; ++i)
                        if (i * 4 / DMAS == s) issue_one(c + 2, i);
                }
                load_step(st, 1, s, fb);
            });
        }
        if (c + 1 < n_chunks) __builtin_amdgcn_s_barrier();  // barrier c + 1: the other group's hand-over
        multiply(fb, [](int) {});
    }

    // Exchange of partial sums.  Everybody is done with the ring (barrier), which the exchange area overlays.
    // Wavefront w, block b: the three quarters of its accumulator that the others finish, 16 bytes per lane
    // each, at position t (t < quad) or t - 1 (t > quad) of its slot.
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    f32x4* xch = reinterpret_cast<f32x4*>(rks_lds);
    auto finish = [&](auto Qc) {
        constexpr int Q = decltype(Qc)::value;
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t == Q) continue;
                const int pos = t < Q ? t : t - 1;
                xch[((wave * RB + b) * 3 + pos) * 64 + lane] = f32x4{acc[b][4 * t], acc[b][4 * t + 1], acc[b][4 * t + 2], acc[b][4 * t + 3]};
            }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < RB; ++b) {
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int o = 0; o < 4; ++o) {                   // owners of quarters 0..3 = (kh, group) = (o / 2, o % 2), one fixed order
                if (o == Q) {
                    sum += f32x4{acc[b][4 * Q], acc[b][4 * Q + 1], acc[b][4 * Q + 2], acc[b][4 * Q + 3]};
                } else {
                    const int pw = (o % 2) * 4 + (o / 2) * 2 + wc;      // that owner's wavefront
                    const int pos = Q < o ? Q : Q - 1;                  // where it put quarter Q
                    sum += xch[((pw * RB + b) * 3 + pos) * 64 + lane];
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = j0 + tile_row(b, 8 * Q + 4 * half + t);
                if (row < J && col < D) W[(int64_t)row * ldw + col] = prox_entry(wreg[b][t] + alpha * sum[t], prox_kind, prox_a);
            }
        }
    };
    switch (quad) {
        case 0: finish(std::integral_constant<int, 0>{}); break;
        case 1: finish(std::integral_constant<int, 1>{}); break;
        case 2: finish(std::integral_constant<int, 2>{}); break;
        default: finish(std::integral_constant<int, 3>{}); break;
    }
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
    if (a.bf16 || a.use_mask || !al(a.u, a.ldu) || !al(a.v, a.ldv) || (a.tile_cols() % kRksBN) != 0 ||
        (a.N % kRksBK) != 0 || a.N < kRksBK || rb < 3 || rb > 5)
        return false;
    return a.conformed || ((a.J % 4) == 0 && a.J >= 4);     // padded copies of U hold J rounded up to 4 columns
}

int reconstruct_ksplit_rows(int64_t J) { return 32 * ksplit_rb(J); }

// True when splitting the pairs leaves the busiest SIMD with clearly less than `other_blocks`
// whole-block times (what the tile it would replace gives it).
bool reconstruct_ksplit_wins(int64_t J, int64_t D, int64_t other_blocks) {
    if ((D % kRksBN) != 0) return false;
    const int rb = ksplit_rb(J);
    if (rb < 3 || rb > 5) return false;
    const int64_t tiles = ((J + 32 * rb - 1) / (32 * rb)) * (D / kRksBN);
    // a tile puts rb half-blocks (rb blocks through half of the pairs, as two wavefronts with a quarter each) on
    // each of the four SIMDs of its compute unit: compare in half-block units
    const int64_t tiles_per_simd = (tiles * 4 + 1023) / 1024;
    return 10 * tiles_per_simd * rb <= 9 * 2 * other_blocks;
}

template <int RB>
static hipError_t launch_ksplit(const ReconArgs& a, hipStream_t s) {
    constexpr int BM = 32 * RB;
    constexpr size_t ring = (size_t)4 * kRksBK * (BM + kRksBN) * sizeof(float), exchange = (size_t)8 * RB * 3 * 1024;
    constexpr size_t lds_bytes = ring > exchange ? ring : exchange;
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_ksplit_kernel<RB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_jb = (a.J + BM - 1) / BM, n_db = a.tile_cols() / kRksBN;
    const int total = n_jb * n_db;
    SFB_LAUNCH(reconstruct_apply_ksplit_kernel<RB>, dim3(total), dim3(512), lds_bytes, s, a.w, a.ldw, a.u, a.ldu,
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
