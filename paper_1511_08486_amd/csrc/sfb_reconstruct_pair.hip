// Reconstruction + update (Section 3, Section 2.1) on 128 x 128 tiles of W with EIGHT wavefronts:
//     W[j][d] <- W[j][d] + alpha * sum_n U[n][j] * V[n][d]
//
// The tile, the staging and the operand layouts are those of the LDS-DMA kernel in
// sfb_reconstruct.hip: a wavefront owns 32 rows x 128 columns (four 32 x 32 blocks, columns
// interleaved by four so that one 16-byte LDS read feeds four matrix instructions and a lane
// finishes four consecutive entries of a row), the factor tiles [k][128] go from L2 straight into
// LDS, alpha and the entrywise proximal operator are applied in the epilogue.  What differs is who
// multiplies what.  That kernel runs four wavefronts, one per SIMD, and every hand-over to the next
// chunk of 32 pairs (wait for the copies, barrier, issue the next copies, first LDS reads) is time
// the matrix pipe of that SIMD stands still: about a seventh of the loop at N = 512.  Here two
// wavefronts share each SIMD and each 32-row strip, in two groups of four that take the chunks in
// turn (group 0 the even chunks, group 1 the odd ones): when one wavefront of a SIMD is at a
// hand-over, the other is in the middle of its own chunk and keeps the pipe busy.  Barrier number c
// is the hand-over to chunk c: the group that owns chunk c reaches it between two chunks, the other
// group in the middle of chunk c - 1 (32 of its 64 matrix instructions issued); every wavefront
// executes every barrier exactly once.  A group stages its own chunks (its four wavefronts, 256
// lanes, 8 copy instructions each; a ring of four stages, two per group; completion counted by hand
// with the in-order vector-memory counter) and only it reads them, so a chunk's stage is free again
// as soon as the group has passed its next hand-over.  At the end the two wavefronts of a strip
// trade halves of their partial sums through LDS and each finishes half of the strip's entries:
// (even chunks) + (odd chunks), then + W: one fixed order, results do not depend on timing.
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

constexpr int kRpBM = 128, kRpBN = 128, kRpBK = 32;

// EDGE: W may have any alignment and leading dimension and end inside the last column tile (the factors
// are then padded copies): its entries are read after the contraction and written one by one within bounds.
template <bool EDGE>
__global__ __launch_bounds__(512) void reconstruct_apply_pair_kernel(
    float* __restrict__ W, int64_t ldw, const float* __restrict__ U, int64_t ldu, const float* __restrict__ V,
    int64_t ldv, int J, int D, int N, float alpha, int n_jb, int total, int prox_kind, float prox_a) {
    constexpr int BM = kRpBM, BN = kRpBN, BK = kRpBK, GT = 256;               // GT: threads of a group
    constexpr int U_LD = BK * BM / 4 / GT, V_LD = BK * BN / 4 / GT;           // 16-byte DMAs per thread and chunk
    constexpr int DMAS = U_LD + V_LD;
    constexpr int STAGE_FLOATS = BK * (BM + BN);
    constexpr int W_LOADS = EDGE ? 0 : 8;        // 16-byte loads in flight during the contraction: a wavefront finishes half of its strip's entries
    static_assert(U_LD == 4 && V_LD == 4, "tile / thread count mismatch");
    static_assert(DMAS + W_LOADS <= 63, "wait count encoding");
    extern __shared__ __attribute__((aligned(16))) float rp_lds[];            // 4 x (U tile, V tile); the exchange area overlays it

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int g = wave >> 2, strip = wave & 3, gtid = tid & (GT - 1);
    const int id = xcd_contiguous_id(blockIdx.x, total);
    const int jb = id % n_jb, db = id / n_jb;
    const int j0 = jb * BM, d0 = db * BN;

    // source of DMA i of a chunk: item idx = gtid + i * GT of the [k][128] tile in row-major order of
    // 16-byte items.  Columns of U beyond J rounded up to 4 are clamped (host: a row of U holds that many
    // floats): they feed rows of W that are never stored.
    const int ju = (J + 3) & ~3;
    const float* pu[U_LD];
    const float* pv[V_LD];
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
    const uint32_t lds0 = (uint32_t)(uintptr_t)rp_lds;
    const int64_t ustep = (int64_t)BK * ldu, vstep = (int64_t)BK * ldv;
    auto issue_one = [&](int chunk, int i) {
        const uint32_t ubase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)((chunk & 3) * STAGE_FLOATS + strip * 64 * 4) * 4u);
        if (i < U_LD) lds_dma16(pu[i] + chunk * ustep, ubase + (uint32_t)(i * GT * 16));
        else lds_dma16(pv[i - U_LD] + chunk * vstep, ubase + (uint32_t)(BK * BM) * 4u + (uint32_t)((i - U_LD) * GT * 16));
    };

    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;

    // MFMA k-step s (0..7) of half h of a chunk covers pairs 16 h + 2 s and + 1: lanes 0-31 carry the first
    // (row l32 of the strip / columns 4 l32 .. 4 l32 + 3), lanes 32-63 the second.
    struct Frags {
        float a[8];
        f32x4 b[8];
    };
    auto load_step = [&](int st, int h, int s, Frags& f) {
        const int k = 16 * h + 2 * s + half;
        f.a[s] = rp_lds[st * STAGE_FLOATS + k * BM + strip * 32 + l32];
        f.b[s] = *reinterpret_cast<const f32x4*>(&rp_lds[st * STAGE_FLOATS + BK * BM + k * BN + 4 * l32]);
    };
    // The matrix instructions of one half chunk; between(s) runs after those of k-step s: LDS reads of the other
    // half and copies of a later chunk go there, a piece per k-step, in the shadow of the matrix pipe.
    auto multiply = [&](const Frags& f, auto between) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[s], f.b[s][n], acc[n], 0, 0, 0);
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

    // The W entries this wavefront finishes: accumulator entries 8 g .. 8 g + 7 of its four blocks = 8 rows x 4
    // consecutive columns per lane.
    f32x4 wreg[8];
    auto w_row = [&](int t) {
        const int e = 8 * g + t;
        return j0 + strip * 32 + 8 * (e / 4) + 4 * half + (e % 4);
    };
    auto load_w = [&]() {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const float* wr = W + (int64_t)min(w_row(t), J - 1) * ldw;
            if constexpr (EDGE) {
#pragma unroll
                for (int q = 0; q < 4; ++q) wreg[t][q] = wr[min(d0 + 4 * l32 + q, D - 1)];
            } else {
                wreg[t] = ldg4(wr + d0 + 4 * l32);
            }
        }
    };
    if (!EDGE && g >= n_chunks) load_w();                    // a single chunk: group 1 has none, but finishes its half
    Frags fa, fb;
    for (int c = g; c < n_chunks; c += 2) {
        // hand-over to chunk c.  In counter order my copies of chunk c are followed by nothing but, once, the W
        // loads (requested during my first chunk, i.e. after the copies of my second one)
        if (c == g + 2) wait_vmcnt<W_LOADS>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();                        // barrier c
        const int st = c & 3;
        const bool more = c + 2 < n_chunks;
#pragma unroll
        for (int s = 0; s < 8; ++s) load_step(st, 0, s, fa);
        if (c == g) {
            // the copies of my second chunk first, then the W entries: they have the whole contraction to arrive
            if (more) {
#pragma unroll
                for (int i = 0; i < DMAS; ++i) issue_one(c + 2, i);
            }
            if (!EDGE) load_w();
            multiply(fa, [&](int s) { load_step(st, 1, s, fb); });
        } else {
            multiply(fa, [&](int s) {
                if (more) issue_one(c + 2, s);               // DMAS == 8: one copy instruction per k-step
                load_step(st, 1, s, fb);
            });
        }
        if (c + 1 < n_chunks) __builtin_amdgcn_s_barrier();  // barrier c + 1: the other group's hand-over
        multiply(fb, [](int) {});
    }
    static_assert(DMAS == 8, "one copy instruction per k-step of a half chunk");

    // Exchange of partial sums.  Everybody is done with the ring (barrier), which the exchange area overlays:
    // slot of wavefront w = the eight accumulator entries of each of its four blocks that its partner finishes,
    // as [entry][lane] items of 16 bytes (the four blocks' values of one entry).
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (EDGE) load_w();
    f32x4* xch = reinterpret_cast<f32x4*>(rp_lds);
    auto finish = [&](auto Gc) {
        constexpr int G = decltype(Gc)::value;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            constexpr int e0 = 8 * (1 - G);
            xch[(wave * 8 + t) * 64 + lane] = f32x4{acc[0][e0 + t], acc[1][e0 + t], acc[2][e0 + t], acc[3][e0 + t]};
        }
        __syncthreads();
        const int partner = wave ^ 4;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const f32x4 p = xch[(partner * 8 + t) * 64 + lane];
            const int e = 8 * G + t;
            const f32x4 mine = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
            const f32x4 sum = G == 0 ? mine + p : p + mine;          // (even chunks) + (odd chunks)
            const int row = w_row(t);
            const f32x4 w = prox_entry4(wreg[t] + alpha * sum, prox_kind, prox_a);
            if constexpr (EDGE) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = d0 + 4 * l32 + q;
                    if (row < J && col < D) W[(int64_t)row * ldw + col] = w[q];
                }
            } else {
                if (row < J) *reinterpret_cast<f32x4*>(W + (int64_t)row * ldw + d0 + 4 * l32) = w;
            }
        }
    };
    if (g == 0) finish(std::integral_constant<int, 0>{});
    else finish(std::integral_constant<int, 1>{});
}

bool reconstruct_pair_ok(const ReconArgs& a) {
    auto al = [](const void* p, int64_t ld) { return ((uintptr_t)p % 16) == 0 && (ld % 4) == 0; };
    if (a.bf16 || a.use_mask || !al(a.u, a.ldu) || !al(a.v, a.ldv) || (a.tile_cols() % kRpBN) != 0 ||
        (a.N % kRpBK) != 0 || a.N < kRpBK)
        return false;
    // padded copies of the factors go with the entry-by-entry form of the W accesses
    return a.conformed || (al(a.w, a.ldw) && (a.J % 4) == 0 && a.J >= 4);
}

template <bool EDGE>
static hipError_t launch_pair(const ReconArgs& a, hipStream_t s) {
    constexpr size_t lds_bytes = (size_t)4 * kRpBK * (kRpBM + kRpBN) * sizeof(float);      // 128 KB; the exchange needs 64 KB
    static std::atomic<bool> raised{false};
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)reconstruct_apply_pair_kernel<EDGE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_jb = (a.J + kRpBM - 1) / kRpBM, n_db = a.tile_cols() / kRpBN;
    const int total = n_jb * n_db;
    SFB_LAUNCH(reconstruct_apply_pair_kernel<EDGE>, dim3(total), dim3(512), lds_bytes, s, a.w, a.ldw, a.u, a.ldu,
               (const float*)a.v, a.ldv, a.J, a.D, a.N, a.alpha, n_jb, total, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

hipError_t launch_reconstruct_pair(const ReconArgs& a, hipStream_t s) {
    return a.conformed ? launch_pair<true>(a, s) : launch_pair<false>(a, s);
}

}  // namespace sfb
