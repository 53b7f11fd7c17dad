// One pass over W per step for the bf16-feature path: the update of iteration t and the scores of
// iteration t+1 in the same kernel.
//
// A bulk-synchronous run alternates  W <- W - eta*scale * U_t^T V_t  (Section 3 reconstruction + the
// update of Section 2.1) with  Z_{t+1} = A_{t+1} W^T  (problem (P)) at the W just produced.  Done as
// two kernels, W crosses HBM three times per step (read for the scores, read and written for the
// update); at 860 MB that is all the step costs.  Here a workgroup owns a band of 128 rows of W and
// a slice of its columns, walks the slice in tiles of 32 columns, and for every tile
//   1. forms the tile's update with the bf16 matrix cores (contraction over the N factor pairs),
//   2. adds it to the tile of W it has prefetched, stores the new tile (the only write of W), and
//      parks the new tile in LDS, rounded to bf16 as the score pass rounds W,
//   3. multiplies the parked tile with the next batch's features for these 32 columns into score
//      accumulators [N x 128] that stay in registers for the whole slice,
// and writes the accumulators once at the end as one split-K partial of Z (summed by the factor
// kernel, like the partials of the separate score pass).  W is read once and written once.
//
// Work split of the 8 wavefronts (two per SIMD):
//   phase 1  wavefront (rb, kh): rows 32*rb.. of the band x the tile's 32 columns, over half kh of the
//            factor pairs.  A operand: its 32 rows of (alpha u)^T for its half, held in registers for
//            the workgroup's whole life (loaded once).  B operand: v^T tile from LDS.  The two wavefronts
//            of a row block trade partial sums through LDS and each finishes two of the block's four row
//            groups, adding in one fixed order ((kh = 0 part) + (kh = 1 part), then W): results do not
//            depend on timing.
//   phase 2  wavefront (rbp, nq): rows 64*rbp.. of the band (two 32-row blocks) x a quarter nq of the
//            samples.  A operand: next features from LDS; B operand: the parked bf16 tile.
// Memory traffic of a tile: the v^T tile and the feature tile (two stages each) and the fp32 W tile (one
// stage) arrive by LDS-DMA, a share per wavefront, completion counted by hand; the new W entries are
// stored from the accumulator layout (a wavefront instruction covers two whole 128-byte lines).  The
// v^T and feature sources were laid out tile by tile, already swizzled, by the packing kernels below,
// so a stage is one linear copy.
#include <type_traits>

#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

typedef __bf16 fu_bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kFuBand = 128;      // rows of W per workgroup
constexpr int kFuCols = 32;       // columns of W per tile
constexpr int kFuThreads = 512;

__device__ __forceinline__ void fu_dma16(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}

// Every LDS access of this wavefront has completed (writes visible, reads returned), then the barrier.
__device__ __forceinline__ void fu_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// LDS swizzles (16-byte items).  v^T tile: chunks of 8 items (64 factor pairs) x 32 columns, 128-byte rows:
// item p of row r sits at p ^ key8(r); sixteen consecutive rows at one logical item cover sixteen
// different 16-byte groups of a 256-byte span.  Feature tile and parked W tile: 64-byte rows
// (32 columns of bf16), item p of row r at p ^ key4(r).
__host__ __device__ __forceinline__ int fu_key8(int r) { return (r >> 1) & 7; }
__host__ __device__ __forceinline__ int fu_key4(int r) { return (r >> 2) & 3; }

// At most n of this wavefront's vector-memory operations may still be in flight (n <= 40).
__device__ __forceinline__ void fu_wait_vm(int n) {
    switch (n) {
#define FU_CASE(k) case k: wait_vmcnt<k>(); break;
        FU_CASE(0) FU_CASE(1) FU_CASE(2) FU_CASE(3) FU_CASE(4) FU_CASE(5) FU_CASE(6) FU_CASE(7) FU_CASE(8) FU_CASE(9)
        FU_CASE(10) FU_CASE(11) FU_CASE(12) FU_CASE(13) FU_CASE(14) FU_CASE(15) FU_CASE(16) FU_CASE(17) FU_CASE(18)
        FU_CASE(19) FU_CASE(20) FU_CASE(21) FU_CASE(22) FU_CASE(23) FU_CASE(24) FU_CASE(25) FU_CASE(26) FU_CASE(27)
        FU_CASE(28) FU_CASE(29) FU_CASE(30) FU_CASE(31) FU_CASE(32) FU_CASE(33) FU_CASE(34) FU_CASE(35) FU_CASE(36)
        FU_CASE(37) FU_CASE(38) FU_CASE(39)
#undef FU_CASE
        default: wait_vmcnt<40>(); break;
    }
}

template <int NQ>   // N = 128 * NQ factor pairs (and next samples)
__global__ __launch_bounds__(kFuThreads) void update_score_kernel(
    float* __restrict__ W, int64_t ldw, const bf16_t* __restrict__ UT, const bf16_t* __restrict__ VTp,
    const bf16_t* __restrict__ AnP, float* __restrict__ Zp, int64_t ldz, int64_t zstride, int J, int D, int k_slice,
    int n_bands, int total) {
    constexpr int N = 128 * NQ;
    constexpr int STAGE = 64 * N;                  // bytes of a v^T tile (32 x N bf16) = bytes of a feature tile (N x 32 bf16)
    constexpr int LD = STAGE / 16 / kFuThreads;    // DMA instructions per lane and v^T / feature stage
    constexpr int W_LD = kFuBand * 8 / kFuThreads; // ... and per W tile (128 rows x 128 bytes)
    constexpr int KS1 = 4 * NQ;                    // 16-deep MFMA steps over a wavefront's half of the pairs
    // LDS: two v^T stages, two feature stages, one fp32 W tile, and the exchange area of the partial sums
    // (2 KB per wavefront), which is reused for the parked bf16 tile once the partial sums have been read
    constexpr int VT_OFF = 0, AN_OFF = 2 * STAGE, WS_OFF = 4 * STAGE, X_OFF = WS_OFF + kFuBand * 128;
    constexpr int TILE_ELEMS = 32 * N;             // bf16 elements of a packed tile

    extern __shared__ __attribute__((aligned(16))) unsigned char fu_lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront-uniform: roles and counters live in scalar registers
    const int l32 = lane & 31, half = lane >> 5;
    const int rb = wave & 3, kh = wave >> 2;       // phase 1 / update role
    const int rbp = wave & 1, nq = wave >> 1;      // phase 2 role

    const int id = xcd_contiguous_id(blockIdx.x, total);    // a die's workgroups share a column slice: its
    const int band = id % n_bands, ks = id / n_bands;       // v^T and feature tiles are fetched once per die
    const int j0 = band * kFuBand, k0 = ks * k_slice;
    const int n_tiles = (min(D, k0 + k_slice) - k0) / kFuCols;
    const int t0 = k0 / kFuCols;

    // this wavefront's rows of (alpha u)^T, its half of the pairs: resident A operand of phase 1
    u32x4 ut[KS1];
    {
        const bf16_t* up = UT + (int64_t)min(j0 + 32 * rb + l32, J - 1) * N + kh * (N / 2) + 8 * half;
#pragma unroll
        for (int s = 0; s < KS1; ++s) ut[s] = *reinterpret_cast<const u32x4*>(up + 16 * s);
    }

    // ---- stage copies (LDS-DMA), issued by every wavefront: lane t moves the 16-byte items t, t + 512, ... of a
    // stage.  A wavefront's loads retire in order, so "all but the n most recent loads have landed" is what
    // s_waitcnt vmcnt(n) gives; `issued` counts this wavefront's copy instructions and a stage's mark is the
    // count just after its copy.  The W stores of the same wavefronts also sit in that counter: they can only
    // make a wait longer, never let it pass early (a load that has not landed keeps every younger load in
    // flight, so more than n operations are outstanding). ----
    const uint32_t lds0 = (uint32_t)(uintptr_t)fu_lds;
    int issued = 0, mark_vt[2] = {0, 0}, mark_an[2] = {0, 0}, mark_w = 0;
    auto issue = [&](const bf16_t* tile, int lds_off) {     // one linear copy of STAGE bytes
        const unsigned char* g = reinterpret_cast<const unsigned char*>(tile) + tid * 16;
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)lds_off + (uint32_t)(wave * 1024));
#pragma unroll
        for (int i = 0; i < LD; ++i) fu_dma16(g + i * (kFuThreads * 16), base + (uint32_t)(i * kFuThreads * 16));
        issued += LD;
    };
    // W tile: item t + 512 i -> row (t + 512 i) / 8 of the band, 16 bytes at column 4 * (t % 8); rows beyond J
    // (last band) are read from row J - 1 and never stored.  Offsets are 32-bit (host: J * ldw < 2^31).
    const int w_row0 = j0 + (tid >> 3);
    const uint32_t w_col = (uint32_t)(k0 + 4 * (tid & 7));
    auto issue_w = [&](int tile) {
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)WS_OFF + (uint32_t)(wave * 1024));
#pragma unroll
        for (int i = 0; i < W_LD; ++i)
            fu_dma16(W + ((uint32_t)min(w_row0 + 64 * i, J - 1) * (uint32_t)ldw + w_col + (uint32_t)(tile * kFuCols)),
                     base + (uint32_t)(i * kFuThreads * 16));
        issued += W_LD;
        mark_w = issued;
    };

    // W stores, accumulator layout: acc[e] <-> row 8*(e/4) + 4*half + e%4 of the row block, column l32.
    // Address = (wavefront-uniform row pointer) + (one 32-bit lane offset shared by all stores).  Only the last
    // band can be ragged: whether this wavefront's 32 rows all exist is wavefront-uniform.
    float* const wblock = W + (int64_t)(j0 + 32 * rb) * ldw + k0;
    const uint32_t wlane = (uint32_t)(4 * half) * (uint32_t)ldw + (uint32_t)l32;
    const bool wfull = J - (j0 + 32 * rb) >= 32;
    const int wlim = J - (j0 + 32 * rb + 4 * half);     // rows 4*half + c of the block with c < wlim exist

    f32x16 zacc[2][NQ];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NQ; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) zacc[a][b][e] = 0.f;

    // lane constants of the fragment reads
    const int hk8 = (half ^ fu_key8(l32)) * 16;
    const int f4 = fu_key4(l32);
    const int it4[2] = {((0 + half) ^ f4) * 16, ((2 + half) ^ f4) * 16};

    issue(VTp + (int64_t)t0 * TILE_ELEMS, VT_OFF);
    mark_vt[0] = issued;
    issue(AnP + (int64_t)t0 * TILE_ELEMS, AN_OFF);
    mark_an[0] = issued;
    issue_w(0);
    if (n_tiles > 1) {
        issue(VTp + (int64_t)(t0 + 1) * TILE_ELEMS, VT_OFF + STAGE);
        mark_vt[1] = issued;
    }

    // The update of the entries this wavefront finishes: acc[8*KH .. 8*KH + 7] (two of the four row groups);
    // the partner's partial sums of the same entries come through LDS.  `own + partner` is formed as
    // (kh = 0 part) + (kh = 1 part) by both wavefronts of a pair, then added to W: one fixed order of additions.
    // The new entries are stored, and parked as bf16 [row][32 columns] over the partner's exchange slot, which
    // only this wavefront reads: neighbouring lanes hold neighbouring columns, so a lane pair trades one value
    // and each lane writes one packed pair (even lane: the row of e, odd lane: the row of e + 1).
    auto finish = [&](auto KHc, const f32x16& acc, int tile) {
        constexpr int KH = decltype(KHc)::value;
        const unsigned char* slot = fu_lds + X_OFF + rb * 4096 + (1 - KH) * 2048;
        f32x4 p[2];
        float w[8];
#pragma unroll
        for (int j = 0; j < 2; ++j) p[j] = *reinterpret_cast<const f32x4*>(slot + j * 1024 + lane * 16);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int rl = 8 * (2 * KH + t / 4) + (t % 4);                       // + 4*half: row of the block
            w[t] = *reinterpret_cast<const float*>(fu_lds + WS_OFF + (32 * rb + rl + 4 * half) * 128 + l32 * 4);
        }
        const bool odd = lane & 1;
        const int pair = l32 >> 1;                                               // dword of the 64-byte row
        unsigned char* park = fu_lds + X_OFF + rb * 4096 + (1 - KH) * 2048;
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
            float wn[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int e = 8 * KH + t + u, c = 8 * (e / 4) + (e % 4);
                wn[u] = w[t + u] + (acc[e] + p[(t + u) / 4][(t + u) % 4]);
                float* const wrowp = wblock + (int64_t)c * ldw + tile * kFuCols;      // uniform
                if (wfull || c < wlim) wrowp[wlane] = wn[u];
            }
            const float send = odd ? wn[0] : wn[1];
            const float recv = __builtin_bit_cast(
                float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));   // lane ^ 1
            const uint32_t pk = odd ? cvt_pk_bf16(recv, wn[1]) : cvt_pk_bf16(wn[0], recv);
            const int rl = 8 * (2 * KH + t / 4) + 4 * half + (t % 4) + (odd ? 1 : 0);     // row of the block
            const int off = (rl & 15) * 64 + (((pair >> 2) ^ fu_key4(rl)) * 16) + (pair & 3) * 4;
            *reinterpret_cast<uint32_t*>(park + off) = pk;
        }
    };

    for (int i = 0; i < n_tiles; ++i) {
        const int st = i & 1;
        // ---- the v^T tile of this step has landed; everybody is done with the previous step's feature tile ----
        fu_wait_vm(issued - mark_vt[st]);
        fu_barrier();
        if (i + 1 < n_tiles) {
            issue(AnP + (int64_t)(t0 + i + 1) * TILE_ELEMS, AN_OFF + (st ^ 1) * STAGE);
            mark_an[st ^ 1] = issued;
        }

        // ---- phase 1: this wavefront's half of the contraction over the factor pairs; fragments four steps ahead ----
        f32x16 acc;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
        {
            const unsigned char* vt = fu_lds + VT_OFF + st * STAGE + (kh * NQ * 32 + l32) * 128;
            auto frag = [&](int s) {
                return *reinterpret_cast<const u32x4*>(vt + (s >> 2) * 4096 + (((2 * (s & 3)) * 16) ^ hk8));
            };
            u32x4 fr[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) fr[s] = frag(s);
#pragma unroll
            for (int s = 0; s < KS1; ++s) {
                __builtin_amdgcn_sched_barrier(0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fu_bf16x8, ut[s]),
                                                              __builtin_bit_cast(fu_bf16x8, fr[s & 3]), acc, 0, 0, 0);
                if (s + 4 < KS1) fr[s & 3] = frag(s + 4);
            }
        }
        // the partner finishes the other two row groups: hand it this wavefront's partial sums of those
        {
            unsigned char* mine = fu_lds + X_OFF + rb * 4096 + kh * 2048;
#pragma unroll
            for (int j = 0; j < 2; ++j)      // kh = 0 hands over entries 8..15, kh = 1 entries 0..7 (a select, no indexing)
                *reinterpret_cast<f32x4*>(mine + j * 1024 + lane * 16) =
                    kh == 0 ? f32x4{acc[8 + 4 * j], acc[9 + 4 * j], acc[10 + 4 * j], acc[11 + 4 * j]}
                            : f32x4{acc[4 * j], acc[1 + 4 * j], acc[2 + 4 * j], acc[3 + 4 * j]};
        }
        // ---- partial sums exchanged, the W tile has landed; the v^T stage is free again ----
        fu_wait_vm(issued - mark_w);
        fu_barrier();
        if (kh == 0) finish(std::integral_constant<int, 0>{}, acc, i);
        else finish(std::integral_constant<int, 1>{}, acc, i);
        // (after the update's stores: this copy has two tiles of lead, the stores are wanted now)
        if (i + 2 < n_tiles) {
            issue(VTp + (int64_t)(t0 + i + 2) * TILE_ELEMS, VT_OFF + st * STAGE);
            mark_vt[st] = issued;
        }

        // ---- the parked tile is complete, the W stage is free, and the feature tile has landed ----
        fu_wait_vm(issued - mark_an[st]);
        fu_barrier();
        if (i + 1 < n_tiles) issue_w(i + 1);

        // ---- phase 2: scores of the next batch from the new tile ----
        {
            const unsigned char* an = fu_lds + AN_OFF + st * STAGE + (nq * NQ * 32 + l32) * 64;
            // row l32 of a block was parked by the wavefront that finished its row group, over its partner's slot
            const unsigned char* parked = fu_lds + X_OFF + (2 * rbp) * 4096 + (1 - (l32 >> 4)) * 2048 + (l32 & 15) * 64;
#pragma unroll
            for (int s = 0; s < 2; ++s) {          // 16 columns at a time: two fragments of the new tile, NQ of the features
                u32x4 wf[2];
#pragma unroll
                for (int a = 0; a < 2; ++a) wf[a] = *reinterpret_cast<const u32x4*>(parked + a * 4096 + it4[s]);
                u32x4 a0 = *reinterpret_cast<const u32x4*>(an + it4[s]), a1;
#pragma unroll
                for (int b = 0; b < NQ; b += 2) {
                    if (b + 1 < NQ) a1 = *reinterpret_cast<const u32x4*>(an + (b + 1) * 2048 + it4[s]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int a = 0; a < 2; ++a)
                        zacc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fu_bf16x8, a0),
                                                                             __builtin_bit_cast(fu_bf16x8, wf[a]),
                                                                             zacc[a][b], 0, 0, 0);
                    if (b + 2 < NQ) a0 = *reinterpret_cast<const u32x4*>(an + (b + 2) * 2048 + it4[s]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (b + 1 < NQ) {
#pragma unroll
                        for (int a = 0; a < 2; ++a)
                            zacc[a][b + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(fu_bf16x8, a1),
                                                                                 __builtin_bit_cast(fu_bf16x8, wf[a]),
                                                                                 zacc[a][b + 1], 0, 0, 0);
                    }
                }
            }
        }
    }

    // this slice's partial scores: zacc[a][b][e] <-> sample 32*(nq*NQ + b) + 8*(e/4) + 4*half + e%4, row 64*rbp + 32*a + l32
    float* zp = Zp + (int64_t)ks * zstride;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int row = j0 + 64 * rbp + 32 * a + l32;
#pragma unroll
        for (int b = 0; b < NQ; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int n = 32 * (nq * NQ + b) + 8 * (e / 4) + 4 * half + (e % 4);
                if (row < J) zp[(int64_t)n * ldz + row] = zacc[a][b][e];
            }
    }
}

// ---------------------------------------------------------------------------------------
// Received factors -> the operands of phase 1, and the next batch's features -> the A operand of phase 2:
//   UT[j][n] = bf16(alpha * U[n][j])                       row-major, n contiguous
//   VTp: v^T tile by tile (32 columns of W x N pairs), each tile in the swizzled LDS order of the kernel
//        above: element (column r of the tile, pair k) at item ((k/64)*32 + r)*8 + ((k/8 % 8) ^ key8(r))
//   AnP: the next features tile by tile (N samples x 32 columns), item p of sample n at n*4 + (p ^ key4(n))
//   V  : takes the next features (v_i = a_i, Section 2.1) once its old contents have been packed
// Rows of dead workers go into UT and VTp as zeros.  64 x 64 tiles through LDS; blocks [0, n_jblk) of a row
// of blocks do U, the rest V.  A V block is the only one that touches its 64 samples x 64 columns of V: it
// reads them (v_t), and after its barrier, when every one of those reads has returned, overwrites them.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fused_pack_kernel(
    const float* __restrict__ U, int64_t ldu, bf16_t* __restrict__ V, int64_t ldv, const bf16_t* __restrict__ A,
    int64_t lda, bf16_t* __restrict__ UT, bf16_t* __restrict__ VTp, bf16_t* __restrict__ AnP, int N, int J, int D, int B,
    float alpha, uint64_t live_mask, bool use_mask, int n_jblk, int n_dblk, bool vec_u) {
    // [column of the source][pair of samples]: a word holds samples 2 w and 2 w + 1 of one column as bf16.  Rows of
    // 36 words (144 bytes); the 4-word group g of row r sits at group g ^ (r / 4 % 8), so that the 64 lanes of a
    // write (16 column quads x 4 pairs) fall two to a bank, and a 16-byte read still finds its 8 samples together.
    __shared__ __attribute__((aligned(16))) uint32_t tile[64][36];
    const int tid = threadIdx.x;
    const int n_cblk = n_jblk + n_dblk;
    const int cb = blockIdx.x % n_cblk, kb = blockIdx.x / n_cblk;
    const bool is_u = cb < n_jblk;
    const int c0 = (is_u ? cb : cb - n_jblk) * 64, k0 = kb * 64;
    const int ncols = is_u ? J : D;
    // the next features of this block's samples and columns: two 16-byte items per thread, requested first
    u32x4 nxt[2];
    if (!is_u) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = tid + 256 * i, n = k0 + idx / 8, c = c0 + 8 * (idx % 8);
            nxt[i] = c < D ? *reinterpret_cast<const u32x4*>(A + (int64_t)n * lda + c) : u32x4{0, 0, 0, 0};
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int np = (tid >> 4) + 16 * i, c = c0 + (tid & 15) * 4;       // samples 2 np and 2 np + 1 of the block
        f32x4 v[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int n = k0 + 2 * np + h;
            bool live = n < N;
            if (use_mask && live) live = (live_mask >> (n / B)) & 1ull;
            v[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (live) {
                // one 16-byte (U) or 8-byte (V: host guarantees 16-byte aligned rows) load where the four entries exist
                if (is_u) v[h] = load4(U + (int64_t)n * ldu, c, ncols, vec_u) * alpha;
                else v[h] = load4(V + (int64_t)n * ldv, c, ncols, true);
            }
        }
        const int word = np ^ (4 * ((tid & 15) & 7));                       // row / 4 = tid & 15
#pragma unroll
        for (int e = 0; e < 4; ++e)
            tile[(tid & 15) * 4 + e][word] = (uint32_t)f32_to_bf16(v[0][e]) | ((uint32_t)f32_to_bf16(v[1][e]) << 16);
    }
    __syncthreads();
    // store: thread -> 2 columns x 8 consecutive n (one 16-byte item)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = (tid >> 3) + 32 * i, p8 = tid & 7;
        if (c0 + c >= ncols) continue;
        const u32x4 item = *reinterpret_cast<const u32x4*>(&tile[c][4 * (p8 ^ ((c >> 2) & 7))]);
        if (is_u) {
            *reinterpret_cast<u32x4*>(UT + (int64_t)(c0 + c) * N + k0 + p8 * 8) = item;
        } else {
            const int col = c0 + c, t = col / kFuCols, r = col % kFuCols;
            const int64_t slot = ((int64_t)kb * 32 + r) * 8 + (p8 ^ fu_key8(r));
            *reinterpret_cast<u32x4*>(VTp + (int64_t)t * (32 * N) + slot * 8) = item;
        }
    }
    if (!is_u) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = tid + 256 * i, n = k0 + idx / 8, c = c0 + 8 * (idx % 8);
            if (c >= D) continue;
            const int t = c / kFuCols, p = (c % kFuCols) / 8;
            *reinterpret_cast<u32x4*>(AnP + (int64_t)t * (32 * N) + ((int64_t)n * 4 + (p ^ fu_key4(n))) * 8) = nxt[i];
            *reinterpret_cast<u32x4*>(V + (int64_t)n * ldv + c) = nxt[i];
        }
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
bool fused_shape_ok(int64_t J, int64_t D, int64_t N) {
    return (N == 128 || N == 256 || N == 512) && D % kFuCols == 0 && D >= kFuCols && J >= 1;
}

// Column slices, each at least 8 tiles long.  One workgroup per compute unit is resident, so the launch takes
// rounds-of-256-workgroups x (tiles of a slice + the fixed cost of a workgroup: its rows of (alpha u)^T in, its
// partial scores out, about 7 tile times), and every slice costs one more write and read of the partial scores
// (N x J x 8 bytes at about 4 TB/s, a tile taking about 2.7 us).  Up to 85 bands that is one round of as many
// slices as fit; beyond (J = 11000: 86 bands) two rounds of shorter slices beat one round that leaves a third of
// the compute units idle.  Ties go to fewer slices.
FusedPlan plan_fused(int64_t J, int64_t D, int64_t N) {
    FusedPlan p{};
    p.n_bands = (int)((J + kFuBand - 1) / kFuBand);
    const int64_t tiles = D / kFuCols;
    int64_t s_max = tiles / 8;
    if (s_max < 1) s_max = 1;
    if (s_max > 64) s_max = 64;
    const double slice_cost = (double)N * (double)J * 8.0 / 4e6 / 2.7;        // in tile times
    int64_t best = 1;
    double best_cost = 1e300;
    for (int64_t s = 1; s <= s_max; ++s) {
        const int64_t per = (tiles + s - 1) / s;
        if ((tiles + per - 1) / per != s) continue;                           // the same cut as a smaller count
        const double rounds = (double)((p.n_bands * s + 255) / 256);
        const double cost = rounds * ((double)per + 7.0) + (double)s * slice_cost;
        if (cost < best_cost * (1.0 - 1e-9)) { best_cost = cost; best = s; }
    }
    const int64_t per = (tiles + best - 1) / best;
    p.slices = (int)((tiles + per - 1) / per);
    p.k_slice = (int)(per * kFuCols);
    p.grid = p.n_bands * p.slices;
    return p;
}

// Extra device scratch beyond the bf16 reconstruction's ((alpha u)^T and v^T, reused as UT and VTp): the staged features.
size_t fused_extra_workspace(int64_t D, int64_t N) { return ((size_t)D * N * 2 + 255) / 256 * 256; }

bool fused_call_ok(const FusedArgs& a) {
    auto al16 = [](const void* p) { return ((uintptr_t)p % 16) == 0; };
    return fused_shape_ok(a.J, a.D, a.N) && (int64_t)a.J * a.ldw < (1LL << 31) && al16(a.a_next) && (a.lda % 8) == 0 &&
           al16(a.v) && (a.ldv % 8) == 0 && al16(a.w) && (a.ldw % 4) == 0;
}

template <int NQ>
static hipError_t launch_update_score(const FusedArgs& a, const FusedPlan& p, const bf16_t* UT, const bf16_t* VTp,
                                      const bf16_t* AnP, hipStream_t s) {
    constexpr int N = 128 * NQ;
    constexpr size_t lds_bytes = (size_t)4 * 64 * N + kFuBand * 128 + 4 * 4096;
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)update_score_kernel<NQ>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    SFB_LAUNCH(update_score_kernel<NQ>, dim3(p.grid), dim3(kFuThreads), lds_bytes, s, a.w, a.ldw, UT, VTp, AnP, a.zp, a.ldz,
               a.zstride, a.J, a.D, p.k_slice, p.n_bands, p.grid);
    return hipGetLastError();
}

// ws_factors: the bf16 reconstruction's scratch ((alpha u)^T [J][N], then v^T, 256-byte rounded), ws_next: fused_extra_workspace bytes.
hipError_t launch_fused(const FusedArgs& a, const FusedPlan& p, void* ws_factors, void* ws_next, hipStream_t s) {
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    bf16_t* UT = (bf16_t*)ws_factors;
    bf16_t* VTp = (bf16_t*)((char*)ws_factors + up((size_t)a.J * a.N * 2));
    bf16_t* AnP = (bf16_t*)ws_next;
    const int n_jblk = (a.J + 63) / 64, n_dblk = a.D / 64 + (a.D % 64 ? 1 : 0), n_kblk = a.N / 64;
    // a plain launch: an armed pair of timing events belongs to the fused kernel below
    hipLaunchKernelGGL(fused_pack_kernel, dim3((n_jblk + n_dblk) * n_kblk), dim3(256), 0, s, a.u, a.ldu, (bf16_t*)a.v, a.ldv,
                       (const bf16_t*)a.a_next, a.lda, UT, VTp, AnP, a.N, a.J, a.D, a.B, a.alpha, a.live_mask, a.use_mask,
                       n_jblk, n_dblk, ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (a.N) {
        case 128: return launch_update_score<1>(a, p, UT, VTp, AnP, s);
        case 256: return launch_update_score<2>(a, p, UT, VTp, AnP, s);
        case 512: return launch_update_score<4>(a, p, UT, VTp, AnP, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace sfb
