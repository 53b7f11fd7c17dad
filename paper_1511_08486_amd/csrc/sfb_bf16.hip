// bf16-feature path (bf16 a_i and v_i, fp32 W, u and accumulation) on the bf16 matrix cores.
//
// With 16x the fp32 MFMA rate, both contractions of the step stop being compute-bound at
// the sizes this path is for (W of hundreds of MB): the score pass must read W once, the
// reconstruction must read and write it once, and everything else is sized so that HBM
// streaming of W is the only thing that cannot be hidden.
//
// One "NT" kernel serves both contractions: C[m][n] = sum_k A[m][k] * B[n][k] with both
// operands contiguous along k, staged HBM/L2 -> LDS by DMA through a ring of stages
// (completion tracked by hand, see lds_dma16), swizzled on the source side so that the
// 128-bit fragment reads are conflict-free, and v_mfma_f32_32x32x16_bf16 (lane l supplies
// 8 consecutive k of row l%32, lanes 32..63 the upper 8 of each 16; A and B use the same
// k order, so the order itself is immaterial).
//   scores (Section 2, z = W a):      A = features [N][D] bf16, B = W [J][D] fp32, widened
//                                     operand rounded to bf16 (RNE) after the LDS read;
//                                     epilogue stores a split-K partial of Z; the feature tiles
//                                     are passed on to V (v_i = a_i), a share per class block.
//   reconstruct (Section 3 + 2.1):    A = (alpha u)^T [J][N] bf16, B = v^T [D][N] bf16, both
//                                     produced by transpose_pack_kernel from the received
//                                     factors; epilogue is the read-modify-write W += C.
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tile shapes.  Reconstruction: 256 x 128 (rows of W x columns of W), 2 x 2 wavefronts, 32-deep
// stages (72 KB of LDS), two workgroups per compute unit: one multiplies while the other sits
// in its read-modify-write of W, whose loads and stores are paced by HBM.
// Scores: 256 samples x 256 classes, 4 x 2 wavefronts (two per SIMD): the feature operand is
// re-read once per class block, so wide class blocks halve that traffic, and 80 tiles x 3
// slices of D fill the chip in a single round.
constexpr int kBfReconBM = 256, kBfReconBN = 128, kBfReconBK = 32, kBfReconWPS = 2;
constexpr int kBfFwdBM = 256, kBfFwdBN = 256, kBfFwdBK = 32;

__device__ __forceinline__ void lds_dma16_raw(const void* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}

// Swizzle for a tile whose rows are IPR items of 16 bytes: item c of row r is stored at
// position c ^ swz<IPR>(r).  For every IPR, sixteen consecutive rows read at the same
// logical item land in sixteen different 16-byte bank groups.
template <int IPR> __device__ __forceinline__ int swz(int r);
template <> __device__ __forceinline__ int swz<4>(int r) { return (r >> 2) & 3; }
template <> __device__ __forceinline__ int swz<8>(int r) { return (r & 7) ^ ((r >> 3) & 1); }
template <> __device__ __forceinline__ int swz<16>(int r) { return r & 15; }

enum BfEpilogue { kStoreZ = 0, kUpdateW = 1 };

// B_FP32: B rows are fp32 in memory (W in the score pass) and are rounded to bf16 after the
// LDS read.  NST: stages in the ring.
// WPS: wavefronts per SIMD the register budget must allow (2 = two workgroups of four
// wavefronts, or one of eight, per compute unit).
// BM x BN tile computed by WGM x WGN wavefronts.
template <bool B_FP32, int EPI, int NST, int BK, int WPS, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(WGM * WGN * 64, WPS) void nt_bf16_kernel(
    const bf16_t* __restrict__ A, int64_t lda, const void* __restrict__ Bv, int64_t ldb, float* __restrict__ C,
    int64_t ldc, int64_t cstride, bf16_t* __restrict__ Vout, int64_t ldv, int M, int N, int K, int k_slice,
    int n_mb, int n_nb, int total, int band, int prox_kind, float prox_a) {
    constexpr int kBfThreads = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN, MT = WM / 32, NT = WN / 32;
    static_assert(MT >= 1 && NT >= 1 && MT * 32 * WGM == BM && NT * 32 * WGN == BN, "tile / wavefront grid mismatch");
    constexpr int IA = BK / 8, IB = B_FP32 ? BK / 4 : BK / 8;      // 16-byte items per tile row
    constexpr int A_ITEMS = BM * IA, B_ITEMS = BN * IB;
    constexpr int A_LD = A_ITEMS / kBfThreads, B_LD = B_ITEMS / kBfThreads;
    constexpr int A_BYTES = A_ITEMS * 16, STAGE_BYTES = (A_ITEMS + B_ITEMS) * 16;
    constexpr int KSTEPS = BK / 16;

    extern __shared__ __attribute__((aligned(16))) unsigned char bf_lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, half = lane >> 5;

    // consecutive ids share the B block (W rows in the score pass: the workgroups that
    // reuse a W block run next to each other on one die)
    int id = xcd_contiguous_id(blockIdx.x, total);
    int mb, nb, ks;
    if (EPI == kUpdateW) {
        // one slice; walk the tile grid in bands of `band` B-blocks with the A block fastest
        // inside a band: a band's B-blocks stay in the die's L2 (the host sizes the band for
        // that, ideally one band per die) while the A blocks stream past them once per band
        ks = 0;
        const int bi = id / (band * n_mb), rem = id - bi * band * n_mb;
        const int width = min(band, n_nb - bi * band);     // the last band may be narrower
        nb = bi * band + rem % width;
        mb = rem / width;
    } else {
        mb = id % n_mb;
        id /= n_mb;
        nb = id % n_nb;
        ks = id / n_nb;
    }
    const int m0 = mb * BM, n0 = nb * BN;
    const int k_begin = ks * k_slice;
    const int n_chunks = (min(K, k_begin + k_slice) - k_begin) / BK;   // host: K % BK == 0

    const bf16_t* pa[A_LD];
    const unsigned char* pb[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int s = tid + i * kBfThreads, r = s / IA, c = (s % IA) ^ swz<IA>(r);
        pa[i] = A + (int64_t)min(m0 + r, M - 1) * lda + k_begin + 8 * c;
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int s = tid + i * kBfThreads;
        const int r = s / IB, c = (s % IB) ^ swz<IB>(r);
        if (B_FP32) {
            pb[i] = (const unsigned char*)((const float*)Bv + (int64_t)min(n0 + r, N - 1) * ldb + k_begin + 4 * c);
        } else {
            pb[i] = (const unsigned char*)((const bf16_t*)Bv + (int64_t)min(n0 + r, N - 1) * ldb + k_begin + 8 * c);
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)bf_lds;
    auto issue = [&](int chunk, int st) {
        const uint32_t abase = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(st * STAGE_BYTES + wave * 1024));
        const uint32_t bbase = abase + (uint32_t)A_BYTES;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) lds_dma16_raw(pa[i] + chunk * BK, abase + (uint32_t)(i * kBfThreads * 16));
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            lds_dma16_raw(pb[i] + (int64_t)chunk * BK * (B_FP32 ? 4 : 2), bbase + (uint32_t)(i * kBfThreads * 16));
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // byte offsets of this lane's items (row base excluded); every row this lane reads is
    // congruent to l32 modulo 32, so the swizzle value is a lane constant
    int a_off[KSTEPS], b_off[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        a_off[s] = 16 * ((2 * s + half) ^ swz<IA>(l32));
        b_off[s] = B_FP32 ? 16 * ((4 * s + 2 * half) ^ swz<IB>(l32)) : 16 * ((2 * s + half) ^ swz<IB>(l32));
    }
    const int swb = swz<IB>(l32);

    struct Frag { u32x4 a[MT]; u32x4 b[NT]; u32x4 b2[B_FP32 ? NT : 1]; };
    auto read_frag = [&](Frag& f, int st, int s) {
        const unsigned char* as = bf_lds + st * STAGE_BYTES + (wm * WM + l32) * (IA * 16);
        const unsigned char* bs = bf_lds + st * STAGE_BYTES + A_BYTES + (wn * WN + l32) * (IB * 16);
#pragma unroll
        for (int i = 0; i < MT; ++i) f.a[i] = *reinterpret_cast<const u32x4*>(as + i * 32 * (IA * 16) + a_off[s]);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            if (B_FP32) {
                // 8 consecutive k of an fp32 row = two 16-byte items (logical 4s+2h and 4s+2h+1)
                const unsigned char* row = bs + j * 32 * (IB * 16);
                f.b[j] = *reinterpret_cast<const u32x4*>(row + b_off[s]);
                f.b2[j] = *reinterpret_cast<const u32x4*>(row + 16 * ((4 * s + 2 * half + 1) ^ swb));
            } else {
                f.b[j] = *reinterpret_cast<const u32x4*>(bs + j * 32 * (IB * 16) + b_off[s]);
            }
        }
    };
    auto mma_frag = [&](const Frag& f) {
        bf16x8 bop[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            if (B_FP32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    bop[j][e] = (__bf16)__uint_as_float(f.b[j][e]);          // round to nearest even
                    bop[j][e + 4] = (__bf16)__uint_as_float(f.b2[j][e]);
                }
            } else {
                bop[j] = __builtin_bit_cast(bf16x8, f.b[j]);
            }
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]), bop[j],
                                                                     acc[i][j], 0, 0, 0);
    };
    auto compute = [&](int st) {
        Frag f0, f1;
        read_frag(f0, st, 0);
#pragma unroll
        for (int s = 0; s < KSTEPS; s += 2) {
            if (s + 1 < KSTEPS) read_frag(f1, st, s + 1);
            __builtin_amdgcn_sched_barrier(0);
            mma_frag(f0);
            __builtin_amdgcn_sched_barrier(0);
            if (s + 1 < KSTEPS) {
                if (s + 2 < KSTEPS) read_frag(f0, st, s + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma_frag(f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // v_i = a_i: the staged feature items go on to V (score pass); the class blocks share the job,
    // block nb takes the chunks c with c % n_nb == nb
    const bool write_v = (EPI == kStoreZ) && (Vout != nullptr);
    auto copy_v = [&](int chunk, int st) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int s = tid + i * kBfThreads, r = s / IA, c = (s % IA) ^ swz<IA>(r);
            const u32x4 v = *reinterpret_cast<const u32x4*>(bf_lds + st * STAGE_BYTES + 16 * s);
            if (m0 + r < M)
                *reinterpret_cast<u32x4*>(Vout + (int64_t)(m0 + r) * ldv + k_begin + chunk * BK + 8 * c) = v;
        }
    };

    // ring of NST stages, NST-1 of them in flight ahead of the one being multiplied
#pragma unroll
    for (int p = 0; p < NST - 1; ++p)
        if (p < n_chunks) issue(p, p);

    auto step = [&](int c, int st) {
        // younger DMAs that may still be in flight: those of the next NST-2 chunks
        const int younger = min(n_chunks - 1 - c, NST - 2);
        if (younger >= 2) wait_vmcnt<2 * (A_LD + B_LD)>();
        else if (younger == 1) wait_vmcnt<A_LD + B_LD>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (c + NST - 1 < n_chunks) issue(c + NST - 1, (st + NST - 1) % NST);
        if (write_v && (c % n_nb) == nb) copy_v(c, st);
        compute(st);
    };
    static_assert(NST == 3 || NST == 4, "ring depth");
    int c = 0;
    for (; c + NST - 1 < n_chunks; c += NST) {
        step(c, 0);
        step(c + 1, 1);
        step(c + 2, 2);
        if (NST == 4) step(c + 3, 3);
    }
    if (c < n_chunks) step(c, 0);
    if (c + 1 < n_chunks) step(c + 1, 1);
    if (NST == 4 && c + 2 < n_chunks) step(c + 2, 2);

    float* cout = C + (int64_t)ks * cstride;
    if (EPI == kUpdateW) {
        // Read-modify-write of the tile in groups of EG 32 x 32 blocks: all loads of a group
        // first (addresses clamped into the matrix, so no branch sits between them and 16*EG
        // loads per lane are in flight), then the adds and the guarded stores.  Each wavefront
        // instruction covers two full 128-byte lines of W.  The other workgroup resident on
        // this compute unit multiplies meanwhile.
        constexpr int EG = 4, NBLK = MT * NT;
        static_assert(NBLK % EG == 0, "epilogue group");
#pragma unroll
        for (int g = 0; g < NBLK; g += EG) {
            float w[EG][16];
#pragma unroll
            for (int b = 0; b < EG; ++b) {
                const int i = (g + b) / NT, j = (g + b) % NT;
                const int cc = min(n0 + wn * WN + j * 32 + l32, N - 1);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                    w[b][e] = cout[(int64_t)min(row, M - 1) * ldc + cc];
                }
            }
#pragma unroll
            for (int b = 0; b < EG; ++b) {
                const int i = (g + b) / NT, j = (g + b) % NT;
                const int col = n0 + wn * WN + j * 32 + l32;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                    if (row < M && col < N) cout[(int64_t)row * ldc + col] = prox_entry(w[b][e] + acc[i][j][e], prox_kind, prox_a);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int col = n0 + wn * WN + j * 32 + l32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                if (row < M && col < N) cout[(int64_t)row * ldc + col] = acc[i][j][e];
            }
        }
}

// ---------------------------------------------------------------------------------------
// Received factors -> the k-contiguous bf16 operands of the reconstruction:
//   UT[j][n] = bf16(alpha * U[n][j]),  VT[d][n] = V[n][d],  n < ldn (zero beyond N and for
//   the rows of dead workers).  64 x 64 tiles through LDS; blocks [0, n_ub) do U, the rest V.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_pack_kernel(
    const float* __restrict__ U, int64_t ldu, const bf16_t* __restrict__ V, int64_t ldv, bf16_t* __restrict__ UT,
    bf16_t* __restrict__ VT, int64_t ldn, int N, int J, int D, int B, float alpha, uint64_t live_mask,
    bool use_mask, int n_jblk, int n_dblk, bool vec_u, bool vec_v) {
    __shared__ __attribute__((aligned(16))) bf16_t tile[64][72];   // [column of the source][n], 144-byte rows
    const int tid = threadIdx.x;
    const int n_cblk = n_jblk + n_dblk;
    const int cb = blockIdx.x % n_cblk, kb = blockIdx.x / n_cblk;
    const bool is_u = cb < n_jblk;
    const int c0 = (is_u ? cb : cb - n_jblk) * 64, k0 = kb * 64;
    const int ncols = is_u ? J : D;
    // load 64 (n) x 64 (columns): thread -> 4 rows x 4 consecutive columns
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = k0 + (tid >> 4) + 16 * i, c = c0 + (tid & 15) * 4;
        bool live = n < N;
        if (use_mask && live) live = (live_mask >> (n / B)) & 1ull;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (live) {
            // one wide load where the host found the rows aligned for it and the four entries exist
            if (is_u) v = load4(U + (int64_t)n * ldu, c, ncols, vec_u) * alpha;
            else v = load4(V + (int64_t)n * ldv, c, ncols, vec_v);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[(tid & 15) * 4 + e][(tid >> 4) + 16 * i] = f32_to_bf16(v[e]);
    }
    __syncthreads();
    // store: thread -> 2 columns x 8 consecutive n (16 bytes)
    bf16_t* out = is_u ? UT : VT;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = (tid >> 3) + 32 * i, n8 = (tid & 7) * 8;
        if (c0 + c < ncols && k0 + n8 < ldn)
            *reinterpret_cast<u32x4*>(out + (int64_t)(c0 + c) * ldn + k0 + n8) =
                *reinterpret_cast<const u32x4*>(&tile[c][n8]);
    }
}

int64_t bf16_ldn(int64_t N) { return (N + 63) / 64 * 64; }

// Device scratch the bf16 reconstruction needs: (alpha u)^T [J][ldn] and v^T [D][ldn], bf16,
// each rounded up to 256 bytes.
size_t bf16_recon_workspace(int64_t J, int64_t D, int64_t N) {
    const size_t ldn = (size_t)bf16_ldn(N);
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    return up((size_t)J * ldn * 2) + up((size_t)D * ldn * 2);
}

int bf16_recon_grid(int64_t J, int64_t D) {
    return (int)(((J + kBfReconBM - 1) / kBfReconBM) * ((D + kBfReconBN - 1) / kBfReconBN));
}

hipError_t launch_reconstruct_bf16(const ReconArgs& a, void* ws, hipStream_t s) {
    const int64_t ldn = bf16_ldn(a.N);
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    bf16_t* UT = (bf16_t*)ws;
    bf16_t* VT = (bf16_t*)((char*)ws + up((size_t)a.J * ldn * 2));
    const int n_jblk = (a.J + 63) / 64, n_dblk = (a.D + 63) / 64, n_kblk = (int)(ldn / 64);
    // plain launch: an armed pair of timing events belongs to the contraction below
    hipLaunchKernelGGL(transpose_pack_kernel, dim3((n_jblk + n_dblk) * n_kblk), dim3(256), 0, s, a.u, a.ldu,
                       (const bf16_t*)a.v, a.ldv, UT, VT, ldn, a.N, a.J, a.D, a.B, a.alpha, a.live_mask, a.use_mask,
                       n_jblk, n_dblk, ((uintptr_t)a.u % 16) == 0 && (a.ldu % 4) == 0,
                       ((uintptr_t)a.v % 8) == 0 && (a.ldv % 4) == 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int NST = 3, BK = kBfReconBK, WPS = kBfReconWPS;
    constexpr int BM = kBfReconBM, BN = kBfReconBN;
    constexpr size_t lds_bytes = (size_t)NST * (BM + BN) * (BK / 8) * 16;
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        e = hipFuncSetAttribute((const void*)nt_bf16_kernel<false, kUpdateW, NST, BK, WPS, BM, BN, 2, 2>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_mb = (a.J + BM - 1) / BM, n_nb = (a.D + BN - 1) / BN;
    const int total = n_mb * n_nb;
    // one band of B-blocks per die if ~3 MB of a 4 MB L2 can hold it, else as many as fit
    int band = (n_nb + kXcds - 1) / kXcds;
    const int64_t fit = (3LL << 20) / ((int64_t)BN * ldn * 2);
    if (band > fit) band = (int)fit;
    if (band < 1) band = 1;
    SFB_LAUNCH((nt_bf16_kernel<false, kUpdateW, NST, BK, WPS, BM, BN, 2, 2>), dim3(total), dim3(256), lds_bytes, s, UT, ldn,
                       (const void*)VT, ldn, a.w, a.ldw, (int64_t)0, (bf16_t*)nullptr, (int64_t)0, a.J, a.D,
                       (int)ldn, (int)ldn, n_mb, n_nb, total, band, a.prox_kind, a.prox_a);
    return hipGetLastError();
}

bool forward_bf16_ok(const FwdArgs& a) {
    return a.bf16 && !a.diff && ((uintptr_t)a.a % 16) == 0 && (a.lda % 8) == 0 && ((uintptr_t)a.w % 16) == 0 &&
           (a.ldw % 4) == 0 && (a.v == nullptr || (((uintptr_t)a.v % 16) == 0 && (a.ldv % 8) == 0)) &&
           (a.D % kBfFwdBK) == 0 && a.D >= kBfFwdBK;
}

FwdPlan plan_forward_bf16(int64_t n_rows, int64_t J, int64_t D) {
    FwdPlan p;
    p.dma = true;
    p.bm = kBfFwdBM;
    p.bn = kBfFwdBN;
    const int64_t tiles = ((n_rows + kBfFwdBM - 1) / kBfFwdBM) * ((J + kBfFwdBN - 1) / kBfFwdBN);
    const int64_t chunks = D / kBfFwdBK > 0 ? D / kBfFwdBK : 1;
    // One workgroup per compute unit is resident (the stage ring fills the LDS) and pulls its rows of W at what
    // one compute unit's outstanding misses allow, about 25 GB/s; all of them together at no more than the
    // pass's share of HBM, about 4.5 TB/s; every slice costs one more write and read of the partial scores.
    // In microseconds (bytes / 1e6 per TB/s):
    const int64_t s_max = chunks / 8 > 0 ? (chunks / 8 < 32 ? chunks / 8 : 32) : 1;
    // (the sample blocks that share rows of W run on one die and fetch them into its L2 once)
    const double w_bytes = (double)((J + kBfFwdBN - 1) / kBfFwdBN * kBfFwdBN) * (double)D * 4.0;
    int64_t best = 1;
    double best_cost = 1e30;
    for (int64_t s = 1; s <= s_max; ++s) {
        const int64_t k = (chunks + s - 1) / s * kBfFwdBK;                    // columns per slice
        const double rounds = (double)((tiles * s + 255) / 256);
        const double per_cu = rounds * (double)kBfFwdBN * (double)k * 4.0 / 25e3;
        const double hbm = w_bytes / 4.5e6;
        const double partials = (double)s * (double)n_rows * (double)J * 8.0 / 4e6;
        const double cost = (per_cu > hbm ? per_cu : hbm) + partials;
        if (cost < best_cost * (1.0 - 1e-9)) { best_cost = cost; best = s; }
    }
    int64_t s = best;
    const int64_t per = (chunks + s - 1) / s;
    s = (chunks + per - 1) / per;
    p.split_k = (int)s;
    p.k_slice = (int)(per * kBfFwdBK);
    p.grid = (int)(tiles * s);
    return p;
}

hipError_t launch_forward_bf16(const FwdArgs& a, const FwdPlan& p, hipStream_t s) {
    constexpr int NST = 3, BK = kBfFwdBK, BM = kBfFwdBM, BN = kBfFwdBN;
    constexpr size_t lds_bytes = (size_t)NST * (BM * (BK / 8) + BN * (BK / 4)) * 16;
    static std::atomic<bool> raised{false};
    if (lds_bytes > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)nt_bf16_kernel<true, kStoreZ, NST, BK, 2, BM, BN, 4, 2>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int n_mb = (a.n_rows + BM - 1) / BM, n_nb = (a.J + BN - 1) / BN;
    const int total = n_mb * n_nb * p.split_k;
    SFB_LAUNCH((nt_bf16_kernel<true, kStoreZ, NST, BK, 2, BM, BN, 4, 2>), dim3(total), dim3(512), lds_bytes, s,
                       (const bf16_t*)a.a, a.lda, (const void*)a.w, a.ldw, a.zp, a.ldz, a.zstride, (bf16_t*)a.v,
                       a.ldv, a.n_rows, a.J, a.D, p.k_slice, n_mb, n_nb, total, 1, 0, 0.f);
    return hipGetLastError();
}

}  // namespace sfb
