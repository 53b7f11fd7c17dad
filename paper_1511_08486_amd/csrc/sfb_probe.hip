// Measurement aids, not part of the method: kernels that do nothing but the memory traffic or
// the matrix-core work of one of the path's kernels, in that kernel's own access shape.  Their
// durations are the floors the real kernels are compared with: what the part delivers for that
// shape when nothing else competes for the compute unit.
//   probe_w_stream   reads W once the way the bf16 score pass does: a workgroup walks a block of
//                    256 rows along its slice of D, 128 bytes of every row per step, several steps
//                    in flight; `dup` workgroups read the same block (the score pass has one per
//                    sample block, so dup = 2 at N = 512)
//   probe_w_rmw      W += c in the tile and lane mapping of the bf16 reconstruction's epilogue:
//                    256 x 128 tiles, 2 x 2 wavefronts, the MFMA accumulator layout (lane = column,
//                    16 rows per 32 x 32 block), four blocks of loads in flight
//   probe_fused_traffic  the memory operations of the one-pass update + score kernel and nothing else: per
//                    tile of 128 rows x 32 columns the same LDS-DMA copies from the same places (the packed
//                    v^T and feature tiles, the fp32 W tile) and the same 4-byte stores of the W tile, with
//                    the one dependency the real kernel has (a W entry is stored after it has arrived) and
//                    no barriers, no matrix work, no LDS reads beyond the W tile
//   probe_empty      an empty kernel: the cost of one dispatch
//   probe_mfma       a register-resident loop of matrix-core instructions (no memory traffic):
//                    the rate the matrix cores sustain at the clock the part holds under that load
#include "sfb_device.h"
#include "sfb_kernels.h"

namespace sfb {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(512) void probe_w_stream_kernel(const float* __restrict__ W, int64_t ldw, int J, int D,
                                                             int k_slice, int n_nb, int dup, float* __restrict__ sink) {
    // 512 lanes x 2 pieces of 32 bytes = 256 rows x 128 bytes per step
    const int bid = blockIdx.x / dup, nb = bid % n_nb, ks = bid / n_nb;
    const int tid = threadIdx.x;
    const int k0 = ks * k_slice, k1 = min(D, k0 + k_slice);
    const int steps = (k1 - k0) / 32;                       // whole 32-float steps only (host: D % 32 == 0)
    if (steps <= 0) return;
    const float* p[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int s = tid + i * 512, r = s / 4, c = s % 4;
        p[i] = W + (int64_t)min(nb * 256 + r, J - 1) * ldw + k0 + c * 8;
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    f32x4 r0[4], r1[4], r2[4];
    auto fetch = [&](f32x4* r, int st) {
        const int o = min(st, steps - 1) * 32;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            r[2 * i] = *reinterpret_cast<const f32x4*>(p[i] + o);
            r[2 * i + 1] = *reinterpret_cast<const f32x4*>(p[i] + o + 4);
        }
    };
    auto use = [&](const f32x4* r) { acc += r[0] + r[1] + r[2] + r[3]; };
    fetch(r0, 0); fetch(r1, 1); fetch(r2, 2);
    int st = 0;
    for (; st + 3 <= steps; st += 3) {
        use(r0); fetch(r0, st + 3); __builtin_amdgcn_sched_barrier(0);
        use(r1); fetch(r1, st + 4); __builtin_amdgcn_sched_barrier(0);
        use(r2); fetch(r2, st + 5); __builtin_amdgcn_sched_barrier(0);
    }
    use(r0); use(r1); use(r2);
    // never true for finite data; keeps the loads alive
    if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[blockIdx.x % 64] = acc[0];
}

__global__ __launch_bounds__(256, 2) void probe_w_rmw_kernel(float* __restrict__ W, int64_t ldw, int J, int D, int n_nb,
                                                             float add) {
    constexpr int BM = 256, BN = 128, WM = BM / 2, WN = BN / 2, MT = WM / 32, NT = WN / 32, EG = 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;
    const int mb = blockIdx.x / n_nb, nb = blockIdx.x % n_nb;
    const int m0 = mb * BM, n0 = nb * BN;
#pragma unroll
    for (int g = 0; g < MT * NT; g += EG) {
        float w[EG][16];
#pragma unroll
        for (int b = 0; b < EG; ++b) {
            const int i = (g + b) / NT, j = (g + b) % NT;
            const int cc = min(n0 + wn * WN + j * 32 + l32, D - 1);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                w[b][e] = W[(int64_t)min(row, J - 1) * ldw + cc];
            }
        }
#pragma unroll
        for (int b = 0; b < EG; ++b) {
            const int i = (g + b) / NT, j = (g + b) % NT;
            const int col = n0 + wn * WN + j * 32 + l32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                if (row < J && col < D) W[(int64_t)row * ldw + col] = w[b][e] + add;
            }
        }
    }
}

// 16 matrix-core instructions per iteration on four independent accumulators
template <bool BF16>
__global__ __launch_bounds__(512) void probe_mfma_kernel(float* __restrict__ sink, int iters, float a0, float b0) {
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
    const float a = a0 + threadIdx.x * 1e-6f, b = b0;
    probe_bf16x8 ab, bb;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ab[e] = (__bf16)a; bb[e] = (__bf16)b; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                if (BF16) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bb, acc[n], 0, 0, 0);
                else acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[n], 0, 0, 0);
            }
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[n][e];
    sink[(blockIdx.x * blockDim.x + threadIdx.x) % 64] = s;       // 64 floats of sink: last writer wins, value unused
}

// The one-pass kernel's traffic.  Workgroup = (band of 128 rows, column slice) exactly as in that kernel
// (same grid, same die-contiguous numbering).  Wavefront w owns rows 16 w .. 16 w + 15 of the band: it copies
// its 2 KB of every W tile into a ring of four private LDS slots three tiles ahead, waits for the oldest
// (its own copies retire in order), reads it back in the store layout (lane = column, two rows per
// instruction) and stores the same values: W keeps its bits, and no other wavefront touches those entries.
// The packed v^T and feature tiles are copied into one LDS area nobody reads (a share per wavefront, as in
// the real kernel).  Rows beyond J are read from row J - 1 and not stored.
template <int NQ>
__global__ __launch_bounds__(512) void probe_fused_traffic_kernel(float* __restrict__ W, int64_t ldw, const bf16_t* __restrict__ VTp,
                                                                  const bf16_t* __restrict__ AnP, int J, int D, int k_slice,
                                                                  int n_bands, int total) {
    constexpr int N = 128 * NQ, STAGE = 64 * N, LD = STAGE / 16 / 512, TILE_ELEMS = 32 * N, AHEAD = 3;
    constexpr int PER_TILE = 2 + 2 * LD;                 // copy instructions per wavefront and tile
    extern __shared__ __attribute__((aligned(16))) unsigned char pf_lds[];   // [STAGE] sink, then [8][4][2 KB] W ring
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int id = xcd_contiguous_id(blockIdx.x, total);
    const int band = id % n_bands, ks = id / n_bands;
    const int j0 = band * 128, k0 = ks * k_slice;
    const int n_tiles = (min(D, k0 + k_slice) - k0) / 32, t0 = k0 / 32;
    const uint32_t lds0 = (uint32_t)(uintptr_t)pf_lds;
    const int r0 = j0 + 16 * wave;
    const float* wsrc[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) wsrc[p] = W + (int64_t)min(r0 + 8 * p + (lane >> 3), J - 1) * ldw + k0 + 4 * (lane & 7);
    auto dma = [&](const void* g, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
    };
    auto issue_tile = [&](int i) {     // W first, then the two packed tiles: PER_TILE instructions
        const uint32_t slot = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)STAGE + (uint32_t)((wave * 4 + (i & 3)) * 2048));
#pragma unroll
        for (int p = 0; p < 2; ++p) dma(wsrc[p] + i * 32, slot + p * 1024);
        const unsigned char* vt = reinterpret_cast<const unsigned char*>(VTp + (int64_t)(t0 + i) * TILE_ELEMS) + tid * 16;
        const unsigned char* an = reinterpret_cast<const unsigned char*>(AnP + (int64_t)(t0 + i) * TILE_ELEMS) + tid * 16;
        const uint32_t sink = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(wave * 1024));
#pragma unroll
        for (int q = 0; q < LD; ++q) dma(vt + q * 8192, sink + q * 8192);
#pragma unroll
        for (int q = 0; q < LD; ++q) dma(an + q * 8192, sink + q * 8192);
    };
    for (int i = 0; i < AHEAD && i < n_tiles; ++i) issue_tile(i);
    for (int i = 0; i < n_tiles; ++i) {
        // tile i's two W copies are followed by its own packed copies and by AHEAD - 1 whole tiles; near the end
        // fewer tiles follow, so everything is waited for (stores also sit in the counter: they can only make a
        // wait longer)
        if (i + AHEAD <= n_tiles) wait_vmcnt<2 * LD + (AHEAD - 1) * PER_TILE>();
        else wait_vmcnt<0>();
        const unsigned char* slot = pf_lds + STAGE + (wave * 4 + (i & 3)) * 2048;
        float w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = *reinterpret_cast<const float*>(slot + (2 * e + half) * 128 + l32 * 4);
        float* wt = W + (int64_t)r0 * ldw + k0 + i * 32 + l32;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (r0 + 2 * e + half < J) wt[(int64_t)(2 * e + half) * ldw] = w[e];
        // the slot of tile i + AHEAD is the one tile i - 1 used: its reads have returned (their values were stored)
        if (i + AHEAD < n_tiles) issue_tile(i + AHEAD);
    }
}

// Nothing at all: what one dispatch costs on this stream (the floor of every launch-bound kernel).
__global__ void probe_empty_kernel(int) {}

hipError_t launch_probe_empty(hipStream_t s) {
    SFB_LAUNCH(probe_empty_kernel, dim3(256), dim3(256), 0, s, 0);
    return hipGetLastError();
}

hipError_t launch_probe_fused_traffic(float* W, int64_t ldw, int J, int D, int N, const FusedPlan& p, const void* ws_factors,
                                      const void* ws_next, hipStream_t s) {
    // same operand placement as launch_fused: (alpha u)^T [J][N], then the packed v^T; the packed features
    const bf16_t* VTp = (const bf16_t*)((const char*)ws_factors + ((size_t)J * N * 2 + 255) / 256 * 256);
    const bf16_t* AnP = (const bf16_t*)ws_next;
    const size_t lds = (size_t)64 * N + 8 * 4 * 2048;
    auto go = [&](auto kernel) -> hipError_t {
        static std::atomic<bool> raised{false};
        if (lds > 64 * 1024 && !raised) {
            hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            raised = true;
        }
        SFB_LAUNCH(kernel, dim3(p.grid), dim3(512), lds, s, W, ldw, VTp, AnP, J, D, p.k_slice, p.n_bands, p.grid);
        return hipGetLastError();
    };
    switch (N) {
        case 128: return go(probe_fused_traffic_kernel<1>);
        case 256: return go(probe_fused_traffic_kernel<2>);
        case 512: return go(probe_fused_traffic_kernel<4>);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_probe_w_stream(const float* W, int64_t ldw, int J, int D, int k_slice, int dup, float* sink,
                                 hipStream_t s) {
    const int n_nb = (J + 255) / 256, n_ks = (D + k_slice - 1) / k_slice;
    SFB_LAUNCH(probe_w_stream_kernel, dim3(n_nb * n_ks * dup), dim3(512), 0, s, W, ldw, J, D, k_slice, n_nb, dup, sink);
    return hipGetLastError();
}

hipError_t launch_probe_w_rmw(float* W, int64_t ldw, int J, int D, float add, hipStream_t s) {
    const int n_mb = (J + 255) / 256, n_nb = (D + 127) / 128;
    SFB_LAUNCH(probe_w_rmw_kernel, dim3(n_mb * n_nb), dim3(256), 0, s, W, ldw, J, D, n_nb, add);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(bool bf16, int waves_per_simd, int iters, float* sink, hipStream_t s) {
    const dim3 grid(256), block(256 * waves_per_simd);            // one workgroup per compute unit
    if (bf16) SFB_LAUNCH(probe_mfma_kernel<true>, grid, block, 0, s, sink, iters, 1.0f, 1e-3f);
    else SFB_LAUNCH(probe_mfma_kernel<false>, grid, block, 0, s, sink, iters, 1.0f, 1e-3f);
    return hipGetLastError();
}

}  // namespace sfb
