// Host-callable launchers of the SFB kernels.  Internal to the library: the public
// surface is include/sfb.h.  Every launcher validates nothing; the C ABI layer has
// already checked shapes and pointers.  Each returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

namespace sfb {

enum Model { kMLR = 0, kDML = 1, kL2SVM = 2 };

// Timing hook.  When a pair of events is armed on the calling thread, the next kernel launched
// through SFB_LAUNCH carries them: they take the start and stop timestamps of that dispatch
// itself, so what they measure is the kernel's duration with no stream packets in between.
struct LaunchEvents {
    hipEvent_t start, stop;
    bool armed;
};
LaunchEvents& launch_events();

#define SFB_LAUNCH(kernel, grid, block, lds, stream, ...)                                                  \
    do {                                                                                                    \
        ::sfb::LaunchEvents& sfb_le_ = ::sfb::launch_events();                                              \
        if (sfb_le_.armed) {                                                                                \
            sfb_le_.armed = false;                                                                          \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, sfb_le_.start, sfb_le_.stop, 0,         \
                                  __VA_ARGS__);                                                             \
        } else {                                                                                            \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                              \
        }                                                                                                   \
    } while (0)

struct FwdPlan {
    int bm, bn;      // output tile: samples x classes
    int split_k;     // slices of the D-long contraction
    int k_slice;     // columns of D per slice (multiple of the K chunk)
    int grid;        // workgroups
    bool dma;        // stage tiles by LDS-DMA where the shape allows
};

// Chooses tile and split for Z[n_rows][J] = A W^T with contraction length D.
FwdPlan plan_forward(int64_t n_rows, int64_t J, int64_t D);
// Recomputes k_slice / grid after bm, bn or split_k were set by hand (split_k is clamped
// so that no slice is empty).
void finish_forward_plan(FwdPlan* p, int64_t n_rows, int64_t J, int64_t D);

struct FwdArgs {
    const void* a;        // [n_rows][lda] features (fp32 or bf16)
    const void* a2;       // second point of the pair (DML) or nullptr
    int64_t lda;
    const float* w;       // [J][ldw]
    int64_t ldw;
    float* zp;            // [split_k][n_rows][ldz] partial scores
    int64_t ldz, zstride;
    void* v;              // [n_rows][ldv] out: a (or a - a2); nullptr = do not write
    int64_t ldv;
    int n_rows, J, D;
    bool bf16, diff;
};
hipError_t launch_forward(const FwdArgs& a, const FwdPlan& p, hipStream_t s);
// fp32 scores as six bf16 term products per product (sfb_forward_split.hip); 64 x 128 tiles
bool forward_split_ok(const FwdArgs& a);
hipError_t launch_forward_split(const FwdArgs& a, const FwdPlan& p, hipStream_t s);

// Dual side of SDCA (Section 2.1): with `dual` set, the MLR factor kernel turns its
// softmax residual r_i into delta u_i = frac * (u_i + r_i), stores that in U and
// u_i - delta u_i back into row sample[i] of `dual`.
struct SdcaDev {
    const int32_t* sample;   // [n_rows] row of `dual` (and entry of `conj`) of every batch row
    float* dual;             // [n_data][ldd]
    int64_t ldd;
    float* conj;             // [n_data] or nullptr: f_i*(-u_i) after the update
    float frac;
    bool vec;                // rows of `dual` are 16-byte aligned
};

struct FactorArgs {
    const float* zp;      // [split_k][n_rows][ldz]
    int64_t ldz, zstride;
    int split_k;
    const int32_t* y;     // [n_rows]
    float* u;             // [n_rows][ldu]
    int64_t ldu;
    float* loss;          // [n_rows] or nullptr
    int n_rows, J;
    Model model;
    SdcaDev sdca;         // dual == nullptr: plain factors
};
hipError_t launch_factor(const FactorArgs& a, hipStream_t s);

struct DensifyArgs {
    const int32_t* rowptr; const int32_t* col; const float* val;
    float* v; int64_t ldv;
    int n_rows, D;
    int64_t nnz;          // length of col / val
};
hipError_t launch_csr_densify(const DensifyArgs& a, hipStream_t s);

// Scores straight from the CSR features (no dense A): Z[n][j] = sum_e val[e] * W[j][col[e]].
// Usable when four W rows fit in LDS (csr_scores_ok); writes one slice (no split-K).
bool csr_scores_ok(int D);
// True when that pass is expected to beat the dense contraction on the densified rows (a fitted cost comparison).
bool csr_scores_wins(int64_t n_rows, int64_t J, int64_t D, int64_t nnz);
hipError_t launch_csr_scores(const DensifyArgs& a, const float* W, int64_t ldw, float* Z, int64_t ldz, int J,
                             hipStream_t s);

// dst[0 .. bytes) = src[0 .. bytes); both 16-byte aligned, bytes a multiple of 16.
hipError_t launch_stream_copy(const void* src, void* dst, int64_t bytes, hipStream_t s);

// Measurement aids (sfb_probe.hip): the bare memory traffic / matrix-core work of a kernel, in its access shape.
hipError_t launch_probe_w_stream(const float* W, int64_t ldw, int J, int D, int k_slice, int dup, float* sink,
                                 hipStream_t s);
hipError_t launch_probe_w_rmw(float* W, int64_t ldw, int J, int D, float add, hipStream_t s);
hipError_t launch_probe_mfma(bool bf16, int waves_per_simd, int iters, float* sink, hipStream_t s);
hipError_t launch_probe_empty(hipStream_t s);
struct FusedPlan;
// ws_factors / ws_next: where launch_fused keeps its packed operands (their contents do not matter here)
hipError_t launch_probe_fused_traffic(float* W, int64_t ldw, int J, int D, int N, const FusedPlan& p, const void* ws_factors,
                                      const void* ws_next, hipStream_t s);

// Proximal step on W (Section 2.1).  kind: 0 identity, 1 squared l2 (param = lam), 2 l1
// (param = lam), 3 projection of every column onto the l2 ball of radius param (needs
// prox_workspace(J, D) bytes of 16-byte aligned device memory).
struct ProxArgs {
    float* w; int64_t ldw;
    int J, D;
    int kind;
    float eta, param;
};
size_t prox_workspace(int64_t J, int64_t D);
hipError_t launch_prox(const ProxArgs& a, void* workspace, hipStream_t s);

struct ReconPlan {
    int variant;          // index into the tile table
    int bm, bn;           // W tile: rows (J) x columns (D)
    int grid;
    // the single-block tiles with few tiles and many factor pairs: slices of the pairs over workgroups
    // (sfb_reconstruct_small.hip); 1 = none.  Planned for n_rows pairs; calls with another count do not split.
    int n_split = 1, k_rows = 0, n_rows = 0;
};
ReconPlan plan_reconstruct(int64_t J, int64_t D, int64_t N);
ReconPlan plan_reconstruct_variant(int64_t J, int64_t D, int variant);
int num_reconstruct_variants();

struct ReconArgs {
    float* w; int64_t ldw;         // [J][ldw] read-modify-write
    const float* u; int64_t ldu;   // [N][ldu]
    const void* v; int64_t ldv;    // [N][ldv] fp32 or bf16
    int J, D, N;
    int B;                         // samples per worker (rows of one mask bit)
    float alpha;                   // -eta * scale
    uint64_t live_mask;            // bit p = worker p contributes
    bool use_mask, bf16;
    int prox_kind = 0;             // entrywise proximal operator applied to the updated entries
    float prox_a = 0.f;            //   before they are stored: see prox_entry (0 = none)
    // Set by launch_reconstruct_conformed only: u and v are the padded copies made by
    // conform_factors_kernel (16-byte aligned, J rounded up to 4 columns, D to Dp columns, N to whole
    // stages of zero rows, dead workers' rows zero), W is whatever the caller passed: any
    // alignment, any leading dimension, D columns.
    bool conformed = false;
    int Dp = 0;                    // columns of the padded v (a multiple of 128); 0: D itself
    float* partial = nullptr;      // room for the plan's n_split planes of J x tile_cols() partial sums (256-byte aligned), or none
    int tile_cols() const { return Dp > 0 ? Dp : D; }
};
hipError_t launch_reconstruct(const ReconArgs& a, const ReconPlan& p, hipStream_t s);
// Ragged or misaligned fp32 factors through the LDS-DMA kernels: the factors are first copied
// into `workspace` (conform_workspace(J, D, N) bytes, 256-byte aligned) with every row padded to
// what those kernels assume, then the plan's kernel runs on the copies and updates W entry by
// entry within its bounds.  `p` comes from plan_reconstruct_padded (variant < 0: the planner's choice
// for the padded shape); returns hipErrorNotSupported (nothing launched) when that plan's kernel has
// no such form (conformed_variant_ok(p.variant) is false: the register-staged variants).
size_t conform_workspace(int64_t J, int64_t D, int64_t N);
int64_t conform_cols(int64_t D);
int64_t conform_rows(int64_t N);
bool conformed_variant_ok(int variant);
ReconPlan plan_reconstruct_padded(int64_t J, int64_t D, int64_t N, int variant);
// True when launch_reconstruct(a, p) ends in one of the LDS-DMA kernels (nothing is launched).
bool reconstruct_takes_dma(const ReconArgs& a, const ReconPlan& p);
hipError_t launch_reconstruct_conformed(const ReconArgs& a, const ReconPlan& p, void* workspace, hipStream_t s);
// A dead worker (a.use_mask) in a call that would otherwise end in an LDS-DMA kernel: U is copied into
// `workspace` (masked_workspace(J, N) bytes, 256-byte aligned) with the dead workers' rows as zeros and the
// plan's kernel runs on the copy without a mask; hipErrorNotSupported (nothing launched) otherwise.
size_t masked_workspace(int64_t J, int64_t N);
hipError_t launch_reconstruct_masked(const ReconArgs& a, const ReconPlan& p, void* workspace, hipStream_t s);
// 64 x 64 tiles, one 32 x 32 block per wavefront (sfb_reconstruct_small.hip): for shapes whose
// block count leaves the larger tiles' busiest SIMD with clearly more work than the average
bool reconstruct_small_ok(const ReconArgs& a);
bool reconstruct_small_wins(int64_t J, int64_t D, int big_bm, int big_waves);
hipError_t launch_reconstruct_small(const ReconArgs& a, hipStream_t s);
// the same tiles with the factor pairs cut into n_split slices of k_rows over workgroups and a second kernel that adds
// the slices' sums in slice order (needs a.partial); reconstruct_small_split picks the count (1: do not split)
int reconstruct_small_split(int64_t J, int64_t D, int64_t N, int* k_rows);
size_t reconstruct_small_split_workspace(int n_split, int64_t J, int64_t D);
hipError_t launch_reconstruct_small_split(const ReconArgs& a, int n_split, int k_rows, hipStream_t s);
// (96..160) x 64 tiles whose eight wavefronts split the two column blocks, every stage's pairs and the stages
// (sfb_reconstruct_ksplit.hip): for shapes where even single blocks leave the busiest SIMD well above the average
bool reconstruct_ksplit_ok(const ReconArgs& a);
bool reconstruct_ksplit_wins(int64_t J, int64_t D, int64_t other_blocks);
int reconstruct_ksplit_rows(int64_t J);
hipError_t launch_reconstruct_ksplit(const ReconArgs& a, hipStream_t s);
// 128 x 128 tiles with eight wavefronts in two groups that take the stages in turn (sfb_reconstruct_pair.hip)
bool reconstruct_pair_ok(const ReconArgs& a);
hipError_t launch_reconstruct_pair(const ReconArgs& a, hipStream_t s);
// fp32 reconstruction as six bf16 term products per product (sfb_reconstruct_split.hip); 128 x 128 tiles
bool reconstruct_split_ok(const ReconArgs& a);
hipError_t launch_reconstruct_split(const ReconArgs& a, hipStream_t s);

// bf16-feature path on the bf16 matrix cores (sfb_bf16.hip)
bool forward_bf16_ok(const FwdArgs& a);                       // alignment / shape the DMA kernel needs
FwdPlan plan_forward_bf16(int64_t n_rows, int64_t J, int64_t D);
hipError_t launch_forward_bf16(const FwdArgs& a, const FwdPlan& p, hipStream_t s);
size_t bf16_recon_workspace(int64_t J, int64_t D, int64_t N);  // bytes of device scratch
int bf16_recon_grid(int64_t J, int64_t D);                     // workgroups of the W += C launch
// ws: bf16_recon_workspace bytes, 256-byte aligned.  Two launches: transpose/pack, then W += C.
hipError_t launch_reconstruct_bf16(const ReconArgs& a, void* ws, hipStream_t s);

// Update of iteration t fused with the scores of iteration t+1, one pass over W (sfb_fused.hip; bf16 contexts).
struct FusedPlan {
    int n_bands, slices, k_slice, grid;
};
struct FusedArgs {
    float* w; int64_t ldw;             // [J][ldw] read-modify-write
    const float* u; int64_t ldu;       // [N][ldu] factors of iteration t
    void* v; int64_t ldv;              // [N][ldv] bf16: v_t on entry, the next batch's features on return
    const void* a_next; int64_t lda;   // [N][lda] bf16 features of iteration t+1
    float* zp; int64_t ldz, zstride;   // [slices][N][ldz] partial scores of iteration t+1 out
    int J, D, N, B;
    float alpha;
    uint64_t live_mask;
    bool use_mask;
};
bool fused_shape_ok(int64_t J, int64_t D, int64_t N);
FusedPlan plan_fused(int64_t J, int64_t D, int64_t N);
size_t fused_extra_workspace(int64_t D, int64_t N);
bool fused_call_ok(const FusedArgs& a);   // alignment and size of this call's operands
hipError_t launch_fused(const FusedArgs& a, const FusedPlan& p, void* ws_factors, void* ws_next, hipStream_t s);

}  // namespace sfb
