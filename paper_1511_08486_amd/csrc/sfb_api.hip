// C ABI of the SFB library (see include/sfb.h): argument validation, launch plans,
// and the order of kernel launches for one bulk-synchronous SFB iteration.
// Host code only; every step of the computation runs in the kernels.
#include "../../include/sfb.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <new>
#include <vector>

#include "sfb_kernels.h"

using namespace sfb;

namespace {
constexpr int kFamilies = 6;  // 0 scores, 1 factor u, 2 reconstruct-apply, 3 sparse helpers, 4 proximal step, 5 one-pass update + next scores
struct EventPair { hipEvent_t a, b; };

// Scratch of the entry point that allocates nothing (sfb_step_noalloc): device memory that belongs
// to the library's code object, one copy per GPU the library is loaded on, held until the process
// ends.  It plays the role of the registered workspace (split-K partial scores, packed bf16
// factors), every byte of which a step writes before reading it, so nothing has to be cleared
// between calls.  In host code the array's NAME is only a handle for hipGetSymbolAddress; kernels
// are given the device address kept in static_scratch_ptr.
constexpr size_t kStaticScratchBytes = SFB_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> static_scratch_ptr[kMaxDevices];     // zero-initialised: not resolved yet

// Device address of `scratch` on the current device, resolved once per device.
hipError_t resolve_static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        static_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread resolves the same address
    }
    *out = p;
    return hipSuccess;
}
}  // namespace

namespace sfb {
LaunchEvents& launch_events() {
    static thread_local LaunchEvents le{nullptr, nullptr, false};
    return le;
}
}  // namespace sfb

struct sfb_ctx {
    sfb_model model;
    int64_t J, D;
    int32_t P, B;
    sfb_dtype dtype;
    hipStream_t stream;
    FwdPlan fwd_all, fwd_worker;   // scores of all N rows / of one worker's B rows
    FwdPlan fwd_bf16;              // all N rows on the bf16 matrix cores (bf16 contexts)
    FwdPlan fwd_split;             // all N rows, fp32 operands split into bf16 terms (64 x 128 tiles)
    bool split_scores;             // use it where the shape allows
    bool split_recon;              // reconstruction with split-bf16 products where the shape allows
    ReconPlan recon;
    ReconPlan recon_padded;        // the plan of the padded shape (ragged fp32 contexts: see padded_factors)
    bool padded_factors;           // fp32 and J, D or P*B not what the LDS-DMA reconstructions take as they are
    FusedPlan fused;               // update fused with the next scores (bf16 contexts whose shape it covers)
    bool fused_ok, use_fused;
    void* ws;
    size_t ws_bytes;
    int last_hip;
    bool timing;
    bool sparse_forward;           // L2SVM: scores from the CSR entries when W rows fit in LDS and that is the cheaper pass
    bool sparse_always;            //   ... whenever they fit (no cost comparison)
    std::vector<EventPair> used[kFamilies], spare;
};

namespace {

inline int64_t round_up4(int64_t x) { return (x + 3) / 4 * 4; }

// Bytes of split-K partial scores (the first region of the workspace), rounded to 256.
size_t scores_need(const sfb_ctx* c) {
    const int64_t ldz = round_up4(c->J);
    size_t need = (size_t)c->fwd_all.split_k * (size_t)c->P * c->B * ldz * sizeof(float);
    const size_t one = (size_t)c->fwd_worker.split_k * (size_t)c->B * ldz * sizeof(float);
    if (one > need) need = one;
    if (c->dtype == SFB_BF16) {
        const size_t bf = (size_t)c->fwd_bf16.split_k * (size_t)c->P * c->B * ldz * sizeof(float);
        if (bf > need) need = bf;
    }
    if (c->split_scores) {
        const size_t sp = (size_t)c->fwd_split.split_k * (size_t)c->P * c->B * ldz * sizeof(float);
        if (sp > need) need = sp;
    }
    if (c->fused_ok) {
        const size_t fu = (size_t)c->fused.slices * (size_t)c->P * c->B * ldz * sizeof(float);
        if (fu > need) need = fu;
    }
    return (need + 255) / 256 * 256;
}

// bf16 contexts append the transposed bf16 factors of the reconstruction.
size_t workspace_need(const sfb_ctx* c) {
    size_t need = scores_need(c);
    if (c->dtype == SFB_BF16) need += bf16_recon_workspace(c->J, c->D, (int64_t)c->P * c->B);
    if (c->fused_ok) need += fused_extra_workspace(c->D, (int64_t)c->P * c->B);   // staged next features, last
    // ragged fp32 shapes: padded copies of the factors, made and used inside one reconstruction, when the
    // partial scores (consumed by the factor kernel of the same call that wrote them) are dead: same bytes
    // few tiles and many factor pairs: planes of partial sums behind those copies (or behind the masked copy of U)
    if (c->padded_factors) {
        const size_t pad = conform_workspace(c->J, c->D, (int64_t)c->P * c->B) +
                           reconstruct_small_split_workspace(c->recon_padded.n_split, c->J, conform_cols(c->D));
        if (pad > need) need = pad;
    } else if (c->dtype == SFB_F32 && c->recon.n_split > 1) {
        const size_t sp = masked_workspace(c->J, (int64_t)c->P * c->B) +
                          reconstruct_small_split_workspace(c->recon.n_split, c->J, c->D);
        if (sp > need) need = sp;
    }
    // the column projection of the proximal step reuses the front of the buffer between steps
    const size_t prox = prox_workspace(c->J, c->D);
    return need > prox ? need : prox;
}

sfb_status hip_fail(sfb_ctx* c, hipError_t e) {
    c->last_hip = (int)e;
    return SFB_EHIP;
}

// Arms a pair of events for the next kernel launch when timing is on (see SFB_LAUNCH).
struct Timed {
    sfb_ctx* c;
    int fam;
    EventPair ev;
    bool on;
    Timed(sfb_ctx* ctx, int family) : c(ctx), fam(family), on(ctx->timing) {
        if (!on) return;
        if (!c->spare.empty()) {
            ev = c->spare.back();
            c->spare.pop_back();
        } else {
            hipError_t e = hipEventCreate(&ev.a);
            if (e == hipSuccess) {
                e = hipEventCreate(&ev.b);
                if (e != hipSuccess) (void)hipEventDestroy(ev.a);
            }
            if (e != hipSuccess) {          // this launch goes untimed; the caller can see why
                c->last_hip = (int)e;
                on = false;
                return;
            }
        }
        LaunchEvents& le = launch_events();
        le.start = ev.a;
        le.stop = ev.b;
        le.armed = true;
    }
    ~Timed() {
        if (!on) return;
        LaunchEvents& le = launch_events();
        if (le.armed) {             // nothing was launched: the events hold no timestamps
            le.armed = false;
            c->spare.push_back(ev);
        } else {
            c->used[fam].push_back(ev);
        }
    }
};

sfb_status check_common(const sfb_ctx* c, const float* W, int64_t ldw, const float* U, int64_t ldu,
                        const void* V, int64_t ldv) {
    if (!c || !W || !U || !V) return SFB_EINVAL;
    if (ldw < c->D || ldu < c->J || ldv < c->D) return SFB_ESHAPE;
    return SFB_OK;
}

sfb_status check_batch(const sfb_ctx* c, const sfb_batch* b, const int32_t* y) {
    if (!b || !y) return SFB_EINVAL;
    if (c->model == SFB_L2SVM) {
        if (!b->csr_rowptr || (b->nnz > 0 && (!b->csr_col || !b->csr_val))) return SFB_EINVAL;
        if (b->nnz < 0) return SFB_ESHAPE;
    } else {
        if (!b->a) return SFB_EINVAL;
        if (c->model == SFB_DML && !b->a2) return SFB_EINVAL;
        if (b->lda < c->D) return SFB_ESHAPE;
    }
    return SFB_OK;
}

// Factor u (and the loss) of `n_rows` samples from the `split_k` partial scores at the front of the workspace.
sfb_status factor_rows(sfb_ctx* c, int split_k, int64_t zstride, const int32_t* y, int64_t row0, int n_rows, float* U,
                       int64_t ldu, float* loss, const sfb_sdca* sdca) {
    FactorArgs g{};
    g.zp = (const float*)c->ws; g.ldz = round_up4(c->J); g.zstride = zstride; g.split_k = split_k;
    g.y = y; g.u = U + row0 * ldu; g.ldu = ldu; g.loss = loss ? loss + row0 : nullptr;
    g.n_rows = n_rows; g.J = (int)c->J; g.model = (Model)c->model;
    if (sdca) {
        const bool vec = ((uintptr_t)sdca->dual % 16) == 0 && (sdca->ld_dual % 4) == 0;
        g.sdca = SdcaDev{sdca->sample, sdca->dual, sdca->ld_dual, sdca->conj, sdca->s, vec};
    }
    Timed t(c, 1);
    hipError_t e = launch_factor(g, c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

// Factors of `n_rows` samples whose outputs start at row `row0` of U, V, loss.
sfb_status factors_rows(sfb_ctx* c, const FwdPlan& plan, const float* W, int64_t ldw, const sfb_batch* b,
                        const int32_t* y, int64_t row0, int n_rows, float* U, int64_t ldu, void* V,
                        int64_t ldv, float* loss, const sfb_sdca* sdca = nullptr) {
    if (c->ws == nullptr || c->ws_bytes < workspace_need(c)) return SFB_EWORKSPACE;
    const bool bf16 = c->dtype == SFB_BF16;
    const size_t vsz = bf16 ? 2 : 4;
    void* v_rows = (char*)V + (size_t)row0 * ldv * vsz;
    const int64_t ldz = round_up4(c->J);

    FwdArgs f{};
    f.w = W; f.ldw = ldw;
    f.zp = (float*)c->ws; f.ldz = ldz; f.zstride = (int64_t)n_rows * ldz;
    f.n_rows = n_rows; f.J = (int)c->J; f.D = (int)c->D;
    f.bf16 = bf16;
    bool sparse_scores = false;
    if (c->model == SFB_L2SVM) {
        // v_i first: the dense rows are what the reconstruction multiplies
        DensifyArgs d{b->csr_rowptr, b->csr_col, b->csr_val, (float*)v_rows, ldv, n_rows, (int)c->D, b->nnz};
        {
            Timed t(c, 3);
            hipError_t e = launch_csr_densify(d, c->stream);
            if (e != hipSuccess) return hip_fail(c, e);
        }
        if (c->sparse_forward && csr_scores_ok((int)c->D) && b->nnz <= (1LL << 30) - 1024 &&
            (c->sparse_always || csr_scores_wins(n_rows, c->J, c->D, b->nnz))) {
            // scores from the stored entries only: 2*nnz*J flops instead of 2*N*J*D
            Timed t(c, 0);
            hipError_t e = launch_csr_scores(d, W, ldw, (float*)c->ws, ldz, (int)c->J, c->stream);
            if (e != hipSuccess) return hip_fail(c, e);
            sparse_scores = true;
        } else {
            // fall back to the dense contraction on the densified rows
            f.a = v_rows; f.a2 = nullptr; f.lda = ldv; f.v = nullptr; f.ldv = 0; f.diff = false;
        }
    } else {
        f.a = b->a; f.a2 = (c->model == SFB_DML) ? b->a2 : nullptr; f.lda = b->lda;
        f.v = v_rows; f.ldv = ldv; f.diff = (c->model == SFB_DML);
    }
    // bf16 features, full batch, aligned: the bf16 matrix-core kernel with its own plan
    const bool on_bf16_cores = bf16 && n_rows == c->P * c->B && n_rows >= 128 && forward_bf16_ok(f);
    // fp32 features, full batch, aligned, and the caller opted in: split-bf16 products
    const bool on_split = !sparse_scores && !bf16 && c->split_scores && n_rows == c->P * c->B && forward_split_ok(f);
    const FwdPlan& used = on_bf16_cores ? c->fwd_bf16 : on_split ? c->fwd_split : plan;
    if (!sparse_scores) {
        Timed t(c, 0);
        hipError_t e = on_bf16_cores ? launch_forward_bf16(f, used, c->stream)
                       : on_split    ? launch_forward_split(f, used, c->stream)
                                     : launch_forward(f, used, c->stream);
        if (e != hipSuccess) return hip_fail(c, e);
    }
    return factor_rows(c, sparse_scores ? 1 : used.split_k, f.zstride, y, row0, n_rows, U, ldu, loss, sdca);
}

sfb_status check_sdca(const sfb_ctx* c, const sfb_sdca* d) {
    if (!d || !d->dual || !d->sample || d->n_data < 1) return SFB_EINVAL;
    if (!std::isfinite(d->lam) || !(d->lam > 0.f) || !std::isfinite(d->s) || !(d->s > 0.f) || d->s > 1.f)
        return SFB_EINVAL;
    if (d->ld_dual < c->J) return SFB_ESHAPE;
    if (c->model != SFB_MLR) return SFB_EUNSUPPORTED;
    return SFB_OK;
}

sfb_status check_recon(const sfb_ctx* c, float eta, float scale, const uint8_t* active) {
    if (!std::isfinite(eta) || !std::isfinite(scale)) return SFB_EINVAL;
    if (active && c->P > 64) return SFB_EUNSUPPORTED;
    return SFB_OK;
}

// n_rows: factor pairs to contract over (0 = all P*B; a single worker's B otherwise, no mask)
sfb_status recon_launch(sfb_ctx* c, float* W, int64_t ldw, const float* U, int64_t ldu, const void* V,
                        int64_t ldv, float eta, float scale, const uint8_t* active, int n_rows = 0,
                        int prox_kind = 0, float prox_a = 0.f) {
    ReconArgs r{};
    r.w = W; r.ldw = ldw; r.u = U; r.ldu = ldu; r.v = V; r.ldv = ldv;
    r.J = (int)c->J; r.D = (int)c->D; r.N = n_rows > 0 ? n_rows : c->P * c->B; r.B = c->B;
    r.alpha = -eta * scale;
    r.bf16 = c->dtype == SFB_BF16;
    r.use_mask = false;
    r.live_mask = ~0ull;
    r.prox_kind = prox_kind; r.prox_a = prox_a;
    if (active) {
        uint64_t m = 0;
        bool all = true;
        for (int p = 0; p < c->P; ++p) {
            if (active[p]) m |= (1ull << p); else all = false;
        }
        r.live_mask = m;
        r.use_mask = !all;
    }
    Timed t(c, 2);
    hipError_t e;
    if (r.bf16) {
        if (c->ws == nullptr || c->ws_bytes < workspace_need(c)) return SFB_EWORKSPACE;
        e = launch_reconstruct_bf16(r, (char*)c->ws + scores_need(c), c->stream);
    } else if (c->split_recon && reconstruct_split_ok(r)) {
        e = launch_reconstruct_split(r, c->stream);
    } else {
        // calls that would end in the register-staged kernel first try a copy of the factors that the LDS-DMA
        // kernels accept: padded ones for ragged shapes, U with a dead worker's rows zeroed for a masked call
        // (N x ceil4(J) floats: never more than the partial scores, whose bytes it takes)
        e = hipErrorNotSupported;
        const bool have_ws = c->ws != nullptr && c->ws_bytes >= workspace_need(c);
        const int64_t n_all = (int64_t)c->P * c->B;
        if (have_ws && !reconstruct_takes_dma(r, c->recon)) {
            if (c->padded_factors && conformed_variant_ok(c->recon_padded.variant)) {
                if (c->recon_padded.n_split > 1) r.partial = (float*)((char*)c->ws + conform_workspace(c->J, c->D, n_all));
                e = launch_reconstruct_conformed(r, c->recon_padded, c->ws, c->stream);
                r.partial = nullptr;
            } else if (r.use_mask && masked_workspace(c->J, r.N) <= scores_need(c)) {
                if (!c->padded_factors && c->recon.n_split > 1) r.partial = (float*)((char*)c->ws + masked_workspace(c->J, n_all));
                e = launch_reconstruct_masked(r, c->recon, c->ws, c->stream);
                r.partial = nullptr;
            }
        }
        if (e == hipErrorNotSupported) {
            if (have_ws && !c->padded_factors && c->recon.n_split > 1)
                r.partial = (float*)((char*)c->ws + masked_workspace(c->J, n_all));
            e = launch_reconstruct(r, c->recon, c->stream);
        }
    }
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

}  // namespace

extern "C" {

sfb_status sfb_create(sfb_ctx** out, sfb_model m, int64_t J, int64_t D, int32_t P, int32_t B,
                      sfb_dtype input_dtype, void* hip_stream) {
    if (!out) return SFB_EINVAL;
    *out = nullptr;
    if (J <= 0 || D <= 0 || P <= 0 || B <= 0) return SFB_EINVAL;
    if (m != SFB_MLR && m != SFB_DML && m != SFB_L2SVM) return SFB_EINVAL;
    if (input_dtype != SFB_F32 && input_dtype != SFB_BF16) return SFB_EDTYPE;
    if (input_dtype == SFB_BF16 && m != SFB_MLR) return SFB_EUNSUPPORTED;
    // kernels index rows and columns with 32-bit ints
    if (J > (1 << 30) || D > (1 << 30) || (int64_t)P * B > (1 << 30)) return SFB_EUNSUPPORTED;
    sfb_ctx* c = new (std::nothrow) sfb_ctx();
    if (!c) return SFB_EINVAL;
    c->model = m; c->J = J; c->D = D; c->P = P; c->B = B; c->dtype = input_dtype;
    c->stream = (hipStream_t)hip_stream;
    c->fwd_all = plan_forward((int64_t)P * B, J, D);
    c->fwd_worker = plan_forward(B, J, D);
    c->fwd_bf16 = plan_forward_bf16((int64_t)P * B, J, D);
    {
        // 64 x 128 tiles; as many slices of D as bring the grid to about two workgroups per compute unit
        FwdPlan sp{};
        sp.bm = 64; sp.bn = 128; sp.dma = false;
        const int64_t tiles = (((int64_t)P * B + 63) / 64) * ((J + 127) / 128);
        // (two workgroups fit a compute unit and overlap each other's splitting and multiplying)
        int64_t s = (512 + tiles / 2) / tiles;
        if (s < 1) s = 1;
        if (s > 8) s = 8;
        sp.split_k = (int)s;
        finish_forward_plan(&sp, (int64_t)P * B, J, D);
        c->fwd_split = sp;
    }
    c->split_scores = false;
    c->split_recon = false;
    c->recon = plan_reconstruct(J, D, (int64_t)P * B);
    {
        const int64_t N = (int64_t)P * B;
        c->padded_factors = input_dtype == SFB_F32 &&
                            !((J % 4) == 0 && J >= 4 && (D % 128) == 0 && (N % 32) == 0 && N >= 32);
        c->recon_padded = plan_reconstruct_padded(J, D, N, -1);
    }
    c->fused_ok = input_dtype == SFB_BF16 && m == SFB_MLR && fused_shape_ok(J, D, (int64_t)P * B);
    c->use_fused = true;
    c->fused = c->fused_ok ? plan_fused(J, D, (int64_t)P * B) : FusedPlan{};
    c->ws = nullptr; c->ws_bytes = 0; c->last_hip = 0; c->timing = false; c->sparse_forward = true; c->sparse_always = false;
    // Set-up for sfb_step_noalloc on the device that is current now: resolve the address of the
    // library's scratch array, so that the entry point itself only reads it.  On a machine without a
    // GPU this fails; the context is still good for everything that can be checked on the host, and
    // the entry point tries again (and reports SFB_EHIP if it still cannot).
    {
        void* unused = nullptr;
        if (resolve_static_scratch(&unused) != hipSuccess) (void)hipGetLastError();
    }
    *out = c;
    return SFB_OK;
}

void sfb_destroy(sfb_ctx* c) {
    if (!c) return;
    for (int f = 0; f < kFamilies; ++f)
        for (auto& e : c->used[f]) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (auto& e : c->spare) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    delete c;
}

sfb_status sfb_workspace_bytes(const sfb_ctx* c, size_t* bytes) {
    if (!c || !bytes) return SFB_EINVAL;
    *bytes = workspace_need(c);
    return SFB_OK;
}

sfb_status sfb_set_workspace(sfb_ctx* c, void* dev, size_t bytes) {
    if (!c || !dev) return SFB_EINVAL;
    if (((uintptr_t)dev % 256) != 0) return SFB_EINVAL;
    if (bytes < workspace_need(c)) return SFB_EWORKSPACE;
    c->ws = dev; c->ws_bytes = bytes;
    return SFB_OK;
}

sfb_status sfb_compute_factors(sfb_ctx* c, const float* W, int64_t ldw, const sfb_batch* batch,
                               const int32_t* y, float* U, int64_t ldu, void* V, int64_t ldv, float* loss) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch, y);
    if (s != SFB_OK) return s;
    return factors_rows(c, c->fwd_all, W, ldw, batch, y, 0, c->P * c->B, U, ldu, V, ldv, loss);
}

sfb_status sfb_compute_factors_worker(sfb_ctx* c, const float* W, int64_t ldw, const sfb_batch* batch_p,
                                      const int32_t* y_p, int32_t p, float* U, int64_t ldu, void* V,
                                      int64_t ldv, float* loss) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch_p, y_p);
    if (s != SFB_OK) return s;
    if (p < 0 || p >= c->P) return SFB_ESHAPE;
    return factors_rows(c, c->fwd_worker, W, ldw, batch_p, y_p, (int64_t)p * c->B, c->B, U, ldu, V, ldv, loss);
}

sfb_status sfb_reconstruct_apply(sfb_ctx* c, float* W, int64_t ldw, const float* U, int64_t ldu,
                                 const void* V, int64_t ldv, float eta, float scale, const uint8_t* active) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    return recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active);
}

sfb_status sfb_reconstruct_apply_worker(sfb_ctx* c, float* W, int64_t ldw, const float* U, int64_t ldu,
                                        const void* V, int64_t ldv, int32_t p, float eta, float scale) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_recon(c, eta, scale, nullptr);
    if (s != SFB_OK) return s;
    if (p < 0 || p >= c->P) return SFB_ESHAPE;
    const size_t vsz = c->dtype == SFB_BF16 ? 2 : 4;
    return recon_launch(c, W, ldw, U + (int64_t)p * c->B * ldu, ldu,
                        (const char*)V + (size_t)p * c->B * (size_t)ldv * vsz, ldv, eta, scale, nullptr, c->B);
}

sfb_status sfb_step(sfb_ctx* c, float* W, int64_t ldw, const sfb_batch* batch, const int32_t* y, float* U,
                    int64_t ldu, void* V, int64_t ldv, float* loss, float eta, const uint8_t* active) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch, y);
    if (s != SFB_OK) return s;
    float scale;                              // mini-batch mean inside a worker (Section 3)
    (void)sfb_default_scale(c, &scale);
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    s = factors_rows(c, c->fwd_all, W, ldw, batch, y, 0, c->P * c->B, U, ldu, V, ldv, loss);
    if (s != SFB_OK) return s;
    return recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active);
}

sfb_status sfb_step_pipelined(sfb_ctx* c, float* W, int64_t ldw, float* U, int64_t ldu, void* V, int64_t ldv,
                              const sfb_batch* next_batch, const int32_t* next_y, float* loss, float eta,
                              const uint8_t* active) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, next_batch, next_y);
    if (s != SFB_OK) return s;
    float scale;
    (void)sfb_default_scale(c, &scale);
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    if (c->ws == nullptr || c->ws_bytes < workspace_need(c)) return SFB_EWORKSPACE;
    const int N = c->P * c->B;
    if (c->fused_ok && c->use_fused) {
        FusedArgs f{};
        f.w = W; f.ldw = ldw; f.u = U; f.ldu = ldu; f.v = V; f.ldv = ldv;
        f.a_next = next_batch->a; f.lda = next_batch->lda;
        f.zp = (float*)c->ws; f.ldz = round_up4(c->J); f.zstride = (int64_t)N * f.ldz;
        f.J = (int)c->J; f.D = (int)c->D; f.N = N; f.B = c->B;
        f.alpha = -eta * scale;
        f.live_mask = ~0ull; f.use_mask = false;
        if (active) {
            uint64_t m = 0;
            bool all = true;
            for (int p = 0; p < c->P; ++p) {
                if (active[p]) m |= (1ull << p); else all = false;
            }
            f.live_mask = m; f.use_mask = !all;
        }
        if (fused_call_ok(f)) {
            char* ws_factors = (char*)c->ws + scores_need(c);
            char* ws_next = ws_factors + bf16_recon_workspace(c->J, c->D, N);
            {
                Timed t(c, 5);
                hipError_t e = launch_fused(f, c->fused, ws_factors, ws_next, c->stream);
                if (e != hipSuccess) return hip_fail(c, e);
            }
            return factor_rows(c, c->fused.slices, f.zstride, next_y, 0, N, U, ldu, loss, nullptr);
        }
    }
    // the same two steps as separate passes over W
    s = recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active);
    if (s != SFB_OK) return s;
    return factors_rows(c, c->fwd_all, W, ldw, next_batch, next_y, 0, N, U, ldu, V, ldv, loss);
}

sfb_status sfb_pipeline_info(const sfb_ctx* c, int32_t* fused, int32_t* grid, int32_t* slices) {
    if (!c) return SFB_EINVAL;
    const bool on = c->fused_ok && c->use_fused;
    if (fused) *fused = on ? 1 : 0;
    if (grid) *grid = on ? c->fused.grid : 0;
    if (slices) *slices = on ? c->fused.slices : 0;
    return SFB_OK;
}

sfb_status sfb_step_noalloc(sfb_ctx* c, float* W, int64_t ldw, const sfb_batch* batch, const int32_t* y, float* U,
                            int64_t ldu, void* V, int64_t ldv, float* loss, float eta, const uint8_t* active) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch, y);
    if (s != SFB_OK) return s;
    float scale;
    (void)sfb_default_scale(c, &scale);
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    if (workspace_need(c) > kStaticScratchBytes) return SFB_ESCRATCH;
    void* ptr = nullptr;
    hipError_t e = resolve_static_scratch(&ptr);     // a table read after sfb_create on this device
    if (e != hipSuccess) return hip_fail(c, e);
    // the kernels take the scratch address where they take the registered workspace in sfb_step
    void* const ws = c->ws;
    const size_t ws_bytes = c->ws_bytes;
    c->ws = ptr; c->ws_bytes = kStaticScratchBytes;
    s = factors_rows(c, c->fwd_all, W, ldw, batch, y, 0, c->P * c->B, U, ldu, V, ldv, loss);
    if (s == SFB_OK) s = recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active);
    c->ws = ws; c->ws_bytes = ws_bytes;
    return s;
}

sfb_status sfb_sdca_compute_factors(sfb_ctx* c, const float* W, int64_t ldw, const sfb_batch* batch,
                                    const int32_t* y, const sfb_sdca* sdca, float* U, int64_t ldu, void* V,
                                    int64_t ldv, float* loss) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch, y);
    if (s != SFB_OK) return s;
    s = check_sdca(c, sdca);
    if (s != SFB_OK) return s;
    return factors_rows(c, c->fwd_all, W, ldw, batch, y, 0, c->P * c->B, U, ldu, V, ldv, loss, sdca);
}

sfb_status sfb_sdca_step(sfb_ctx* c, float* W, int64_t ldw, const sfb_batch* batch, const int32_t* y,
                         const sfb_sdca* sdca, float* U, int64_t ldu, void* V, int64_t ldv, float* loss) {
    if (!c || !sdca) return SFB_EINVAL;
    // Z <- Z - (1/n_data) sum delta u a^T and W = Z / lam, folded into one scale (Section 2.1)
    const float scale = (float)(1.0 / ((double)sdca->lam * (double)sdca->n_data));
    if (!std::isfinite(scale)) return SFB_EINVAL;
    sfb_status s = sfb_sdca_compute_factors(c, W, ldw, batch, y, sdca, U, ldu, V, ldv, loss);
    if (s != SFB_OK) return s;
    return recon_launch(c, W, ldw, U, ldu, V, ldv, 1.0f, scale, nullptr);
}

// kind and parameters of a proximal step; the workspace only matters for the column projection
static sfb_status check_prox(const sfb_ctx* c, sfb_prox_kind kind, float eta, float param, bool need_workspace) {
    if ((int)kind < SFB_PROX_NONE || (int)kind > SFB_PROX_COLUMN_BALL) return SFB_EINVAL;
    if (!std::isfinite(eta) || !std::isfinite(param) || eta < 0.f || param < 0.f) return SFB_EINVAL;
    if (kind == SFB_PROX_COLUMN_BALL && !(param > 0.f)) return SFB_EINVAL;
    if (need_workspace && kind == SFB_PROX_COLUMN_BALL && (c->ws == nullptr || c->ws_bytes < workspace_need(c)))
        return SFB_EWORKSPACE;
    return SFB_OK;
}

sfb_status sfb_prox(sfb_ctx* c, float* W, int64_t ldw, sfb_prox_kind kind, float eta, float param) {
    if (!c || !W) return SFB_EINVAL;
    sfb_status s = check_prox(c, kind, eta, param, false);
    if (s != SFB_OK) return s;
    if (ldw < c->D) return SFB_ESHAPE;
    if (kind == SFB_PROX_NONE) return SFB_OK;
    s = check_prox(c, kind, eta, param, true);
    if (s != SFB_OK) return s;
    ProxArgs a{W, ldw, (int)c->J, (int)c->D, (int)kind, eta, param};
    Timed t(c, 4);
    hipError_t e = launch_prox(a, c->ws, c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

// The proximal step after an update: the entrywise kinds ride in the reconstruction's epilogue
// (no extra pass over W), the column projection runs as its own kernels afterwards.
static sfb_status recon_then_prox(sfb_ctx* c, float* W, int64_t ldw, const float* U, int64_t ldu, const void* V,
                                  int64_t ldv, float eta, float scale, const uint8_t* active, sfb_prox_kind kind,
                                  float param) {
    if (kind == SFB_PROX_L2SQ)
        return recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active, 0, 1, 1.0f / (1.0f + eta * param));
    if (kind == SFB_PROX_L1) return recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active, 0, 2, eta * param);
    sfb_status s = recon_launch(c, W, ldw, U, ldu, V, ldv, eta, scale, active);
    if (s != SFB_OK || kind == SFB_PROX_NONE) return s;
    return sfb_prox(c, W, ldw, kind, eta, param);
}

sfb_status sfb_reconstruct_apply_prox(sfb_ctx* c, float* W, int64_t ldw, const float* U, int64_t ldu, const void* V,
                                      int64_t ldv, float eta, float scale, const uint8_t* active,
                                      sfb_prox_kind kind, float param) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    s = check_prox(c, kind, eta, param, true);
    if (s != SFB_OK) return s;
    return recon_then_prox(c, W, ldw, U, ldu, V, ldv, eta, scale, active, kind, param);
}

sfb_status sfb_step_prox(sfb_ctx* c, float* W, int64_t ldw, const sfb_batch* batch, const int32_t* y, float* U,
                         int64_t ldu, void* V, int64_t ldv, float* loss, float eta, const uint8_t* active,
                         sfb_prox_kind kind, float param) {
    sfb_status s = check_common(c, W, ldw, U, ldu, V, ldv);
    if (s != SFB_OK) return s;
    s = check_batch(c, batch, y);
    if (s != SFB_OK) return s;
    float scale;
    (void)sfb_default_scale(c, &scale);
    s = check_recon(c, eta, scale, active);
    if (s != SFB_OK) return s;
    s = check_prox(c, kind, eta, param, true);
    if (s != SFB_OK) return s;
    s = factors_rows(c, c->fwd_all, W, ldw, batch, y, 0, c->P * c->B, U, ldu, V, ldv, loss);
    if (s != SFB_OK) return s;
    return recon_then_prox(c, W, ldw, U, ldu, V, ldv, eta, scale, active, kind, param);
}

sfb_status sfb_shape(const sfb_ctx* c, int64_t* J, int64_t* D, int32_t* P, int32_t* B, int32_t* input_dtype) {
    if (!c) return SFB_EINVAL;
    if (J) *J = c->J;
    if (D) *D = c->D;
    if (P) *P = c->P;
    if (B) *B = c->B;
    if (input_dtype) *input_dtype = (int32_t)c->dtype;
    return SFB_OK;
}

sfb_status sfb_default_scale(const sfb_ctx* c, float* scale) {
    if (!c || !scale) return SFB_EINVAL;
    *scale = 1.0f / (float)c->B;
    return SFB_OK;
}

sfb_status sfb_sync(sfb_ctx* c) {
    if (!c) return SFB_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

const char* sfb_strerror(sfb_status s) {
    switch (s) {
        case SFB_OK: return "ok";
        case SFB_EINVAL: return "invalid argument (null pointer, non-positive size, non-finite eta or scale)";
        case SFB_ESHAPE: return "shape mismatch (leading dimension shorter than the row, negative nnz, worker index out of range)";
        case SFB_EDTYPE: return "unknown dtype";
        case SFB_EWORKSPACE: return "workspace missing or too small";
        case SFB_EUNSUPPORTED: return "unsupported model/dtype combination or size";
        case SFB_EHIP: return "HIP runtime error";
        case SFB_ESCRATCH: return "the context needs more scratch than the library's fixed array holds (use sfb_step with a registered workspace)";
    }
    return "unknown status";
}

int sfb_last_hip_error(const sfb_ctx* c) { return c ? c->last_hip : 0; }

sfb_status sfb_plan_info(const sfb_ctx* c, int32_t* fwd_split_k, int32_t* fwd_grid, int32_t* recon_grid) {
    if (!c) return SFB_EINVAL;
    const FwdPlan& f = c->dtype == SFB_BF16 ? c->fwd_bf16 : c->fwd_all;
    if (fwd_split_k) *fwd_split_k = f.split_k;
    if (fwd_grid) *fwd_grid = f.grid;
    if (recon_grid) {
        // ragged fp32 shapes run the padded shape's plan once a workspace is registered (recon_launch)
        const bool padded = c->padded_factors && conformed_variant_ok(c->recon_padded.variant) && c->ws != nullptr &&
                            c->ws_bytes >= workspace_need(c);
        *recon_grid = c->dtype == SFB_BF16 ? bf16_recon_grid(c->J, c->D) : padded ? c->recon_padded.grid : c->recon.grid;
    }
    return SFB_OK;
}

sfb_status sfb_set_plan(sfb_ctx* c, int32_t fwd_bm, int32_t fwd_bn, int32_t fwd_split_k, int32_t recon_variant,
                        int32_t fwd_dma) {
    if (!c) return SFB_EINVAL;
    if ((fwd_bm > 0 && fwd_bm != 64 && fwd_bm != 128) || (fwd_bn > 0 && fwd_bn != 64 && fwd_bn != 128))
        return SFB_EINVAL;
    if (recon_variant >= num_reconstruct_variants() || fwd_split_k > 64) return SFB_EINVAL;
    FwdPlan p = c->fwd_all;
    if (fwd_bm > 0) p.bm = fwd_bm;
    if (fwd_bn > 0) p.bn = fwd_bn;
    if (fwd_split_k > 0) p.split_k = fwd_split_k;
    if (fwd_dma >= 0) p.dma = (fwd_dma & 1) != 0;
    if (fwd_dma >= 0) c->sparse_forward = (fwd_dma & 2) == 0;   // bit 1 set: dense scores for CSR input
    if (fwd_dma >= 0) c->sparse_always = (fwd_dma & 32) != 0;   // bit 5 set: from the entries whenever the kernel can take them
    if (fwd_dma >= 0) c->split_scores = (fwd_dma & 4) != 0;     // bit 2 set: fp32 scores as split-bf16 products
    if (fwd_dma >= 0) c->split_recon = (fwd_dma & 8) != 0;      // bit 3 set: the reconstruction likewise
    if (fwd_dma >= 0) c->use_fused = (fwd_dma & 16) == 0;       // bit 4 set: sfb_step_pipelined runs two separate passes
    finish_forward_plan(&p, (int64_t)c->P * c->B, c->J, c->D);
    c->fwd_all = p;
    if (recon_variant >= 0) {
        c->recon = plan_reconstruct_variant(c->J, c->D, recon_variant);
        c->recon_padded = plan_reconstruct_padded(c->J, c->D, (int64_t)c->P * c->B, recon_variant);
    }
    return SFB_OK;
}

sfb_status sfb_stream_copy(sfb_ctx* c, void* dst, const void* src, size_t bytes) {
    if (!c || !dst || !src) return SFB_EINVAL;
    if (((uintptr_t)dst % 16) != 0 || ((uintptr_t)src % 16) != 0 || (bytes % 16) != 0) return SFB_EINVAL;
    if (bytes == 0) return SFB_OK;
    Timed t(c, 3);
    hipError_t e = launch_stream_copy(src, dst, (int64_t)bytes, c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

sfb_status sfb_probe(sfb_ctx* c, sfb_probe_kind kind, float* W, int64_t ldw, int32_t param) {
    if (!c) return SFB_EINVAL;
    if (c->ws == nullptr || c->ws_bytes < 256) return SFB_EWORKSPACE;      // 64 floats of sink
    hipError_t e;
    switch (kind) {
        case SFB_PROBE_W_STREAM: {
            if (!W || (param != 1 && param != 2)) return SFB_EINVAL;
            if (ldw < c->D) return SFB_ESHAPE;
            if (((uintptr_t)W % 16) != 0 || (ldw % 4) != 0 || (c->D % 32) != 0) return SFB_EUNSUPPORTED;
            Timed t(c, 3);
            e = launch_probe_w_stream(W, ldw, (int)c->J, (int)c->D, c->fwd_bf16.k_slice, param, (float*)c->ws, c->stream);
            break;
        }
        case SFB_PROBE_W_RMW: {
            if (!W) return SFB_EINVAL;
            if (ldw < c->D) return SFB_ESHAPE;
            Timed t(c, 3);
            e = launch_probe_w_rmw(W, ldw, (int)c->J, (int)c->D, 0.0f, c->stream);
            break;
        }
        case SFB_PROBE_MFMA_F32:
        case SFB_PROBE_MFMA_BF16: {
            if (param != 1 && param != 2) return SFB_EINVAL;
            Timed t(c, 3);
            e = launch_probe_mfma(kind == SFB_PROBE_MFMA_BF16, param, SFB_PROBE_MFMA_ITERS, (float*)c->ws, c->stream);
            break;
        }
        case SFB_PROBE_EMPTY: {
            Timed t(c, 3);
            e = launch_probe_empty(c->stream);
            break;
        }
        case SFB_PROBE_FUSED_TRAFFIC: {
            if (!W) return SFB_EINVAL;
            if (ldw < c->D) return SFB_ESHAPE;
            // the shapes and operands the one-pass kernel takes, and its packed-operand areas of the workspace
            const int N = c->P * c->B;
            if (!c->fused_ok || (int64_t)c->J * ldw >= (1LL << 31) || ((uintptr_t)W % 16) != 0 || (ldw % 4) != 0)
                return SFB_EUNSUPPORTED;
            if (c->ws_bytes < workspace_need(c)) return SFB_EWORKSPACE;
            char* ws_factors = (char*)c->ws + scores_need(c);
            char* ws_next = ws_factors + bf16_recon_workspace(c->J, c->D, N);
            Timed t(c, 3);
            e = launch_probe_fused_traffic(W, ldw, (int)c->J, (int)c->D, N, c->fused, ws_factors, ws_next, c->stream);
            break;
        }
        default: return SFB_EINVAL;
    }
    if (e != hipSuccess) return hip_fail(c, e);
    return SFB_OK;
}

sfb_status sfb_enable_timing(sfb_ctx* c, int enable) {
    if (!c) return SFB_EINVAL;
    c->timing = enable != 0;
    return SFB_OK;
}

sfb_status sfb_kernel_time_ms(sfb_ctx* c, int which, double* ms, int64_t* launches) {
    if (!c || which < 0 || which >= kFamilies || !ms) return SFB_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    double total = 0.0;
    for (auto& p : c->used[which]) {
        float t = 0.f;
        e = hipEventElapsedTime(&t, p.a, p.b);
        if (e != hipSuccess) return hip_fail(c, e);
        total += t;
    }
    *ms = total;
    if (launches) *launches = (int64_t)c->used[which].size();
    return SFB_OK;
}

sfb_status sfb_reset_timing(sfb_ctx* c) {
    if (!c) return SFB_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e);
    for (int f = 0; f < kFamilies; ++f) {
        for (auto& p : c->used[f]) c->spare.push_back(p);
        c->used[f].clear();
    }
    return SFB_OK;
}

}  // extern "C"
