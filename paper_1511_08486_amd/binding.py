"""ctypes binding of libsfb.so.  Argument marshalling only: every step of the path runs in
the library's kernels.  Tensors are torch CUDA tensors used as plain device buffers
(data_ptr + row stride); torch does no arithmetic here."""
from __future__ import annotations

import ctypes as C
import os

import torch

SFB_MLR, SFB_DML, SFB_L2SVM = 0, 1, 2
SFB_F32, SFB_BF16 = 0, 1
SFB_EINVAL = -1
_MODELS = {"mlr": SFB_MLR, "dml": SFB_DML, "l2svm": SFB_L2SVM}
_DTYPES = {"f32": SFB_F32, "bf16": SFB_BF16}

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path():
    return os.path.join(_HERE, "libsfb.so")


class sfb_batch(C.Structure):
    _fields_ = [("a", C.c_void_p), ("a2", C.c_void_p), ("lda", C.c_int64),
                ("csr_rowptr", C.c_void_p), ("csr_col", C.c_void_p), ("csr_val", C.c_void_p),
                ("nnz", C.c_int64)]


class sfb_sdca(C.Structure):
    _fields_ = [("dual", C.c_void_p), ("ld_dual", C.c_int64), ("n_data", C.c_int64), ("sample", C.c_void_p),
                ("conj", C.c_void_p), ("lam", C.c_float), ("s", C.c_float)]


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python paper_1511_08486_amd/build.py` "
                          "(there is no fallback path)")
    try:
        lib = C.CDLL(path)
    except OSError as e:  # pragma: no cover
        raise ImportError(f"cannot load {path}: {e}") from e
    vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_float
    pb = C.POINTER(sfb_batch)
    pd = C.POINTER(sfb_sdca)
    sigs = {
        "sfb_create": (C.c_int, [C.POINTER(vp), C.c_int, i64, i64, i32, i32, C.c_int, vp]),
        "sfb_destroy": (None, [vp]),
        "sfb_workspace_bytes": (C.c_int, [vp, C.POINTER(C.c_size_t)]),
        "sfb_set_workspace": (C.c_int, [vp, vp, C.c_size_t]),
        "sfb_compute_factors": (C.c_int, [vp, vp, i64, pb, vp, vp, i64, vp, i64, vp]),
        "sfb_compute_factors_worker": (C.c_int, [vp, vp, i64, pb, vp, i32, vp, i64, vp, i64, vp]),
        "sfb_reconstruct_apply": (C.c_int, [vp, vp, i64, vp, i64, vp, i64, f32, f32, vp]),
        "sfb_step": (C.c_int, [vp, vp, i64, pb, vp, vp, i64, vp, i64, vp, f32, vp]),
        "sfb_step_pipelined": (C.c_int, [vp, vp, i64, vp, i64, vp, i64, pb, vp, vp, f32, vp]),
        "sfb_pipeline_info": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "sfb_step_noalloc": (C.c_int, [vp, vp, i64, pb, vp, vp, i64, vp, i64, vp, f32, vp]),
        "sfb_default_scale": (C.c_int, [vp, C.POINTER(f32)]),
        "sfb_sync": (C.c_int, [vp]),
        "sfb_strerror": (C.c_char_p, [C.c_int]),
        "sfb_last_hip_error": (C.c_int, [vp]),
        "sfb_plan_info": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "sfb_set_plan": (C.c_int, [vp, i32, i32, i32, i32, i32]),
        "sfb_stream_copy": (C.c_int, [vp, vp, vp, C.c_size_t]),
        "sfb_probe": (C.c_int, [vp, C.c_int, vp, i64, i32]),
        "sfb_enable_timing": (C.c_int, [vp, C.c_int]),
        "sfb_kernel_time_ms": (C.c_int, [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]),
        "sfb_reset_timing": (C.c_int, [vp]),
        "sfb_reconstruct_apply_worker": (C.c_int, [vp, vp, i64, vp, i64, vp, i64, i32, f32, f32]),
        "sfb_shape": (C.c_int, [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]),
        "sfb_sdca_compute_factors": (C.c_int, [vp, vp, i64, pb, vp, pd, vp, i64, vp, i64, vp]),
        "sfb_sdca_step": (C.c_int, [vp, vp, i64, pb, vp, pd, vp, i64, vp, i64, vp]),
        "sfb_prox": (C.c_int, [vp, vp, i64, C.c_int, f32, f32]),
        "sfb_reconstruct_apply_prox": (C.c_int, [vp, vp, i64, vp, i64, vp, i64, f32, f32, vp, C.c_int, f32]),
        "sfb_step_prox": (C.c_int, [vp, vp, i64, pb, vp, vp, i64, vp, i64, vp, f32, vp, C.c_int, f32]),
        "sfb_ssp_create": (C.c_int, [C.POINTER(vp), vp, i32, C.POINTER(vp), i64, vp, i64, vp, i64, i32]),
        "sfb_ssp_destroy": (None, [vp]),
        "sfb_ssp_worker_step": (C.c_int, [vp, i32, pb, vp, f32, vp, C.POINTER(i32)]),
        "sfb_ssp_deliver": (C.c_int, [vp, i32, i32, i32]),
        "sfb_ssp_set_receivers": (C.c_int, [vp, vp]),
        "sfb_halton_receivers": (C.c_int, [i32, i32, vp]),
        "sfb_ssp_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32)]),
    }
    for name, (res, args) in sigs.items():
        try:
            fn = getattr(lib, name)
        except AttributeError as e:
            raise ImportError(f"{path} lacks {name}: it is older than this binding, rebuild it with "
                              "`python paper_1511_08486_amd/build.py`") from e
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def sfb_strerror(status):
    return lib.sfb_strerror(int(status)).decode()


class SfbError(RuntimeError):
    def __init__(self, status, where, hip=0):
        self.status, self.hip = int(status), int(hip)
        super().__init__(f"{where}: {sfb_strerror(status)} (status {int(status)}, hip error {int(hip)})")


class SfbBatch:
    """One minibatch as device tensors.  Dense: a [N, D] (and a2 for DML pairs).
    Sparse (L2-SVM): rowptr int32 [N+1], col int32 [nnz], val float32 [nnz]."""

    def __init__(self, a=None, a2=None, rowptr=None, col=None, val=None):
        self.a, self.a2, self.rowptr, self.col, self.val = a, a2, rowptr, col, val

    def c_struct(self):
        s = sfb_batch()
        if self.a is not None:
            s.a, s.lda = self.a.data_ptr(), self.a.stride(0)
        if self.a2 is not None:
            s.a2 = self.a2.data_ptr()
            if self.a is not None and self.a2.stride(0) != self.a.stride(0):
                raise ValueError("a and a2 must share their row stride")
        if self.rowptr is not None:
            s.csr_rowptr = self.rowptr.data_ptr()
            s.csr_col = self.col.data_ptr() if self.col is not None and self.col.numel() else None
            s.csr_val = self.val.data_ptr() if self.val is not None and self.val.numel() else None
            s.nnz = int(self.col.numel()) if self.col is not None else 0
        return s


def _ptr(t):
    return None if t is None else t.data_ptr()


class Sfb:
    """Owns one sfb_ctx plus its workspace; methods mirror the C entry points."""

    def __init__(self, model, J, D, P, B, dtype="f32", stream=None, device="cuda:0"):
        self.model = _MODELS[model] if isinstance(model, str) else int(model)
        self.dtype = _DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
        self.J, self.D, self.P, self.B = int(J), int(D), int(P), int(B)
        self.device = torch.device(device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        self.stream = int(stream)
        self._ctx = C.c_void_p()
        self._check(lib.sfb_create(C.byref(self._ctx), self.model, self.J, self.D, self.P, self.B,
                                   self.dtype, C.c_void_p(self.stream)), "sfb_create")
        self._ws = None
        self._ensure_workspace()

    # -- plumbing ---------------------------------------------------------
    def _check(self, status, where):
        if status != 0:
            hip = lib.sfb_last_hip_error(self._ctx) if self._ctx else 0
            raise SfbError(status, where, hip)

    def _ensure_workspace(self):
        need = C.c_size_t()
        self._check(lib.sfb_workspace_bytes(self._ctx, C.byref(need)), "sfb_workspace_bytes")
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = torch.empty(max(int(need.value), 16), dtype=torch.uint8, device=self.device)
        self._check(lib.sfb_set_workspace(self._ctx, self._ws.data_ptr(), self._ws.numel()),
                    "sfb_set_workspace")

    def close(self):
        if getattr(self, "_ctx", None):
            lib.sfb_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self):
        need = C.c_size_t()
        self._check(lib.sfb_workspace_bytes(self._ctx, C.byref(need)), "sfb_workspace_bytes")
        return int(need.value)

    # -- the path -----------------------------------------------------------
    def compute_factors(self, W, batch, y, U, V, loss=None):
        b = batch.c_struct()
        self._check(lib.sfb_compute_factors(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(),
                                            U.data_ptr(), U.stride(0), V.data_ptr(), V.stride(0),
                                            _ptr(loss)), "sfb_compute_factors")

    def compute_factors_worker(self, W, batch_p, y_p, p, U, V, loss=None):
        b = batch_p.c_struct()
        self._check(lib.sfb_compute_factors_worker(self._ctx, W.data_ptr(), W.stride(0), C.byref(b),
                                                   y_p.data_ptr(), int(p), U.data_ptr(), U.stride(0),
                                                   V.data_ptr(), V.stride(0), _ptr(loss)),
                    "sfb_compute_factors_worker")

    def default_scale(self):
        """1/B as the library's fp32 (what sfb_step passes to the reconstruction)."""
        v = C.c_float()
        self._check(lib.sfb_default_scale(self._ctx, C.byref(v)), "sfb_default_scale")
        return v.value

    @staticmethod
    def _mask(active):
        if active is None:
            return None, None
        buf = (C.c_uint8 * len(active))(*[1 if a else 0 for a in active])
        return buf, C.cast(buf, C.c_void_p)

    def reconstruct_apply(self, W, U, V, eta, scale=None, active=None):
        if scale is None:
            scale = self.default_scale()
        if active is not None and len(active) != self.P:
            raise ValueError("active mask must have P entries")
        keep, ptr = self._mask(active)
        self._check(lib.sfb_reconstruct_apply(self._ctx, W.data_ptr(), W.stride(0), U.data_ptr(), U.stride(0),
                                              V.data_ptr(), V.stride(0), float(eta), float(scale), ptr),
                    "sfb_reconstruct_apply")

    def reconstruct_apply_worker(self, W, U, V, p, eta, scale=None):
        if scale is None:
            scale = self.default_scale()
        self._check(lib.sfb_reconstruct_apply_worker(self._ctx, W.data_ptr(), W.stride(0), U.data_ptr(), U.stride(0),
                                                     V.data_ptr(), V.stride(0), int(p), float(eta), float(scale)),
                    "sfb_reconstruct_apply_worker")

    def step(self, W, batch, y, U, V, eta, loss=None, active=None):
        if active is not None and len(active) != self.P:
            raise ValueError("active mask must have P entries")
        b = batch.c_struct()
        keep, ptr = self._mask(active)
        self._check(lib.sfb_step(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(), U.data_ptr(),
                                 U.stride(0), V.data_ptr(), V.stride(0), _ptr(loss), float(eta), ptr),
                    "sfb_step")

    def update_and_next_factors(self, W, U, V, next_batch, next_y, eta, loss=None, active=None):
        """sfb_step_pipelined: apply the pending factors in U, V to W, then leave the next batch's factors there."""
        if active is not None and len(active) != self.P:
            raise ValueError("active mask must have P entries")
        b = next_batch.c_struct()
        keep, ptr = self._mask(active)
        self._check(lib.sfb_step_pipelined(self._ctx, W.data_ptr(), W.stride(0), U.data_ptr(), U.stride(0),
                                           V.data_ptr(), V.stride(0), C.byref(b), next_y.data_ptr(), _ptr(loss),
                                           float(eta), ptr), "sfb_step_pipelined")

    def pipeline_info(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(lib.sfb_pipeline_info(self._ctx, C.byref(a), C.byref(b), C.byref(c)), "sfb_pipeline_info")
        return {"fused": bool(a.value), "grid": b.value, "slices": c.value}

    def pipeline_ok(self):
        """True if sfb_step_pipelined would run its one-pass kernel for this context's shape."""
        return self.pipeline_info()["fused"]

    def step_noalloc(self, W, batch, y, U, V, eta, loss=None, active=None):
        """sfb_step on the library's own fixed scratch array (no workspace, nothing allocated)."""
        if active is not None and len(active) != self.P:
            raise ValueError("active mask must have P entries")
        b = batch.c_struct()
        keep, ptr = self._mask(active)
        self._check(lib.sfb_step_noalloc(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(),
                                         U.data_ptr(), U.stride(0), V.data_ptr(), V.stride(0), _ptr(loss),
                                         float(eta), ptr), "sfb_step_noalloc")

    # -- proximal step ---------------------------------------------------------
    PROX_KINDS = {"none": 0, "l2sq": 1, "l1": 2, "column_ball": 3}

    def prox(self, W, kind, eta, param):
        self._check(lib.sfb_prox(self._ctx, W.data_ptr(), W.stride(0), self.PROX_KINDS[kind], float(eta), float(param)),
                    "sfb_prox")

    def reconstruct_apply_prox(self, W, U, V, eta, kind, param, scale=None, active=None):
        if scale is None:
            scale = self.default_scale()
        keep, ptr = self._mask(active)
        self._check(lib.sfb_reconstruct_apply_prox(self._ctx, W.data_ptr(), W.stride(0), U.data_ptr(), U.stride(0),
                                                   V.data_ptr(), V.stride(0), float(eta), float(scale), ptr,
                                                   self.PROX_KINDS[kind], float(param)), "sfb_reconstruct_apply_prox")

    def step_prox(self, W, batch, y, U, V, eta, kind, param, loss=None, active=None):
        b = batch.c_struct()
        keep, ptr = self._mask(active)
        self._check(lib.sfb_step_prox(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(), U.data_ptr(),
                                      U.stride(0), V.data_ptr(), V.stride(0), _ptr(loss), float(eta), ptr,
                                      self.PROX_KINDS[kind], float(param)), "sfb_step_prox")

    # -- SDCA ------------------------------------------------------------------
    @staticmethod
    def _sdca(dual, sample, lam, s, conj):
        return sfb_sdca(dual.data_ptr(), dual.stride(0), dual.shape[0], sample.data_ptr(), _ptr(conj), float(lam),
                        float(s))

    def sdca_compute_factors(self, W, batch, y, dual, sample, lam, s, U, V, loss=None, conj=None):
        b, d = batch.c_struct(), self._sdca(dual, sample, lam, s, conj)
        self._check(lib.sfb_sdca_compute_factors(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(),
                                                 C.byref(d), U.data_ptr(), U.stride(0), V.data_ptr(), V.stride(0),
                                                 _ptr(loss)), "sfb_sdca_compute_factors")

    def sdca_step(self, W, batch, y, dual, sample, lam, s, U, V, loss=None, conj=None):
        b, d = batch.c_struct(), self._sdca(dual, sample, lam, s, conj)
        self._check(lib.sfb_sdca_step(self._ctx, W.data_ptr(), W.stride(0), C.byref(b), y.data_ptr(), C.byref(d),
                                      U.data_ptr(), U.stride(0), V.data_ptr(), V.stride(0), _ptr(loss)),
                    "sfb_sdca_step")

    def sync(self):
        self._check(lib.sfb_sync(self._ctx), "sfb_sync")

    # -- plan / timing -------------------------------------------------------
    def plan_info(self):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(lib.sfb_plan_info(self._ctx, C.byref(a), C.byref(b), C.byref(c)), "sfb_plan_info")
        return {"fwd_split_k": a.value, "fwd_grid": b.value, "recon_grid": c.value}

    def set_plan(self, fwd_bm=0, fwd_bn=0, fwd_split_k=0, recon_variant=-1, fwd_dma=-1):
        self._check(lib.sfb_set_plan(self._ctx, fwd_bm, fwd_bn, fwd_split_k, recon_variant, fwd_dma),
                    "sfb_set_plan")
        self._ensure_workspace()

    def stream_copy(self, dst, src):
        nbytes = src.numel() * src.element_size()
        self._check(lib.sfb_stream_copy(self._ctx, dst.data_ptr(), src.data_ptr(), nbytes), "sfb_stream_copy")

    PROBES = {"w_stream": 0, "w_rmw": 1, "mfma_f32": 2, "mfma_bf16": 3, "empty": 4, "fused_traffic": 5}
    PROBE_MFMA_ITERS = 4000

    def probe(self, kind, W=None, param=1):
        """One launch of a measurement aid (sfb_probe); time it with enable_timing / kernel_time_ms(3)."""
        self._check(lib.sfb_probe(self._ctx, self.PROBES[kind], _ptr(W), W.stride(0) if W is not None else 0,
                                  int(param)), "sfb_probe")

    def enable_timing(self, on=True):
        self._check(lib.sfb_enable_timing(self._ctx, 1 if on else 0), "sfb_enable_timing")

    def kernel_time_ms(self, which):
        ms, n = C.c_double(), C.c_int64()
        self._check(lib.sfb_kernel_time_ms(self._ctx, int(which), C.byref(ms), C.byref(n)), "sfb_kernel_time_ms")
        return ms.value, n.value

    def reset_timing(self):
        self._check(lib.sfb_reset_timing(self._ctx), "sfb_reset_timing")


def halton_receivers(P, Q):
    """receivers[p] = sorted workers that p broadcasts to under Halton sequence broadcast
    (computed by the library: sfb_halton_receivers)."""
    m = (C.c_uint8 * (P * P))()
    status = lib.sfb_halton_receivers(int(P), int(Q), m)
    if status != 0:
        raise SfbError(status, "sfb_halton_receivers")
    return [[r for r in range(P) if m[p * P + r]] for p in range(P)]


class SspSimulator:
    """Stale-synchronous SFB on one device: owns P replicas of W and the ring of factor sets,
    forwards every event to the sfb_ssp_* entry points (which keep the clocks and the rules).
    receivers[q] (optional) = the workers q broadcasts to; default: everybody."""

    def __init__(self, ctx, W0, staleness, ring_slots=None, receivers=None):
        self.ctx, self.s = ctx, int(staleness)
        self.slots = int(ring_slots) if ring_slots is not None else 2 * self.s + 2
        dev = ctx.device
        vdt = torch.bfloat16 if ctx.dtype == SFB_BF16 else torch.float32
        N = ctx.P * ctx.B
        self.W = [W0.to(dev).clone() for _ in range(ctx.P)]
        self.U_ring = torch.zeros((self.slots, N, ctx.J), dtype=torch.float32, device=dev)
        self.V_ring = torch.zeros((self.slots, N, ctx.D), dtype=vdt, device=dev)
        ptrs = (C.c_void_p * ctx.P)(*[w.data_ptr() for w in self.W])
        self._ssp = C.c_void_p()
        ctx._check(lib.sfb_ssp_create(C.byref(self._ssp), ctx._ctx, self.s, ptrs, self.W[0].stride(0),
                                      self.U_ring.data_ptr(), self.U_ring.stride(1), self.V_ring.data_ptr(),
                                      self.V_ring.stride(1), self.slots), "sfb_ssp_create")
        if receivers is not None:
            P = ctx.P
            m = (C.c_uint8 * (P * P))()
            for q, rs in enumerate(receivers):
                for r in rs:
                    m[q * P + int(r)] = 1
            ctx._check(lib.sfb_ssp_set_receivers(self._ssp, m), "sfb_ssp_set_receivers")

    def worker_step(self, p, batch_p, y_p, eta, loss=None):
        """True if worker p ran its next iteration, False if it had to pause (the staleness rule,
        or its send queue -- the ring -- is full); self.last_blocked says which (1 or 2)."""
        b = batch_p.c_struct()
        blocked = C.c_int32(0)
        self.ctx._check(lib.sfb_ssp_worker_step(self._ssp, int(p), C.byref(b), y_p.data_ptr(), float(eta),
                                                _ptr(loss), C.byref(blocked)), "sfb_ssp_worker_step")
        self.last_blocked = blocked.value
        return blocked.value == 0

    def deliver(self, p, q, count=1):
        """True if replica p applied the next `count` factor sets of worker q, False if refused."""
        status = lib.sfb_ssp_deliver(self._ssp, int(p), int(q), int(count))
        if status == SFB_EINVAL:
            return False
        self.ctx._check(status, "sfb_ssp_deliver")
        return True

    def state(self):
        P = self.ctx.P
        t = (C.c_int32 * P)()
        tau = (C.c_int32 * (P * P))()
        self.ctx._check(lib.sfb_ssp_state(self._ssp, t, tau), "sfb_ssp_state")
        return list(t), [list(tau[p * P:(p + 1) * P]) for p in range(P)]

    def close(self):
        if getattr(self, "_ssp", None):
            lib.sfb_ssp_destroy(self._ssp)
            self._ssp = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
