"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and its host-side validation rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_1511_08486_amd as sfb
    return sfb.lib


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sfb.h")).read()
    return sorted(set(re.findall(r"SFB_API[^;(]*?\b(sfb_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_symbols()
    for must in ("sfb_create", "sfb_destroy", "sfb_compute_factors", "sfb_compute_factors_worker",
                 "sfb_reconstruct_apply", "sfb_step", "sfb_sync", "sfb_strerror", "sfb_workspace_bytes",
                 "sfb_set_workspace"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    raw = C.CDLL(os.path.join(ROOT, "paper_1511_08486_amd", "libsfb.so"))
    for name in declared_symbols():
        assert hasattr(raw, name), f"libsfb.so lacks {name}"


def test_create_validates_arguments(lib):
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(None, 0, 10, 10, 1, 1, 0, None) == -1
    assert lib.sfb_create(C.byref(ctx), 0, 0, 10, 1, 1, 0, None) == -1
    assert lib.sfb_create(C.byref(ctx), 0, 10, 10, 0, 1, 0, None) == -1
    assert lib.sfb_create(C.byref(ctx), 7, 10, 10, 1, 1, 0, None) == -1
    assert lib.sfb_create(C.byref(ctx), 0, 10, 10, 1, 1, 5, None) == -3
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_DML, 10, 10, 1, 1, sfb.SFB_BF16, None) == -6
    assert not ctx.value
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 1000, 4096, 8, 64, sfb.SFB_F32, None) == 0
    need = C.c_size_t()
    assert lib.sfb_workspace_bytes(ctx, C.byref(need)) == 0
    k, g, r = C.c_int32(), C.c_int32(), C.c_int32()
    assert lib.sfb_plan_info(ctx, C.byref(k), C.byref(g), C.byref(r)) == 0
    assert need.value == k.value * 512 * 1000 * 4 and g.value >= 256 and r.value >= 256
    lib.sfb_destroy(ctx)


def test_ragged_fp32_contexts_reserve_room_for_padded_factor_copies(lib):
    """A context whose J, D or P*B is not what the LDS-DMA reconstructions take as they are (J % 4,
    D % 128, P*B % 32) asks for room for padded copies of the factors: rows of J rounded up to 4 and D
    rounded up to 128 floats, P*B rounded up to 32 rows, each copy rounded to 256 bytes, overlaying the
    partial scores.  Whole shapes and bf16 contexts ask for what they asked for before."""
    import paper_1511_08486_amd as sfb
    need, k, g, r = C.c_size_t(), C.c_int32(), C.c_int32(), C.c_int32()

    def ask(model, J, D, P, B, dtype):
        ctx = C.c_void_p()
        assert lib.sfb_create(C.byref(ctx), model, J, D, P, B, dtype, None) == 0
        assert lib.sfb_workspace_bytes(ctx, C.byref(need)) == 0
        assert lib.sfb_plan_info(ctx, C.byref(k), C.byref(g), C.byref(r)) == 0
        lib.sfb_destroy(ctx)
        return need.value, k.value

    def padded(J, D, N):
        up = lambda x, m: (x + m - 1) // m * m
        return up(up(N, 32) * up(J, 4) * 4, 256) + up(up(N, 32) * up(D, 128) * 4, 256)

    def expect(J, D, N, split, pad):
        up = lambda x, m: (x + m - 1) // m * m
        scores = up(split * N * up(J, 4) * 4, 256)
        return max(scores, padded(J, D, N)) if pad else scores

    got, split = ask(sfb.SFB_DML, 600, 780, 8, 128, sfb.SFB_F32)           # the metric of Section 6 on 780 features
    assert got == expect(600, 780, 1024, split, True)
    got, split = ask(sfb.SFB_MLR, 10, 100, 4, 16, sfb.SFB_F32)             # the smallest benchmark shape: the copies decide
    assert got == expect(10, 100, 64, split, True) == padded(10, 100, 64) == 64 * 12 * 4 + 64 * 128 * 4
    got, split = ask(sfb.SFB_MLR, 10, 784, 8, 64, sfb.SFB_F32)             # ten classes on 784 pixels
    assert got == expect(10, 784, 512, split, True) == padded(10, 784, 512)
    got, split = ask(sfb.SFB_MLR, 1000, 4096, 8, 60, sfb.SFB_F32)          # 480 rows: whole stages, nothing to pad
    assert got == expect(1000, 4096, 480, split, False)
    got, split = ask(sfb.SFB_MLR, 1000, 4096, 8, 61, sfb.SFB_F32)          # 488 rows
    assert got == expect(1000, 4096, 488, split, True) == padded(1000, 4096, 488)
    got32, _ = ask(sfb.SFB_MLR, 300, 1004, 3, 30, sfb.SFB_F32)             # ragged in every way
    assert got32 >= padded(300, 1004, 90)


def test_calls_reject_bad_arguments_before_launching(lib):
    """Fake non-null pointers are safe here: validation fails first, nothing is launched."""
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    fake = C.c_void_p(0x1000)
    b = sfb.binding.sfb_batch()
    b.a, b.lda = 0x1000, 16
    # null W / U / V
    assert lib.sfb_compute_factors(ctx, None, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -1
    assert lib.sfb_reconstruct_apply(ctx, fake, 16, None, 8, fake, 16, 0.1, 1.0, None) == -1
    # leading dimensions shorter than the rows
    assert lib.sfb_compute_factors(ctx, fake, 15, C.byref(b), fake, fake, 8, fake, 16, None) == -2
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 7, fake, 16, None) == -2
    assert lib.sfb_reconstruct_apply(ctx, fake, 16, fake, 8, fake, 15, 0.1, 1.0, None) == -2
    b.lda = 15
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -2
    b.lda = 16
    # missing batch / labels / features
    assert lib.sfb_compute_factors(ctx, fake, 16, None, fake, fake, 8, fake, 16, None) == -1
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), None, fake, 8, fake, 16, None) == -1
    b.a = None
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -1
    b.a = 0x1000
    # worker index out of range
    assert lib.sfb_compute_factors_worker(ctx, fake, 16, C.byref(b), fake, 2, fake, 8, fake, 16, None) == -2
    # no workspace registered yet
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -5
    assert lib.sfb_set_workspace(ctx, fake, 1) == -5
    assert lib.sfb_set_workspace(ctx, C.c_void_p(0x1010), 1 << 20) == -1      # not 256-byte aligned
    # non-finite learning rate
    assert lib.sfb_reconstruct_apply(ctx, fake, 16, fake, 8, fake, 16, float("nan"), 1.0, None) == -1
    assert lib.sfb_step(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None, float("inf"), None) == -1
    # plan override outside the table
    assert lib.sfb_set_plan(ctx, 96, 0, 0, -1, -1) == -1 and lib.sfb_set_plan(ctx, 0, 0, 0, 99, -1) == -1
    lib.sfb_destroy(ctx)
    # a mask needs P <= 64
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 65, 1, sfb.SFB_F32, None) == 0
    mask = (C.c_uint8 * 65)(*([1] * 65))
    assert lib.sfb_reconstruct_apply(ctx, fake, 16, fake, 8, fake, 16, 0.1, 1.0, C.cast(mask, C.c_void_p)) == -6
    lib.sfb_destroy(ctx)
    # DML needs both points; L2SVM needs the CSR arrays
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_DML, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -1
    lib.sfb_destroy(ctx)
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_L2SVM, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    assert lib.sfb_compute_factors(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None) == -1
    lib.sfb_destroy(ctx)


def test_strerror_covers_every_status(lib):
    import paper_1511_08486_amd as sfb
    seen = {sfb.sfb_strerror(s) for s in (0, -1, -2, -3, -5, -6, -7)}
    assert len(seen) == 7 and "unknown status" not in seen
    assert sfb.sfb_strerror(-99) == "unknown status"


def test_ssp_and_per_sender_calls_validate_before_launching(lib):
    """Host-side rules of the stale-synchronous scheduler need no GPU: creation checks, a
    delivery nobody has produced, a worker index out of range."""
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 3, 4, sfb.SFB_F32, None) == 0
    J, D, P, B, dt = C.c_int64(), C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32()
    assert lib.sfb_shape(ctx, C.byref(J), C.byref(D), C.byref(P), C.byref(B), C.byref(dt)) == 0
    assert (J.value, D.value, P.value, B.value, dt.value) == (8, 16, 3, 4, 0)
    assert lib.sfb_shape(None, None, None, None, None, None) == -1
    fake = C.c_void_p(0x1000)
    assert lib.sfb_reconstruct_apply_worker(ctx, fake, 16, fake, 8, fake, 16, 3, 0.1, 0.25) == -2
    assert lib.sfb_reconstruct_apply_worker(ctx, fake, 16, fake, 8, fake, 16, -1, 0.1, 0.25) == -2
    assert lib.sfb_reconstruct_apply_worker(ctx, fake, 16, fake, 8, fake, 16, 0, float("nan"), 0.25) == -1
    assert lib.sfb_reconstruct_apply_worker(ctx, None, 16, fake, 8, fake, 16, 0, 0.1, 0.25) == -1
    ssp = C.c_void_p()
    reps = (C.c_void_p * 3)(0x1000, 0x2000, 0x3000)
    assert lib.sfb_ssp_create(None, ctx, 1, reps, 16, fake, 8, fake, 16, 4) == -1
    assert lib.sfb_ssp_create(C.byref(ssp), None, 1, reps, 16, fake, 8, fake, 16, 4) == -1
    assert lib.sfb_ssp_create(C.byref(ssp), ctx, -1, reps, 16, fake, 8, fake, 16, 4) == -1
    assert lib.sfb_ssp_create(C.byref(ssp), ctx, 1, reps, 15, fake, 8, fake, 16, 4) == -2       # ldw < D
    assert lib.sfb_ssp_create(C.byref(ssp), ctx, 1, reps, 16, fake, 8, fake, 16, 3) == -2       # ring < 2s + 2
    holes = (C.c_void_p * 3)(0x1000, None, 0x3000)
    assert lib.sfb_ssp_create(C.byref(ssp), ctx, 1, holes, 16, fake, 8, fake, 16, 4) == -1
    assert not ssp.value
    assert lib.sfb_ssp_create(C.byref(ssp), ctx, 1, reps, 16, fake, 8, fake, 16, 4) == 0
    t = (C.c_int32 * 3)()
    tau = (C.c_int32 * 9)(*([7] * 9))
    assert lib.sfb_ssp_state(ssp, t, tau) == 0 and list(t) == [0, 0, 0] and list(tau) == [0] * 9
    assert lib.sfb_ssp_deliver(ssp, 0, 0, 1) == -1          # a worker does not receive from itself
    assert lib.sfb_ssp_deliver(ssp, 0, 1, 1) == -1          # worker 1 has produced nothing yet
    assert lib.sfb_ssp_deliver(ssp, 0, 3, 1) == -2
    assert lib.sfb_ssp_deliver(ssp, 0, 1, 0) == 0           # nothing to apply, nothing launched
    blocked = C.c_int32(5)
    assert lib.sfb_ssp_worker_step(ssp, 3, None, None, 0.1, None, C.byref(blocked)) == -2
    assert lib.sfb_ssp_worker_step(ssp, 0, None, None, 0.1, None, None) == -1
    assert lib.sfb_ssp_worker_step(ssp, 0, None, fake, 0.1, None, C.byref(blocked)) == -1     # no batch: refused by the factor call
    assert list(t) == [0, 0, 0]
    # partial broadcast: 0 -> 1 -> 2 -> 0
    assert lib.sfb_ssp_set_receivers(ssp, None) == -1 and lib.sfb_ssp_set_receivers(None, reps) == -1
    ring = (C.c_uint8 * 9)(0, 1, 0, 0, 0, 1, 1, 0, 0)
    assert lib.sfb_ssp_set_receivers(ssp, ring) == 0
    assert lib.sfb_ssp_deliver(ssp, 0, 1, 0) == -1          # worker 1 does not send to worker 0 (even for count 0)
    assert lib.sfb_ssp_deliver(ssp, 1, 0, 0) == 0
    m = (C.c_uint8 * 36)()
    assert lib.sfb_halton_receivers(6, 2, m) == 0
    assert [[r for r in range(6) if m[p * 6 + r]] for p in range(6)] == [[1, 3], [2, 4], [3, 5], [0, 4], [1, 5], [0, 2]]
    assert lib.sfb_halton_receivers(0, 2, m) == -1 and lib.sfb_halton_receivers(6, -1, m) == -1
    assert lib.sfb_halton_receivers(6, 2, None) == -1
    lib.sfb_ssp_destroy(ssp)
    lib.sfb_destroy(ctx)


def test_sdca_calls_validate_before_launching(lib):
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    fake = C.c_void_p(0x1000)
    b = sfb.binding.sfb_batch()
    b.a, b.lda = 0x1000, 16

    def sd(**kw):
        d = sfb.binding.sfb_sdca(dual=0x1000, ld_dual=8, n_data=100, sample=0x1000, conj=None, lam=0.1, s=0.5)
        for k, v in kw.items():
            setattr(d, k, v)
        return C.byref(d)

    def call(d, fn=lib.sfb_sdca_compute_factors):
        return fn(ctx, fake, 16, C.byref(b), fake, d, fake, 8, fake, 16, None)
    assert call(None) == -1
    assert call(sd(dual=None)) == -1 and call(sd(sample=None)) == -1 and call(sd(n_data=0)) == -1
    assert call(sd(lam=0.0)) == -1 and call(sd(lam=float("nan"))) == -1
    assert call(sd(s=0.0)) == -1 and call(sd(s=1.5)) == -1 and call(sd(s=float("nan"))) == -1
    assert call(sd(ld_dual=7)) == -2
    assert call(sd()) == -5                                   # all valid: stops at the missing workspace
    assert call(sd(), lib.sfb_sdca_step) == -5
    assert call(None, lib.sfb_sdca_step) == -1
    assert call(sd(lam=1e-45, n_data=1), lib.sfb_sdca_step) == -1       # 1 / (lam n_data) overflows
    lib.sfb_destroy(ctx)
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_DML, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    b.a2 = 0x1000
    assert call(sd()) == -6                                   # the dual update exists for the logistic loss only
    lib.sfb_destroy(ctx)


def test_prox_validates_before_launching(lib):
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    fake = C.c_void_p(0x1000)
    assert lib.sfb_prox(ctx, None, 16, 1, 0.1, 0.1) == -1
    assert lib.sfb_prox(None, fake, 16, 1, 0.1, 0.1) == -1
    assert lib.sfb_prox(ctx, fake, 16, 4, 0.1, 0.1) == -1 and lib.sfb_prox(ctx, fake, 16, -1, 0.1, 0.1) == -1
    assert lib.sfb_prox(ctx, fake, 16, 1, -0.1, 0.1) == -1 and lib.sfb_prox(ctx, fake, 16, 2, 0.1, -1.0) == -1
    assert lib.sfb_prox(ctx, fake, 16, 1, float("nan"), 0.1) == -1 and lib.sfb_prox(ctx, fake, 16, 2, 0.1, float("inf")) == -1
    assert lib.sfb_prox(ctx, fake, 16, 3, 0.1, 0.0) == -1           # a ball of radius 0
    assert lib.sfb_prox(ctx, fake, 15, 1, 0.1, 0.1) == -2
    assert lib.sfb_prox(ctx, fake, 16, 3, 0.1, 1.0) == -5           # the column projection needs the workspace
    assert lib.sfb_prox(ctx, fake, 16, 0, 0.1, 0.1) == 0            # identity: nothing is launched
    # the fused forms refuse the same things, before anything is launched
    b = sfb.binding.sfb_batch()
    b.a, b.lda = 0x1000, 16
    assert lib.sfb_reconstruct_apply_prox(ctx, fake, 16, fake, 8, fake, 16, 0.1, 1.0, None, 7, 0.1) == -1
    assert lib.sfb_reconstruct_apply_prox(ctx, fake, 16, fake, 8, fake, 16, 0.1, 1.0, None, 2, -0.1) == -1
    assert lib.sfb_reconstruct_apply_prox(ctx, fake, 16, fake, 8, fake, 16, 0.1, 1.0, None, 3, 1.0) == -5
    assert lib.sfb_reconstruct_apply_prox(ctx, None, 16, fake, 8, fake, 16, 0.1, 1.0, None, 1, 0.1) == -1
    assert lib.sfb_step_prox(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None, 0.1, None, 9, 0.1) == -1
    assert lib.sfb_step_prox(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None, 0.1, None, 3, 0.0) == -1
    assert lib.sfb_step_prox(ctx, fake, 16, C.byref(b), fake, fake, 8, fake, 16, None, 0.1, None, 1, 0.1) == -5
    lib.sfb_destroy(ctx)


def test_launch_plans_of_the_benchmark_shapes(lib):
    """The planner is host code: tile counts for the five benchmark shapes (no GPU needed).
    mlr_medium: 128x128 tiles, one per compute unit; dml: 600 rows take four row tiles of five row blocks x 64
    column tiles, one workgroup per compute unit;
    l2svm: 128x128 tiles, four per compute unit; mlr_large: 256x128 bf16 tiles."""
    import paper_1511_08486_amd as sfb
    want = {("mlr", 10, 100, 4, 16, "f32"): 1, ("mlr", 1000, 4096, 8, 64, "f32"): 256,
            ("dml", 600, 4096, 8, 128, "f32"): 256, ("l2svm", 2000, 8192, 16, 64, "f32"): 1024}
    for (model, J, D, P, B, dt), grid in want.items():
        ctx = C.c_void_p()
        assert lib.sfb_create(C.byref(ctx), sfb.binding._MODELS[model], J, D, P, B, sfb.binding._DTYPES[dt], None) == 0
        k, g, r = C.c_int32(), C.c_int32(), C.c_int32()
        assert lib.sfb_plan_info(ctx, C.byref(k), C.byref(g), C.byref(r)) == 0
        assert r.value == grid, (model, J, D, r.value)
        assert k.value >= 1 and g.value >= 1
        # every variant of the table can be selected; one past the end cannot
        for v in range(13):
            assert lib.sfb_set_plan(ctx, 0, 0, 0, v, -1) == 0
        assert lib.sfb_set_plan(ctx, 0, 0, 0, 13, -1) == -1
        lib.sfb_destroy(ctx)


def test_measurement_aids_validate_their_arguments(lib):
    import paper_1511_08486_amd as sfb
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 8, 16, 2, 4, sfb.SFB_F32, None) == 0
    fake = C.c_void_p(0x1000)
    assert lib.sfb_stream_copy(ctx, fake, fake, 24) == -1                    # not a multiple of 16 bytes
    assert lib.sfb_stream_copy(ctx, C.c_void_p(0x1008), fake, 32) == -1      # destination not 16-byte aligned
    assert lib.sfb_stream_copy(ctx, None, fake, 32) == -1 and lib.sfb_stream_copy(None, fake, fake, 32) == -1
    ms, n = C.c_double(-1.0), C.c_int64(-1)
    assert lib.sfb_kernel_time_ms(ctx, 9, C.byref(ms), C.byref(n)) == -1     # no such kernel family
    assert lib.sfb_kernel_time_ms(ctx, 0, None, C.byref(n)) == -1
    assert lib.sfb_enable_timing(None, 1) == -1 and lib.sfb_reset_timing(None) == -1
    assert lib.sfb_plan_info(None, None, None, None) == -1
    assert lib.sfb_last_hip_error(ctx) == 0
    lib.sfb_destroy(ctx)
    lib.sfb_destroy(None)                                                     # harmless


def test_noalloc_step_rejects_what_its_fixed_scratch_cannot_hold(lib):
    """Fake non-null pointers are safe here: the size check fails first, nothing is launched."""
    import paper_1511_08486_amd as sfb
    assert "sfb_step_noalloc" in declared_symbols()
    fake = C.c_void_p(0x1000)
    b = sfb.binding.sfb_batch()
    ctx = C.c_void_p()
    # 10000 x 21504 bf16: 61 MB of partial scores + 32 MB of packed factors > the 16 MiB array
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 10000, 21504, 16, 32, sfb.SFB_BF16, None) == 0
    need = C.c_size_t()
    assert lib.sfb_workspace_bytes(ctx, C.byref(need)) == 0 and need.value > (16 << 20)
    b.a, b.lda = 0x1000, 21504
    assert lib.sfb_step_noalloc(ctx, fake, 21504, C.byref(b), fake, fake, 10000, fake, 21504, None, 0.1, None) == -8
    assert b"scratch" in lib.sfb_strerror(-8)
    # the other argument checks come first, as in sfb_step
    assert lib.sfb_step_noalloc(ctx, None, 21504, C.byref(b), fake, fake, 10000, fake, 21504, None, 0.1, None) == -1
    assert lib.sfb_step_noalloc(ctx, fake, 21503, C.byref(b), fake, fake, 10000, fake, 21504, None, 0.1, None) == -2
    lib.sfb_destroy(ctx)


def test_pipelined_step_and_probes_validate_their_arguments(lib):
    """Fake non-null pointers are safe here: every call below is refused before anything is launched."""
    import paper_1511_08486_amd as sfb
    for name in ("sfb_step_pipelined", "sfb_pipeline_info", "sfb_probe", "sfb_default_scale"):
        assert name in declared_symbols()
    fake = C.c_void_p(0x1000)
    b = sfb.binding.sfb_batch()
    b.a, b.lda = 0x1000, 1024
    ctx = C.c_void_p()
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 300, 1024, 4, 32, sfb.SFB_BF16, None) == 0
    fused, grid, slices = C.c_int32(), C.c_int32(), C.c_int32()
    assert lib.sfb_pipeline_info(ctx, C.byref(fused), C.byref(grid), C.byref(slices)) == 0
    assert fused.value == 1 and grid.value == 3 * slices.value and slices.value >= 1      # 3 bands of 128 rows
    scale = C.c_float()
    assert lib.sfb_default_scale(ctx, C.byref(scale)) == 0 and scale.value == 1.0 / 32
    assert lib.sfb_default_scale(ctx, None) == -1
    # argument checks of the pipelined step: null W, short leading dimension, missing batch, bad eta; then no workspace
    args = lambda W, ldw, batch, eta: lib.sfb_step_pipelined(ctx, W, ldw, fake, 300, fake, 1024, batch, fake, None, eta, None)
    assert args(None, 1024, C.byref(b), 0.1) == -1
    assert args(fake, 1023, C.byref(b), 0.1) == -2
    assert args(fake, 1024, None, 0.1) == -1
    assert args(fake, 1024, C.byref(b), float("nan")) == -1
    assert args(fake, 1024, C.byref(b), 0.1) == -5
    # probes: no workspace registered -> refused; unknown kind and bad parameters are refused too
    assert lib.sfb_probe(ctx, 2, None, 0, 1) == -5
    assert lib.sfb_probe(None, 2, None, 0, 1) == -1
    lib.sfb_destroy(ctx)
    # shapes the one-pass kernel does not take report so
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 300, 1004, 3, 30, sfb.SFB_BF16, None) == 0
    assert lib.sfb_pipeline_info(ctx, C.byref(fused), None, None) == 0 and fused.value == 0
    lib.sfb_destroy(ctx)
    assert lib.sfb_create(C.byref(ctx), sfb.SFB_MLR, 1000, 4096, 8, 64, sfb.SFB_F32, None) == 0
    assert lib.sfb_pipeline_info(ctx, C.byref(fused), None, None) == 0 and fused.value == 0
    lib.sfb_destroy(ctx)
