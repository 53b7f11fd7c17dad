"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  fp32 configs: max relative error 1e-4 (with a floor of 1e-2 of the
largest magnitude); bf16-input config: 2e-2."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import alloc_factors, assert_close, fresh_update, make_clear_of_kink, run_chain, to_device

pytestmark = pytest.mark.gpu

TOL32 = 1e-4
TOLBF = 2e-2


@pytest.fixture(scope="module")
def sfb():
    import paper_1511_08486_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return m


def test_mlr_tiny_five_steps(sfb):
    wl = workloads.make("mlr_tiny")
    worst = run_chain(wl, wl.steps, TOL32)
    print("mlr_tiny worst error/allowance", worst)


@pytest.mark.parametrize("J,D,P,B", [(1, 1, 1, 1), (3, 2, 1, 1), (37, 203, 3, 5), (130, 131, 2, 33),
                                     (333, 1111, 5, 77), (64, 128, 2, 16), (257, 516, 4, 40)])
def test_mlr_ragged_shapes(sfb, J, D, P, B):
    wl = workloads.make("mlr_tiny", seed=J + D, J=J, D=D, P=P, B=B, steps=3)
    run_chain(wl, 3, TOL32)


@pytest.mark.parametrize("pad", [1, 4])
def test_padded_leading_dimensions(sfb, pad):
    """ld > row length; pad=1 also breaks 16-byte row alignment (scalar paths)."""
    wl = workloads.make("mlr_tiny", seed=5, J=70, D=300, P=3, B=20, steps=2)
    run_chain(wl, 2, TOL32, pad=pad)


@pytest.mark.parametrize("variant,J,D,P,B", [(12, 260, 384, 3, 32), (11, 388, 320, 2, 48), (9, 100, 192, 3, 32)])
def test_padded_leading_dimensions_through_the_lds_dma_reconstructions(sfb, variant, J, D, P, B):
    """ld = row length + 4 keeps the rows 16-byte aligned: the LDS-DMA kernels run (not their fallbacks) and must
    honour ldw, ldu, ldv."""
    wl = workloads.make("mlr_medium", seed=variant, J=J, D=D, P=P, B=B, steps=2, pool=2)
    run_chain(wl, 2, TOL32, pad=4, plan=dict(recon_variant=variant))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("variant", [-1, 9, 11, 12, 7, 8, 10, 0])
@pytest.mark.parametrize("name,over", [("dml", dict(J=600, D=780, P=4, B=40)),      # the metric of Section 6 on 780 features
                                       ("mlr_tiny", dict(J=10, D=784, P=4, B=16)),   # ten classes on 784 pixels
                                       ("mlr_tiny", dict(J=1001, D=260, P=3, B=21)),
                                       ("l2svm", dict(J=130, D=515, P=2, B=33, density=0.05))])
def test_ragged_fp32_shapes_through_padded_factor_copies(sfb, name, over, variant):
    """J % 4, D % 128 or P*B % 32 not zero: the reconstruction copies the factors into padded rows and
    runs its LDS-DMA kernels on the copies (the planner's choice for the padded shape, or the
    single-block / two-group / pair kernel that stands for the variant asked for; variant 0 is
    register-staged and takes the factors as they are).  W has a leading dimension of D + 1."""
    wl = make_clear_of_kink(name, 77, 2, steps=2, pool=2, **over)
    run_chain(wl, 2, TOL32, pad=1, plan=None if variant < 0 else dict(recon_variant=variant))


def test_padded_factor_copies_are_what_the_reconstruction_reads(sfb):
    """Ragged shape: after sfb_reconstruct_apply the workspace holds the factors as [32 x 40] and
    [32 x 256] (37 -> 40 columns, 203 -> 256, 15 -> 32 rows), zero outside, and a dead worker's rows
    zero whatever its slot held.  A register-staged variant, or a shape the kernels take as it is,
    leaves the workspace alone."""
    dev = "cuda:0"
    J, D, P, B, eta = 37, 203, 3, 5, 0.1
    N, Np, Jp, Dp = P * B, 32, 40, 256
    rng = np.random.default_rng(5)
    W0 = rng.standard_normal((J, D)).astype(np.float32)
    Uh = rng.standard_normal((N, J)).astype(np.float32)
    Vh = rng.standard_normal((N, D)).astype(np.float32)
    active = [1, 0, 1]
    Uh_dead = Uh.copy()
    Uh_dead[B:2 * B] = np.nan                                   # what a dead worker's slot may hold
    ctx = sfb.Sfb("mlr", J, D, P, B, device=dev)
    assert ctx.workspace_bytes() >= (Np * Jp + Np * Dp) * 4
    ws = ctx._ws.view(torch.float32)
    for variant, mask in ((-1, None), (-1, active), (0, None)):
        if variant >= 0:
            ctx.set_plan(recon_variant=variant)
            ws = ctx._ws.view(torch.float32)
        ws.fill_(float("nan"))
        W = torch.from_numpy(W0).to(dev)
        U = torch.from_numpy(Uh_dead if mask else Uh).to(dev)
        V = torch.from_numpy(Vh).to(dev)
        ctx.reconstruct_apply(W, U, V, eta, active=mask)
        ctx.sync()
        live = np.repeat(np.asarray(mask if mask else [1] * P, dtype=bool), B)
        dW = oracle.delta_w(np.where(live[:, None], Uh, 0.0), Vh.astype(np.float64), P, B, active=mask)
        assert_close(W.cpu().numpy(), oracle.apply_update(W0.astype(np.float64), dW, eta), TOL32, f"W, variant {variant}")
        if variant == 0:
            assert bool(torch.isnan(ws).all())
            continue
        Uc = ws[:Np * Jp].view(Np, Jp).cpu().numpy()
        Vc = ws[Np * Jp:Np * Jp + Np * Dp].view(Np, Dp).cpu().numpy()     # 32 * 40 * 4 bytes is a multiple of 256
        want_u, want_v = np.zeros((Np, Jp), np.float32), np.zeros((Np, Dp), np.float32)
        want_u[:N, :J] = np.where(live[:, None], Uh, 0.0)
        want_v[:N, :D] = np.where(live[:, None], Vh, 0.0)
        assert np.array_equal(Uc, want_u) and np.array_equal(Vc, want_v)
    ctx.close()
    whole = sfb.Sfb("mlr", 64, 128, 2, 16, device=dev)
    ws = whole._ws.view(torch.float32)
    ws.fill_(float("nan"))
    W = torch.zeros((64, 128), device=dev)
    whole.reconstruct_apply(W, torch.ones((32, 64), device=dev), torch.ones((32, 128), device=dev), eta)
    whole.sync()
    assert bool(torch.isnan(ws).all())
    assert torch.equal(W, torch.full((64, 128), -eta * 32 / 16, device=dev))
    whole.close()


def test_a_dead_worker_in_a_whole_shape_goes_through_a_masked_copy_of_u(sfb):
    """Whole shape, one dead worker: the reconstruction copies U with that worker's rows as zeros
    (whatever the slot held) into the front of the workspace and runs its usual kernel without a
    mask.  With V off the 16-byte grid the call falls back to the register-staged kernel, which
    carries the mask itself and leaves the workspace alone.  Both match the oracle."""
    dev = "cuda:0"
    J, D, P, B, eta = 260, 512, 4, 32, 0.1
    N = P * B
    rng = np.random.default_rng(9)
    W0 = rng.standard_normal((J, D)).astype(np.float32)
    Uh = rng.standard_normal((N, J)).astype(np.float32)
    Vh = rng.standard_normal((N, D)).astype(np.float32)
    active = [1, 1, 0, 1]
    live = np.repeat(np.asarray(active, dtype=bool), B)
    U_masked = np.where(live[:, None], Uh, np.float32(0))
    want = oracle.apply_update(W0.astype(np.float64), oracle.delta_w(U_masked, Vh, P, B, active=active), eta)
    Uh_dead = np.where(live[:, None], Uh, np.float32("nan"))
    ctx = sfb.Sfb("mlr", J, D, P, B, device=dev)
    ws = ctx._ws.view(torch.float32)
    for misaligned in (False, True):
        ws.fill_(float("nan"))
        W = torch.from_numpy(W0).to(dev)
        U = torch.from_numpy(Uh_dead).to(dev)
        if misaligned:
            V = torch.empty(N * D + 1, dtype=torch.float32, device=dev)[1:].view(N, D)
            V.copy_(torch.from_numpy(Vh))
        else:
            V = torch.from_numpy(Vh).to(dev)
        ctx.reconstruct_apply(W, U, V, eta, active=active)
        ctx.sync()
        assert_close(W.cpu().numpy(), want, TOL32, f"W, dead worker, V {'off' if misaligned else 'on'} the 16-byte grid")
        if misaligned:
            assert bool(torch.isnan(ws).all())
        else:
            assert np.array_equal(ws[:N * J].view(N, J).cpu().numpy(), U_masked)
    ctx.close()


@pytest.mark.parametrize("name,over,tiles", [
    ("mlr_tiny", dict(J=10, D=784, P=12, B=100), 14),        # ragged: padded copies, then slices of their 1216 rows
    ("mlr_tiny", dict(J=64, D=128, P=16, B=128), 2),         # whole: two tiles, 64 stages
    ("dml", dict(J=100, D=192, P=8, B=256), 8),              # 192 -> 256 columns: 2 x 4 tiles
    ("l2svm", dict(J=48, D=320, P=4, B=300, density=0.05), 6),   # 320 -> 384 columns
])
def test_few_tiles_many_pairs_split_the_pairs_over_workgroups(sfb, name, over, tiles):
    """J x D of a few 64 x 64 tiles with thousands of factor pairs: the plan cuts the pairs into slices, one
    workgroup per tile and slice stores bare sums, a second kernel adds them in slice order.  Two steps against
    the oracle, the same call twice bit for bit, and with a dead worker."""
    wl = make_clear_of_kink(name, 91, 2, steps=2, pool=2, **over)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    grid = ctx.plan_info()["recon_grid"]
    assert grid % tiles == 0 and grid // tiles > 1, f"the plan does not split: {grid} workgroups for {tiles} tiles"
    ctx.close()
    run_chain(wl, 2, TOL32, pad=0)
    # determinism and the mask, on the reconstruction alone
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    rng = np.random.default_rng(3)
    Uh = rng.standard_normal((wl.N, wl.J)).astype(np.float32)
    Vh = rng.standard_normal((wl.N, wl.D)).astype(np.float32)
    active = [1] * wl.P
    active[1] = 0
    for mask in (None, active):
        got = []
        for _ in range(2):
            W = torch.from_numpy(wl.W0).to(dev)
            ctx.reconstruct_apply(W, torch.from_numpy(Uh).to(dev), torch.from_numpy(Vh).to(dev), wl.eta, active=mask)
            ctx.sync()
            got.append(W)
        assert torch.equal(got[0], got[1])
        dW = oracle.delta_w(Uh, Vh, wl.P, wl.B, active=mask)
        mag = wl.eta * oracle.delta_w(np.abs(Uh), np.abs(Vh), wl.P, wl.B, active=mask)
        assert_close(got[0].cpu().numpy(), oracle.apply_update(wl.W0.astype(np.float64), dW, wl.eta), TOL32,
                     f"W, mask {mask}", terms=mag)
    ctx.close()


def test_w_alone_off_the_16_byte_grid_keeps_the_pair_kernel(sfb):
    """Whole shape with 256 tiles of 128 x 128 (the pair kernel's plan), aligned U and V, and a W whose leading
    dimension is D + 1: the reconstruction takes W entry by entry instead of falling back to register staging.
    Checked against the oracle on the update itself."""
    dev = "cuda:0"
    J, D, P, B, eta = 2048, 2048, 2, 32, 0.1
    N = P * B
    rng = np.random.default_rng(17)
    W0 = (0.1 * rng.standard_normal((J, D))).astype(np.float32)
    Uh = rng.standard_normal((N, J)).astype(np.float32)
    Vh = rng.standard_normal((N, D)).astype(np.float32)
    ctx = sfb.Sfb("mlr", J, D, P, B, device=dev)
    assert ctx.plan_info()["recon_grid"] == 256
    Wbuf = torch.full((J, D + 1), 7.0, dtype=torch.float32, device=dev)
    W = Wbuf[:, :D]
    W.copy_(torch.from_numpy(W0))
    ctx.reconstruct_apply(W, torch.from_numpy(Uh).to(dev), torch.from_numpy(Vh).to(dev), eta)
    ctx.sync()
    dW = oracle.delta_w(Uh, Vh, P, B)
    mag = eta * oracle.delta_w(np.abs(Uh), np.abs(Vh), P, B)
    assert_close(W.cpu().numpy(), oracle.apply_update(W0.astype(np.float64), dW, eta), TOL32, "W", terms=mag)
    assert bool((Wbuf[:, D] == 7.0).all())                               # the column beyond D is not W's
    ctx.close()


def test_scores_far_beyond_the_range_of_exp_do_not_overflow(sfb):
    """Scores of +-150 and more (exp overflows fp32 beyond 88.7): the factor kernel subtracts the row maximum, so
    u = softmax - e_y and the loss stay finite and match the oracle.  The bar is 1e-2 here: an fp32 score of
    magnitude 150 carries an absolute error of 1e-5 to 1e-4, which the softmax turns into that relative error of
    a probability, so the 1e-4 bar of the other tests does not apply to this input."""
    dev = "cuda:0"
    wl = workloads.make("mlr_tiny", seed=13, J=40, D=64, P=4, B=32, steps=1, pool=1)
    W0 = (wl.W0 * 2000.0).astype(np.float32)
    b = wl.batch(0)
    Z = oracle.scores(W0.astype(np.float64), b["A"].astype(np.float64))
    assert np.abs(Z).max() > 150.0
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    db, dy = to_device(wl, b, dev)
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(torch.from_numpy(W0).to(dev), db, dy, U, V, loss)
    ctx.sync()
    assert bool(torch.isfinite(U).all()) and bool(torch.isfinite(loss).all())
    Uo, Vo, _, fo = oracle.step(wl.model, W0.astype(np.float64), b, wl.P, wl.B, wl.eta)
    assert_close(U.cpu().numpy(), Uo, 1e-2, "U")
    assert_close(loss.cpu().numpy(), fo, 1e-4, "loss")       # the loss is a difference of scores: no such amplification
    ctx.close()


def test_mlr_medium_hundred_steps(sfb):
    wl = workloads.make("mlr_medium")
    worst = run_chain(wl, wl.steps, TOL32, check_every=7)
    print("mlr_medium worst error/allowance", worst)


@pytest.mark.parametrize("plan", [dict(fwd_bm=64, fwd_bn=64, fwd_split_k=3, recon_variant=0),
                                  dict(fwd_bm=128, fwd_bn=64, fwd_split_k=1, recon_variant=2),
                                  dict(fwd_bm=64, fwd_bn=128, fwd_split_k=16, recon_variant=3),
                                  dict(fwd_bm=128, fwd_bn=128, fwd_split_k=5, recon_variant=1),
                                  dict(fwd_bm=128, fwd_bn=128, fwd_split_k=2, recon_variant=4),
                                  dict(fwd_bm=64, fwd_bn=64, fwd_split_k=2, recon_variant=5),
                                  dict(fwd_bm=128, fwd_bn=64, fwd_split_k=7, recon_variant=6)])
def test_every_tile_variant(sfb, plan):
    wl = workloads.make("mlr_medium", J=520, D=1000, P=4, B=50, steps=2, pool=2)
    run_chain(wl, 2, TOL32, plan=plan)


@pytest.mark.parametrize("variant", [7, 8, 10, 12])
@pytest.mark.parametrize("J,D,P,B", [(520, 1024, 4, 48), (1000, 4096, 8, 64), (36, 256, 1, 32), (2000, 8192, 1, 16)])
def test_lds_dma_reconstruct_variants(sfb, variant, J, D, P, B):
    """Shapes the LDS-DMA staging accepts (D % 128 == 0, J % 4 == 0, N % 32 == 0)."""
    wl = workloads.make("mlr_medium", seed=variant, J=J, D=D, P=P, B=B, steps=3, pool=2)
    run_chain(wl, 3, TOL32, plan=dict(recon_variant=variant))


@pytest.mark.parametrize("J,D,P,B", [(260, 384, 3, 32), (128, 128, 2, 32), (132, 256, 5, 32), (4, 128, 1, 32),
                                     (1000, 4096, 8, 64), (516, 512, 7, 32)])
def test_two_group_reconstruct_variant(sfb, J, D, P, B):
    """Variant 12 (128 x 128 tiles, eight wavefronts in two groups that take the stages of 32 pairs in turn;
    D % 128 == 0, J % 4 == 0, N % 32 == 0): one stage (the second group has none), two, three, five, seven
    (odd counts) and sixteen; ragged last strip and last row tile; a tile of four rows."""
    wl = workloads.make("mlr_medium", seed=12, J=J, D=D, P=P, B=B, steps=3, pool=2)
    run_chain(wl, 3, TOL32, plan=dict(recon_variant=12))


@pytest.mark.parametrize("J,D,P,B", [(600, 4096, 8, 128), (520, 1024, 4, 48), (36, 256, 1, 32), (64, 64, 2, 32),
                                     (100, 192, 3, 32), (4, 64, 1, 128), (1000, 4096, 8, 64)])
def test_single_block_reconstruct_variant(sfb, J, D, P, B):
    """Variant 9 (64 x 64 tiles, one 32 x 32 block per wavefront; D % 64 == 0, J % 4 == 0, N % 32 == 0):
    ring of one to many stages (N = 32 ... 1024), ragged last row tile, a single tile."""
    wl = workloads.make("mlr_medium", seed=9, J=J, D=D, P=P, B=B, steps=3, pool=2)
    run_chain(wl, 3, TOL32, plan=dict(recon_variant=9))


@pytest.mark.parametrize("J,D,P,B", [(600, 4096, 8, 128), (388, 1024, 4, 48), (256, 256, 1, 32), (96, 64, 2, 32),
                                     (352, 192, 3, 32), (68, 64, 1, 128), (1000, 4096, 8, 64), (440, 128, 1, 64),
                                     (600, 128, 5, 32), (104, 64, 7, 32)])
def test_pair_split_reconstruct_variant(sfb, J, D, P, B):
    """Variant 11 (tiles of 3 to 5 row blocks x 64 columns, eight wavefronts = two column blocks x two halves of
    every stage's pairs x two groups that take the stages in turn; D % 64 == 0, J % 4 == 0, N % 32 == 0): each of
    the three tile heights (J = 600, 388, 1000, 440: five row blocks; 256, 352: four; 96, 68: three), ragged
    last row tile and ragged last row block, one stage (N = 32: the second group has none), two, three (N = 96:
    an odd count) and many (N = 1024), a single tile."""
    wl = workloads.make("mlr_medium", seed=11, J=J, D=D, P=P, B=B, steps=3, pool=2)
    run_chain(wl, 3, TOL32, plan=dict(recon_variant=11))


def test_pair_split_variant_is_what_the_plan_picks_for_600_rows_and_falls_back_when_it_must(sfb):
    import paper_1511_08486_amd as m
    ctx = m.Sfb("dml", 600, 4096, 8, 128, device="cuda:0")
    assert ctx.plan_info()["recon_grid"] == 4 * 64           # four row tiles of five row blocks x 64-column tiles
    ctx.close()
    # shapes the kernel does not take run the single-block kernel or, failing that too, the others: J = 40
    # (two row blocks), D % 64 != 0, N % 32 != 0
    wl = workloads.make("mlr_medium", seed=12, J=40, D=128, P=2, B=32, steps=2, pool=2)
    run_chain(wl, 2, TOL32, plan=dict(recon_variant=11))
    wl = workloads.make("mlr_medium", seed=13, J=600, D=200, P=3, B=20, steps=2, pool=2)
    run_chain(wl, 2, TOL32, plan=dict(recon_variant=11))


def test_single_block_variant_falls_back_when_it_must(sfb):
    import paper_1511_08486_amd as m
    ctx = m.Sfb("mlr", 1000, 4096, 8, 64, device="cuda:0")
    assert ctx.plan_info()["recon_grid"] == 256              # a tie in the block count keeps the 128 x 128 tiles
    ctx.close()
    # shapes the kernel does not take (D % 64 != 0, N % 32 != 0, a dead worker) run the other kernels
    wl = workloads.make("mlr_medium", seed=10, J=72, D=200, P=3, B=20, steps=2, pool=2)
    run_chain(wl, 2, TOL32, plan=dict(recon_variant=9))


def test_dml_twenty_steps(sfb):
    wl = workloads.make("dml", seed=1)    # seed 1 keeps every pair > 1e-4 from the hinge kink
    worst = run_chain(wl, wl.steps, TOL32, check_every=3)
    print("dml worst error/allowance", worst)


def test_dml_ragged(sfb):
    wl = make_clear_of_kink("dml", 2, 3, J=45, D=333, P=3, B=21, steps=3)
    run_chain(wl, 3, TOL32)


@pytest.mark.timeout(600)
def test_l2svm_twenty_steps(sfb):
    wl = workloads.make("l2svm")
    worst = run_chain(wl, wl.steps, TOL32, check_every=4)
    print("l2svm worst error/allowance", worst)


@pytest.mark.parametrize("dense_scores", [False, True])
def test_l2svm_ragged_and_empty_rows(sfb, dense_scores):
    wl = workloads.make("l2svm", seed=3, J=77, D=501, P=3, B=11, steps=2, density=0.05)
    # make two rows empty and one row a single entry
    for b in wl.batches:
        per = b["rowptr"][1]
        counts = np.full(wl.N, per)
        counts[[0, 7]] = 0
        counts[3] = 1
        keep = np.concatenate([np.arange(r * per, r * per + counts[r]) for r in range(wl.N)]).astype(np.int64)
        b["col"], b["val"] = b["col"][keep], b["val"][keep]
        b["rowptr"] = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    run_chain(wl, 2, TOL32, plan=dict(fwd_dma=3) if dense_scores else dict(fwd_dma=33))


def test_l2svm_rows_longer_than_the_score_kernel_prefetches(sfb):
    """The score kernel requests the first 3 x 64 stored entries of a row up front and loops over the rest: rows of
    451 entries (eight slabs), and of 193, 192, 191, 129, 128, 65, 64, 63, 1 and 0 entries around the slab
    boundaries, the last row ending exactly at the end of the arrays."""
    wl = workloads.make("l2svm", seed=31, J=37, D=2048, P=3, B=7, steps=2, density=0.22)
    lengths = [451, 193, 192, 191, 129, 128, 65, 64, 63, 1, 0]
    for b in wl.batches:
        per = b["rowptr"][1]
        assert per == 451
        counts = np.array([lengths[r % len(lengths)] for r in range(wl.N)])
        counts[-1] = 451
        keep = np.concatenate([np.arange(r * per, r * per + counts[r]) for r in range(wl.N)]).astype(np.int64)
        b["col"], b["val"] = b["col"][keep], b["val"][keep]
        b["rowptr"] = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    run_chain(wl, 2, TOL32, plan=dict(fwd_dma=33))          # from the entries, whatever the cost comparison says


def test_l2svm_dense_score_fallback_full_size(sfb):
    wl = workloads.make("l2svm", pool=2)
    run_chain(wl, 2, TOL32, plan=dict(fwd_dma=3))


@pytest.mark.timeout(900)
def test_l2svm_batch_with_no_stored_entries(sfb):
    """nnz = 0: every score is 0, u_j = -2 t_j, V = 0, and W still moves by eta/B * sum u v^T = 0."""
    wl = workloads.make("l2svm", seed=5, J=40, D=256, P=2, B=8, steps=1, pool=1)
    b = wl.batch(0)
    b["col"], b["val"] = b["col"][:0], b["val"][:0]
    b["rowptr"] = np.zeros(wl.N + 1, dtype=np.int32)
    for plan in (None, dict(fwd_dma=33), dict(fwd_dma=3)):
        run_chain(wl, 1, TOL32, plan=plan)


@pytest.mark.parametrize("model,J", [("mlr", 13001), ("dml", 12800), ("l2svm", 12290)])
def test_rows_longer_than_the_register_kernel_covers(sfb, model, J):
    """J > 12288 takes the three-pass factor kernel."""
    name = {"mlr": "mlr_tiny", "dml": "dml", "l2svm": "l2svm"}[model]
    over = dict(J=J, D=64, P=2, B=3, steps=2, pool=1)
    if model == "l2svm":
        over["density"] = 0.2
    wl = workloads.make(name, seed=7, **over)
    if model == "dml":
        wl.W0 *= 0.05          # keep |z|^2 well below the hinge kink with 12800 latent dimensions
    run_chain(wl, 2, TOL32)


@pytest.mark.timeout(1500)
def test_mlr_large_bf16_twenty_steps(sfb, capsys):
    """The configuration's whole chain (20 steps, pool of 4 batches): bf16 rounding of the W tiles in
    the score pass and of U in the reconstruction compounds over the steps; U, V, W, the loss and the
    update itself are compared with the oracle at steps 0, 3, 6, ..., 18, 19."""
    wl = workloads.make("mlr_large")
    assert wl.steps == 20 and len(wl.batches) == 4
    def say(line):                      # the fp64 oracle needs several seconds per step at this size
        with capsys.disabled():
            print(line, flush=True)
    worst = run_chain(wl, wl.steps, TOLBF, check_every=3, progress=say)
    print("mlr_large worst error/allowance", worst)


def test_bf16_ragged(sfb):
    wl = workloads.make("mlr_large", seed=4, J=300, D=1004, P=3, B=30, steps=2, pool=2)
    run_chain(wl, 2, TOLBF)


@pytest.mark.parametrize("J,D,P,B", [(300, 1024, 4, 40), (130, 96, 2, 64), (1000, 2048, 8, 64)])
def test_bf16_matrix_core_path(sfb, J, D, P, B):
    """Shapes that take the bf16 MFMA kernels (D % 32 == 0, N >= 128, aligned rows)."""
    wl = workloads.make("mlr_large", seed=J, J=J, D=D, P=P, B=B, steps=3, pool=2)
    run_chain(wl, 3, TOLBF)


def test_bf16_dead_worker_and_plain_sum(sfb):
    wl = workloads.make("mlr_large", seed=9, J=260, D=512, P=4, B=48, steps=1, pool=1)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype="bf16", device=dev)
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(W, db, dy, U, V, loss)
    active = [1, 0, 1, 1]
    U[wl.B:2 * wl.B] = float("nan")                     # a dead worker's slot may hold anything
    ctx.reconstruct_apply(W, U, V, eta=0.2, scale=1.0, active=active)
    ctx.sync()
    Uo, Vo, fo = oracle.factors(wl.model, wl.W0, b)
    want = oracle.apply_update(wl.W0, oracle.delta_w(Uo, Vo, wl.P, wl.B, active) * wl.B, 0.2)
    assert_close(W.cpu().numpy(), want, TOLBF, "W, bf16, dead worker")
    U[wl.B:2 * wl.B] = float("nan")
    upd = fresh_update(ctx, U, V, 0.2, W, scale=1.0, active=active)
    mag = 0.2 * wl.B * oracle.delta_w(np.abs(Uo), np.abs(Vo), wl.P, wl.B, active)      # sum of |terms| (scale 1)
    assert_close(upd.cpu().numpy(), want - wl.W0, TOLBF, "-eta*dW, bf16, dead worker", terms=mag)
    assert np.array_equal(V.float().cpu().numpy(), b["A"])
    ctx.close()


def test_worker_calls_equal_batched_call_and_mask_drops_a_worker(sfb):
    wl = workloads.make("mlr_medium", J=200, D=520, P=4, B=24, steps=1, pool=1)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(W, db, dy, U, V, loss)
    U2, V2, loss2 = alloc_factors(wl, dev)
    for p in reversed(range(wl.P)):          # any commit order gives the same buffers
        rows = slice(p * wl.B, (p + 1) * wl.B)
        ctx.compute_factors_worker(W, sfb.SfbBatch(a=db.a[rows]), dy[rows], p, U2, V2, loss2)
    ctx.sync()
    Uo, Vo, fo = oracle.factors(wl.model, wl.W0, b)
    for got in (U, U2):
        assert_close(got.cpu().numpy(), Uo, TOL32, "U")
    assert torch.equal(V, V2) and np.array_equal(V.cpu().numpy(), b["A"])      # v = a, bit for bit
    assert_close(loss2.cpu().numpy(), fo, TOL32, "loss")
    # MLR invariant on the device buffer: residual rows sum to zero
    assert float(U.sum(dim=1).abs().max()) < 1e-5
    # reconstruction with worker 2 dead, plain-sum scale
    active = [1, 1, 0, 1]
    W1 = W.clone()
    ctx.reconstruct_apply(W1, U, V, eta=0.3, scale=1.0, active=active)
    ctx.sync()
    want = oracle.apply_update(wl.W0, oracle.delta_w(Uo, Vo, wl.P, wl.B, active) * wl.B, 0.3)
    assert_close(W1.cpu().numpy(), want, TOL32, "W with dead worker")
    upd = fresh_update(ctx, U, V, 0.3, W, scale=1.0, active=active)
    mag = 0.3 * wl.B * oracle.delta_w(np.abs(Uo), np.abs(Vo), wl.P, wl.B, active)
    assert_close(upd.cpu().numpy(), want - wl.W0, TOL32, "-eta*dW with dead worker", terms=mag)
    # a dead worker's buffers may hold anything, even NaN
    U3, V3 = U.clone(), V.clone()
    U3[2 * wl.B:3 * wl.B] = float("nan")
    V3[2 * wl.B:3 * wl.B] = float("inf")
    W2 = W.clone()
    ctx.reconstruct_apply(W2, U3, V3, eta=0.3, scale=1.0, active=active)
    ctx.sync()
    assert torch.equal(W1, W2)
    ctx.close()


def test_zero_factors_leave_w_bit_identical_and_eta_zero_is_identity(sfb):
    wl = workloads.make("dml", seed=1, J=96, D=260, P=2, B=40, steps=1, pool=1)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    db, dy = to_device(wl, wl.batch(0), dev)
    U, V, loss = alloc_factors(wl, dev)
    W = torch.zeros((wl.J, wl.D), device=dev)            # z = 0 -> u = 0 -> W stays 0
    ctx.step(W, db, dy, U, V, 0.5, loss=loss)
    ctx.sync()
    assert not U.any() and not W.any()
    assert np.array_equal(loss.cpu().numpy(), np.where(wl.batch(0)["y"] == 1, 0.0, 1.0).astype(np.float32))
    W = torch.from_numpy(wl.W0).to(dev)
    ctx.step(W, db, dy, U, V, 0.0)
    ctx.sync()
    assert torch.equal(W.cpu(), torch.from_numpy(wl.W0))
    ctx.close()


def test_results_do_not_depend_on_the_launch_plan_beyond_rounding(sfb):
    """Same inputs, two different tilings: W agrees to fp32 rounding (replicas that tile
    differently would drift only at this level)."""
    wl = workloads.make("mlr_medium", J=300, D=700, P=4, B=32, steps=1, pool=1)
    outs = []
    for plan in (dict(fwd_split_k=1, recon_variant=0), dict(fwd_split_k=4, recon_variant=2)):
        dev = "cuda:0"
        ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
        ctx.set_plan(**plan)
        db, dy = to_device(wl, wl.batch(0), dev)
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, _ = alloc_factors(wl, dev)
        ctx.step(W, db, dy, U, V, wl.eta)
        ctx.sync()
        outs.append(W.cpu().numpy())
        ctx.close()
    assert_close(outs[0], outs[1], 1e-6, "W across plans")


def test_determinism_same_call_twice_is_bit_identical(sfb):
    wl = workloads.make("mlr_medium", J=500, D=2048, P=8, B=32, steps=1, pool=1)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    db, dy = to_device(wl, wl.batch(0), dev)
    res = []
    for _ in range(2):
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, _ = alloc_factors(wl, dev)
        ctx.step(W, db, dy, U, V, wl.eta)
        ctx.sync()
        res.append((W.clone(), U.clone()))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    ctx.close()


@pytest.mark.parametrize("name,seed,steps,override", [
    ("mlr_medium", 0, 100, {}),
    ("dml", 1, 20, {}),
    ("mlr_tiny", 5, 3, dict(J=130, D=256, P=3, B=40)),      # ragged tiles, one slice of D
    ("mlr_tiny", 6, 3, dict(J=64, D=96, P=2, B=16)),        # D = 3 chunks: the loop's tail
    ("mlr_tiny", 7, 3, dict(J=37, D=203, P=3, B=5)),        # D % 32 != 0: the switch is ignored
])
def test_split_bf16_scores(sfb, name, seed, steps, override):
    """fp32 scores computed as six bf16 term products per product (plan bit 2): same parity bar
    as the fp32 matrix-core kernels, for all steps of a chain."""
    wl = workloads.make(name, seed=seed, **override)
    worst = run_chain(wl, steps, TOL32, check_every=1 if steps <= 20 else 5, plan=dict(fwd_dma=5))
    print(f"{name} {override}: split-bf16 scores, worst error/allowance {worst}")


@pytest.mark.parametrize("name,seed,steps,override", [
    ("mlr_medium", 0, 100, {}),
    ("dml", 1, 20, {}),
    ("l2svm", 0, 5, {}),
    ("mlr_tiny", 5, 3, dict(J=132, D=260, P=2, B=32)),      # ragged tiles in both directions
    ("mlr_tiny", 6, 3, dict(J=64, D=128, P=3, B=32)),       # N = 96 = 3 chunks: the loop's tail
    ("mlr_tiny", 8, 3, dict(J=8, D=4, P=1, B=32)),          # one chunk, tile far larger than W
    ("mlr_tiny", 7, 3, dict(J=37, D=203, P=3, B=5)),        # J % 4 != 0, N % 32 != 0: the switch is ignored
])
def test_split_bf16_scores_and_reconstruction(sfb, name, seed, steps, override):
    """Both contractions as split-bf16 products (plan bits 2 and 3), whole chains against the oracle."""
    wl = workloads.make(name, seed=seed, **override)
    worst = run_chain(wl, steps, TOL32, check_every=1 if steps <= 20 else 5, plan=dict(fwd_dma=13))
    print(f"{name} {override}: split-bf16 scores and reconstruction, worst error/allowance {worst}")


def test_split_bf16_reconstruction_with_a_dead_worker_falls_back(sfb):
    """A mask of live workers is not covered by the split kernel: the call must still be right."""
    dev = "cuda:0"
    wl = workloads.make("mlr_tiny", seed=9, J=64, D=128, P=4, B=32)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    ctx.set_plan(fwd_dma=13)
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, _ = alloc_factors(wl, dev)
    active = [1, 0, 1, 1]
    ctx.step(W, db, dy, U, V, wl.eta, active=active)
    ctx.sync()
    _, _, want, _ = oracle.step(wl.model, wl.W0, b, wl.P, wl.B, wl.eta, active=active)
    assert_close(W.cpu().numpy(), want, TOL32, "W, split plan, dead worker")
    ctx.close()


def test_split_bf16_scores_are_as_accurate_as_fp32_mfma(sfb):
    """The exact three-way split keeps fp32's 24 bits: against the fp64 oracle the split-bf16
    scores are at least as close as the fp32 matrix-core scores."""
    dev = "cuda:0"
    wl = workloads.make("mlr_medium")
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    want = oracle.scores(wl.W0.astype(np.float64), b["A"].astype(np.float64))
    errs = {}
    for mode in (1, 5):
        ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
        ctx.set_plan(fwd_dma=mode)
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, loss = alloc_factors(wl, dev)
        ctx.compute_factors(W, db, dy, U, V, loss)
        ctx.sync()
        # the loss is logsumexp(z) - z_y: compare it and the factors, both smooth functions of the scores
        fo, Uo = oracle.loss_and_u(wl.model, want, b["y"])
        errs[mode] = (float(np.abs(U.cpu().numpy() - Uo).max()), float(np.abs(loss.cpu().numpy() - fo).max()))
        ctx.close()
    print("max abs error of (U, loss): fp32 mfma", errs[1], " split-bf16", errs[5])
    assert errs[5][0] <= 2.0 * errs[1][0] + 1e-9 and errs[5][1] <= 2.0 * errs[1][1] + 1e-7


@pytest.mark.parametrize("dtype,P,B", [("f32", 1, 32), ("bf16", 4, 32)])
def test_w_with_more_than_2_to_31_entries(sfb, dtype, P, B):
    """J * D = 34000 * 65536 = 2.2e9 entries (8.9 GB): every kernel's addressing past 2^31 elements.
    W is the fp32 outer product of two vectors, so the oracle can form any block of it without holding
    it; the scores, U and the loss are compared in full, the updated W on sampled rows (first, last,
    and around the 2^31-th element) and columns."""
    import paper_1511_08486_amd as m
    J, D, N = 34000, 65536, P * B
    tol = TOL32 if dtype == "f32" else 2e-2
    vdt = torch.float32 if dtype == "f32" else torch.bfloat16
    rng = np.random.default_rng(11)
    a = (0.1 * rng.standard_normal(J)).astype(np.float32)
    b = rng.standard_normal(D).astype(np.float32)
    A = (rng.standard_normal((N, D)) / np.sqrt(D)).astype(np.float32)
    if dtype == "bf16":
        A = workloads.bf16_round(A)[1]
    y = rng.integers(0, J, size=N).astype(np.int32)
    dev = "cuda:0"
    W = torch.outer(torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev))          # fl32(a_j * b_d)
    ctx = m.Sfb("mlr", J, D, P, B, dtype=dtype, device=dev)
    U = torch.empty((N, J), dtype=torch.float32, device=dev)
    V = torch.empty((N, D), dtype=vdt, device=dev)
    loss = torch.empty((N,), dtype=torch.float32, device=dev)
    eta = 0.5
    ctx.step(W, m.SfbBatch(a=torch.from_numpy(A).to(vdt).to(dev)), torch.from_numpy(y).to(dev), U, V, eta, loss=loss)
    ctx.sync()

    def w_block(rows, cols):                    # the same fp32 products, widened
        return (a[rows, None] * b[None, cols]).astype(np.float64)
    A64 = A.astype(np.float64)
    Z = np.empty((N, J))
    for r0 in range(0, J, 2000):
        rows = np.arange(r0, min(J, r0 + 2000))
        Z[:, rows] = A64 @ w_block(rows, np.arange(D)).T
    want_loss, Uo = oracle.loss_and_u("mlr", Z, y)                  # the oracle's pinned factor step
    assert_close(U.cpu().numpy(), Uo, tol, "U")
    assert_close(loss.cpu().numpy(), want_loss, tol, "loss")
    assert torch.equal(V.float().cpu(), torch.from_numpy(A))
    edge = (1 << 31) // D                                           # the row holding the 2^31-th element
    rows = np.unique(np.concatenate([np.arange(0, 3), np.arange(edge - 2, edge + 3), np.arange(J - 3, J),
                                     rng.integers(0, J, size=40), y[:4]]))
    cols = np.unique(np.concatenate([np.arange(0, 4), np.arange(D - 4, D), rng.integers(0, D, size=120)]))
    want_w = oracle.apply_update(w_block(rows, cols), oracle.delta_w(Uo[:, rows], A64[:, cols], P, B), eta)
    got_w = W[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
    assert_close(got_w, want_w, tol, "sampled W")
    # the update really happened on those entries
    assert np.abs(want_w - w_block(rows, cols)).max() > 1e-4
    ctx.prox(W, "l2sq", 0.5, 1.0)                                   # streaming kernels past 2^31 elements too
    ctx.sync()
    got_p = W[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
    assert_close(got_p, oracle.prox("l2sq", want_w, 0.5, 1.0), tol, "sampled W after the proximal step")
    ctx.close()


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        model = ("mlr", "dml", "l2svm")[i % 3]
        # a mix of ragged sizes and sizes on the kernels' alignment boundaries (4, 32, 64, 128)
        J = int(rng.choice([rng.integers(1, 300), 4 * rng.integers(1, 80), 64 * rng.integers(1, 6)]))
        D = int(rng.choice([rng.integers(1, 700), 64 * rng.integers(1, 12), 128 * rng.integers(1, 6)]))
        P = int(rng.integers(1, 6))
        B = int(rng.choice([rng.integers(1, 40), 16, 32]))
        pad = int(rng.choice([0, 0, 1, 4]))
        out.append((model, J, D, P, B, pad, 100 + i))
    return out


@pytest.mark.parametrize("model,J,D,P,B,pad,seed", _random_shapes(36, 2024))
def test_random_shapes_through_the_default_plan(sfb, model, J, D, P, B, pad, seed):
    """Whatever kernel the planner picks for a shape (LDS-DMA or register staging, 128-, 64-row or
    single-block tiles, CSR or dense scores), two steps match the oracle."""
    name = {"mlr": "mlr_tiny", "dml": "dml", "l2svm": "l2svm"}[model]
    over = dict(J=J, D=D, P=P, B=B, steps=2, pool=2)
    if model == "l2svm":
        over["density"] = max(0.05, 1.5 / D)
    wl = make_clear_of_kink(name, seed, 2, **over)      # metric learning: a seed whose pairs stay 1e-4 off the kink
    run_chain(wl, 2, TOL32, pad=pad)


@pytest.mark.parametrize("name,over", [("mlr_medium", dict(J=256, D=512, P=80, B=50)),
                                       ("dml", dict(J=64, D=256, P=32, B=128)),
                                       ("l2svm", dict(J=128, D=1024, P=64, B=64, density=0.02))])
def test_many_workers_and_long_contractions(sfb, name, over):
    """N = P*B of 4000-4096 factor pairs (125-128 stages of the reconstruction ring), more than
    64 workers (no mask is involved, so the 64-worker limit of the mask does not apply)."""
    wl = make_clear_of_kink(name, 5, 2, steps=2, pool=2, **over)
    run_chain(wl, 2, TOL32)


@pytest.mark.parametrize("dense_scores", [False, True])
def test_csr_worker_calls_address_the_shared_arrays_through_their_row_pointers(sfb, dense_scores):
    """A worker's share of a CSR batch handed over without copying: the slice rowptr[p*B : (p+1)*B + 1] of
    the batch's row pointers (first entry non-zero for p > 0) with the batch's own col / val arrays."""
    wl = workloads.make("l2svm", seed=3, J=68, D=300, P=4, B=9, density=0.06, steps=1, pool=1)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    ctx.set_plan(fwd_dma=3 if dense_scores else 33)
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(W, db, dy, U, V, loss)
    U2, V2, loss2 = alloc_factors(wl, dev)
    for p in (2, 0, 3, 1):
        rp = db.rowptr[p * wl.B:(p + 1) * wl.B + 1]
        assert p == 0 or int(rp[0]) > 0
        share = sfb.SfbBatch(rowptr=rp, col=db.col, val=db.val)
        ctx.compute_factors_worker(W, share, dy[p * wl.B:(p + 1) * wl.B], p, U2, V2, loss2)
    ctx.sync()
    Uo, Vo, fo = oracle.factors(wl.model, wl.W0, b)
    assert torch.equal(V, V2) and np.array_equal(V.cpu().numpy(), Vo.astype(np.float32))
    for got in (U, U2):
        assert_close(got.cpu().numpy(), Uo, TOL32, "U")
    assert_close(loss2.cpu().numpy(), fo, TOL32, "loss")
    ctx.close()


@pytest.mark.parametrize("dense_scores", [False, True])
def test_csr_columns_in_any_order_within_a_row(sfb, dense_scores):
    """The CSR rows need not be sorted by column (the header promises it): every row's entries are
    shuffled, the step must not change beyond rounding."""
    wl = workloads.make("l2svm", seed=8, J=96, D=640, P=3, B=11, density=0.05, steps=2, pool=2)
    rng = np.random.default_rng(8)
    for b in wl.batches:
        for r in range(wl.N):
            lo, hi = int(b["rowptr"][r]), int(b["rowptr"][r + 1])
            perm = rng.permutation(hi - lo)
            b["col"][lo:hi] = b["col"][lo:hi][perm]
            b["val"][lo:hi] = b["val"][lo:hi][perm]
        assert np.any(np.diff(b["col"][:int(b["rowptr"][1])]) < 0)
    run_chain(wl, 2, TOL32, plan=dict(fwd_dma=3) if dense_scores else dict(fwd_dma=33))


@pytest.mark.parametrize("dense_scores,D,density", [(False, 320, 0.05), (True, 320, 0.05), (False, 16500, 0.002)])
def test_csr_column_repeated_inside_a_row_counts_as_the_sum_of_its_values(sfb, dense_scores, D, density):
    """The header defines it: a column that appears twice in a row contributes the sum of its values,
    in the scores (from the stored entries or from the dense rows) and in v_i alike.  D = 16500: a row
    no longer fits the LDS buffer the dense rows are built in (the entries are added in memory) nor do
    four rows of W fit for the scores from the stored entries (dense scores on the densified rows)."""
    wl = workloads.make("l2svm", seed=21, J=52, D=D, P=3, B=10, density=density, steps=2, pool=2)
    rng = np.random.default_rng(21)
    for b in wl.batches:
        per = int(b["rowptr"][1])
        for r in range(wl.N):
            lo = r * per
            # entries 0 and 1 of the row move onto the columns of entries 2 and 3: two doubled columns
            b["col"][lo:lo + 2] = b["col"][lo + 2:lo + 4]
            perm = rng.permutation(per)
            b["col"][lo:lo + per] = b["col"][lo:lo + per][perm]
            b["val"][lo:lo + per] = b["val"][lo:lo + per][perm]
        first = b["col"][:per]
        assert len(np.unique(first)) == per - 2
    run_chain(wl, 2, TOL32, plan=dict(fwd_dma=3) if dense_scores else dict(fwd_dma=33))


def _misaligned(t, off=1):
    """A copy of the 2-D tensor t whose rows start `off` elements into rows `off + 2` elements longer:
    neither the base address nor the row stride keeps the 16-byte alignment of the fast paths."""
    buf = torch.zeros((t.shape[0], t.shape[1] + off + 2), dtype=t.dtype, device=t.device)
    view = buf[:, off:off + t.shape[1]]
    view.copy_(t)
    return view


@pytest.mark.parametrize("name,over,tol", [("mlr_medium", dict(J=200, D=512, P=4, B=32), TOL32),
                                           ("dml", dict(J=64, D=256, P=2, B=64), TOL32),
                                           ("l2svm", dict(J=64, D=512, P=2, B=32, density=0.04), TOL32),
                                           ("mlr_large", dict(J=300, D=1024, P=4, B=40), TOLBF)])
def test_any_alignment_is_accepted(sfb, name, over, tol):
    """Every dense operand starts one element past an aligned address and has a row stride that is not a
    multiple of four elements: the kernels must take their scalar paths and still match the oracle."""
    wl = workloads.make(name, seed=12, steps=2, pool=2, **over)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    vdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    W = _misaligned(torch.from_numpy(wl.W0).to(dev))
    U = _misaligned(torch.zeros((wl.N, wl.J), device=dev))
    V = _misaligned(torch.zeros((wl.N, wl.D), dtype=vdt, device=dev))
    loss = torch.zeros(wl.N + 1, device=dev)[1:]
    Wo = wl.W0.astype(np.float64)
    for t in range(2):
        b = wl.batch(t)
        db, dy = to_device(wl, b, dev)
        if db.a is not None:
            db.a = _misaligned(db.a)
        if db.a2 is not None:
            db.a2 = _misaligned(db.a2)
        assert W.data_ptr() % 16 != 0 and W.stride(0) % 4 != 0
        ctx.step(W, db, dy, U, V, wl.eta, loss=loss)
        ctx.sync()
        Uo, Vo, Wo, fo = oracle.step(wl.model, Wo, b, wl.P, wl.B, wl.eta)
        assert_close(U.cpu().numpy(), Uo, tol, f"U step {t}")
        assert_close(V.float().cpu().numpy(), Vo, tol, f"V step {t}")
        assert_close(W.cpu().numpy(), Wo, tol, f"W step {t}")
        assert_close(loss.cpu().numpy(), fo, tol, f"loss step {t}")
    # nothing was written outside the views
    for view in (W, U, V):
        base = view._base
        assert float(base[:, 0].float().abs().max()) == 0.0 and float(base[:, view.shape[1] + 1:].float().abs().max()) == 0.0
    ctx.close()


def test_labels_outside_the_class_range_drop_the_one_hot_term(sfb):
    """The header documents it: class ids outside [0, J) are not detected; the one-hot term is absent,
    so u is the plain softmax (rows sum to 1) and the loss is logsumexp(z).  Nothing else is disturbed."""
    wl = workloads.make("mlr_tiny", seed=13, J=12, D=64, P=2, B=8)
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    b = wl.batch(0)
    db, dy = to_device(wl, b, dev)
    bad = dy.clone()
    bad[3], bad[7] = wl.J + 5, -1
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(W, db, bad, U, V, loss)
    ctx.sync()
    Z = oracle.scores(wl.W0, b["A"])
    fo, Uo = oracle.loss_and_u("mlr", Z, b["y"])
    got = U.cpu().numpy()
    for i in range(wl.N):
        if i in (3, 7):
            soft = np.exp(Z[i] - Z[i].max())
            soft /= soft.sum()
            assert_close(got[i], soft, TOL32, f"row {i}: plain softmax")
            assert abs(float(loss[i]) - float(np.log(np.exp(Z[i]).sum()))) < 1e-5
        else:
            assert_close(got[i], Uo[i], TOL32, f"row {i}")
    ctx.close()


def test_two_contexts_on_two_streams_do_not_disturb_each_other(sfb):
    """Distinct contexts are independent: steps of two models interleaved on two streams (default
    priority), without synchronising in between, give what each gives alone."""
    dev = "cuda:0"
    wls = [workloads.make("mlr_medium", seed=14, J=200, D=512, P=4, B=32, steps=4, pool=2),
           workloads.make("dml", seed=15, J=96, D=256, P=2, B=64, steps=4, pool=2)]

    def setup(wl, stream):
        with torch.cuda.stream(stream):
            ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
            W = torch.from_numpy(wl.W0).to(dev)
            U, V, loss = alloc_factors(wl, dev)
            pool = [to_device(wl, b, dev) for b in wl.batches]
        stream.synchronize()
        return ctx, W, U, V, pool

    alone = []
    for wl in wls:
        s = torch.cuda.Stream(device=dev)
        ctx, W, U, V, pool = setup(wl, s)
        for t in range(4):
            ctx.step(W, *pool[t % 2], U, V, wl.eta)
        ctx.sync()
        alone.append(W.clone())
        ctx.close()
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]
    state = [setup(wl, s) for wl, s in zip(wls, streams)]
    for t in range(4):
        for (ctx, W, U, V, pool), wl in zip(state, wls):
            ctx.step(W, *pool[t % 2], U, V, wl.eta)          # enqueue only
    for (ctx, W, U, V, pool), want in zip(state, alone):
        ctx.sync()
        assert torch.equal(W, want)
        ctx.close()
