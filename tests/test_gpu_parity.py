"""GPU parity: every C-ABI call against the fp64 CPU oracle on the same seeded inputs.

Tolerances (the benchmark spec): factors and preconditioned gradients relative Frobenius error
<= 1e-4 in fp32 (<= 2e-2 with bf16 inputs); eigenpairs: ||F - Q diag(lam) Q^T||_F <= 1e-5 ||F||_F and
eigenvalues within 1e-5 * lam_max of the oracle's; unfold is bit-exact (data movement only).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2007_00784_amd import kfac as K
from paper_2007_00784_amd import synthetic as S
from gpu_util import Ctx, relfro, ndt_to_rows

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
TOL_RES = 1e-5
TOL_LAM = 1e-5


@pytest.fixture(scope="module")
def ctx():
    c = Ctx(1 << 30)
    yield c
    c.close()


# ------------------------------------------------------------------ unfold
UNFOLD_CASES = [
    # N, C, H, k, stride, pad
    (2, 3, 5, 3, 1, 1),
    (1, 1, 5, 7, 1, 3),
    (2, 2, 7, 3, 2, 1),
    (3, 4, 8, 1, 2, 0),
    (2, 3, 37, 7, 2, 3),       # several row chunks per plane after staging limits
    (4, 16, 8, 3, 1, 1),       # config-1 layer
    (2, 64, 14, 3, 1, 1),
    (2, 130, 7, 3, 2, 1),      # many channels per workgroup, ragged channel tail
    (1, 3, 224, 7, 2, 3),      # stem geometry: chunked rows
    (2, 8, 56, 3, 1, 1),
    (2, 5, 28, 3, 2, 1),       # stride 2 onto a 14 x 14 map: the tile holds the output
    (1, 2, 14, 5, 2, 2),
    (3, 20, 7, 3, 1, 1),       # 7 x 7 map, several channels per workgroup with a ragged tail
    (2, 4, 56, 3, 2, 1),       # stride 2 onto 28 x 28: one channel per workgroup
]


@pytest.mark.parametrize("case", UNFOLD_CASES)
@pytest.mark.parametrize("bf16", [False, True])
def test_unfold_bit_exact(ctx, case, bf16):
    N, C, H, k, s, p = case
    x = np.random.default_rng(1).standard_normal((N, C, H, H)).astype(np.float32)
    if bf16:
        x = S.bf16_bits_to_f32(S.to_bf16_bits(x)).reshape(x.shape)
    out = ctx.unfold(x, k, k, s, p, bf16=bf16).float().cpu().numpy()
    ref = oracle.unfold(x, k, k, s, s, p, p)
    assert np.array_equal(ndt_to_rows(out), ref)


# ------------------------------------------------------------------ factors
FACTOR_CASES = [
    # layout, N, d, T, ones
    ("RD", 64, 10, 1, 0),
    ("RD", 300, 65, 1, 1),
    ("RD", 2048, 144, 1, 1),
    ("NDT", 32, 144, 64, 1),       # config-1 A factor
    ("NDT", 32, 16, 64, 0),        # config-1 G factor
    ("NDT", 7, 130, 49, 1),        # T = 49, ragged tiles
    ("NDT", 3, 257, 196, 0),
    ("NDT", 5, 300, 5, 1),         # T < K slab
    ("RD", 5000, 33, 1, 1),        # split-K on a single tile
    ("NDT", 64, 64, 784, 1),       # deep split-K
    ("NDT", 9, 200, 9, 1),         # bf16 engine: every example ends in a group that overlaps the one before by 7
    ("NDT", 4, 130, 8, 0),         # bf16 engine: exactly one group per example
    ("NDT", 40, 257, 100, 1),      # bf16 engine: T = 12.5 groups, three tiles per side, contraction ends mid-slab
    ("NDT", 6, 70, 4, 1),          # grouped engine, fp32: one group per example (bf16: element-wise engine, T < 8)
    ("NDT", 6, 70, 7, 1),          # grouped engine, fp32: second group overlaps the first by one position
    ("NDT", 3, 20, 15, 0),         # grouped engine: bf16 second group overlaps by one, fp32 fourth by one
    ("NDT", 600, 129, 49, 1),      # T = 49 with split-K: several jobs per tile, column sums across splits, ragged tile
]


def test_unfold_batched_bit_exact(ctx):
    """Every unfold case, fp32 and bf16 mixed, in one batched call (one launch per element type; a workgroup finds
    its layer by binary search over the layers' first workgroup indices), bit-exact against the oracle; an empty
    batch is a no-op and two layers writing the same output are rejected."""
    rng = np.random.default_rng(3)
    K.kfac_unfold_batched(ctx.h, [], [], [])
    xs, convs, outs, refs = [], [], [], []
    for (N, C, H, k, s, p) in UNFOLD_CASES:
        for bf16 in (False, True):
            x = rng.standard_normal((N, C, H, H)).astype(np.float32)
            if bf16:
                x = S.bf16_bits_to_f32(S.to_bf16_bits(x)).reshape(x.shape)
            Ho = (H + 2 * p - k) // s + 1
            xd = ctx.to_dev(x, bf16)
            xs.append(xd); convs.append((k, k, s, p))
            outs.append(torch.full((N, C * k * k, Ho * Ho), float("nan"), dtype=xd.dtype, device=ctx.dev))
            refs.append(oracle.unfold(x, k, k, s, s, p, p))
    assert K.kfac_unfold_workspace_bytes(len(xs)) <= ctx.ws.numel()
    K.kfac_unfold_batched(ctx.h, xs, convs, outs)
    torch.cuda.synchronize()
    for o, ref in zip(outs, refs):
        assert np.array_equal(ndt_to_rows(o.float().cpu().numpy()), ref)
    with pytest.raises(K.KfacError):
        K.kfac_unfold_batched(ctx.h, xs[:2], convs[:2], [outs[0], outs[0]])


@pytest.mark.parametrize("case", FACTOR_CASES)
@pytest.mark.parametrize("bf16", [False, True])
def test_update_factors_matches_oracle(ctx, case, bf16):
    layout, N, d, T, ones = case
    rng = np.random.default_rng(2)
    D = d + ones
    F = None
    Fd = torch.full((D, D), float("nan"), dtype=torch.float32, device=ctx.dev)
    for upd, decay in enumerate([0.0, 0.95, 0.95]):
        X = np.maximum(rng.standard_normal((N, d, T)), 0).astype(np.float32) if layout == "NDT" else \
            np.maximum(rng.standard_normal((N * T, d)), 0).astype(np.float32)
        if bf16:
            X = S.bf16_bits_to_f32(S.to_bf16_bits(X)).reshape(X.shape)
        rows = ndt_to_rows(X) if layout == "NDT" else X.astype(np.float64)
        R = rows.shape[0]
        Fb = oracle.gram(rows, ones, 1.0 / R)
        F = Fb if upd == 0 else oracle.ema(F, Fb, decay)
        Xd = ctx.to_dev(X, bf16)
        ctx.update_factors(Xd, K.KFAC_LAYOUT_NDT if layout == "NDT" else K.KFAC_LAYOUT_RD, N, d, T, ones,
                           1.0 / R, decay, Fd)
        torch.cuda.synchronize()
        got = Fd.cpu().numpy()
        assert np.isfinite(got).all()
        assert np.array_equal(got, got.T)
        assert relfro(got, F) <= TOL_F32
    if ones:
        assert abs(got[D - 1, D - 1] - 1.0) < 1e-6


def test_update_factors_batched_matches_oracle(ctx):
    """Every case above, fp32 and bf16 operands mixed, in ONE batched call per update (all four operand forms
    in the same call; job tables, per-factor partial buffers, the shared reducer), two updates so the
    running average of each factor is exercised, plus an empty batch."""
    rng = np.random.default_rng(5)
    K.kfac_update_factors_batched(ctx.h, [])
    F = [None] * (2 * len(FACTOR_CASES))
    Fd = [torch.full((d + ones, d + ones), float("nan"), dtype=torch.float32, device=ctx.dev)
          for (_, _, d, _, ones) in FACTOR_CASES for _ in range(2)]
    for upd, decay in enumerate([0.0, 0.9]):
        items = []
        for ci, (layout, N, d, T, ones) in enumerate(FACTOR_CASES):
            for bf16 in (False, True):
                j = 2 * ci + int(bf16)
                X = np.maximum(rng.standard_normal((N, d, T)), 0).astype(np.float32) if layout == "NDT" else \
                    np.maximum(rng.standard_normal((N * T, d)), 0).astype(np.float32)
                if bf16:
                    X = S.bf16_bits_to_f32(S.to_bf16_bits(X)).reshape(X.shape)
                rows = ndt_to_rows(X) if layout == "NDT" else X.astype(np.float64)
                R = rows.shape[0]
                Fb = oracle.gram(rows, ones, 1.0 / R)
                F[j] = Fb if upd == 0 else oracle.ema(F[j], Fb, decay)
                items.append(dict(X=ctx.to_dev(X, bf16), layout=K.KFAC_LAYOUT_NDT if layout == "NDT" else K.KFAC_LAYOUT_RD,
                                  N=N, d=d, T=T, append_ones=ones, scale=1.0 / R, decay=decay, F=Fd[j]))
        assert K.kfac_update_factors_workspace_bytes(items) <= ctx.ws.numel()
        K.kfac_update_factors_batched(ctx.h, items)
        torch.cuda.synchronize()
        for j in range(len(F)):
            got = Fd[j].cpu().numpy()
            assert np.isfinite(got).all(), j
            assert np.array_equal(got, got.T), j
            assert relfro(got, F[j]) <= TOL_F32, (j, relfro(got, F[j]))
    # the same factor twice in one batch is rejected
    with pytest.raises(K.KfacError):
        K.kfac_update_factors_batched(ctx.h, [items[0], items[0]])


def test_update_factors_deterministic(ctx):
    rng = np.random.default_rng(3)
    X = ctx.to_dev(rng.standard_normal((20000, 70)).astype(np.float32))
    outs = []
    for _ in range(2):
        Fd = torch.zeros((71, 71), dtype=torch.float32, device=ctx.dev)
        ctx.update_factors(X, K.KFAC_LAYOUT_RD, 20000, 70, 1, 1, 1.0 / 20000, 0.0, Fd)
        torch.cuda.synchronize()
        outs.append(Fd.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


# ------------------------------------------------------------------ eig
def gram_factor(n, rows, seed, ones=True):
    rng = np.random.default_rng(seed)
    X = np.maximum(rng.standard_normal((rows, n - (1 if ones else 0))), 0)
    return oracle.gram(X, 1 if ones else 0, 1.0 / rows).astype(np.float32)


def check_eigpairs(F32, lam, Q, label=""):
    F = F32.astype(np.float64)
    lam = lam.astype(np.float64)
    Q = Q.astype(np.float64)
    n = F.shape[0]
    nf = np.linalg.norm(F)
    assert np.isfinite(lam).all() and np.isfinite(Q).all(), label
    assert np.all(np.diff(lam) >= 0), label
    res = np.linalg.norm(F - (Q * lam) @ Q.T) / nf
    orth = np.linalg.norm(Q.T @ Q - np.eye(n), 2)
    ref, _ = oracle.eigh(F)
    lerr = np.abs(lam - ref).max() / max(abs(ref).max(), 1e-300)
    print("%s n=%d residual=%.2e orth2=%.2e lam_err=%.2e" % (label, n, res, orth, lerr))
    assert res <= TOL_RES, label
    assert lerr <= TOL_LAM, label
    assert orth <= 1e-4, label


EIG_SIZES = [(1, 1), (2, 5), (16, 40), (17, 9), (65, 200), (128, 64), (129, 300), (145, 2048), (257, 100),
             (289, 600), (577, 300), (640, 2000)]


@pytest.mark.parametrize("n,rows", EIG_SIZES)
def test_eig_single(ctx, n, rows):
    F = gram_factor(n, rows, seed=n)
    Ld, Qd, info = ctx.eig([F])
    assert info[0][2], info
    check_eigpairs(F, Ld[0].cpu().numpy(), Qd[0].cpu().numpy(), "single")


def test_eig_batch_mixed_sizes(ctx):
    sizes = [(16, 50), (145, 500), (10, 3), (145, 700), (289, 100), (64, 64), (300, 1000), (33, 100), (289, 900)]
    mats = [gram_factor(n, r, seed=100 + i, ones=(i % 2 == 0)) for i, (n, r) in enumerate(sizes)]
    Ld, Qd, info = ctx.eig(mats)
    for i, F in enumerate(mats):
        assert info[i][2]
        check_eigpairs(F, Ld[i].cpu().numpy(), Qd[i].cpu().numpy(), "batch[%d]" % i)


def test_eig_known_spectrum_and_diagonal(ctx):
    n = 200
    u = np.random.default_rng(5).standard_normal(n); u /= np.linalg.norm(u)
    H = np.eye(n) - 2 * np.outer(u, u)
    D = np.concatenate([np.zeros(50), np.full(60, 0.5), np.linspace(1, 9, 89), [100.0]])
    F = (H @ np.diag(D) @ H).astype(np.float32)
    Dg = np.diag(np.random.default_rng(6).random(150)).astype(np.float32)
    Ld, Qd, info = ctx.eig([F, Dg])
    lam = Ld[0].cpu().numpy()
    assert np.abs(lam - np.sort(D)).max() <= TOL_LAM * 100
    check_eigpairs(F, lam, Qd[0].cpu().numpy(), "householder")
    assert np.array_equal(Ld[1].cpu().numpy(), np.sort(np.diag(Dg)))
    assert info[1][0] == 0


def test_eig_warm_start(ctx):
    """A slowly moving factor (running average with 5 % of a new batch, Sec. IV-B) decomposed again from the
    previous eigenvectors: the same invariants hold, in fewer sweeps than from the identity; a flat-path
    factor and a two-level one, plus a small one (which ignores the option) in the same batch.  Starting from
    the exact eigenvectors of the same matrix converges at once."""
    sizes = [(577, 1500), (2100, 3000), (65, 200)]
    F0 = [gram_factor(n, r, seed=40 + i) for i, (n, r) in enumerate(sizes)]
    F1 = [(0.95 * a.astype(np.float64) + 0.05 * gram_factor(n, r, seed=50 + i)).astype(np.float32)
          for i, (a, (n, r)) in enumerate(zip(F0, sizes))]
    Fd0 = [ctx.to_dev(f) for f in F0]
    Fd1 = [ctx.to_dev(f) for f in F1]
    Q = [torch.zeros_like(f) for f in Fd0]
    lam = [torch.zeros(f.shape[0], dtype=torch.float32, device=ctx.dev) for f in Fd0]
    info0 = K.kfac_eig(ctx.h, Fd0, Q, lam)
    again = K.kfac_eig(ctx.h, Fd0, Q, lam, warm_start=True)          # Q holds the eigenvectors of the same matrices
    torch.cuda.synchronize()
    assert all(c for (_, _, c) in again) and again[0][0] <= 1 and again[1][0] <= 1, again
    for i, F in enumerate(F0):
        check_eigpairs(F, lam[i].cpu().numpy(), Q[i].cpu().numpy(), "warm-same[%d]" % i)
    warm = K.kfac_eig(ctx.h, Fd1, Q, lam, warm_start=True)
    torch.cuda.synchronize()
    for i, F in enumerate(F1):
        check_eigpairs(F, lam[i].cpu().numpy(), Q[i].cpu().numpy(), "warm[%d]" % i)
    cold = K.kfac_eig(ctx.h, Fd1, Q, lam)
    torch.cuda.synchronize()
    print("sweeps cold", [x[0] for x in cold], "warm", [x[0] for x in warm], "first", [x[0] for x in info0])
    assert all(c for (_, _, c) in warm) and all(c for (_, _, c) in cold)
    assert warm[0][0] < cold[0][0] and warm[1][0] < cold[1][0]


def test_eig_max_sweeps_reports_noconv(ctx):
    F = gram_factor(300, 500, seed=7)
    with pytest.raises(K.KfacError) as e:
        ctx.eig([F], max_sweeps=1, tol=1e-7)
    assert e.value.code == K.KFAC_ENOCONV
    Ld, Qd, info = ctx.eig([F], max_sweeps=1, tol=1e-7, raise_on_noconv=False)
    assert not info[0][2] and info[0][0] == 1
    assert np.isfinite(Qd[0].cpu().numpy()).all()


def test_eig_many_factors_of_one_size(ctx):
    """200 factors of one blocked size class advance as one group: every one of them gets its own norms,
    flags and eigenpairs (the group's bookkeeping is sized by its member count, not by a fixed launch)."""
    n, count = 160, 200
    mats = [gram_factor(n, 200 + 3 * i, seed=1000 + i, ones=(i % 2 == 0)) for i in range(count)]
    Ld, Qd, info = ctx.eig(mats)
    assert all(c for (_, _, c) in info), [i for i, x in enumerate(info) if not x[2]]
    for i in list(range(0, count, 7)) + [127, 128, 129, count - 1]:
        check_eigpairs(mats[i], Ld[i].cpu().numpy(), Qd[i].cpu().numpy(), "many[%d]" % i)
    for i in range(count):      # the cheap invariants on every member: trace and orthonormal first/last columns
        lam, Q = Ld[i].cpu().numpy().astype(np.float64), Qd[i].cpu().numpy().astype(np.float64)
        assert abs(lam.sum() - np.trace(mats[i].astype(np.float64))) <= 1e-5 * abs(lam).max() * n, i
        assert abs(np.linalg.norm(Q[:, 0]) - 1) < 1e-4 and abs(np.linalg.norm(Q[:, -1]) - 1) < 1e-4, i


def test_eig_is_reproducible(ctx):
    """Same input, same bits: the norms that decide convergence and the Rayleigh quotients are summed in a
    fixed order (small, flat and two-level path)."""
    mats = [gram_factor(n, r, seed=70 + i) for i, (n, r) in enumerate([(100, 300), (577, 900), (2100, 2500)])]
    L1, Q1, i1 = ctx.eig(mats)
    L2, Q2, i2 = ctx.eig(mats)
    assert i1 == i2
    for a, b in zip(L1 + Q1, L2 + Q2):
        assert torch.equal(a, b)


@pytest.mark.parametrize("n", [40, 230, 300, 2100])
def test_eig_non_finite_input(ctx, n):
    """A NaN in the factor: KFAC_ENOCONV, and every element of that factor's outputs is non-finite, while a
    healthy factor of the same call is decomposed as usual."""
    bad = gram_factor(n, 2 * n, seed=3)
    bad[n // 2, n // 3] = np.nan
    bad[n // 3, n // 2] = np.nan
    good = gram_factor(n, 2 * n, seed=4)
    with pytest.raises(K.KfacError) as e:
        ctx.eig([bad, good])
    assert e.value.code == K.KFAC_ENOCONV
    Ld, Qd, info = ctx.eig([bad, good], raise_on_noconv=False)
    assert not info[0][2] and info[1][2], info
    assert not np.isfinite(Ld[0].cpu().numpy()).any() and not np.isfinite(Qd[0].cpu().numpy()).any()
    check_eigpairs(good, Ld[1].cpu().numpy(), Qd[1].cpu().numpy(), "beside NaN")


# ------------------------------------------------------------------ precondition
# (230, 100) and (97, 200): edge tiles between 65 and 127 wide and tall (accumulator blocks masked under the full
# wave map); the others: edge tiles at most 64 wide or tall (the waves share them in slices)
PRECOND_CASES = [(10, 4), (145, 16), (65, 10), (289, 32), (577, 64), (130, 257), (230, 100), (97, 200)]


@pytest.mark.parametrize("dA,dG", PRECOND_CASES)
@pytest.mark.parametrize("bf16", [False, True])
def test_precondition_matches_oracle(ctx, dA, dG, bf16):
    rng = np.random.default_rng(8)
    A = gram_factor(dA, 3 * dA, seed=dA).astype(np.float64)
    G = oracle.gram(rng.standard_normal((3 * dG, dG)) * 1e-2, 0, 1.0 / (3 * dG))
    lamA, QA = oracle.eigh(A)
    lamG, QG = oracle.eigh(G)
    gamma = 1e-3 * lamA.mean() * lamG.mean()
    grad = (rng.standard_normal((dG, dA)) * 1e-2).astype(np.float32)
    if bf16:
        grad = S.bf16_bits_to_f32(S.to_bf16_bits(grad)).reshape(grad.shape)
    ref = oracle.precondition(QA, lamA, QG, lamG, gamma, grad)
    gd = ctx.to_dev(grad, bf16)
    K.kfac_precondition(ctx.h, ctx.to_dev(QA.astype(np.float32)), ctx.to_dev(lamA.astype(np.float32)),
                        ctx.to_dev(QG.astype(np.float32)), ctx.to_dev(lamG.astype(np.float32)), gamma, gd)
    torch.cuda.synchronize()
    got = gd.float().cpu().numpy()
    assert relfro(got, ref) <= (TOL_BF16 if bf16 else TOL_F32)


@pytest.mark.parametrize("dA,dG", PRECOND_CASES + [(1000, 300), (4, 1)])
@pytest.mark.parametrize("bf16", [False, True])
def test_precondition_split_f16_matches_oracle(ctx, dA, dG, bf16):
    """The same step with the GEMM chain on the split-fp16 engine (operands of any extent and alignment, per-layer
    power-of-two scales from the gradient's and V2's Frobenius norms), to the same bar as the fp32 chain; a
    gradient scaled far outside fp16's range (1e-9, 1e+6) must come out the same, and a zero gradient stays zero."""
    rng = np.random.default_rng(8)
    A = gram_factor(dA, 3 * dA, seed=dA).astype(np.float64)
    G = oracle.gram(rng.standard_normal((3 * dG, dG)) * 1e-2, 0, 1.0 / (3 * dG))
    lamA, QA = oracle.eigh(A)
    lamG, QG = oracle.eigh(G)
    gamma = 1e-3 * lamA.mean() * lamG.mean()
    dev = [ctx.to_dev(QA.astype(np.float32)), ctx.to_dev(lamA.astype(np.float32)),
           ctx.to_dev(QG.astype(np.float32)), ctx.to_dev(lamG.astype(np.float32))]
    for mag in (1e-2, 1e-9, 1e6, 0.0):
        grad = (rng.standard_normal((dG, dA)) * mag).astype(np.float32)
        if bf16:
            grad = S.bf16_bits_to_f32(S.to_bf16_bits(grad)).reshape(grad.shape)
        ref = oracle.precondition(QA, lamA, QG, lamG, gamma, grad)
        gd = ctx.to_dev(grad, bf16)
        K.kfac_precondition_batched(ctx.h, [dev[0]], [dev[1]], [dev[2]], [dev[3]], gamma, [gd], split_f16=True)
        torch.cuda.synchronize()
        got = gd.float().cpu().numpy()
        assert np.isfinite(got).all()
        if mag == 0.0:
            assert not got.any()
        else:
            assert relfro(got, ref) <= (TOL_BF16 if bf16 else TOL_F32), (mag, relfro(got, ref))


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("split", [False, True])
def test_precondition_batched_with_gradient_scaling(ctx, bf16, split):
    """Sec. V-C: the batched preconditioner followed by nu = min(1, sqrt(kappa / (lr^2 sum_l |<P_l, g_l>|))).
    Three layers of different tile counts (one tile, ragged tiles, several tiles) in one call, against the oracle
    end to end, against the oracle's nu on the library's own unscaled output, and with a kappa that does not clip."""
    rng = np.random.default_rng(11)
    dims = [(65, 16), (300, 130), (145, 257)]
    QAs, lAs, QGs, lGs, grads, refs = [], [], [], [], [], []
    gamma = None
    for dA, dG in dims:
        A = gram_factor(dA, 3 * dA, seed=dA).astype(np.float64)
        G = oracle.gram(rng.standard_normal((3 * dG, dG)), 0, 1.0 / (3 * dG))
        lamA, QA = oracle.eigh(A)
        lamG, QG = oracle.eigh(G)
        gamma = 1e-2
        grad = (rng.standard_normal((dG, dA)) * 1e-2).astype(np.float32)
        if bf16:
            grad = S.bf16_bits_to_f32(S.to_bf16_bits(grad)).reshape(grad.shape)
        refs.append(oracle.precondition(QA, lamA, QG, lamG, gamma, grad))
        QAs.append(ctx.to_dev(QA.astype(np.float32))); lAs.append(ctx.to_dev(lamA.astype(np.float32)))
        QGs.append(ctx.to_dev(QG.astype(np.float32))); lGs.append(ctx.to_dev(lamG.astype(np.float32)))
        grads.append(grad)
    tol = TOL_BF16 if bf16 else TOL_F32
    # unscaled output of the library, for the same inputs
    plain = [ctx.to_dev(g, bf16) for g in grads]
    K.kfac_precondition_batched(ctx.h, QAs, lAs, QGs, lGs, gamma, plain, split_f16=split)
    torch.cuda.synchronize()
    plain = [p.float().cpu().numpy().astype(np.float64) for p in plain]
    lr = 0.1
    s_sum = sum(abs(float((p * g).sum())) for p, g in zip(plain, grads))
    for kappa, clipped in [(1e-3 * lr * lr * s_sum, True), (10.0 * lr * lr * s_sum, False)]:
        gd = [ctx.to_dev(g, bf16) for g in grads]
        nu_d = torch.full((1,), float("nan"), dtype=torch.float32, device=ctx.dev)
        K.kfac_precondition_batched_scaled(ctx.h, QAs, lAs, QGs, lGs, gamma, gd, kappa, lr, nu_d, split_f16=split)
        torch.cuda.synchronize()
        nu = float(nu_d.item())
        nu_own = oracle.grad_scale(plain, grads, kappa, lr)          # oracle formula on the library's own P_l
        nu_ref = oracle.grad_scale(refs, grads, kappa, lr)           # oracle end to end
        assert (nu < 1.0) == clipped
        assert abs(nu - nu_own) <= 2e-6 * nu_own
        assert abs(nu - nu_ref) <= tol * nu_ref
        if clipped:
            assert nu == pytest.approx(np.sqrt(1e-3), rel=1e-5)
        for j in range(len(dims)):
            got = gd[j].float().cpu().numpy()
            assert relfro(got, nu_ref * refs[j]) <= tol
            assert relfro(got, nu * plain[j]) <= (4e-3 if bf16 else 1e-6)   # bf16: one more rounding of the product
    with pytest.raises(K.KfacError):
        K.kfac_precondition_batched_scaled(ctx.h, QAs, lAs, QGs, lGs, gamma, gd, 0.0, lr, nu_d)


@pytest.mark.parametrize("dA,dG", [(145, 16), (300, 130), (577, 64), (230, 100)])
def test_explicit_inverse_method_matches_cholesky_oracle(ctx, dA, dG):
    """Sec. II-C, Eq. (kfac-damped): (G + gamma I)^-1 grad (A + gamma I)^-1.  The library forms it in the eigenbasis
    of its own eigendecompositions (factored denominator); the oracle by two Cholesky solves with no
    eigendecomposition at all, so this checks factors -> eig -> precondition against an independent route."""
    rng = np.random.default_rng(dA)
    # zero-mean unit-variance samples on both sides: spectra within [0.1, 3], so that one damping value means the same
    # for both factors and the damped inverses are well conditioned (the sensitivity to the eigensolver's 1e-6 ||F||
    # stays below the 1e-4 bar; ill-conditioned cases are exercised in test_gpu_configs.py)
    X = rng.standard_normal((3 * dA, dA - 1)).astype(np.float32)
    Gr = rng.standard_normal((4 * dG, dG)).astype(np.float32)
    Ad = torch.zeros((dA, dA), dtype=torch.float32, device=ctx.dev)
    Gd = torch.zeros((dG, dG), dtype=torch.float32, device=ctx.dev)
    ctx.update_factors(ctx.to_dev(X), K.KFAC_LAYOUT_RD, X.shape[0], dA - 1, 1, 1, 1.0 / X.shape[0], 0.0, Ad)
    ctx.update_factors(ctx.to_dev(Gr), K.KFAC_LAYOUT_RD, Gr.shape[0], dG, 1, 0, 1.0 / Gr.shape[0], 0.0, Gd)
    Ld, Qd, info = ctx.eig([Ad, Gd])
    assert all(c for (_, _, c) in info)
    A = oracle.gram(X, 1, 1.0 / X.shape[0])
    G = oracle.gram(Gr, 0, 1.0 / Gr.shape[0])
    grad = (rng.standard_normal((dG, dA)) * 1e-2).astype(np.float32)
    for gamma in (0.3, 1.0):
        ref = oracle.precondition_inverse(G, A, gamma, grad)
        gd = ctx.to_dev(grad)
        K.kfac_precondition_batched(ctx.h, [Qd[0]], [Ld[0]], [Qd[1]], [Ld[1]], gamma, [gd], factored_damping=True)
        torch.cuda.synchronize()
        got = gd.cpu().numpy()
        assert relfro(got, ref) <= TOL_F32, (gamma, relfro(got, ref))
        # and it is not the hot path's damping
        g2 = ctx.to_dev(grad)
        K.kfac_precondition_batched(ctx.h, [Qd[0]], [Ld[0]], [Qd[1]], [Ld[1]], gamma, [g2])
        torch.cuda.synchronize()
        assert relfro(g2.cpu().numpy(), ref) > 1e-3


def _spd_factor(rng, n, rows, relu=True):
    X = rng.standard_normal((rows, n - 1))
    if relu:
        X = np.maximum(X, 0)
    X = X.astype(np.float32)
    return oracle.gram(X, 1, 1.0 / rows)


@pytest.mark.parametrize("n,rows", [(1, 8), (5, 40), (64, 256), (128, 300), (129, 300), (300, 200), (577, 1200), (1153, 1500)])
def test_invert_factors_matches_cholesky_oracle(ctx, n, rows):
    """Sec. II-C, Eq. (kfac-damped): (F + gamma I)^-1 by the library's blocked Cholesky inverse against the oracle's
    Cholesky solve of (F + gamma I) X = I in fp64.  Sizes straddle the 128-wide blocks; (300, 200) is rank deficient
    (only the damping makes it definite).  An fp32 inverse carries a relative error of the order of
    cond(F + gamma I) * 6e-8, so the bound is max(2e-6, 2e-7 * cond) with cond from the fp64 spectrum (measured:
    0.02 .. 0.1 of it)."""
    rng = np.random.default_rng(31 * n + rows)
    F = _spd_factor(rng, n, rows)
    lam = np.linalg.eigvalsh(F)
    Fd = ctx.to_dev(F.astype(np.float32))
    F32 = Fd.cpu().numpy().astype(np.float64)
    for gamma in (1e-1, 1e-3):
        ref = oracle.spd_solve(F32 + gamma * np.eye(n), np.eye(n))
        out = torch.full((n, n), float("nan"), dtype=torch.float32, device=ctx.dev)
        K.kfac_invert_factors(ctx.h, [Fd], gamma, [out])
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        cond = (max(lam[-1], 0) + gamma) / (max(lam[0], 0) + gamma)
        err = relfro(got, ref)
        assert err <= max(2e-6, 2e-7 * cond), (n, gamma, err, cond)
        # the defining property, in fp64 on the fp32 result
        res = np.linalg.norm(got @ (F32 + gamma * np.eye(n)) - np.eye(n)) / np.sqrt(n)
        assert res <= max(2e-6, 2e-7 * cond), (n, gamma, res, cond)


def test_invert_factors_batch_of_mixed_sizes(ctx):
    """Several factors in one call share the workspace one after another; every inverse is checked."""
    rng = np.random.default_rng(77)
    dims = [257, 16, 130, 257, 400]
    Fs = [_spd_factor(rng, n, 3 * n, relu=False) for n in dims]
    Fd = [ctx.to_dev(F.astype(np.float32)) for F in Fs]
    outs = [torch.zeros((n, n), dtype=torch.float32, device=ctx.dev) for n in dims]
    assert 0 < K.kfac_invert_workspace_bytes(dims) <= K.kfac_workspace_bytes(max(dims), 1, 1)
    K.kfac_invert_factors(ctx.h, Fd, 0.05, outs)
    torch.cuda.synchronize()
    for F, o, n in zip(Fd, outs, dims):
        ref = oracle.spd_solve(F.cpu().numpy().astype(np.float64) + 0.05 * np.eye(n), np.eye(n))
        assert relfro(o.cpu().numpy(), ref) <= 1e-5, n
    with pytest.raises(K.KfacError):
        K.kfac_invert_factors(ctx.h, Fd, 0.0, outs)
    with pytest.raises(K.KfacError):
        K.kfac_invert_factors(ctx.h, Fd, 0.05, Fd)


@pytest.mark.parametrize("dA,dG", [(145, 16), (300, 130), (577, 64), (230, 100)])
@pytest.mark.parametrize("bf16", [False, True])
def test_precondition_inverse_matches_oracle(ctx, dA, dG, bf16):
    """The whole inverse method, factors -> Cholesky inverses -> Ginv grad Ainv, against the oracle's two Cholesky
    solves (Sec. II-C, Eq. (kfac-damped)); well-conditioned factors as in
    test_explicit_inverse_method_matches_cholesky_oracle, fp32 and bf16 gradients."""
    rng = np.random.default_rng(dA + 5)
    X = rng.standard_normal((3 * dA, dA - 1)).astype(np.float32)
    Gr = rng.standard_normal((4 * dG, dG)).astype(np.float32)
    Ad = torch.zeros((dA, dA), dtype=torch.float32, device=ctx.dev)
    Gd = torch.zeros((dG, dG), dtype=torch.float32, device=ctx.dev)
    ctx.update_factors(ctx.to_dev(X), K.KFAC_LAYOUT_RD, X.shape[0], dA - 1, 1, 1, 1.0 / X.shape[0], 0.0, Ad)
    ctx.update_factors(ctx.to_dev(Gr), K.KFAC_LAYOUT_RD, Gr.shape[0], dG, 1, 0, 1.0 / Gr.shape[0], 0.0, Gd)
    A = oracle.gram(X, 1, 1.0 / X.shape[0])
    G = oracle.gram(Gr, 0, 1.0 / Gr.shape[0])
    grad = (rng.standard_normal((dG, dA)) * 1e-2).astype(np.float32)
    if bf16:
        grad = S.bf16_bits_to_f32(S.to_bf16_bits(grad)).reshape(grad.shape)
    Ai, Gi = torch.empty_like(Ad), torch.empty_like(Gd)
    for gamma in (0.3, 1.0):
        ref = oracle.precondition_inverse(G, A, gamma, grad)
        K.kfac_invert_factors(ctx.h, [Ad, Gd], gamma, [Ai, Gi])
        gd = ctx.to_dev(grad, bf16)
        K.kfac_precondition_inverse(ctx.h, Ai, Gi, gd)
        torch.cuda.synchronize()
        got = gd.float().cpu().numpy()
        assert relfro(got, ref) <= (TOL_BF16 if bf16 else TOL_F32), (gamma, relfro(got, ref))


def test_precondition_inverse_batched_equals_per_layer(ctx):
    """One batched call over layers of different shapes and gradient types gives, bit for bit, what the per-layer call
    gives (same tiles, same order of operations)."""
    rng = np.random.default_rng(9)
    shapes = [(145, 16, False), (300, 130, True), (64, 257, False), (129, 128, True)]
    Ai, Gi, g1, g2 = [], [], [], []
    for dA, dG, bf16 in shapes:
        A = _spd_factor(rng, dA, 2 * dA, relu=False)
        G = _spd_factor(rng, dG, 2 * dG, relu=False)
        Ai.append(ctx.to_dev(np.linalg.inv(A + 0.5 * np.eye(dA)).astype(np.float32)))
        Gi.append(ctx.to_dev(np.linalg.inv(G + 0.5 * np.eye(dG)).astype(np.float32)))
        g = rng.standard_normal((dG, dA)).astype(np.float32)
        g1.append(ctx.to_dev(g, bf16))
        g2.append(ctx.to_dev(g, bf16))
    K.kfac_precondition_inverse_batched(ctx.h, Ai, Gi, g1)
    for a, g, x in zip(Ai, Gi, g2):
        K.kfac_precondition_inverse(ctx.h, a, g, x)
    torch.cuda.synchronize()
    for x, y in zip(g1, g2):
        assert torch.equal(x, y)


@pytest.mark.parametrize("dA,dG,rows", [(145, 16, 2048), (577, 64, 1500), (289, 32, 200)])
def test_explicit_inverse_method_at_the_papers_damping(ctx, dA, dG, rows):
    """The explicit-inverse method where it is hard: ReLU-activation A factors (one eigenvalue ~ 0.16 d_A over a bulk
    of ~0.3; rank deficient in the last case), gradient factors of size 1e-6, damping 1e-3 (the paper's ImageNet
    value, Sec. VI) -- against the oracle's two Cholesky solves.  The inverse of F + gamma I amplifies a perturbation
    of F by cond(F + gamma I) = (lam_max + gamma) / (lam_min + gamma), and an fp32 eigendecomposition is a
    perturbation of F of the order of fp32's unit roundoff, so the bound is
    max(1e-4, 6e-8 * (cond_A + cond_G)), from the oracle's spectra (measured: 2e-9 .. 5e-9 times that sum)."""
    rng = np.random.default_rng(1000 + dA)
    X = np.maximum(rng.standard_normal((rows, dA - 1)), 0).astype(np.float32)
    Gr = (rng.standard_normal((rows, dG)) * 1e-3).astype(np.float32)
    Ad = torch.zeros((dA, dA), dtype=torch.float32, device=ctx.dev)
    Gd = torch.zeros((dG, dG), dtype=torch.float32, device=ctx.dev)
    ctx.update_factors(ctx.to_dev(X), K.KFAC_LAYOUT_RD, rows, dA - 1, 1, 1, 1.0 / rows, 0.0, Ad)
    ctx.update_factors(ctx.to_dev(Gr), K.KFAC_LAYOUT_RD, rows, dG, 1, 0, 1.0 / rows, 0.0, Gd)
    Ld, Qd, info = ctx.eig([Ad, Gd])
    assert all(c for (_, _, c) in info)
    A = oracle.gram(X, 1, 1.0 / rows)
    G = oracle.gram(Gr, 0, 1.0 / rows)
    gamma = 1e-3
    la, lg = np.linalg.eigvalsh(A), np.linalg.eigvalsh(G)
    cond = (la.max() + gamma) / (max(la.min(), 0.0) + gamma) + (lg.max() + gamma) / (max(lg.min(), 0.0) + gamma)
    bound = max(TOL_F32, 6e-8 * cond)
    grad = (rng.standard_normal((dG, dA)) * 1e-2).astype(np.float32)
    ref = oracle.precondition_inverse(G, A, gamma, grad)
    gd = ctx.to_dev(grad)
    K.kfac_precondition_batched(ctx.h, [Qd[0]], [Ld[0]], [Qd[1]], [Ld[1]], gamma, [gd], factored_damping=True)
    torch.cuda.synchronize()
    err = relfro(gd.cpu().numpy(), ref)
    print("explicit inverse dA=%d dG=%d rows=%d: cond %.1e, error %.2e (bound %.1e)" % (dA, dG, rows, cond, err, bound))
    assert err <= bound


# ------------------------------------------------------------------ whole path, config 1
def test_single_conv_layer_end_to_end(ctx):
    """3x3 conv 16->16 on 8x8, batch 32: three factor updates, eig, precondition, against the oracle and
    against brute-force inversion of the damped Kronecker product."""
    wl = S.workload("single_conv")
    lay = wl.layers[0]
    A = G = None
    Ad = torch.full((145, 145), float("nan"), dtype=torch.float32, device=ctx.dev)
    Gd = torch.full((16, 16), float("nan"), dtype=torch.float32, device=ctx.dev)
    for upd in range(3):
        t = S.layer_inputs(wl, 0, update=upd)
        P = oracle.unfold(t["x"], 3, 3, 1, 1, 1, 1)
        gr = t["g"].transpose(0, 2, 3, 1).reshape(-1, lay.c_out)
        R = P.shape[0]
        Ab, Gb = oracle.gram(P, 1, 1.0 / R), oracle.gram(gr, 0, 1.0 / R)
        A = Ab if A is None else oracle.ema(A, Ab, wl.decay)
        G = Gb if G is None else oracle.ema(G, Gb, wl.decay)
        decay = 0.0 if upd == 0 else wl.decay
        Pd = ctx.unfold(t["x"], 3, 3, 1, 1)
        ctx.update_factors(Pd, K.KFAC_LAYOUT_NDT, wl.batch, 144, lay.T, 1, 1.0 / R, decay, Ad)
        gd = ctx.to_dev(t["g"].reshape(wl.batch, lay.c_out, lay.T))
        ctx.update_factors(gd, K.KFAC_LAYOUT_NDT, wl.batch, 16, lay.T, 0, 1.0 / R, decay, Gd)
    torch.cuda.synchronize()
    assert relfro(Ad.cpu().numpy(), A) <= TOL_F32
    assert relfro(Gd.cpu().numpy(), G) <= TOL_F32
    Ld, Qd, info = ctx.eig([Ad, Gd])
    check_eigpairs(Ad.cpu().numpy(), Ld[0].cpu().numpy(), Qd[0].cpu().numpy(), "A")
    check_eigpairs(Gd.cpu().numpy(), Ld[1].cpu().numpy(), Qd[1].cpu().numpy(), "G")
    lamA, QA = oracle.eigh(A)
    lamG, QG = oracle.eigh(G)
    for gamma in (wl.damping, 1e-3 * lamA.mean() * lamG.mean()):
        ref = oracle.precondition(QA, lamA, QG, lamG, gamma, t["gradw"])
        gd = ctx.to_dev(t["gradw"])
        K.kfac_precondition(ctx.h, Qd[0], Ld[0], Qd[1], Ld[1], gamma, gd)
        torch.cuda.synchronize()
        got = gd.cpu().numpy()
        assert relfro(got, ref) <= TOL_F32
        assert relfro(got, oracle.bruteforce(G, A, gamma, t["gradw"])) <= TOL_F32


# ------------------------------------------------------------------ error paths (host-side validation)
def test_invalid_arguments_are_rejected(ctx):
    F = torch.zeros((4, 4), device=ctx.dev)
    X = torch.zeros((8, 4), device=ctx.dev)
    L = K.lib()
    assert L.kfac_update_factors(ctx.h, None, 0, 0, 8, 4, 1, 0, 1.0, 0.0, F.data_ptr()) == K.KFAC_EINVAL
    assert L.kfac_update_factors(ctx.h, X.data_ptr(), 7, 0, 8, 4, 1, 0, 1.0, 0.0, F.data_ptr()) == K.KFAC_EINVAL
    assert L.kfac_update_factors(ctx.h, X.data_ptr(), 0, 0, 8, 4, 1, 0, 1.0, 1.5, F.data_ptr()) == K.KFAC_EINVAL
    assert L.kfac_update_factors(ctx.h, X.data_ptr(), 0, 0, 0, 4, 1, 0, 1.0, 0.5, F.data_ptr()) == K.KFAC_EINVAL
    assert L.kfac_precondition(ctx.h, F.data_ptr(), F.data_ptr(), 4, F.data_ptr(), F.data_ptr(), 4, 0.0,
                               F.data_ptr(), 0) == K.KFAC_EINVAL
    d = K.kfac_conv_desc(1, 1, 4, 4, 3, 3, 0, 1, 1, 1, 0)
    import ctypes
    assert L.kfac_unfold(ctx.h, ctypes.byref(d), X.data_ptr(), F.data_ptr()) == K.KFAC_EINVAL
    small = Ctx(1 << 16)
    big = torch.zeros((300, 300), device=ctx.dev)
    with pytest.raises(K.KfacError) as e:
        K.kfac_eig(small.h, [big], [torch.empty_like(big)], [torch.empty(300, device=ctx.dev)])
    assert e.value.code == K.KFAC_EWORKSPACE
    small.close()
