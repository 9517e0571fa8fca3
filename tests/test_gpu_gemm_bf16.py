"""GPU parity of hpsgd_gemm_bf16_nt: every tile form of the bf16 product of the local step
against the float64 product of the same bf16 values, plain and as the in-place SGD update."""
import numpy as np
import pytest
import torch

from oracle import hpsgd_oracle as oc
from paper_2009_02701_amd import binding as hb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FORMS = ["128x128", "128x256", "192x256", "256x256"]

# (groups, M, N, Kd): tails in every dimension against every tile (128 / 192 / 256 rows, 128 / 256
# columns, k-tiles of 64 with Kd a multiple of 8 only), one tile, several tiles per group, a
# contraction of one chunk, more groups than XCDs
SHAPES = [
    (2, 200, 72, 40),
    (3, 1117, 301, 1000),
    (1, 130, 520, 2600),
    (2, 257, 259, 72),
    (1, 385, 513, 136),
    (9, 96, 40, 8),
    (1, 1, 1, 8),
    (2, 192, 256, 64),
    (1, 600, 1030, 320),
]


def _operands(seed, G, M, N, Kd):
    rng = np.random.default_rng(seed)
    A = torch.from_numpy(rng.uniform(-1, 1, (G, M, Kd)).astype(np.float32)).to(torch.bfloat16)
    B = torch.from_numpy(rng.uniform(-1, 1, (G, N, Kd)).astype(np.float32)).to(torch.bfloat16)
    W = rng.standard_normal((G, M, N)).astype(np.float32)
    return A, B, W


def _want(A, B, W, lr):
    a, b = A.to(torch.float64).numpy(), B.to(torch.float64).numpy()
    prod = np.stack([oc._mm(a[g], b[g].T, None) for g in range(a.shape[0])])
    mag = np.stack([np.abs(a[g]) @ np.abs(b[g]).T for g in range(a.shape[0])])
    if W is None:
        return prod, mag
    upd = np.stack([oc.commit({"w": W[g]}, {"w": prod[g]}, lr)["w"] for g in range(a.shape[0])])
    return upd, mag


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("commit", [False, True], ids=["plain", "sgd"])
def test_every_form_matches_float64_product(shape, commit):
    G, M, N, Kd = shape
    A, B, W = _operands(7 + M + N + Kd, G, M, N, Kd)
    lr = 0.37
    want, mag = _want(A, B, W if commit else None, lr)
    # fp32 accumulation of Kd exact products: well inside Kd * 2^-24 * sum |a||b|; a dropped or
    # doubled chunk of 8 products is ~1e-3 of that sum
    tol = (lr if commit else 1.0) * 1e-5 * mag + 2e-7 * np.abs(want)
    Ad, Bd = A.to(DEV), B.to(DEV)
    results = {}
    for form in ["auto"] + FORMS:
        out = torch.full((G, M, N), float("nan"), dtype=torch.float32, device=DEV)
        win = None
        if commit:
            out.copy_(torch.from_numpy(W))  # in place: win is the output
            win = out
        hb.gemm_bf16_nt(Ad, Bd, out, win=win, lr=lr, form=form)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        err = np.abs(got.astype(np.float64) - want)
        assert (err <= tol).all(), (form, float((err / tol).max()), np.unravel_index(np.argmax(err / tol), err.shape))
        results[form] = got
    # every form runs the same sequence of MFMAs per element
    for form in FORMS:
        assert np.array_equal(results[form], results["128x128"]), form
    assert np.array_equal(results["auto"], results["128x128"])


def test_seeded_random_shapes_every_form():
    """40 seeded shapes with tails against every tile size; guard rows around C catch a store
    outside the matrix."""
    rng = np.random.default_rng(20090270)
    for case in range(40):
        G = int(rng.integers(1, 4))
        M, N = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        Kd = 8 * int(rng.integers(1, 150))
        commit = bool(case & 1)
        A, B, W = _operands(1000 + case, G, M, N, Kd)
        lr = 0.25
        want, mag = _want(A, B, W if commit else None, lr)
        tol = (lr if commit else 1.0) * 1e-5 * mag + 2e-7 * np.abs(want)
        Ad, Bd = A.to(DEV), B.to(DEV)
        first = None
        for form in FORMS:
            # one guard row of the matrix's width before and after the G * M rows
            buf = torch.full(((G * M + 2) * N,), 12345.0, dtype=torch.float32, device=DEV)
            out = buf[N:N + G * M * N].view(G, M, N)
            win = None
            if commit:
                out.copy_(torch.from_numpy(W))
                win = out
            hb.gemm_bf16_nt(Ad, Bd, out, win=win, lr=lr, form=form)
            torch.cuda.synchronize()
            host = buf.cpu().numpy()
            assert (host[:N] == 12345.0).all() and (host[-N:] == 12345.0).all(), (case, form, "guard")
            got = host[N:N + G * M * N].reshape(G, M, N)
            err = np.abs(got.astype(np.float64) - want)
            assert (err <= tol).all(), (case, (G, M, N, Kd), form, float((err / tol).max()))
            if first is None:
                first = got
            else:
                assert np.array_equal(got, first), (case, form)


def test_padded_pitches_and_untouched_padding():
    """Row pitches larger than the rows (as for the operand copies inside the local step): the
    padding of C keeps its contents."""
    G, M, N, Kd, lda, ldb, ldc = 2, 150, 270, 72, 80, 88, 272
    rng = np.random.default_rng(3)
    A = torch.zeros((G, M, lda), dtype=torch.bfloat16)
    B = torch.zeros((G, N, ldb), dtype=torch.bfloat16)
    A[:, :, :Kd] = torch.from_numpy(rng.uniform(-1, 1, (G, M, Kd)).astype(np.float32)).to(torch.bfloat16)
    B[:, :, :Kd] = torch.from_numpy(rng.uniform(-1, 1, (G, N, Kd)).astype(np.float32)).to(torch.bfloat16)
    A[:, :, Kd:] = 100.0  # must not be read as part of the contraction
    B[:, :, Kd:] = 100.0
    want, mag = _want(A[:, :, :Kd], B[:, :, :Kd], None, 0.0)
    Ad, Bd = A.to(DEV), B.to(DEV)
    lib = hb.load_library()
    for form in range(5):
        out = torch.full((G, M, ldc), -7.0, dtype=torch.float32, device=DEV)
        rc = lib.hpsgd_gemm_bf16_nt(Ad.data_ptr(), lda, M * lda, Bd.data_ptr(), ldb, N * ldb, out.data_ptr(), ldc,
                                    M * ldc, None, 0, 0.0, M, N, Kd, G, form, None)
        assert rc == 0
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (np.abs(got[:, :, :N] - want) <= 1e-5 * mag).all(), form
        assert (got[:, :, N:] == -7.0).all(), form


def test_rejects_bad_arguments():
    lib = hb.load_library()
    A = torch.zeros((1, 16, 16), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((1, 16, 16), dtype=torch.float32, device=DEV)
    ok = dict(lda=16, sA=256, ldb=16, sB=256, ldc=16, sC=256, M=16, N=16, Kd=16, G=1, form=0)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.hpsgd_gemm_bf16_nt(A.data_ptr() + a.get("offA", 0), a["lda"], a["sA"], A.data_ptr(), a["ldb"], a["sB"],
                                      out.data_ptr(), a["ldc"], a["sC"], None, 0, 0.0, a["M"], a["N"], a["Kd"], a["G"],
                                      a["form"], None)

    assert call() == 0
    einval, ealign = call(Kd=12), call(offA=2)
    assert einval != 0 and ealign != 0 and einval != ealign
    assert call(form=5) == einval and call(M=0) == einval and call(lda=8) == einval
    assert call(lda=20) == ealign
    torch.cuda.synchronize()
