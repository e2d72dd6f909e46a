"""Pins for the CPU oracle: it is checked against what the problem itself fixes, never
against the HIP path.  Each pin is chosen so that a plausible slip in the oracle (a
dropped term or scale, a transposed operand, a wrong segment index) breaks it.

Paper passages: LoRA branch Y = XW + XAB (Sec. 2.1); S = XA, Y = S_i B_i + Y_base,
dS = scale dY B_i^T, dX = dS A_i^T, dA_i = X_i^T dS_i, dB_i = S_i^T dY_i (Sec. 5.1);
flat token buffer with per-adapter offsets (App. A.1).
"""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import workloads as wl


def tiny(seed=0, k=7, n=5, ranks=(1, 2, 3), lens=(3, 5, 4), scales=(0.5, -1.5, 2.0), grid=None):
    """Tiny fp32 case with distinct non-square shapes; optional rounding of every input to
    a dyadic grid so that +-h perturbations stay exact in float32."""
    w = wl.make_workload("tiny", "f32", k, n, ranks, lens, scales, seed, b_sigma=0.7)
    if grid:
        q = lambda a: (np.round(a * grid) / grid).astype(np.float32)
        w.X, w.W, w.dY = q(w.X), q(w.W), q(w.dY)
        w.A, w.B = [q(a) for a in w.A], [q(b) for b in w.B]
    return w


def f64(a):
    return np.asarray(a, dtype=np.float64)


def loss(w, X=None, A=None, B=None):
    """L = <Y, dY>, whose gradients w.r.t. X, A_i, B_i are what backward must return."""
    fw = orc.forward(w.X if X is None else X, w.W, w.A if A is None else A,
                     w.B if B is None else B, w.scales, w.offsets)
    return float(np.sum(fw.Y * f64(w.dY)))


# ---- pin 1: B = 0 reproduces X W exactly -------------------------------------------------
def test_zero_B_gives_plain_XW_exactly():
    w = tiny(seed=1, k=19, n=11, ranks=(2, 5, 3), lens=(4, 6, 5))
    zB = [np.zeros_like(b) for b in w.B]
    fw = orc.forward(w.X, w.W, w.A, zB, w.scales, w.offsets, want_base=True)
    # separately coded X W: plain python-order sum in fp64
    ref = np.zeros((w.T, w.n))
    for t in range(w.T):
        for nu in range(w.n):
            acc = 0.0
            for kappa in range(w.k):
                acc += float(w.X[t, kappa]) * float(w.W[kappa, nu])
            ref[t, nu] = acc
    assert np.array_equal(fw.Y, ref)          # bit-for-bit
    assert np.array_equal(fw.Ybase, ref)
    bw = orc.backward(w.dY, w.X, w.W, w.A, zB, w.scales, w.offsets)
    for i in range(w.N):
        assert np.all(bw.dS[i] == 0.0) and np.all(bw.dA[i] == 0.0)
    np.testing.assert_allclose(bw.dX, f64(w.dY) @ f64(w.W).T, rtol=1e-13, atol=1e-13)
    # dB does not vanish with B: it is s S^T dY
    S = [f64(w.X[w.offsets[i]:w.offsets[i + 1]]) @ f64(w.A[i]) for i in range(w.N)]
    for i in range(w.N):
        ref_dB = w.scales[i] * S[i].T @ f64(w.dY[w.offsets[i]:w.offsets[i + 1]])
        np.testing.assert_allclose(bw.dB[i], ref_dB, rtol=1e-12, atol=1e-12)


# ---- pin 2: merged weights W + s A B equal the unmerged path -----------------------------
def test_merged_weight_identity_forward_and_backward():
    w = wl.small_case(seed=3, dtype="f32", k=96, n=72, ranks=(4, 16, 0, 33, 5, 8),
                      seg_lens=(17, 1, 9, 31, 12, 0), b_sigma=0.5)
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    for i in range(w.N):
        lo, hi = w.offsets[i], w.offsets[i + 1]
        Wm = f64(w.W) + w.scales[i] * f64(w.A[i]) @ f64(w.B[i])       # merged weight, fp64
        Xi, dYi = f64(w.X[lo:hi]), f64(w.dY[lo:hi])
        np.testing.assert_allclose(fw.Y[lo:hi], Xi @ Wm, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(bw.dX[lo:hi], dYi @ Wm.T, rtol=1e-12, atol=1e-12)
        G = Xi.T @ dYi                                                  # dense gradient of a merged layer
        np.testing.assert_allclose(bw.dA[i], w.scales[i] * G @ f64(w.B[i]).T, rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(bw.dB[i], w.scales[i] * f64(w.A[i]).T @ G, rtol=1e-11, atol=1e-11)


# ---- pin 3: adapter permutation invariance ----------------------------------------------
def test_adapter_permutation_invariance_exact():
    w = tiny(seed=5, k=13, n=9, ranks=(2, 4, 1, 3), lens=(3, 0, 6, 4), scales=(0.5, 2.0, -1.0, 3.0))
    perm = [2, 0, 3, 1]
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    segs = [(w.offsets[i], w.offsets[i + 1]) for i in range(w.N)]
    Xp = np.concatenate([w.X[lo:hi] for lo, hi in (segs[p] for p in perm)])
    dYp = np.concatenate([w.dY[lo:hi] for lo, hi in (segs[p] for p in perm)])
    lens_p = [segs[p][1] - segs[p][0] for p in perm]
    off_p = [0] + list(np.cumsum(lens_p))
    Ap, Bp, sp = [w.A[p] for p in perm], [w.B[p] for p in perm], [w.scales[p] for p in perm]
    fwp = orc.forward(Xp, w.W, Ap, Bp, sp, off_p)
    bwp = orc.backward(dYp, Xp, w.W, Ap, Bp, sp, off_p)
    for j, p in enumerate(perm):
        lo, hi = segs[p]
        assert np.array_equal(fwp.Y[off_p[j]:off_p[j + 1]], fw.Y[lo:hi])
        assert np.array_equal(bwp.dX[off_p[j]:off_p[j + 1]], bw.dX[lo:hi])
        assert np.array_equal(fwp.S[j], fw.S[p])
        assert np.array_equal(bwp.dA[j], bw.dA[p]) and np.array_equal(bwp.dB[j], bw.dB[p])


# ---- pin 4: central finite differences (exact for this multilinear layer) ---------------
def test_finite_differences_fix_scale_on_dB_and_base_term_in_dX():
    w = tiny(seed=7, k=7, n=5, ranks=(1, 2, 3), lens=(3, 5, 4), scales=(0.5, -1.5, 2.0), grid=64)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    h = np.float32(2.0 ** -4)

    def central(arr_name, idx, pos):
        def bumped(sign):
            if arr_name == "X":
                X = w.X.copy(); X[pos] += sign * h
                return loss(w, X=X)
            lst = [a.copy() for a in (w.A if arr_name == "A" else w.B)]
            lst[idx][pos] += sign * h
            return loss(w, A=lst) if arr_name == "A" else loss(w, B=lst)
        return (bumped(+1) - bumped(-1)) / (2.0 * float(h))

    for t in range(w.T):
        for kappa in range(w.k):
            assert abs(central("X", None, (t, kappa)) - bw.dX[t, kappa]) <= 1e-9 * max(1.0, abs(bw.dX[t, kappa]))
    for i in range(w.N):
        for kappa in range(w.k):
            for rho in range(w.ranks[i]):
                fd = central("A", i, (kappa, rho))
                assert abs(fd - bw.dA[i][kappa, rho]) <= 1e-9 * max(1.0, abs(fd))
        for rho in range(w.ranks[i]):
            for nu in range(w.n):
                fd = central("B", i, (rho, nu))
                assert abs(fd - bw.dB[i][rho, nu]) <= 1e-9 * max(1.0, abs(fd))


# ---- pin 5: linearity ------------------------------------------------------------------
def test_linearity_in_scale_dY_and_X():
    w = tiny(seed=9, k=12, n=10, ranks=(3, 2, 4), lens=(4, 4, 5), scales=(0.5, 1.25, -2.0), grid=256)
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets, want_base=True)
    s2 = list(w.scales); s2[1] *= 2.0
    fw2 = orc.forward(w.X, w.W, w.A, w.B, s2, w.offsets, want_base=True)
    lo, hi = w.offsets[1], w.offsets[2]
    np.testing.assert_allclose(fw2.Y[lo:hi] - fw2.Ybase[lo:hi], 2.0 * (fw.Y[lo:hi] - fw.Ybase[lo:hi]), rtol=1e-13, atol=1e-14)
    mask = np.ones(w.T, bool); mask[lo:hi] = False
    assert np.array_equal(fw2.Y[mask], fw.Y[mask])
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw4 = orc.backward(w.dY * np.float32(4.0), w.X, w.W, w.A, w.B, w.scales, w.offsets)
    assert np.array_equal(bw4.dX, 4.0 * bw.dX)
    for i in range(w.N):
        assert np.array_equal(bw4.dA[i], 4.0 * bw.dA[i]) and np.array_equal(bw4.dB[i], 4.0 * bw.dB[i])
    # <dY, Y(X+V) - Y(X)> == <dX, V>: the layer is linear in X
    rng = np.random.default_rng(0)
    V = (np.round(rng.standard_normal(w.X.shape) * 16) / 16).astype(np.float32)
    fwv = orc.forward(w.X + V, w.W, w.A, w.B, w.scales, w.offsets)
    lhs = np.sum(f64(w.dY) * (fwv.Y - fw.Y)); rhs = np.sum(bw.dX * f64(V))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(rhs))


# ---- pin 6: closed forms ----------------------------------------------------------------
def test_closed_forms_all_ones_and_one_hot():
    k, n, ranks, lens, scales = 6, 4, [2, 3], [3, 2], [0.5, 2.0]
    off = [0, 3, 5]
    wv, av, bv = 0.25, 0.5, 2.0
    X = np.ones((5, k), np.float32); W = np.full((k, n), wv, np.float32)
    A = [np.full((k, r), av, np.float32) for r in ranks]; B = [np.full((r, n), bv, np.float32) for r in ranks]
    fw = orc.forward(X, W, A, B, scales, off)
    for i in range(2):
        assert np.all(fw.Y[off[i]:off[i + 1]] == k * wv + scales[i] * k * ranks[i] * av * bv)
        assert np.all(fw.S[i] == k * av)
    # one-hot rows pick rows of W + s A B
    w = tiny(seed=11, k=6, n=4, ranks=(2, 3), lens=(3, 2), scales=(0.5, 2.0), grid=32)
    Xh = np.zeros_like(w.X)
    hot = [1, 4, 0, 5, 2]
    for t, c in enumerate(hot):
        Xh[t, c] = 1.0
    fwh = orc.forward(Xh, w.W, w.A, w.B, w.scales, w.offsets)
    for t, c in enumerate(hot):
        i = 0 if t < 3 else 1
        row = f64(w.W[c]) + w.scales[i] * f64(w.A[i][c]) @ f64(w.B[i])
        np.testing.assert_allclose(fwh.Y[t], row, rtol=1e-14, atol=1e-15)


# ---- pin 7: library cross-check: one adapter is an ordinary LoRA linear under autograd ----
def test_torch_float64_autograd_per_adapter():
    w = wl.small_case(seed=13, dtype="f32", k=48, n=40, ranks=(4, 16, 0, 7), seg_lens=(9, 1, 5, 20),
                      scales=(2.0, 0.5, 1.0, 16.0 / 7.0), b_sigma=0.3)
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    Wt = torch.tensor(w.W, dtype=torch.float64)
    for i in range(w.N):
        lo, hi = w.offsets[i], w.offsets[i + 1]
        Xi = torch.tensor(w.X[lo:hi], dtype=torch.float64, requires_grad=True)
        Ai = torch.tensor(w.A[i], dtype=torch.float64, requires_grad=True)
        Bi = torch.tensor(w.B[i], dtype=torch.float64, requires_grad=True)
        Yi = Xi @ Wt + w.scales[i] * (Xi @ Ai) @ Bi
        Yi.backward(torch.tensor(w.dY[lo:hi], dtype=torch.float64))
        np.testing.assert_allclose(fw.Y[lo:hi], Yi.detach().numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(fw.S[i], (Xi @ Ai).detach().numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(bw.dX[lo:hi], Xi.grad.numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(bw.dA[i], Ai.grad.numpy(), rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(bw.dB[i], Bi.grad.numpy(), rtol=1e-11, atol=1e-11)
        dS_ref = w.scales[i] * torch.tensor(w.dY[lo:hi], dtype=torch.float64) @ Bi.detach().T
        np.testing.assert_allclose(bw.dS[i], dS_ref.numpy(), rtol=1e-12, atol=1e-12)


# ---- pin 8: isolation between adapters (only diagonal blocks exist, Sec. 5.1) -------------
def test_isolation_between_adapters():
    w = tiny(seed=15, k=10, n=8, ranks=(2, 3, 4), lens=(4, 3, 5))
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    A2 = [a.copy() for a in w.A]; B2 = [b.copy() for b in w.B]; s2 = list(w.scales)
    A2[1] += 1.0; B2[1] -= 2.0; s2[1] = 7.0
    fw2 = orc.forward(w.X, w.W, A2, B2, s2, w.offsets)
    bw2 = orc.backward(w.dY, w.X, w.W, A2, B2, s2, w.offsets)
    lo, hi = w.offsets[1], w.offsets[2]
    mask = np.ones(w.T, bool); mask[lo:hi] = False
    assert np.array_equal(fw2.Y[mask], fw.Y[mask]) and np.array_equal(bw2.dX[mask], bw.dX[mask])
    assert not np.array_equal(fw2.Y[lo:hi], fw.Y[lo:hi])
    for i in (0, 2):
        assert np.array_equal(bw2.dA[i], bw.dA[i]) and np.array_equal(bw2.dB[i], bw.dB[i])


# ---- sampling: a requested subset equals the same entries of the full result ---------------
def test_row_and_column_sampling_matches_full_results():
    w = wl.small_case(seed=17, dtype="bf16", k=64, n=80, ranks=(4, 16, 0, 33, 9, 8),
                      seg_lens=(17, 1, 9, 31, 12, 0))
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    rows = np.array([0, 16, 17, 18, 26, 27, 57, 58, 69]); cols = np.array([0, 3, 63, 79, 17])
    fws = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets, rows=rows, cols=cols)
    assert np.array_equal(fws.Y, fw.Y[np.ix_(rows, cols)])
    kc = np.array([0, 5, 63]); bc = np.array([79, 1])
    bws = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets, rows=rows, cols=kc,
                       a_rows=kc, b_cols=bc, adapters=[0, 3])
    assert np.array_equal(bws.dX, bw.dX[np.ix_(rows, kc)])
    assert np.array_equal(bws.dA[3], bw.dA[3][kc]) and np.array_equal(bws.dB[0], bw.dB[0][:, bc])
    assert bws.dA[1] is None


def test_segment_validation_and_owner():
    with pytest.raises(ValueError):
        orc.forward(np.zeros((4, 2), np.float32), np.zeros((2, 2), np.float32), [], [], [], [0, 3])
    with pytest.raises(ValueError):
        orc.shrink(np.zeros((4, 2), np.float32), [np.zeros((2, 1), np.float32)] * 2, [0, 3, 2, 4][:3])
    off = [0, 3, 3, 7]
    assert list(orc.owner_of_rows(off, np.arange(7))) == [0, 0, 0, 2, 2, 2, 2]


def test_bf16_rounding_helper_is_rne_and_exact_roundtrip():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.14159, 0.0], np.float32)
    r = wl.round_to_bf16(x)
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, ref)
    assert np.array_equal(wl.bf16_bits_to_f32(wl.bf16_bits(r)), r)
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(wl.round_to_bf16(big), torch.tensor(big).to(torch.bfloat16).to(torch.float32).numpy())


def test_flop_count_formula():
    # only diagonal blocks are useful work: sum_i T_i r_i, not (sum T_i)(sum r_i)   (Sec. 5.1)
    assert orc.flop_count(16384, 4096, 4096, [8, 8, 16, 16, 32, 32, 64, 64], [2048] * 8) == \
        4 * 16384 * 4096 * 4096 + 6 * 491520 * 8192
