"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded
inputs.  Tolerances (fp32 GPU path against the fp64 oracle):
  - permutation and keys: bit-exact;
  - deterministic kernels (objective, gap, v = A x, decision values): relative error <= 1e-5;
  - asynchronous solver: final objective within 1e-4 relative of the oracle's converged objective;
  - v = A x after every epoch: relative error (2-norm) <= 1e-4."""
import numpy as np
import pytest
import torch

import datagen
import oracle
import paper_1803_06333_amd as snap

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rel(a, b):
    return abs(a - b) / max(abs(b), 1e-300)


def relnorm(a, b):
    return np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300)


def close(got, want, rtol=1e-4, atol_rel=2e-6):
    """Element by element: |got - want| <= rtol |want| + atol_rel max|want| for every entry, so that an entry
    a thousand times smaller than the largest one still has to be right to a few digits (a norm over
    the whole vector would not notice it)."""
    want = np.asarray(want, dtype=np.float64)
    np.testing.assert_allclose(np.asarray(got, dtype=np.float64), want, rtol=rtol,
                               atol=atol_rel * max(float(np.abs(want).max(initial=0.0)), 1e-300))
    return True


def expected_chunks(ptr, chunk_bytes):
    """Chunks of consecutive coordinates: as many as fit chunk_bytes of index + value (8 bytes per nonzero),
    at least one coordinate each (the rule of the streaming layer, Section 3.2)."""
    cap, m, bounds, c0 = max(1, chunk_bytes // 8), len(ptr) - 1, [0], 0
    while c0 < m:
        c1 = c0 + 1
        while c1 < m and ptr[c1 + 1] - ptr[c0] <= cap:
            c1 += 1
        bounds.append(c1)
        c0 = c1
    return bounds


def executed_order(perm, lengths, small_max=4096, bounds=None):
    """The order the asynchronous engine runs and reports: inside every chunk the split coordinates
    (longer than small_max) of the permutation first, the others after them, each class in the
    permutation's order.  perm: absolute coordinate numbers, chunk after chunk."""
    perm = np.asarray(perm, dtype=np.int64)
    lengths = np.asarray(lengths)
    bounds = [0, perm.size] if bounds is None else bounds
    out = []
    for a, b in zip(bounds, bounds[1:]):
        seg = perm[a:b]
        big = lengths[seg] > small_max
        out += [seg[big], seg[~big]]
    return np.concatenate(out) if out else perm


def gpu_solver(p, **kw):
    # the tests choose the epoch engine themselves: no search for groups unless a test asks for it
    kw.setdefault("auto_groups", False)
    return snap.Solver.from_problem(p.to(DEV), **kw)


def small_problems():
    return {
        "cfg1_sparse_logistic": datagen.uniform_sparse_logistic(),
        "cfg2_dense_ridge": datagen.dense_ridge(n=20_000, d=300),
        "cfg3_zipf_svm": datagen.zipf_sparse_svm(n=40_000, d=5_000, lam=1e-4),
        "cfg4_onehot_logistic": datagen.onehot_fields(n=200_000, d=5_000, lam=1e-4),
        "stream_onehot_logistic": datagen.onehot_fields(n=100_000, d=3_000, lam=1e-3, seed=77),
        "stream_uniform_logistic": datagen.uniform_sparse_logistic(n=50_000, d=5_000, k=20, seed=78),
    }


PROBLEMS = None


def problem(name):
    global PROBLEMS
    if PROBLEMS is None:
        PROBLEMS = small_problems()
    return PROBLEMS[name]


NAMES = ["cfg1_sparse_logistic", "cfg2_dense_ridge", "cfg3_zipf_svm", "cfg4_onehot_logistic"]


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("m", [1, 2, 63, 64, 65, 2047, 2048, 2049, 5000, 300_001])
def test_permutation_bit_exact(m):
    # a matrix with m empty columns is enough to drive the permutation
    ptr = np.zeros(m + 1, dtype=np.int64)
    s = snap.Solver("csc", 4, m, ptr, np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32),
                    np.ones(4, dtype=np.float32), "ridge", 0.1)
    for seed in [0, 1, 2 ** 64 - 1, 180306333]:
        s.epoch(seed)
        perm, keys = s.perm(want_keys=True)
        operm, okeys = oracle.permutation(seed, m, want_keys=True)
        assert np.array_equal(keys, okeys), "keys differ for m=%d seed=%d" % (m, seed)
        assert np.array_equal(perm, operm), "perm differs for m=%d seed=%d" % (m, seed)
    s.close()


@pytest.mark.parametrize("name", NAMES)
def test_deterministic_kernels(name):
    """objective / gap / v = A x / decision values at a fixed model, against the oracle."""
    p = problem(name)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = gpu_solver(p)
    o = oracle.Solver(A, y, p.loss, p.lam)
    rng = np.random.default_rng(7)
    # state 0: the zero model
    P0 = g.objective()
    assert rel(P0, o.primal()) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 1e-5
    # a random model (alpha in [0,1] for the dual form)
    if o.form == "dual":
        x = rng.random(o.m).astype(np.float32)
    else:
        x = (0.05 * rng.standard_normal(o.m)).astype(np.float32)
    g.set_model(x)
    o.x[:] = x.astype(np.float64)
    o.v[:] = o.shared_from_model()
    assert relnorm(g.shared(), o.v) <= 1e-5
    close(g.shared(), o.v, rtol=1e-5, atol_rel=1e-6)           # fp64 sums rounded once, entry by entry
    if o.form == "dual":
        P, D = g.objective(want_dual=True)
        oP, oD = o.primal_dual()
        assert rel(P, oP) <= 1e-5 and rel(D, oD) <= 1e-5
    else:
        assert rel(g.objective(), o.primal()) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 1e-5
    # deterministic: same bits on a second call
    assert g.duality_gap() == g.duality_gap() and g.objective() == g.objective()
    w, xc = g.model()
    assert np.array_equal(xc, x)
    assert relnorm(w, o.weights()) <= 1e-5
    close(w, o.weights(), rtol=1e-5, atol_rel=1e-6)
    # decision values on the training matrix in the layouts predict supports, entry by entry (the weights
    # the oracle multiplies with are the library's fp32 ones, so only the summation differs)
    want = A.matvec(w.astype(np.float64))
    if p.layout == "dense_colmajor":
        out = g.predict("dense_colmajor", p.n, None, None, p.val.numpy())
        assert relnorm(out, want) <= 1e-5 and close(out, want, rtol=1e-5, atol_rel=1e-6)
        rm = np.ascontiguousarray(p.val.numpy().reshape(p.d, p.n).T).reshape(-1)
        out = g.predict("dense_rowmajor", p.n, None, None, torch.from_numpy(rm).to(DEV))
        assert relnorm(out.cpu().numpy(), want) <= 1e-5 and close(out.cpu().numpy(), want, rtol=1e-5, atol_rel=1e-6)
    else:
        out = g.predict(p.layout, p.n, p.ptr.numpy(), p.idx.numpy(), p.val.numpy())
        assert relnorm(out, want) <= 1e-5 and close(out, want, rtol=1e-5, atol_rel=1e-6)
        if "csr" in p.meta:
            rp, ri, rv = (t.to(DEV) for t in p.meta["csr"])
            out = g.predict("csr", p.n, rp, ri, rv)
            assert relnorm(out.cpu().numpy(), want) <= 1e-5 and close(out.cpu().numpy(), want, rtol=1e-5, atol_rel=1e-6)
    g.close()


@pytest.mark.parametrize("name,epochs", [("cfg1_sparse_logistic", 10), ("cfg2_dense_ridge", 20),
                                         ("cfg3_zipf_svm", 30), ("cfg4_onehot_logistic", 40)])
def test_solver_reaches_oracle_objective(name, epochs):
    p = problem(name)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    ref = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-6)
    dual = ref.form == "dual"
    target = ref.dual() if dual else ref.primal()
    g = gpu_solver(p)
    best = None
    for e in range(epochs):
        g.epoch(e)
        # invariant: the maintained v equals A x recomputed from the model (oracle product, fp64)
        _, x = g.model()
        ref_v = oracle.Solver(A, y, p.loss, p.lam)
        ref_v.x[:] = x
        assert relnorm(g.shared(), ref_v.shared_from_model()) <= 1e-4, "v != A x after epoch %d" % e
        if dual:
            assert x.min() >= 0.0 and x.max() <= 1.0
            val = g.objective(want_dual=True)[1]
        else:
            val = g.objective()
        best = val if best is None else (max(best, val) if dual else min(best, val))
    assert rel(best, target) <= 1e-4, "objective %r vs oracle %r" % (best, target)
    assert g.duality_gap() >= 0.0
    g.close()


def test_permutation_is_the_oracles_on_a_real_problem():
    p = problem("cfg4_onehot_logistic")
    g = gpu_solver(p)
    g.epoch(42)
    lengths = np.diff(p.ptr.numpy())
    assert (lengths > 4096).any()                        # the data has coordinates of both classes
    assert np.array_equal(g.perm(), executed_order(oracle.permutation(42, p.d), lengths))
    assert np.array_equal(g.perm(want_keys=True)[1], oracle.permutation(42, p.d, want_keys=True)[1])
    g.close()


def test_orthogonal_columns_match_sequential_result():
    """With mutually orthogonal columns the asynchronous epoch equals the sequential one."""
    n, d = 50_000, 300
    rng = np.random.default_rng(3)
    cols = rng.integers(0, d, size=n)
    order = np.argsort(cols, kind="stable")
    ptr = np.zeros(d + 1, dtype=np.int64)
    ptr[1:] = np.cumsum(np.bincount(cols, minlength=d))
    idx = order.astype(np.int32)
    val = rng.standard_normal(n).astype(np.float32)
    y = rng.standard_normal(n).astype(np.float32)
    g = snap.Solver("csc", n, d, ptr, idx, val, y, "ridge", 0.01)
    g.epoch(5)
    o = oracle.solve(oracle.Matrix("csc", n, d, ptr, idx, val), y, "ridge", 0.01, epochs=1, seed0=5)
    _, x = g.model()
    np.testing.assert_allclose(x, o.x, rtol=2e-5, atol=1e-7)
    assert relnorm(g.shared(), o.v) <= 1e-5
    g.close()


def test_edge_cases_empty_and_ragged():
    # empty columns, a single huge column spanning several segments, one-element columns
    n = 40_000
    lens = [0, 1, 0, 4096, 4097, 8192, 8193, 30_000, 0, 63, 64, 65]
    d = len(lens)
    rng = np.random.default_rng(11)
    ptr = np.zeros(d + 1, dtype=np.int64)
    ptr[1:] = np.cumsum(lens)
    idx = np.concatenate([np.sort(rng.choice(n, size=l, replace=False)) for l in lens]).astype(np.int32)
    val = rng.standard_normal(idx.size).astype(np.float32)
    for loss in ["ridge", "logistic"]:
        y = (rng.standard_normal(n) if loss == "ridge" else np.where(rng.random(n) < 0.5, 1.0, -1.0)).astype(np.float32)
        A = oracle.Matrix("csc", n, d, ptr, idx, val)
        ref = oracle.solve(A, y, loss, 0.05, epochs=300, tol=1e-12)
        g = snap.Solver("csc", n, d, ptr, idx, val, y, loss, 0.05)
        for e in range(60):
            g.epoch(e)
        assert rel(g.objective(), ref.primal()) <= 1e-4
        _, x = g.model()
        assert x[0] == 0.0 and x[2] == 0.0 and x[8] == 0.0
        g.close()
    # dual form with an empty row: alpha = 1
    rows = 3000
    rl = rng.integers(1, 40, size=rows)
    rl[7] = 0
    rptr = np.zeros(rows + 1, dtype=np.int64)
    rptr[1:] = np.cumsum(rl)
    ridx = np.concatenate([np.sort(rng.choice(500, size=l, replace=False)) for l in rl]).astype(np.int32)
    rval = rng.standard_normal(ridx.size).astype(np.float32)
    y = np.where(rng.random(rows) < 0.5, 1.0, -1.0).astype(np.float32)
    g = snap.Solver("csr", rows, 500, rptr, ridx, rval, y, "hinge", 0.01)
    ref = oracle.solve(oracle.Matrix("csr", rows, 500, rptr, ridx, rval), y, "hinge", 0.01, epochs=2000, tol=1e-9)
    for e in range(200):
        g.epoch(e)
    _, a = g.model()
    assert a[7] == 1.0 and a.min() >= 0 and a.max() <= 1
    assert rel(g.objective(want_dual=True)[1], ref.dual()) <= 1e-4
    g.close()


def test_error_paths():
    ptr = np.array([0, 2, 3], dtype=np.int64)
    idx = np.array([0, 1, 2], dtype=np.int32)
    val = np.ones(3, dtype=np.float32)
    y = np.array([1, -1, 1], dtype=np.float32)
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 3, 2, ptr, idx, val, y, "hinge", 0.1)
    assert e.value.code == -2
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 3, 2, ptr, idx, val, y, "ridge", -1.0)
    assert e.value.code == -1
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 2, 2, ptr, idx, val, y[:2], "ridge", 0.1)       # row index 2 out of range
    assert e.value.code == -1
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 3, 2, ptr, idx, val, np.array([1, 0.5, 1], dtype=np.float32), "logistic", 0.1)
    assert e.value.code == -1
    bad = np.array([0, 3, 2], dtype=np.int64)
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 3, 2, bad, idx, val, y, "ridge", 0.1)
    assert e.value.code == -1


def _ragged_matrix(lengths, minor, seed):
    """Compressed arrays whose major slices have the given lengths: distinct minor indices, N(0,1) values."""
    r = np.random.default_rng(seed)
    ptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    idx = np.concatenate([np.sort(r.choice(minor, size=k, replace=False)) for k in lengths] or [np.zeros(0)]).astype(np.int32)
    val = (r.standard_normal(ptr[-1]) / np.sqrt(max(1.0, np.mean(lengths)))).astype(np.float32)
    return ptr, idx, val


@pytest.mark.parametrize("loss,layout", [("ridge", "csc"), ("logistic", "csc"), ("hinge", "csr"), ("logistic", "csr")])
def test_one_coordinate_in_flight_is_the_sequential_method(loss, layout):
    """With a cap of one wavefront the asynchronous kernel visits the coordinates one after the other in
    the epoch order, each seeing all earlier updates: the oracle's sequential pass, step by step, for
    coordinates of every length around the kernel's register rounds (64 and 256 nonzeros) and its loops."""
    lengths = np.array([0, 1, 2, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 1000, 4096] * 3)
    np.random.default_rng(5).shuffle(lengths)
    minor = 5000
    ptr, idx, val = _ragged_matrix(lengths, minor, 6)
    m = len(lengths)
    r = np.random.default_rng(7)
    n, d = (minor, m) if layout == "csc" else (m, minor)
    y = r.standard_normal(n).astype(np.float32) if loss == "ridge" else np.sign(r.standard_normal(n)).astype(np.float32)
    lam = 1e-2
    g = snap.Solver(layout, n, d, ptr, idx, val, y, loss, lam, max_inflight_nnz=1, adaptive=False, auto_groups=False)
    assert g.epoch_stats()["n_large"] == 0
    o = oracle.Solver(oracle.Matrix(layout, n, d, ptr, idx, val), y, loss, lam)
    for e in range(3):
        g.epoch(e)
        o.epoch(e)
        assert np.array_equal(g.perm(), o.last_perm)
        _, x = g.model()
        assert relnorm(x, o.x) <= 2e-5, (e, relnorm(x, o.x))
        assert relnorm(g.shared(), o.v) <= 2e-5
        close(x, o.x, rtol=1e-4, atol_rel=2e-6)
        close(g.shared(), o.v, rtol=1e-4, atol_rel=2e-6)
    assert rel(g.objective(), o.primal()) <= 1e-5
    g.close()


@pytest.mark.parametrize("loss,layout", [("ridge", "csc"), ("logistic", "csc"), ("hinge", "csr"), ("logistic", "csr")])
def test_one_workgroup_in_flight_with_split_coordinates_follows_the_reported_order(monkeypatch, loss, layout):
    """Coordinates longer than the one-wavefront limit are split into segments and run before the
    others.  With one workgroup and one wavefront in flight the epoch is sequential in exactly the
    order that snap_get_perm reports, and equals the oracle visiting the coordinates in that order."""
    monkeypatch.setenv("SNAP_SMALL_MAX", "100")          # limit of the one-wavefront class
    monkeypatch.setenv("SNAP_SEG", "256")                # nonzeros per work item of a split coordinate
    lengths = np.array([0, 1, 64, 100, 101, 255, 256, 257, 511, 512, 513, 1000, 3000] * 3)
    np.random.default_rng(15).shuffle(lengths)
    minor = 4000
    ptr, idx, val = _ragged_matrix(lengths, minor, 16)
    m = len(lengths)
    r = np.random.default_rng(17)
    n, d = (minor, m) if layout == "csc" else (m, minor)
    y = r.standard_normal(n).astype(np.float32) if loss == "ridge" else np.sign(r.standard_normal(n)).astype(np.float32)
    lam = 1e-2
    g = snap.Solver(layout, n, d, ptr, idx, val, y, loss, lam, max_inflight_nnz=1, adaptive=False, auto_groups=False)
    assert g.epoch_stats()["n_large"] == int(np.sum(lengths > 100))
    o = oracle.Solver(oracle.Matrix(layout, n, d, ptr, idx, val), y, loss, lam)
    for e in range(3):
        g.epoch(e)
        want_order = executed_order(oracle.permutation(e, m), lengths, 100)
        got_order, keys = g.perm(want_keys=True)
        assert np.array_equal(got_order.astype(np.int64), want_order)
        assert np.array_equal(keys, oracle.permutation(e, m, want_keys=True)[1])
        o.visit(want_order)
        _, x = g.model()
        np.testing.assert_allclose(x, o.x, rtol=2e-5, atol=2e-6 * np.abs(o.x).max())
        np.testing.assert_allclose(g.shared(), o.v, rtol=2e-5, atol=2e-6 * np.abs(o.v).max())
    assert rel(g.objective(), o.primal()) <= 1e-5
    g.close()


@pytest.mark.parametrize("mean_len", [3, 20, 50, 100, 400])
def test_predict_csr_rows_of_every_length(mean_len):
    """Decision values for CSR rows from empty to long: every lanes-per-row variant of the row kernel
    (chosen from the mean row length) against the oracle's x_i . w."""
    r = np.random.default_rng(100 + mean_len)
    d = 3000
    lengths = np.clip(r.poisson(mean_len, size=700), 0, d)
    lengths[:12] = [0, 1, 7, 8, 9, 15, 16, 17, 63, 64, 65, min(d, 4 * mean_len)]
    lengths[-1] = 0                                                       # a ragged tail that ends empty
    ptr, idx, val = _ragged_matrix(lengths, d, 200 + mean_len)
    n = len(lengths)
    # any trained model will do: a few epochs of ridge on a small CSC problem with the same d
    cl = r.integers(1, 40, size=d)
    cptr, cidx, cval = _ragged_matrix(cl, 500, 300 + mean_len)
    y = r.standard_normal(500).astype(np.float32)
    g = snap.Solver("csc", 500, d, cptr, cidx, cval, y, "ridge", 1e-2, auto_groups=False)
    o = oracle.Solver(oracle.Matrix("csc", 500, d, cptr, cidx, cval), y, "ridge", 1e-2)
    for e in range(2):
        o.epoch(e)
    g.set_model(o.x.astype(np.float32))
    o.x[:] = o.x.astype(np.float32)
    want = o.predict(oracle.Matrix("csr", n, d, ptr, idx, val))
    got = g.predict("csr", n, ptr, idx, val)
    scale = np.abs(want).max()
    assert np.abs(got - want).max() <= 1e-6 * scale
    assert got[0] == 0.0 and got[-1] == 0.0
    got_dev = g.predict("csr", n, torch.from_numpy(ptr).to(DEV), torch.from_numpy(idx).to(DEV), torch.from_numpy(val).to(DEV))
    assert np.array_equal(got_dev.cpu().numpy(), got)                     # fixed summation order
    g.close()


def test_predict_column_layout_agrees_with_the_row_layout_to_the_last_bit_of_its_fp64_sums():
    """The contract of the compressed-column layouts (predict, and v = A x in set_model / recompute_shared):
    every entry is an fp64 sum of its terms rounded once to fp32.  The terms are added with fp64 atomics, so
    the order is not fixed, but the fp64 sum moves by at most a few units in its last place (2^-52 relative
    to the largest partial sum), which changes the fp32 result only when the sum sits within that distance
    of a rounding boundary: against the row layout (fixed order) at most one fp32 ulp, and almost always none."""
    r = np.random.default_rng(77)
    rows, d = 30_000, 2_000
    lengths = np.clip(r.poisson(25, size=rows), 0, d)
    ptr, idx, val = _ragged_matrix(lengths, d, 78)
    rr = np.repeat(np.arange(rows), np.diff(ptr))
    order = np.lexsort((rr, idx))
    cptr = np.concatenate([[0], np.cumsum(np.bincount(idx, minlength=d))]).astype(np.int64)
    cidx, cval = rr[order].astype(np.int32), val[order]
    y = np.sign(r.standard_normal(rows)).astype(np.float32)
    g = snap.Solver("csc", rows, d, cptr, cidx, cval, y, "logistic", 1e-3, auto_groups=False)
    w = r.standard_normal(d).astype(np.float32)
    g.set_model(w)
    by_rows = g.predict("csr", rows, ptr, idx, val)
    want = oracle.Matrix("csr", rows, d, ptr, idx, val).matvec(w.astype(np.float64))
    ulp = np.spacing(np.abs(by_rows).astype(np.float32)).astype(np.float64)
    differing = 0
    for _ in range(3):
        by_cols = g.predict("csc", rows, cptr, cidx, cval)
        assert np.all(np.abs(by_cols.astype(np.float64) - by_rows) <= ulp)
        differing = max(differing, int(np.sum(by_cols != by_rows)))
        assert np.all(np.abs(by_cols - want) <= 0.5 * ulp + 1e-12 * np.abs(want).max() + 1e-6 * ulp)
    assert differing <= rows // 1000
    # the maintained v after set_model is the same product through the same kernel
    v = g.shared()
    assert np.all(np.abs(v.astype(np.float64) - by_rows) <= ulp) and int(np.sum(v != by_rows)) <= rows // 1000
    g.close()


def test_predict_checks_compressed_input():
    """ptr and idx of the matrix handed to predict are checked before any kernel follows them."""
    ptr = np.array([0, 2, 3], dtype=np.int64)
    idx = np.array([0, 1, 2], dtype=np.int32)
    val = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    y = np.array([1, -1, 1], dtype=np.float32)
    g = snap.Solver("csc", 3, 2, ptr, idx, val, y, "ridge", 0.1)
    g.set_model(np.array([0.5, -2.0], dtype=np.float32))
    np.testing.assert_allclose(g.predict("csc", 3, ptr, idx, val), [0.5, 1.0, -6.0], rtol=1e-6)
    rptr = np.array([0, 1, 2, 3], dtype=np.int64)
    ridx = np.array([0, 0, 1], dtype=np.int32)
    np.testing.assert_allclose(g.predict("csr", 3, rptr, ridx, val), [0.5, 1.0, -6.0], rtol=1e-6)
    cases = [("csr", np.array([0, 1, 2, 3], dtype=np.int64), np.array([0, 2, 1], dtype=np.int32)),    # column 2 of 2
             ("csr", np.array([0, 1, 2, 3], dtype=np.int64), np.array([0, -1, 1], dtype=np.int32)),
             ("csr", np.array([0, 2, 1, 3], dtype=np.int64), ridx),                                   # decreasing
             ("csr", np.array([0, 1, 2, 4], dtype=np.int64), ridx),                                   # past nnz
             ("csr", np.array([1, 1, 2, 3], dtype=np.int64), ridx),                                   # not from 0
             ("csc", np.array([0, 2, 3], dtype=np.int64), np.array([0, 3, 2], dtype=np.int32))]       # row 3 of 3
    for layout, p_, i_ in cases:
        with pytest.raises(snap.SnapError) as e:
            g.predict(layout, 3, p_, i_, val)
        assert e.value.code == -1
        if torch.cuda.is_available():                    # the same on device arrays
            with pytest.raises(snap.SnapError) as e:
                g.predict(layout, 3, torch.from_numpy(p_).to(DEV), torch.from_numpy(i_).to(DEV), torch.from_numpy(val).to(DEV))
            assert e.value.code == -1
    np.testing.assert_allclose(g.predict("csr", 3, rptr, ridx, val), [0.5, 1.0, -6.0], rtol=1e-6)   # still usable
    g.close()


# ---------------------------------------------------------------------------------------------
# streaming (Section 3.2): chunks of coordinates copied from pinned host memory while the previous
# chunk is processed; chunk order fixed, permutation inside each chunk
def _pinned(p):
    q = p.to("cpu")
    for name in ("ptr", "idx", "val", "y"):
        setattr(q, name, getattr(q, name).pin_memory())
    return q


@pytest.mark.parametrize("name,chunk_bytes,budget,unit", [("stream_uniform_logistic", 1 << 20, 2 << 20, True),
                                                          ("stream_uniform_logistic", 1 << 20, 2 << 20, False),
                                                          ("stream_onehot_logistic", 5 << 20, 4 << 20, True)])
def test_streamed_epochs_match_oracle_and_resident(name, chunk_bytes, budget, unit):
    p = problem(name)
    if not unit:                                         # general values: the value array is streamed too
        p = p.to("cpu")
        p.val = torch.from_numpy((0.5 + np.random.default_rng(2).random(p.nnz)).astype(np.float32))
    q = _pinned(p)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = snap.Solver.from_problem(q, device_budget_bytes=budget, chunk_bytes=chunk_bytes, auto_groups=False, profile=True)
    ptr = p.ptr.numpy()
    bounds = expected_chunks(ptr, chunk_bytes)           # the chunking rule, applied here to the same offsets
    assert g.chunk_bounds() == bounds
    assert len(bounds) - 1 >= 6 and bounds[0] == 0 and bounds[-1] == p.d
    assert g.stream_bytes() == (4 if unit else 8) * p.nnz      # all-ones values are not copied again
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=bounds)
    r = gpu_solver(p)                                    # resident twin for the deterministic kernels
    assert r.stream_bytes() == 0
    assert rel(g.duality_gap(), r.duality_gap()) <= 1e-12
    epochs = 30
    for e in range(epochs):
        g.epoch(e)
        o.epoch(e)
        assert np.array_equal(g.perm().astype(np.int64), executed_order(o.last_perm, np.diff(ptr), bounds=bounds)), \
            "chunked permutation differs"
        if e % 8 == 0:
            _, x = g.model()
            chk = oracle.Solver(A, y, p.loss, p.lam)
            chk.x[:] = x
            assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4
    if name == "stream_uniform_logistic":
        # columns without field structure: the chunked order converges, compare with the converged oracle
        target = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-6, chunk_bounds=bounds).primal()
        assert rel(g.objective(), target) <= 1e-4
    else:
        # one field after another is a slow order for the sequential oracle too (one block sweep per
        # epoch): at equal epoch count the asynchronous solver tracks it ...
        assert rel(g.objective(), o.primal()) <= 2e-3
        assert g.objective() < 0.75 * np.log(2.0)
        # ... and run on, it reaches the converged objective (the minimum is unique, whatever the order:
        # the oracle gets there with a permutation over all coordinates) to the stated 1e-4
        target = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-6).primal()
        e = epochs
        while rel(g.objective(), target) > 1e-4 and e < 4000:
            for _ in range(50):
                g.epoch(e)
                e += 1
        assert rel(g.objective(), target) <= 1e-4, "after %d epochs" % e
        print("streamed one-hot: %d epochs to 1e-4 of the converged objective" % e)
    st = g.epoch_stats()
    assert st["n_chunks"] == len(bounds) - 1 and st["copy_ms"] > 0 and st["scd_ms"] > 0
    # deterministic kernels through the streaming path equal the resident ones at the same model
    _, x = g.model()
    r.set_model(x)
    g.set_model(x)                                       # recomputes v chunk by chunk
    assert relnorm(g.shared(), r.shared().astype(np.float64)) <= 1e-6
    # (the two v differ by the order of their fp32 atomics; the gap, a squared gradient norm near
    # the optimum, amplifies that)
    assert rel(g.duality_gap(), r.duality_gap()) <= 1e-3
    assert rel(g.objective(), r.objective()) <= 1e-6
    g.close()
    r.close()


def test_profiling_a_streamed_epoch_copies_nothing_extra():
    """options.profile times the chunk copies that an epoch makes anyway: the same bytes cross the host
    link as without it, one matrix per epoch (the first chunk of an epoch is fetched during the epoch
    before), and the copy and kernel times it reports are those of all chunks."""
    p = problem("stream_uniform_logistic")
    q = _pinned(p)
    copied = []
    for profile in (False, True):
        g = snap.Solver.from_problem(q, device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False, profile=profile)
        C = len(g.chunk_bounds()) - 1
        assert C > 2
        g.epoch(0)
        base = g.bytes_copied()
        for e in range(1, 4):
            g.epoch(e)
        copied.append(g.bytes_copied() - base)
        if profile:
            st = g.epoch_stats()
            assert st["n_chunks"] == C and st["copy_ms"] > 0.0 and st["scd_ms"] > 0.0
        g.close()
    assert copied[0] == copied[1] == 3 * g_stream_bytes(p)


def g_stream_bytes(p):
    return 4 * p.nnz          # unit values: the indices alone are streamed


# ---------------------------------------------------------------------------------------------
# passes over part of the chunks, chosen by their share in the duality gap (Section 3.2)
def test_chunk_gap_shares_match_the_oracle_streamed_and_grouped():
    # streamed chunks, at a model a few epochs in
    p = problem("stream_uniform_logistic")
    q = _pinned(p)
    A = oracle.Matrix.from_problem(p)
    g = snap.Solver.from_problem(q, device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False)
    bounds = g.chunk_bounds()
    o = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=bounds)
    for e in range(3):
        o.epoch(e)
    g.set_model(o.x.astype(np.float32))
    chk = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=bounds)
    chk.x[:] = o.x.astype(np.float32)
    chk.v[:] = chk.shared_from_model()
    want = chk.chunk_gaps()
    got = g.chunk_gaps()
    assert got.shape == want.shape and got.min() >= 0.0
    np.testing.assert_allclose(got, want, rtol=1e-3, atol=1e-3 * want.max())
    assert rel(got.sum(), g.duality_gap()) <= 1e-9          # the shares add up to the gap the library reports
    g.close()
    # groups of the exact sweeps, with an l1 term (Fenchel form of the shares)
    p = _onehot_variant("logistic", True)
    groups = p.meta["field_starts"] + [p.d]
    g = gpu_solver(p, group_bounds=groups, lam1=2e-4)
    o = oracle.Solver(oracle.Matrix.from_problem(p), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True,
                      lam1=2e-4)
    for e in range(2):
        g.epoch(e)
        o.epoch(e)
    got, want = g.chunk_gaps(), o.chunk_gaps()
    np.testing.assert_allclose(got, want, rtol=2e-3, atol=1e-3 * want.max())
    assert rel(got.sum(), g.duality_gap()) <= 1e-6
    g.close()


@pytest.mark.parametrize("loss", ["hinge", "logistic"])
def test_chunk_gap_shares_dual_forms_streamed(loss):
    """Shares of streamed batches of examples in P - D, dual forms, against the oracle at the same alpha."""
    p = problem("cfg3_zipf_svm") if loss == "hinge" else _dual_logistic_problem()
    A = oracle.Matrix.from_problem(p)
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, chunk_bytes=1 << 19)
    bounds = g.chunk_bounds()
    assert len(bounds) > 4
    o = oracle.Solver(A, p.y.numpy(), loss, p.lam, chunk_bounds=bounds)
    for e in range(2):
        o.epoch(e)
    g.set_model(o.x.astype(np.float32))
    chk = oracle.Solver(A, p.y.numpy(), loss, p.lam, chunk_bounds=bounds)
    chk.x[:] = o.x.astype(np.float32)
    chk.v[:] = chk.shared_from_model()
    # v = X^T (y alpha) of a trained model is what is left of large terms that cancel (partial sums of
    # the frequent features: thousands of times the result); the library sums it in fp64
    assert relnorm(g.shared(), chk.v) <= 1e-6
    want, got = chk.chunk_gaps(), g.chunk_gaps()
    assert got.shape == want.shape and got.min() >= 0.0
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=1e-6 * want.max())
    assert rel(got.sum(), g.duality_gap()) <= 1e-6
    # the selected solve runs on them as well and ends below the tolerance
    tol = 0.2 * got.sum()
    passes, visits, gap = g.solve_selected(10, 60, tol, 2, max(1, (len(bounds) - 1) // 2))
    assert gap <= tol and passes < 60
    g.close()


def test_pass_over_selected_groups_equals_the_oracle():
    p = _onehot_variant("logistic", True)
    groups = p.meta["field_starts"] + [p.d]
    g = gpu_solver(p, group_bounds=groups)
    o = oracle.Solver(oracle.Matrix.from_problem(p), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    g.epoch(0)
    o.epoch(0)
    for e, chunks in enumerate([[5, 0, 17], [38], [20, 21, 22, 1], list(range(39))]):
        before = g.model()[1].copy()
        g.epoch_chunks(10 + e, chunks)
        o.epoch(10 + e, chunks=chunks)
        _, x = g.model()
        assert relnorm(x, o.x) <= 2e-5
        assert relnorm(g.shared(), o.v) <= 2e-5
        close(x, o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
        untouched = np.ones(p.d, dtype=bool)
        for c in chunks:
            untouched[groups[c]:groups[c + 1]] = False
        assert np.array_equal(x[untouched], before[untouched])
    g.epoch_chunks(99, [])                                   # a pass over nothing
    assert np.array_equal(g.model()[1], x)
    for bad in ([39], [-1], [3, 3]):
        with pytest.raises(snap.SnapError) as e:
            g.epoch_chunks(0, bad)
        assert e.value.code == -1
    g.close()


def test_streamed_pass_over_selected_chunks_and_the_selected_solve():
    p = problem("stream_uniform_logistic")
    q = _pinned(p)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = snap.Solver.from_problem(q, device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False)
    bounds = g.chunk_bounds()
    C = len(bounds) - 1
    chunk_nnz = np.diff(p.ptr.numpy()[bounds])
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=bounds)
    g.epoch(0)
    o.epoch(0)
    assert g.bytes_copied() >= 4 * p.nnz
    # a working set of two chunks is copied at most once, however often it is swept
    base = g.bytes_copied()
    for e in range(4):
        g.epoch_chunks(20 + e, [C - 1, 2])
        o.epoch(20 + e, chunks=[C - 1, 2])
        gp = g.perm().astype(np.int64)                    # chunk by chunk; the visited ones hold the new order
        n_last = bounds[C] - bounds[C - 1]
        assert np.array_equal(gp[bounds[C - 1]:bounds[C]], o.last_perm[:n_last])
        assert np.array_equal(gp[bounds[2]:bounds[3]], o.last_perm[n_last:])
    assert g.bytes_copied() - base <= 4 * (chunk_nnz[C - 1] + chunk_nnz[2])
    _, x = g.model()
    chk = oracle.Solver(A, y, p.loss, p.lam)
    chk.x[:] = x
    assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4
    assert rel(g.objective(), o.primal()) <= 1e-3            # asynchronous against sequential, five passes in
    # three chunks rotate through the two buffers
    base = g.bytes_copied()
    g.epoch_chunks(30, [1, 3, 0])
    assert 0 < g.bytes_copied() - base <= 4 * (chunk_nnz[1] + chunk_nnz[3] + chunk_nnz[0] + chunk_nnz[1])
    g.close()
    # the selected solve ends at the same optimum as plain epochs, with fewer chunk visits per pass
    g = snap.Solver.from_problem(q, device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False)
    target = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-6, chunk_bounds=bounds).primal()
    passes, visits, gap = g.solve_selected(0, 400, 1e-5, 4, max(2, C // 2))
    assert gap <= 1e-5 and passes < 400
    assert visits < passes * C
    assert rel(g.objective(), target) <= 1e-4
    o2 = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=bounds)
    po, vo, go = oracle.solve_selected(o2, 0, 400, 1e-5, 4, max(2, C // 2))
    assert go <= 1e-5 and abs(po - passes) <= max(4, passes // 4)          # the sequential oracle needs about as many
    g.close()


def test_keys_made_on_the_host_give_the_same_epoch_order():
    """options.host_keys: the keys come from host threads through pinned memory and the copy stream
    (third pipeline stage of Section 3.2); generator and order are the same as with device-made keys."""
    # resident, a permutation long enough for several host threads, and many epochs through the two buffers
    p = datagen.uniform_sparse_logistic(n=3_000, d=300_000, k=2, seed=31)
    g = gpu_solver(p, host_keys=True)
    r = gpu_solver(p)
    for e in (0, 1, 2, 7):
        g.epoch(e)
        r.epoch(e)
        pg, kg = g.perm(want_keys=True)
        pr, kr = r.perm(want_keys=True)
        assert np.array_equal(kg, kr) and np.array_equal(pg, pr)
    assert np.array_equal(pg.astype(np.int64), oracle.permutation(7, p.d))
    g.close()
    r.close()
    # streamed: chunk by chunk, against the chunked oracle, and the solver still converges
    p = problem("stream_uniform_logistic")
    q = _pinned(p)
    A = oracle.Matrix.from_problem(p)
    g = snap.Solver.from_problem(q, device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False, host_keys=True)
    bounds = g.chunk_bounds()
    o = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=bounds)
    for e in range(30):
        g.epoch(e)
        o.epoch(e)
        assert np.array_equal(g.perm().astype(np.int64), o.last_perm)
    target = oracle.solve(A, p.y.numpy(), p.loss, p.lam, epochs=500, tol=1e-6, chunk_bounds=bounds).primal()
    assert rel(g.objective(), target) <= 1e-4
    g.close()


def test_streaming_needs_pinned_memory():
    p = problem("cfg1_sparse_logistic")
    with pytest.raises(snap.SnapError) as e:
        snap.Solver.from_problem(p, device_budget_bytes=1 << 10, chunk_bytes=1 << 16)
    assert e.value.code == -1


# ---------------------------------------------------------------------------------------------
# exact group sweeps: the coordinates of one group (the columns of a one-hot field) do not share
# rows, so a sweep over the groups equals sequential SCD visiting the groups in the same (seeded
# random) order -- the oracle with those groups as shuffled chunks -- update for update, not just in
# the limit
# element-wise bounds of the group sweeps against the fp64 oracle: fp32 data path, fixed-point sums with a
# resolution of 2^-20 of the largest |value| per term
GROUP_RTOL, GROUP_ATOL = 2e-4, 5e-6


def _onehot_variant(loss, unit):
    p = datagen.onehot_fields(n=150_000, d=4_000, lam=1e-4, seed=91)
    rng = np.random.default_rng(4)
    if not unit:
        p.val = torch.from_numpy((0.5 + rng.random(p.nnz)).astype(np.float32))
    if loss == "ridge":
        p.loss = "ridge"
        p.y = torch.from_numpy(rng.standard_normal(p.n).astype(np.float32))
    return p


@pytest.mark.parametrize("loss,unit", [("logistic", True), ("logistic", False), ("ridge", True), ("ridge", False)])
def test_group_sweeps_equal_sequential_oracle(loss, unit):
    p = _onehot_variant(loss, unit)
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = gpu_solver(p, group_bounds=groups)
    assert g.chunk_bounds() == groups
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(6):
        g.epoch(e)
        o.epoch(e)
        _, x = g.model()
        # same trajectory as the sequential oracle (fp32 against fp64), coordinate by coordinate
        assert relnorm(x, o.x) <= 2e-5, "model differs from the sequential oracle after epoch %d" % e
        assert relnorm(g.shared(), o.v) <= 2e-5
        close(x, o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
        close(g.shared(), o.v, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
        assert rel(g.objective(), o.primal()) <= 1e-5
        assert g.epoch_stats()["rejected"] == 0
    assert np.array_equal(g.perm().astype(np.int64), o.last_perm)
    assert rel(g.duality_gap(), o.gap()) <= 1e-3        # squared gradient norm, amplifies fp32 differences
    # continue to convergence of the gap
    for e in range(6, 40):
        g.epoch(e)
        o.epoch(e)
    assert rel(g.objective(), o.primal()) <= 1e-5
    g.close()


# The default launch shape (256 workgroups of 1024 threads, 8 rows per thread and iteration) gives every
# thread at most one iteration on the small problems above, and their few short coordinates never fill
# a wavefront's staging ring.  The tuning knobs (read at creation) shrink the launch and the LDS tables,
# so that the same comparison also covers threads with several iterations, wavefronts cut short in their
# last iteration, rings flushed inside the loop, steps gathered from beyond the LDS table, and the
# alternative layouts (two workgroups per compute unit, two-word sums, no dense buffer).
@pytest.mark.parametrize("knobs", [
    {"SNAP_ROW_WGS": "16", "SNAP_HOT_MAX": "8"},
    {"SNAP_ROW_WGS": "3", "SNAP_HOT_MAX": "40", "SNAP_DELTA_LDS": "16"},
    {"SNAP_ROW_WGS": "16", "SNAP_HOT_MAX": "8", "SNAP_COMPACT": "0"},
    {"SNAP_WGS_PER_CU": "2", "SNAP_HOT_ROWS": "128"},
    {"SNAP_PACK": "0", "SNAP_ROW_WGS": "24"},
], ids=lambda k: ",".join("%s=%s" % (n[5:].lower(), v) for n, v in k.items()))
@pytest.mark.parametrize("loss,unit", [("logistic", True), ("logistic", False), ("ridge", True), ("ridge", False)])
def test_group_sweeps_other_launch_shapes(monkeypatch, knobs, loss, unit):
    for name, value in knobs.items():
        monkeypatch.setenv(name, value)
    p = _onehot_variant(loss, unit)
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    g = gpu_solver(p, group_bounds=groups)
    o = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(4):
        g.epoch(e)
        o.epoch(e)
        _, x = g.model()
        assert relnorm(x, o.x) <= 2e-5, "model differs from the sequential oracle after epoch %d" % e
        assert relnorm(g.shared(), o.v) <= 2e-5
        close(x, o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
        close(g.shared(), o.v, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert rel(g.objective(), o.primal()) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 1e-3
    g.close()


@pytest.mark.parametrize("loss,unit", [("logistic", True), ("logistic", False), ("ridge", True)])
def test_group_sweeps_read_the_maps_of_small_groups_as_bytes(monkeypatch, loss, unit):
    """Resident maps: a group of at most 255 columns has its map read as one byte per row, the others as two;
    every pairing of the two widths in a row pass occurs (13 fields of 64 columns among 26 of 500), and the
    results are those of two-byte maps throughout, bit for bit, with the accept check's fused loss sums too."""
    p = datagen.onehot_fields(n=90_011, d=13 * 64 + 26 * 500, lam=1e-4, seed=29)
    rng = np.random.default_rng(6)
    if not unit:
        p.val = torch.from_numpy((0.5 + rng.random(p.nnz)).astype(np.float32))
    if loss == "ridge":
        p.loss = "ridge"
        p.y = torch.from_numpy(rng.standard_normal(p.n).astype(np.float32))
    groups = p.meta["field_starts"] + [p.d]
    G = len(groups) - 1
    small = sum(1 for a, b in zip(groups, groups[1:]) if b - a <= 255)
    assert 0 < small < G
    a = gpu_solver(p, group_bounds=groups, adaptive=True)
    monkeypatch.setenv("SNAP_MAP8", "0")
    b = gpu_solver(p, group_bounds=groups, adaptive=True)
    monkeypatch.delenv("SNAP_MAP8")
    o = oracle.Solver(oracle.Matrix.from_problem(p), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    assert a.duality_gap() == b.duality_gap()
    pairs = set()
    for e in range(5):
        a.epoch(e)
        b.epoch(e)
        o.epoch(e)
        assert np.array_equal(a.model()[1], b.model()[1]) and np.array_equal(a.shared(), b.shared())
        assert a.objective() == b.objective()
        order = [c for c in snap.block_order(e, G)]
        pairs |= {(groups[u + 1] - groups[u] <= 255, groups[w + 1] - groups[w] <= 255) for u, w in zip(order, order[1:])}
    assert len(pairs) == 4
    sa, sb = a.epoch_stats(), b.epoch_stats()
    assert sa["byte_map_groups"] == small and sb["byte_map_groups"] == 0 and sa["row_map_bytes"] == sb["row_map_bytes"] == 2
    assert sa["rejected"] == 0
    close(a.model()[1], o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert a.duality_gap() == b.duality_gap()
    assert np.array_equal(a.chunk_gaps(), b.chunk_gaps())
    a.epoch_chunks(9, [0, 20, 1])
    b.epoch_chunks(9, [0, 20, 1])
    assert np.array_equal(a.model()[1], b.model()[1])
    a.close()
    b.close()


# ---------------------------------------------------------------------------------------------
# group sweeps on streamed data (Section 3.2): the matrix stays in pinned host memory; what is streamed
# per epoch are the row maps, which the library builds at creation into pinned memory of its own
@pytest.mark.parametrize("knobs", [{}, {"SNAP_ROW_WGS": "16", "SNAP_HOT_MAX": "8"}, {"SNAP_HOT_ROWS": "1000000000"},
                                   {"SNAP_ROW_WGS": "3", "SNAP_HOT_MAX": "40", "SNAP_DELTA_LDS": "16"}, {"SNAP_MAP8": "0"},
                                   {"SNAP_PFX": "0"}],
                         ids=lambda k: ",".join("%s=%s" % (n[5:].lower(), v) for n, v in k.items()) or "default")
@pytest.mark.parametrize("loss", ["logistic", "ridge"])
def test_streamed_group_sweeps_equal_resident_ones_bit_for_bit_and_the_oracle(monkeypatch, knobs, loss):
    for name, value in knobs.items():
        monkeypatch.setenv(name, value)
    p = _onehot_variant(loss, True)
    groups = p.meta["field_starts"] + [p.d]
    G = len(groups) - 1
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    r = gpu_solver(p, group_bounds=groups)                                  # resident twin
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, chunk_bytes=4 << 20, group_bounds=groups,
                                 profile=True)
    assert g.chunk_bounds() == groups
    n_pad = (p.n + 7) // 8 * 8
    # one row map per field: a byte per row for fields of at most 255 columns (all of them here), else two
    small = [b - a <= 255 and knobs.get("SNAP_MAP8") != "0" for a, b in zip(groups, groups[1:])]
    assert all(small) or not any(small)
    plain = sum(n_pad * (1 if s8 else 2) for s8 in small)
    prefix_coded = knobs.get("SNAP_PFX") != "0" and knobs.get("SNAP_MAP8") != "0"      # (the default: fewer bytes still)
    assert (0.3 * plain < g.stream_bytes() <= 0.9 * plain if prefix_coded else g.stream_bytes() == plain) and r.stream_bytes() == 0
    mb = 1 if small[0] else 2
    assert g.objective() == r.objective()
    assert rel(g.duality_gap(), r.duality_gap()) <= (0 if "SNAP_HOT_ROWS" not in knobs else 1e-6)
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    # (without any hot rank the resident sweeps sum the short coordinates straight from v, a wavefront each,
    # the streamed ones from the dense buffer, 16 lanes each: same terms, another order of the fp32 additions)
    same = (lambda a, b: np.array_equal(a, b)) if "SNAP_HOT_ROWS" not in knobs else (lambda a, b: relnorm(a, b.astype(np.float64)) <= 1e-6)
    base = g.bytes_copied()
    for e in range(5):
        g.epoch(e)
        r.epoch(e)
        o.epoch(e)
        xg, xr = g.model()[1], r.model()[1]
        assert same(xg, xr), "streamed and resident sweeps differ after epoch %d" % e
        assert same(g.shared(), r.shared())
        np.testing.assert_allclose(xg, o.x, rtol=2e-4, atol=2e-5 * np.abs(o.x).max())
        assert relnorm(xg, o.x) <= 2e-5
        assert rel(g.objective(), o.primal()) <= 1e-5
    # (a map still in the ring is not copied)
    assert 5 * (g.stream_bytes() - 2 * n_pad * mb) <= g.bytes_copied() - base <= 5 * g.stream_bytes()
    st = g.epoch_stats()
    assert st["n_chunks"] == G and st["copy_ms"] > 0 and st["scd_ms"] > 0 and st["row_map_bytes"] == 2 and st["unit_values"] == 1
    assert np.array_equal(g.perm(), r.perm())
    assert rel(g.duality_gap(), r.duality_gap()) <= (0 if "SNAP_HOT_ROWS" not in knobs else 1e-2)   # the gradient pass streams the maps too
    if "SNAP_HOT_ROWS" not in knobs:
        assert np.array_equal(g.chunk_gaps(), r.chunk_gaps())
    else:   # (squared gradients near the optimum amplify the different order of the fp32 sums)
        np.testing.assert_allclose(g.chunk_gaps(), r.chunk_gaps(), rtol=2e-2, atol=1e-3 * r.chunk_gaps().max())
    for e, chunks in enumerate([[5, 0, 17], [38], [20, 21], list(range(G))]):   # passes over part of the fields
        g.epoch_chunks(10 + e, chunks)
        r.epoch_chunks(10 + e, chunks)
        o.epoch(10 + e, chunks=chunks)
        assert same(g.model()[1], r.model()[1]) and same(g.shared(), r.shared())
    assert relnorm(g.model()[1], o.x) <= 2e-5
    assert g.epoch_stats()["n_chunks"] == G                  # (a pass over listed fields is not timed: no stale figures)
    base = g.bytes_copied()
    g.epoch_chunks(50, [3, 9])
    g.epoch_chunks(51, [3, 9])                                            # the two maps are still in the ring
    assert g.bytes_copied() - base <= 2 * n_pad * mb
    # a new model goes through the caller's (borrowed) column arrays
    w = (0.1 * np.random.default_rng(3).standard_normal(p.d)).astype(np.float32)
    g.set_model(w)
    r.set_model(w)
    assert np.array_equal(g.shared(), r.shared()) or relnorm(g.shared(), r.shared().astype(np.float64)) <= 1e-6
    g.close()
    r.close()


@pytest.mark.parametrize("row_wgs", [None, "5"])
def test_streamed_group_sweeps_escape_coded_row_maps(monkeypatch, row_wgs):
    """Fields of 256 ... 65535 columns whose rows concentrate on the low ranks cross the host link as one
    byte per row plus the two-byte ranks of the rows that do not fit (rank >= 254), and are decoded on the
    device: same sweeps bit for bit as with resident maps, and the bytes per pass are the coded sizes."""
    if row_wgs:
        monkeypatch.setenv("SNAP_ROW_WGS", row_wgs)
    monkeypatch.setenv("SNAP_PFX", "0")              # (the prefix code, which is shorter still, has a test of its own)
    p = datagen.onehot_fields(n=100_003, d=13 * 64 + 26 * 1000, lam=1e-4, seed=23)    # 26 Zipf fields of 1000 columns
    groups = p.meta["field_starts"] + [p.d]
    G = len(groups) - 1
    lengths = np.diff(p.ptr.numpy())
    n_pad = (p.n + 7) // 8 * 8
    n_esc = (n_pad + 4095) // 4096 * 4096
    want_bytes, coded = 0, 0
    for a, b in zip(groups, groups[1:]):
        by_rank = np.sort(lengths[a:b], kind="stable")[::-1]
        if b - a <= 255:
            want_bytes += n_pad
        else:
            blob = (n_esc + 4 * (n_esc // 4096) + 2 * int(by_rank[254:].sum()) + 7) // 8 * 8
            assert 10 * blob <= 9 * 2 * n_pad          # the generator's Zipf fields are concentrated enough
            want_bytes += blob
            coded += 1
    assert coded == 26
    r = gpu_solver(p, group_bounds=groups)
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, group_bounds=groups)
    assert g.stream_bytes() == want_bytes < 0.75 * G * n_pad * 2
    o = oracle.Solver(oracle.Matrix.from_problem(p), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(4):
        g.epoch(e)
        r.epoch(e)
        o.epoch(e)
        assert np.array_equal(g.model()[1], r.model()[1]) and np.array_equal(g.shared(), r.shared())
    close(g.model()[1], o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert g.duality_gap() == r.duality_gap()
    g.close()
    # a field whose rows spread evenly over 3000 columns gains nothing from the coding: two bytes per row
    n, d1, d2 = 60_000, 3_000, 40
    rng = np.random.default_rng(5)
    cols = np.concatenate([rng.integers(0, d1, size=n), d1 + rng.integers(0, d2, size=n)])
    rows = np.concatenate([np.arange(n), np.arange(n)])
    order = np.lexsort((rows, cols))
    ptr = np.concatenate([[0], np.cumsum(np.bincount(cols, minlength=d1 + d2))]).astype(np.int64)
    idx = rows[order].astype(np.int32)
    y = np.where(rng.random(n) < 0.4, 1.0, -1.0).astype(np.float32)
    pin = lambda a: torch.from_numpy(a).pin_memory()
    u = snap.Solver("csc", n, d1 + d2, pin(ptr), pin(idx), None, pin(y), "logistic", 1e-4, group_bounds=[0, d1, d1 + d2],
                    device_budget_bytes=1 << 16)
    assert u.stream_bytes() == 2 * n + n
    ou = oracle.Solver(oracle.Matrix("csc", n, d1 + d2, ptr, idx, np.ones(idx.size, dtype=np.float32)), y, "logistic", 1e-4,
                       chunk_bounds=[0, d1, d1 + d2], shuffle_chunks=True)
    for e in range(3):
        u.epoch(e)
        ou.epoch(e)
    close(u.model()[1], ou.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    u.close()
    r.close()


def _entropy_bits(counts):
    c = np.asarray([x for x in counts if x > 0], dtype=np.float64)
    return float(-(c * np.log2(c / c.sum())).sum())


@pytest.mark.parametrize("row_wgs", [None, "7"])
def test_streamed_group_sweeps_prefix_coded_row_maps(monkeypatch, row_wgs):
    """By default a streamed row map crosses the host link prefix-coded (a Huffman code of rank classes, whole
    ranks for small groups, quarter octaves with extra bits for large ones) and is decoded on the device: the
    sweeps are those of resident maps bit for bit, and the bytes per pass lie between the entropy of the ranks
    and a little above it.  Groups of every kind: 64-bin fields, Zipf fields of 1000 columns, a field that
    covers only part of the rows, evenly spread columns, a group of one column."""
    if row_wgs:
        monkeypatch.setenv("SNAP_ROW_WGS", row_wgs)
    p = datagen.onehot_fields(n=100_003, d=13 * 64 + 26 * 1000, lam=1e-4, seed=23)
    groups = p.meta["field_starts"] + [p.d]
    G = len(groups) - 1
    lengths = np.diff(p.ptr.numpy())
    n_pad = (p.n + 7) // 8 * 8
    n_esc = (n_pad + 4095) // 4096 * 4096
    floor_bits = sum(_entropy_bits(list(lengths[a:b]) + [n_esc - int(lengths[a:b].sum())]) for a, b in zip(groups, groups[1:]))
    overhead = G * (8 * (n_esc // 2048) + 2 * (n_esc // 64) + 16)
    r = gpu_solver(p, group_bounds=groups)
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, group_bounds=groups)
    assert floor_bits / 8 <= g.stream_bytes() - overhead <= 1.05 * floor_bits / 8
    assert g.stream_bytes() < 0.62 * (13 * n_pad + 26 * 2 * n_pad)
    o = oracle.Solver(oracle.Matrix.from_problem(p), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(4):
        g.epoch(e)
        r.epoch(e)
        o.epoch(e)
        assert np.array_equal(g.model()[1], r.model()[1]) and np.array_equal(g.shared(), r.shared())
    close(g.model()[1], o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert g.duality_gap() == r.duality_gap()
    g.close()
    r.close()
    # hand-made groups: 3000 evenly spread columns over all rows; 100 columns over the first half of the rows
    # only; one column that holds every third row; 40 columns over two thirds of the rows; 62 and 63 columns (the
    # largest group coded rank by rank, the smallest coded by classes); 65535 columns (the highest classes)
    n = 70_001
    rng = np.random.default_rng(12)
    parts, d0, bounds = [], 0, [0]
    for width, rows in ((3000, np.arange(n)), (100, np.arange(n // 2)), (1, np.arange(0, n, 3)), (40, np.arange(n)[np.arange(n) % 3 != 1]),
                        (62, np.arange(n)), (63, np.arange(n)), (65535, np.arange(n))):
        cols = d0 + (rng.integers(0, width, size=rows.size) if width > 100 else np.minimum(rng.geometric(0.08, size=rows.size) - 1, width - 1))
        parts.append((cols, rows))
        d0 += width
        bounds.append(d0)
    # ... and 16 columns whose lengths halve from 32768 down to 1: an unlimited Huffman code would need 16 bits
    parts.append((d0 + np.repeat(np.arange(16), 2 ** np.arange(15, -1, -1)), np.arange(65535)))
    d0 += 16
    bounds.append(d0)
    cols = np.concatenate([c for c, _ in parts])
    rows = np.concatenate([r_ for _, r_ in parts])
    order = np.lexsort((rows, cols))
    ptr = np.concatenate([[0], np.cumsum(np.bincount(cols, minlength=d0))]).astype(np.int64)
    idx = rows[order].astype(np.int32)
    y = np.where(rng.random(n) < 0.4, 1.0, -1.0).astype(np.float32)
    pin = lambda a: torch.from_numpy(a).pin_memory()
    u = snap.Solver("csc", n, d0, pin(ptr), pin(idx), None, pin(y), "logistic", 1e-4, group_bounds=bounds, device_budget_bytes=1 << 16)
    ur = snap.Solver("csc", n, d0, ptr, idx, None, y, "logistic", 1e-4, group_bounds=bounds, auto_groups=False)
    n_pad = (n + 7) // 8 * 8
    assert u.stream_bytes() < 0.85 * (2 * 2 * n_pad + 6 * n_pad)      # (uncoded: two bytes for the wide groups, one for the others)
    ou = oracle.Solver(oracle.Matrix("csc", n, d0, ptr, idx, np.ones(idx.size, dtype=np.float32)), y, "logistic", 1e-4,
                       chunk_bounds=bounds, shuffle_chunks=True)
    for e in range(4):
        u.epoch(e)
        ur.epoch(e)
        ou.epoch(e)
        assert np.array_equal(u.model()[1], ur.model()[1]) and np.array_equal(u.shared(), ur.shared())
    close(u.model()[1], ou.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert u.duality_gap() == ur.duality_gap()
    u.close()
    ur.close()


def test_streamed_group_sweeps_are_declined_without_pinned_memory_for_the_maps(monkeypatch):
    """The row maps need pinned host memory of the library's own; when that cannot be had (forced here), the
    handle streams column chunks with the asynchronous engine instead of failing."""
    monkeypatch.setenv("SNAP_NO_PINNED_MAPS", "1")
    p = problem("stream_onehot_logistic")
    groups = p.meta["field_starts"] + [p.d]
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=4 << 20, chunk_bytes=5 << 20, group_bounds=groups)
    bounds = g.chunk_bounds()
    assert bounds == expected_chunks(p.ptr.numpy(), 5 << 20) and g.stream_bytes() == 4 * p.nnz
    P0 = g.objective()
    for e in range(10):
        g.epoch(e)
    assert g.objective() < 0.8 * P0
    assert np.array_equal(g.perm().astype(np.int64),
                          executed_order(_chunked_perm(9, bounds), np.diff(p.ptr.numpy()), bounds=bounds))
    g.close()


def _chunked_perm(seed, bounds):
    """The oracle's permutation chunk by chunk (absolute coordinate numbers)."""
    return np.concatenate([oracle.permutation(seed, b - a, chunk=k).astype(np.int64) + a
                           for k, (a, b) in enumerate(zip(bounds, bounds[1:]))])


def test_streamed_group_sweeps_wide_group_and_error_paths(monkeypatch):
    # a field with more than 65535 categories: 4-byte row maps through the ring
    monkeypatch.setenv("SNAP_ROW_WGS", "16")
    n, d1, d2 = 200_000, 70_000, 50
    rng = np.random.default_rng(8)
    c1 = np.where(rng.random(n) < 0.5, rng.integers(0, 100, size=n), rng.integers(0, d1, size=n))
    c2 = rng.integers(0, d2, size=n)
    cols = np.concatenate([c1, d1 + c2])
    rows = np.concatenate([np.arange(n), np.arange(n)])
    order = np.lexsort((rows, cols))
    d = d1 + d2
    ptr = np.zeros(d + 1, dtype=np.int64)
    ptr[1:] = np.cumsum(np.bincount(cols, minlength=d))
    idx = rows[order].astype(np.int32)
    val = np.ones(idx.size, dtype=np.float32)
    y = np.where(rng.random(n) < 0.3, 1.0, -1.0).astype(np.float32)
    groups = [0, d1, d]
    pin = lambda a: torch.from_numpy(a).pin_memory()
    g = snap.Solver("csc", n, d, pin(ptr), pin(idx), pin(val), pin(y), "logistic", 1e-4, group_bounds=groups,
                    device_budget_bytes=1 << 20, chunk_bytes=1 << 20)
    assert g.stream_bytes() == 2 * n * 4
    o = oracle.Solver(oracle.Matrix("csc", n, d, ptr, idx, val), y, "logistic", 1e-4, chunk_bounds=groups,
                      shuffle_chunks=True)
    for e in range(4):
        g.epoch(e)
        o.epoch(e)
        assert relnorm(g.model()[1], o.x) <= 2e-5
    assert rel(g.objective(), o.primal()) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 1e-3
    g.close()
    # values other than 1 are not streamed as maps: refused, the asynchronous streamed epoch remains
    val2 = (0.5 + rng.random(idx.size)).astype(np.float32)
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", n, d, pin(ptr), pin(idx), pin(val2), pin(y), "logistic", 1e-4, group_bounds=groups,
                    device_budget_bytes=1 << 20, chunk_bytes=1 << 20)
    assert e.value.code == -2
    # overlapping groups are found while the maps are built
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", n, d, pin(ptr), pin(idx), pin(val), pin(y), "logistic", 1e-4, group_bounds=[0, d],
                    device_budget_bytes=1 << 20, chunk_bytes=1 << 20)
    assert e.value.code == -1


def test_pattern_only_matrix_without_a_value_array():
    """val = NULL at creation stands for "every stored value is 1": same results as an array of ones in the
    three engines that take compressed columns (asynchronous, group sweeps, group sweeps on streamed maps)
    and in the streamed asynchronous epoch."""
    p = _onehot_variant("logistic", True)
    groups = p.meta["field_starts"] + [p.d]
    q = p.to("cpu")
    q.val = None
    assert q.nnz == p.nnz
    o = oracle.Solver(oracle.Matrix.from_problem(q), p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(3):
        o.epoch(e)
    for kw, pin in [({"group_bounds": groups}, False), ({"group_bounds": groups, "device_budget_bytes": 1 << 20}, True)]:
        a = snap.Solver.from_problem(_pinned(p) if pin else p.to(DEV), auto_groups=False, **kw)
        b = snap.Solver.from_problem(_pinned_some(q) if pin else q.to(DEV), auto_groups=False, **kw)
        for e in range(3):
            a.epoch(e)
            b.epoch(e)
        assert np.array_equal(a.model()[1], b.model()[1]) and np.array_equal(a.shared(), b.shared())
        assert relnorm(b.model()[1], o.x) <= 2e-5
        assert a.duality_gap() == b.duality_gap()
        a.close()
        b.close()
    # asynchronous engines: resident with one wavefront in flight (sequential, hence comparable), and streamed
    a = gpu_solver(p, max_inflight_nnz=1, adaptive=False)
    b = gpu_solver(q, max_inflight_nnz=1, adaptive=False)
    a.epoch(0)
    b.epoch(0)
    assert relnorm(b.model()[1], a.model()[1].astype(np.float64)) <= 1e-6
    a.close()
    b.close()
    s = snap.Solver.from_problem(_pinned_some(q), device_budget_bytes=1 << 20, chunk_bytes=4 << 20, auto_groups=False)
    t = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, chunk_bytes=4 << 20, auto_groups=False)
    assert s.stream_bytes() == t.stream_bytes() == 4 * p.nnz and s.epoch_stats()["unit_values"] == 1
    assert s.objective() == t.objective() and s.duality_gap() == t.duality_gap()
    for e in range(20):
        s.epoch(e)
        t.epoch(e)
    # (two asynchronous runs: the same trajectory up to the order of their atomics)
    assert rel(s.objective(), t.objective()) <= 1e-3 and s.objective() < 0.8 * np.log(2.0)
    chk = oracle.Solver(oracle.Matrix.from_problem(q), p.y.numpy(), p.loss, p.lam)
    chk.x[:] = s.model()[1]
    assert relnorm(s.shared(), chk.shared_from_model()) <= 1e-4
    s.close()
    t.close()


def _pinned_some(p):
    q = p.to("cpu")
    for name in ("ptr", "idx", "val", "y"):
        if getattr(q, name) is not None:
            setattr(q, name, getattr(q, name).pin_memory())
    return q


@pytest.mark.parametrize("loss", ["logistic", "ridge"])
def test_group_sweeps_are_bit_reproducible(loss):
    """No floating-point atomics and no order left to chance (integer sums in LDS, fixed orders
    elsewhere): two runs from the same seeds end in the same bits."""
    p = _onehot_variant(loss, True)
    groups = p.meta["field_starts"] + [p.d]
    models, shared = [], []
    for profile in (0, 0, 1, 2):                           # timing the row passes (all, or one in four) changes nothing
        g = gpu_solver(p, group_bounds=groups, profile=profile)
        for e in range(3):
            g.epoch(100 + e)
        models.append(g.model()[1].copy())
        shared.append(np.array(g.shared(), copy=True))
        if profile:
            st = g.epoch_stats()
            assert st["n_items"] == len(groups) and 0.0 < st["large_ms"] < st["epoch_ms"]
        g.close()
    for k in range(1, 4):
        assert np.array_equal(models[0], models[k])
        assert np.array_equal(shared[0], shared[k])


def test_group_sweeps_reject_overlapping_groups():
    p = problem("cfg1_sparse_logistic")                  # uniform columns: any two groups of columns overlap
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(p, group_bounds=[0, 500, 1000])
    assert e.value.code == -1
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(p, group_bounds=[0, 500, 999])
    assert e.value.code == -1
    # one coordinate per group is always valid (and equals the plain sequential order of the groups)
    q = datagen.uniform_sparse_logistic(n=2000, d=60, k=5, seed=3)
    g = gpu_solver(q, group_bounds=list(range(61)))
    o = oracle.Solver(oracle.Matrix.from_problem(q), q.y.numpy(), q.loss, q.lam, chunk_bounds=list(range(61)),
                      shuffle_chunks=True)
    for e in range(5):
        g.epoch(e)
        o.epoch(e)
    assert rel(g.objective(), o.primal()) <= 1e-5
    g.close()


@pytest.mark.parametrize("skewed", [False, True], ids=["uniform", "skewed"])
def test_group_sweeps_wide_group_uses_32_bit_maps(monkeypatch, skewed):
    """A group with more than 65535 coordinates takes the 32-bit row-map path.  Uniform categories:
    every coordinate of the wide group is short (no LDS sums at all for it); skewed: a hundred long
    coordinates beside the short ones (LDS sums, and the dense buffer for the short coordinates' rows, with
    four rows per thread and iteration), on a launch small enough for several iterations per thread."""
    n, d1, d2 = 200_000, 70_000, 50
    rng = np.random.default_rng(8)
    c1 = rng.integers(0, d1, size=n)                     # field 1: 70 000 categories
    if skewed:
        monkeypatch.setenv("SNAP_ROW_WGS", "16")
        c1 = np.where(rng.random(n) < 0.5, rng.integers(0, 100, size=n), c1)
    c2 = rng.integers(0, d2, size=n)                     # field 2: 50 categories
    cols = np.concatenate([c1, d1 + c2])
    rows = np.concatenate([np.arange(n), np.arange(n)])
    order = np.lexsort((rows, cols))
    d = d1 + d2
    ptr = np.zeros(d + 1, dtype=np.int64)
    ptr[1:] = np.cumsum(np.bincount(cols, minlength=d))
    idx = rows[order].astype(np.int32)
    val = np.ones(idx.size, dtype=np.float32)
    y = np.where(rng.random(n) < 0.3, 1.0, -1.0).astype(np.float32)
    groups = [0, d1, d]
    g = snap.Solver("csc", n, d, ptr, idx, val, y, "logistic", 1e-4, group_bounds=groups)
    o = oracle.Solver(oracle.Matrix("csc", n, d, ptr, idx, val), y, "logistic", 1e-4, chunk_bounds=groups,
                      shuffle_chunks=True)
    for e in range(5):
        g.epoch(e)
        o.epoch(e)
        _, x = g.model()
        assert relnorm(x, o.x) <= 2e-5
        close(x, o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
    assert rel(g.objective(), o.primal()) <= 1e-5
    g.close()


@pytest.mark.parametrize("loss,stream", [("logistic", False), ("ridge", False), ("logistic", True)])
def test_group_sweeps_with_the_accept_check(loss, stream):
    """With the accept check on, the group sweeps keep the state before an epoch by writing into a second
    array (no copy) and sum the objective in their last pass.  Accepted epochs are the same epochs bit for
    bit; a discarded one (forced here by steps scaled far beyond a Newton step) leaves model and shared
    vector exactly as they were, halves the step scale, and the solver still reaches the oracle's objective."""
    p = _onehot_variant(loss, True)
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    mk = (lambda **kw: snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, group_bounds=groups, **kw)) if stream \
        else (lambda **kw: gpu_solver(p, group_bounds=groups, **kw))
    a, b = mk(adaptive=True, profile=True), mk(adaptive=False)
    for e in range(5):
        a.epoch(e)
        b.epoch(e)
        assert a.epoch_stats()["rejected"] == 0
        assert np.array_equal(a.model()[1], b.model()[1]) and np.array_equal(a.shared(), b.shared())
        assert rel(a.objective(), b.objective()) == 0.0
    a.epoch_chunks(7, [3, 1])                                # a pass over part of the fields, checked as well
    b.epoch_chunks(7, [3, 1])
    assert np.array_equal(a.model()[1], b.model()[1]) and np.array_equal(a.shared(), b.shared())
    a.close()
    b.close()
    # steps 24 times too long make the first epochs worse: discarded, state untouched, scale halved (24, 12, 6,
    # 3, then 1.5, which converges; a power of two would pass through 2, where exact steps on a quadratic
    # leave the objective where it is)
    target = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-7).primal()
    g = mk(adaptive=True, damping=24.0, profile=True)
    rejected, prev_x, prev_v, prev_P = 0, g.model()[1].copy(), np.array(g.shared(), copy=True), g.objective()
    scales = []
    for e in range(80):
        g.epoch(e)
        st = g.epoch_stats()
        scales.append(st["damping"])
        if st["rejected"]:
            rejected += 1
            assert np.array_equal(g.model()[1], prev_x) and np.array_equal(g.shared(), prev_v)
            assert g.objective() == prev_P
        else:
            assert g.objective() <= prev_P * (1 + 2e-6)
        prev_x, prev_v, prev_P = g.model()[1].copy(), np.array(g.shared(), copy=True), g.objective()
    assert rejected >= 2 and scales[-1] < scales[0]
    assert rel(prev_P, target) <= 1e-4
    chk = oracle.Solver(A, y, p.loss, p.lam)
    chk.x[:] = prev_x
    assert relnorm(prev_v, chk.shared_from_model()) <= 1e-4
    g.close()


# ---------------------------------------------------------------------------------------------
# the accept check (Section 3.1, "Adaptive Damping"): too much work in flight makes an epoch worse;
# the epoch is discarded, the cap on work in flight halved, and the solver still converges
def test_accept_check_discards_bad_epochs_and_recovers():
    p = problem("cfg4_onehot_logistic")
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    target = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-6).primal()
    g = gpu_solver(p, max_inflight_nnz=1 << 30, profile=True)      # everything in flight: Jacobi on one-hot data
    rejected, caps, prev = 0, [], g.objective()
    for e in range(80):
        g.epoch(e)
        st = g.epoch_stats()
        cur = g.objective()
        if st["rejected"]:
            rejected += 1
            assert cur == pytest.approx(prev, rel=1e-12), "a discarded epoch must leave the state untouched"
        else:
            assert cur <= prev * (1 + 2e-6)
        caps.append(st["inflight_nnz"])
        prev = cur
    assert rejected >= 1 and caps[-1] < caps[0]
    assert rel(prev, target) <= 1e-4
    # without the check the same setting does not get there
    u = gpu_solver(p, max_inflight_nnz=1 << 30, adaptive=False)
    for e in range(20):
        u.epoch(e)
    assert not (rel(u.objective(), target) <= 1e-4)
    g.close()
    u.close()


def test_options_damping_and_refresh():
    p = problem("cfg1_sparse_logistic")
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    target = oracle.solve(A, y, p.loss, p.lam, epochs=200, tol=1e-9).primal()
    g = gpu_solver(p, damping=0.5, refresh_v_every=3, profile=True)
    for e in range(60):
        g.epoch(e)
    assert g.epoch_stats()["damping"] == pytest.approx(0.5)
    assert rel(g.objective(), target) <= 1e-4              # half steps still converge, more slowly
    _, x = g.model()
    chk = oracle.Solver(A, y, p.loss, p.lam)
    chk.x[:] = x
    assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-5
    g.close()


# ---------------------------------------------------------------------------------------------
# l1 / elastic-net term (eq. (1): lasso and elastic-net regularisers)
@pytest.mark.parametrize("name,lam1", [("cfg1_sparse_logistic", 2e-3), ("cfg2_dense_ridge", 1e-4),
                                       ("cfg4_onehot_logistic", 2e-4)])
def test_elastic_net_objective_and_gap_at_a_given_model(name, lam1):
    p = problem(name)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    rng = np.random.default_rng(12)
    w = (0.05 * rng.standard_normal(p.d) * (rng.random(p.d) < 0.3)).astype(np.float32)
    o = oracle.Solver(A, y, p.loss, p.lam, lam1=lam1)
    o.x[:] = w
    o.v[:] = o.shared_from_model()
    g = gpu_solver(p, lam1=lam1)
    g.set_model(w)
    assert relnorm(g.shared(), o.v) <= 1e-5
    assert rel(g.objective(), o.primal()) <= 1e-5
    P, D = g.objective(want_dual=True)
    gap = g.duality_gap()
    assert rel(gap, o.gap()) <= 1e-4
    assert abs((P - D) - gap) <= 1e-12 * max(1.0, abs(P))
    # without the l1 term the same handle type gives the plain objective (the term is really added)
    g0 = gpu_solver(p)
    g0.set_model(w)
    assert rel(g.objective() - g0.objective(), lam1 * np.abs(w.astype(np.float64)).sum()) <= 1e-6
    g.close()
    g0.close()


@pytest.mark.parametrize("loss,unit", [("logistic", True), ("ridge", False)])
def test_elastic_net_group_sweeps_equal_sequential_oracle(loss, unit):
    p = _onehot_variant(loss, unit)
    lam1 = 2e-4 if loss == "logistic" else 2e-3
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = gpu_solver(p, group_bounds=groups, lam1=lam1)
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True, lam1=lam1)
    for e in range(8):
        g.epoch(e)
        o.epoch(e)
        _, x = g.model()
        assert relnorm(x, o.x) <= 5e-5, "model differs from the sequential oracle after epoch %d" % e
        assert relnorm(g.shared(), o.v) <= 5e-5
        assert rel(g.objective(), o.primal()) <= 1e-5
    _, x = g.model()
    zg, zo = x == 0.0, o.x == 0.0
    assert zo.sum() > 0.2 * p.d                      # the term does produce a sparse model here
    # a coordinate sitting on the threshold may fall on either side in fp32: allow a handful
    assert np.sum(zg != zo) <= max(3, p.d // 1000)
    assert np.abs(o.x[zg != zo]).max(initial=0.0) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 2e-3 or abs(g.duality_gap() - o.gap()) <= 1e-7
    g.close()


@pytest.mark.parametrize("name,lam1,epochs", [("cfg1_sparse_logistic", 2e-3, 12), ("cfg2_dense_ridge", 1e-4, 25),
                                              ("cfg4_onehot_logistic", 2e-4, 40)])
def test_elastic_net_async_reaches_oracle_objective(name, lam1, epochs):
    p = problem(name)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    ref = oracle.solve(A, y, p.loss, p.lam, epochs=500, tol=1e-7, lam1=lam1)
    target = ref.primal()
    assert 0 < np.sum(ref.x == 0.0) < p.d
    g = gpu_solver(p, lam1=lam1)
    best = None
    for e in range(epochs):
        g.epoch(e)
        _, x = g.model()
        chk = oracle.Solver(A, y, p.loss, p.lam, lam1=lam1)
        chk.x[:] = x
        assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4, "v != A x after epoch %d" % e
        val = g.objective()
        best = val if best is None else min(best, val)
    assert rel(best, target) <= 1e-4, "objective %r vs oracle %r" % (best, target)
    gap = g.duality_gap()
    assert gap >= g.objective() - target - 1e-6 * abs(target)
    _, x = g.model()
    assert abs(np.mean(x == 0.0) - np.mean(ref.x == 0.0)) <= 0.05     # exact zeros are kept
    g.close()


def test_elastic_net_error_paths():
    p = problem("cfg3_zipf_svm")
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(p, lam1=0.1)
    assert e.value.code == -2
    q = problem("cfg1_sparse_logistic")
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(q, lam1=-1.0)
    assert e.value.code == -1


# ---------------------------------------------------------------------------------------------
# dense data: exact tile sweeps (ridge) and the asynchronous dense path (any loss)
def _tile_bounds(d, b=128):
    return list(range(0, d, b)) + [d]


@pytest.mark.parametrize("n,d,lam1", [(20_000, 300, 0.0), (20_001, 70, 0.0), (5_003, 64, 0.0), (20_000, 300, 1e-4),
                                      (900, 130, 0.0), (5, 1, 0.0), (3, 200, 0.0), (1, 129, 0.0), (1026, 257, 1e-5)])
def test_dense_tile_sweeps_equal_sequential_oracle(n, d, lam1):
    p = datagen.dense_ridge(n=n, d=d, seed=5)
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    bounds = _tile_bounds(d)
    g = gpu_solver(p, lam1=lam1, dense_tiles=True)
    assert g.chunk_bounds() == bounds
    o = oracle.Solver(A, y, "ridge", p.lam, chunk_bounds=bounds, shuffle_chunks=True, lam1=lam1)
    for e in range(6):
        g.epoch(e)
        o.epoch(e)
        _, x = g.model()
        assert relnorm(x, o.x) <= 2e-5, "model differs from the sequential oracle after epoch %d" % e
        assert relnorm(g.shared(), o.v) <= 2e-5
        close(x, o.x, rtol=1e-4, atol_rel=5e-6)
        close(g.shared(), o.v, rtol=1e-4, atol_rel=5e-6)
        assert rel(g.objective(), o.primal()) <= 1e-5
        assert g.epoch_stats()["rejected"] == 0
    assert np.array_equal(g.perm().astype(np.int64), o.last_perm)
    # the maintained v is A x recomputed from the model
    chk = oracle.Solver(A, y, "ridge", p.lam)
    chk.x[:] = g.model()[1]
    assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-5
    g.close()


def test_dense_tile_sweeps_are_the_default_and_can_be_switched_off():
    p = problem("cfg2_dense_ridge")
    A = oracle.Matrix.from_problem(p)
    ref = oracle.solve(A, p.y.numpy(), "ridge", p.lam, epochs=500, tol=1e-6)
    g = gpu_solver(p)
    assert g.chunk_bounds() == _tile_bounds(p.d)            # tiles in use
    a = gpu_solver(p, dense_tiles=False)
    assert a.chunk_bounds() == [0, p.d]                      # one chunk: asynchronous epoch
    for e in range(20):
        g.epoch(e)
        a.epoch(e)
    assert rel(g.objective(), ref.primal()) <= 1e-4
    assert rel(a.objective(), ref.primal()) <= 1e-4
    g.close()
    a.close()
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(problem("cfg1_sparse_logistic"), dense_tiles=True)
    assert e.value.code == -2


def test_dense_logistic_asynchronous_path():
    p = datagen.dense_ridge(n=20_000, d=300, seed=8)
    rng = np.random.default_rng(8)
    X = p.val.numpy().reshape(p.d, p.n).T.astype(np.float64)
    wstar = rng.standard_normal(p.d)
    p.y = torch.from_numpy(np.where(X @ wstar + 0.1 * rng.standard_normal(p.n) > 0, 1.0, -1.0).astype(np.float32))
    p.loss, p.lam = "logistic", 1e-3
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    ref = oracle.solve(A, y, "logistic", p.lam, epochs=500, tol=1e-6)
    g = gpu_solver(p)
    assert g.chunk_bounds() == [0, p.d]
    best = None
    for e in range(25):
        g.epoch(e)
        chk = oracle.Solver(A, y, "logistic", p.lam)
        chk.x[:] = g.model()[1]
        assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4
        val = g.objective()
        best = val if best is None else min(best, val)
    assert rel(best, ref.primal()) <= 1e-4
    g.close()


# ---------------------------------------------------------------------------------------------
# logistic regression in the dual form (CSR, examples as coordinates)
def _dual_logistic_problem():
    p = datagen.zipf_sparse_svm(n=40_000, d=5_000, lam=1e-5, seed=31)
    p.loss = "logistic"
    return p


def test_dual_logistic_deterministic_kernels():
    p = _dual_logistic_problem()
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    o = oracle.Solver(A, y, "logistic", p.lam)
    g = gpu_solver(p)
    # start: alpha = 1/2, v = X^T (y/2)
    _, x = g.model()
    assert np.all(x == 0.5)
    assert relnorm(g.shared(), o.v) <= 1e-5
    P, D = g.objective(want_dual=True)
    Po, Do = o.primal_dual()
    assert rel(P, Po) <= 1e-5 and rel(D, Do) <= 1e-5
    # a random interior point, and the clipping of values outside (0,1)
    rng = np.random.default_rng(3)
    a = rng.random(p.n).astype(np.float32)
    a[:10] = [0.0, 1.0, -3.0, 7.0, 1e-9, 1 - 1e-9, 0.5, 0.25, 2.0 ** -20, 1 - 2.0 ** -20]
    g.set_model(a)
    o.x[:] = np.clip(a.astype(np.float64), 2.0 ** -20, 1 - 2.0 ** -20)
    o.v[:] = o.shared_from_model()
    _, x = g.model()
    assert np.array_equal(x.astype(np.float64), o.x.astype(np.float32).astype(np.float64))
    assert relnorm(g.shared(), o.v) <= 1e-5
    P, D = g.objective(want_dual=True)
    Po, Do = o.primal_dual()
    assert rel(P, Po) <= 1e-5 and rel(D, Do) <= 1e-5
    assert rel(g.duality_gap(), Po - Do) <= 1e-5
    w, _ = g.model()
    assert relnorm(w, o.weights()) <= 1e-5
    g.close()


def test_dual_logistic_solver_reaches_oracle_objective():
    p = _dual_logistic_problem()
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    ref = oracle.solve(A, y, "logistic", p.lam, epochs=500, tol=1e-7)
    target = ref.dual()
    # the dual optimum is the primal optimum (primal oracle on the transposed storage)
    cptr, cidx, cval = datagen.csr_to_csc(p.n, p.d, p.ptr, p.idx, p.val)
    Ac = oracle.Matrix("csc", p.n, p.d, cptr.numpy(), cidx.numpy(), cval.numpy())
    prim = oracle.solve(Ac, y, "logistic", p.lam, epochs=500, tol=1e-7)
    assert rel(target, prim.primal()) <= 1e-5
    g = gpu_solver(p)
    best = None
    for e in range(40):
        g.epoch(e)
        _, x = g.model()
        assert x.min() >= 2.0 ** -20 and x.max() <= 1 - 2.0 ** -20
        chk = oracle.Solver(A, y, "logistic", p.lam)
        chk.x[:] = x
        assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4, "v != A alpha after epoch %d" % e
        D = g.objective(want_dual=True)[1]
        best = D if best is None else max(best, D)
    assert rel(best, target) <= 1e-4, "dual objective %r vs oracle %r" % (best, target)
    # at the optimum P - D is the difference of two fp32-data sums of size 0.6: zero up to their rounding
    assert -1e-6 <= g.duality_gap() <= 1e-3
    w, _ = g.model()
    assert relnorm(w, prim.weights()) <= 2e-2
    g.close()


def test_dual_logistic_streamed_row_chunks():
    # the terabyte-scale setting of Section 3.2 / 4: examples streamed chunk by chunk, v in R^d resident
    p = _dual_logistic_problem()
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    q = _pinned(p)
    g = snap.Solver.from_problem(q, device_budget_bytes=4 << 20, chunk_bytes=2 << 20)
    bounds = g.chunk_bounds()
    assert len(bounds) - 1 >= 6
    # Visiting the examples chunk by chunk (permuted inside a chunk only) converges much more slowly on
    # this ill-conditioned problem than a permutation over all examples -- for the sequential oracle as
    # well (0.576 against the optimum 0.589 after 40 epochs) -- so the streamed solver is compared with
    # the oracle that takes the same chunked order, at equal epochs.
    o = oracle.Solver(A, y, "logistic", p.lam, chunk_bounds=bounds)
    for e in range(40):
        g.epoch(e)
        o.epoch(e)
        if e % 10 == 9:
            assert rel(g.objective(want_dual=True)[1], o.dual()) <= 1e-3, "epoch %d" % e
    assert np.array_equal(g.perm().astype(np.int64), o.last_perm)
    chk = oracle.Solver(A, y, "logistic", p.lam)
    chk.x[:] = g.model()[1]
    assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4
    # run on to the converged dual objective (unique maximum; the oracle reaches it with a permutation
    # over all examples): the stated 1e-4
    target = oracle.solve(A, y, "logistic", p.lam, epochs=500, tol=1e-7).dual()
    e = 40
    while rel(g.objective(want_dual=True)[1], target) > 1e-4 and e < 6000:
        for _ in range(100):
            g.epoch(e)
            e += 1
    assert rel(g.objective(want_dual=True)[1], target) <= 1e-4, "after %d epochs" % e
    print("streamed dual logistic: %d epochs to 1e-4 of the converged objective" % e)
    g.close()


# ---------------------------------------------------------------------------------------------
# automatic search for ranges of coordinates with disjoint supports
@pytest.mark.parametrize("loss,unit", [("logistic", True), ("ridge", False)])
def test_auto_groups_finds_the_fields_of_one_hot_data(loss, unit):
    p = _onehot_variant(loss, unit)
    fields = p.meta["field_starts"] + [p.d]
    g = gpu_solver(p, auto_groups=None)                  # default: look for groups
    assert g.chunk_bounds() == fields
    A = oracle.Matrix.from_problem(p)
    o = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=fields, shuffle_chunks=True)
    for e in range(4):
        g.epoch(e)
        o.epoch(e)
        assert relnorm(g.model()[1], o.x) <= 2e-5
        close(g.model()[1], o.x, rtol=GROUP_RTOL, atol_rel=GROUP_ATOL)
        assert g.epoch_stats()["rejected"] == 0
    g.close()
    # required and found: the same
    g = gpu_solver(p, auto_groups=True)
    assert g.chunk_bounds() == fields
    g.close()


def test_auto_groups_merges_what_can_be_merged_and_handles_empty_columns():
    # three "fields" over disjoint row sets can share one range; empty columns belong anywhere
    n, d = 3000, 40
    rng = np.random.default_rng(9)
    cols = np.empty(n, dtype=np.int64)
    cols[:1000] = rng.integers(0, 10, 1000)              # rows 0..999 use columns 0..9
    cols[1000:2000] = rng.integers(12, 20, 1000)         # columns 10, 11 stay empty
    cols[2000:] = rng.integers(20, 30, 1000)
    second = rng.integers(30, 40, n)                     # every row also has a column in 30..39
    ptr = np.zeros(d + 1, dtype=np.int64)
    rows = []
    for c in range(d):
        r = np.nonzero((cols == c) | (second == c))[0]
        rows.append(r)
        ptr[c + 1] = ptr[c] + r.size
    idx = np.concatenate(rows).astype(np.int32)
    val = np.ones(idx.size, dtype=np.float32)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    g = snap.Solver("csc", n, d, ptr, idx, val, y, "logistic", 1e-3, auto_groups=True)
    assert g.chunk_bounds() == [0, 30, 40]
    A = oracle.Matrix("csc", n, d, ptr, idx, val)
    o = oracle.Solver(A, y, "logistic", 1e-3, chunk_bounds=[0, 30, 40], shuffle_chunks=True)
    for e in range(5):
        g.epoch(e)
        o.epoch(e)
    assert relnorm(g.model()[1], o.x) <= 2e-5
    g.close()


def test_auto_groups_on_streamed_data_rides_on_the_creation_pass():
    """Streamed pattern-only data: the search is advanced chunk by chunk while the creation pass has each chunk
    on the device (several chunks per field and several fields per chunk here), finds the same fields and
    the sweeps equal those with the fields given; the search copies nothing of its own over the host link."""
    p = _onehot_variant("logistic", True)
    fields = p.meta["field_starts"] + [p.d]
    ref = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, chunk_bytes=1 << 19, group_bounds=fields)
    g = snap.Solver.from_problem(_pinned(p), device_budget_bytes=1 << 20, chunk_bytes=1 << 19)        # default: search
    assert g.chunk_bounds() == fields and g.stream_bytes() == ref.stream_bytes()
    assert g.bytes_copied() == ref.bytes_copied()
    for e in range(3):
        g.epoch(e)
        ref.epoch(e)
        assert np.array_equal(g.model()[1], ref.model()[1]) and np.array_equal(g.shared(), ref.shared())
    assert g.epoch_stats()["rejected"] == 0 and g.epoch_stats()["unit_values"] == 1
    g.close()
    ref.close()
    # values other than 1: streamed maps do not apply; by default the asynchronous streamed epoch runs, on request an error
    q = _onehot_variant("logistic", False)
    g = snap.Solver.from_problem(_pinned(q), device_budget_bytes=1 << 20, chunk_bytes=1 << 19)
    b = g.chunk_bounds()
    g.epoch(0)
    st = g.epoch_stats()
    assert b != fields and st["n_chunks"] == len(b) - 1 > 2 and st["unit_values"] == 0 and g.stream_bytes() == 8 * q.nnz
    g.close()
    with pytest.raises(snap.SnapError) as e:
        snap.Solver.from_problem(_pinned(q), device_budget_bytes=1 << 20, chunk_bytes=1 << 19, auto_groups=True)
    assert e.value.code == -2
    # data without such structure: the search gives up during the pass, nothing else changes
    u = problem("stream_uniform_logistic")
    g = snap.Solver.from_problem(_pinned(u), device_budget_bytes=2 << 20, chunk_bytes=1 << 20)
    a = snap.Solver.from_problem(_pinned(u), device_budget_bytes=2 << 20, chunk_bytes=1 << 20, auto_groups=False)
    assert g.chunk_bounds() == a.chunk_bounds() and g.stream_bytes() == a.stream_bytes()
    g.close()
    a.close()


def test_auto_groups_gives_up_on_unstructured_data():
    p = problem("cfg1_sparse_logistic")
    g = gpu_solver(p, auto_groups=None)
    assert g.chunk_bounds() == [0, p.d]                  # asynchronous epoch
    g.epoch(0)
    assert np.array_equal(g.perm(), oracle.permutation(0, p.d))
    g.close()
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(p, auto_groups=True)
    assert e.value.code == -2
    # a column that repeats a row cannot be in any group
    ptr = np.array([0, 2, 3], dtype=np.int64)
    idx = np.array([1, 1, 0], dtype=np.int32)
    with pytest.raises(snap.SnapError) as e:
        snap.Solver("csc", 3, 2, ptr, idx, np.ones(3, dtype=np.float32), np.ones(3, dtype=np.float32), "ridge", 0.1,
                    auto_groups=True)
    assert e.value.code == -2


@pytest.mark.parametrize("loss,unit,lam1", [("logistic", True, 0.0), ("logistic", False, 2e-4), ("ridge", True, 0.0),
                                            ("ridge", False, 1e-3)])
def test_group_sweeps_objective_and_gap_at_a_given_model(loss, unit, lam1):
    # with groups the gradient pass behind the duality gap runs as row passes, not column gathers
    p = _onehot_variant(loss, unit)
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    rng = np.random.default_rng(21)
    w = (0.2 * rng.standard_normal(p.d) * (rng.random(p.d) < 0.5)).astype(np.float32)
    o = oracle.Solver(A, y, p.loss, p.lam, lam1=lam1)
    o.x[:] = w
    o.v[:] = o.shared_from_model()
    g = gpu_solver(p, group_bounds=groups, lam1=lam1)
    a = gpu_solver(p, lam1=lam1)                           # column-wise gradient pass on the same model
    for s in (g, a):
        s.set_model(w)
    assert rel(g.objective(), o.primal()) <= 1e-5
    assert rel(g.duality_gap(), o.gap()) <= 1e-5
    assert rel(g.duality_gap(), a.duality_gap()) <= 1e-5
    P, D = g.objective(want_dual=True)
    assert abs((P - D) - g.duality_gap()) <= 1e-12 * max(1.0, abs(P))
    # at the zero model too (closed form: every loss' is -y/2 resp. -y)
    z = np.zeros(p.d, dtype=np.float32)
    g.set_model(z)
    o.x[:] = 0
    o.v[:] = 0
    assert rel(g.duality_gap(), o.gap()) <= 1e-5
    g.close()
    a.close()


def test_solve_runs_epochs_until_the_gap_target():
    p = _onehot_variant("logistic", True)
    groups = p.meta["field_starts"] + [p.d]
    A = oracle.Matrix.from_problem(p)
    y = p.y.numpy()
    g = gpu_solver(p, group_bounds=groups)
    epochs, gap = g.solve(100, 200, 1e-4, check_every=4)
    assert 0 < epochs < 200 and epochs % 4 == 0 and gap <= 1e-4
    assert rel(gap, g.duality_gap()) <= 1e-12
    # the same epochs by hand (same seeds) reach the same model: group sweeps are deterministic
    r = gpu_solver(p, group_bounds=groups)
    for e in range(epochs):
        r.epoch(100 + e)
    assert np.array_equal(r.model()[1], g.model()[1])
    # the oracle taking the same epochs agrees on where that is
    o = oracle.Solver(A, y, p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(epochs):
        o.epoch(100 + e)
    assert rel(g.objective(), o.primal()) <= 1e-5
    assert o.gap() <= 1.1e-4
    # budget exhausted: reports the gap it stopped at; zero epochs: just the gap
    e2, gap2 = r.solve(0, 3, 0.0, check_every=5)
    assert e2 == 3 and gap2 > 0.0
    e3, gap3 = r.solve(0, 0, 1.0)
    assert e3 == 0 and rel(gap3, r.duality_gap()) <= 1e-12
    with pytest.raises(snap.SnapError):
        r.solve(0, 5, 1e-3, check_every=0)
    g.close()
    r.close()


def test_group_sweeps_leave_for_the_asynchronous_engine_beyond_their_fixed_point_range():
    """Ridge terms a (v - y) of 2^14 and more do not fit the 64-bit fixed-point sums of the group sweeps.  The
    epoch that meets one is discarded and done again by the asynchronous engine, which the handle keeps
    from then on: the caller gets the oracle's objective, not an error."""
    p = _onehot_variant("ridge", False)
    groups = p.meta["field_starts"] + [p.d]
    p.y = p.y * 1e6                                        # residuals of 1e6: a (v - y) far beyond 2^14
    A = oracle.Matrix.from_problem(p)
    target = oracle.solve(A, p.y.numpy(), "ridge", p.lam, epochs=500, tol=1e-7).primal()
    g = gpu_solver(p, group_bounds=groups)
    assert g.chunk_bounds() == groups
    P0 = g.objective()
    g.epoch(0)
    assert g.chunk_bounds() == [0, p.d]                    # the groups are gone: one chunk, asynchronous epoch
    assert np.array_equal(g.perm(), executed_order(oracle.permutation(0, p.d), np.diff(p.ptr.numpy())))
    assert g.objective() < P0
    for e in range(1, 60):
        g.epoch(e)
    assert rel(g.objective(), target) <= 1e-4
    chk = oracle.Solver(A, p.y.numpy(), "ridge", p.lam)
    chk.x[:] = g.model()[1]
    assert relnorm(g.shared(), chk.shared_from_model()) <= 1e-4
    g.close()
    # the gradient pass of the duality gap meets the limit first when no epoch has run yet
    g = gpu_solver(p, group_bounds=groups)
    o = oracle.Solver(A, p.y.numpy(), "ridge", p.lam)
    assert rel(g.duality_gap(), o.gap()) <= 1e-5
    assert g.chunk_bounds() == [0, p.d]
    g.close()
    # moderate residuals stay with the group sweeps
    p.y = p.y * 1e-4                                       # residuals of 100
    g = gpu_solver(p, group_bounds=groups)
    for e in range(3):
        g.epoch(e)
    assert g.chunk_bounds() == groups
    g.close()


def test_group_sweeps_are_declined_when_lambda_n_is_below_their_resolution():
    """Logistic terms enter the fixed-point sums with 2^-20 / 2^-23 of resolution; with lambda n below 1/16 (for
    values up to 1) a perfectly separated coordinate's step could show it, so such a handle runs the
    asynchronous engine, also when groups were given."""
    p = datagen.onehot_fields(n=20_000, d=1_500, lam=1e-6, seed=17)          # lambda n = 0.02
    groups = p.meta["field_starts"] + [p.d]
    g = gpu_solver(p, group_bounds=groups)
    assert g.chunk_bounds() == [0, p.d]
    A = oracle.Matrix.from_problem(p)
    g.epoch(0)
    assert np.array_equal(g.perm(), executed_order(oracle.permutation(0, p.d), np.diff(p.ptr.numpy())))
    g.close()
    with pytest.raises(snap.SnapError) as e:
        gpu_solver(p, auto_groups=True)
    assert e.value.code == -2
    p.lam = 1e-5                                                              # lambda n = 0.2: group sweeps
    g = gpu_solver(p, group_bounds=groups)
    assert g.chunk_bounds() == groups
    o = oracle.Solver(A, p.y.numpy(), p.loss, p.lam, chunk_bounds=groups, shuffle_chunks=True)
    for e in range(3):
        g.epoch(e)
        o.epoch(e)
    assert relnorm(g.model()[1], o.x) <= 2e-5
    g.close()


# ---------------------------------------------------------------------------------------------
# the measurement aid: bare streaming kernels
def test_stream_probe_reports_plausible_times_and_rejects_bad_arguments():
    rows = 8_000_000
    for kind, per_row in ((0, 4), (1, 8), (2, 12)):
        us = snap.stream_probe(kind, rows, 10)
        tbps = per_row * rows / (us * 1e-6) / 1e12
        assert 0.3 < tbps < 20.0, (kind, us)             # (small arrays may be served by the caches: above the HBM peak)
    assert snap.stream_probe(2, 1001, 2) > 0             # ragged size
    for bad in ((3, 100, 1), (-1, 100, 1), (0, 0, 1), (0, 100, 0), (0, 100, 1001), (0, (1 << 32) + 1, 1)):
        with pytest.raises(snap.SnapError) as e:
            snap.stream_probe(*bad)
        assert e.value.code == -1
