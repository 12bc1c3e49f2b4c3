"""snap_predict_static -- decision values without any allocation (scratch in a static device array of
the library) -- against snap_predict, through the C ABI: every layout, two calls in a row on the same
GPU with the second input smaller than the first (the shared scratch keeps the first call's contents),
the size limit, and the error paths.  The values are those of snap_predict (same kernels): the row
layouts bit for bit, the compressed-column layout to the last bit of its fp64 sums."""
import numpy as np
import pytest
import torch

import oracle
import paper_1803_06333_amd as snap

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
STATIC_ROWS_MAX = 4 << 20


def _csr(rows, d, mean_len, seed):
    r = np.random.default_rng(seed)
    lengths = np.clip(r.poisson(mean_len, size=rows), 0, d)
    if rows > 3:
        lengths[0] = lengths[-1] = 0
    ptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    idx = np.concatenate([np.sort(r.choice(d, size=k, replace=False)) for k in lengths] + [np.zeros(0)]).astype(np.int32)
    val = r.standard_normal(ptr[-1]).astype(np.float32)
    return ptr, idx, val


def _csc_from_csr(rows, d, ptr, idx, val):
    r = np.repeat(np.arange(rows), np.diff(ptr))
    order = np.lexsort((r, idx))
    cptr = np.concatenate([[0], np.cumsum(np.bincount(idx, minlength=d))]).astype(np.int64)
    return cptr, r[order].astype(np.int32), val[order]


def _dense(rows, d, ptr, idx, val):
    X = np.zeros((rows, d), dtype=np.float32)
    X[np.repeat(np.arange(rows), np.diff(ptr)), idx] = val
    return X


def _trained(d, form):
    """A handle with a non-trivial model: primal (CSC training data) or dual (CSR training data)."""
    r = np.random.default_rng(5)
    n = 600
    ptr, idx, val = _csr(n, d, 12, 6)
    y = np.sign(r.standard_normal(n)).astype(np.float32)
    if form == "primal":
        cptr, cidx, cval = _csc_from_csr(n, d, ptr, idx, val)
        g = snap.Solver("csc", n, d, cptr, cidx, cval, y, "logistic", 1e-2, auto_groups=False)
    else:
        g = snap.Solver("csr", n, d, ptr, idx, val, y, "hinge", 1e-2)
    for e in range(3):
        g.epoch(e)
    return g


def _dev(*arrays):
    return [None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in arrays]


@pytest.mark.parametrize("form", ["primal", "dual"])
def test_static_predict_equals_predict_on_two_calls_in_a_row(form):
    d = 900
    g = _trained(d, form)
    w, _ = g.model()
    for rows in (5000, 37):                           # the second call is the smaller one
        ptr, idx, val = _csr(rows, d, 20, 100 + rows)
        want = oracle.Matrix("csr", rows, d, ptr, idx, val).matvec(w.astype(np.float64))
        scale = max(np.abs(want).max(), 1e-30)
        cptr, cidx, cval = _csc_from_csr(rows, d, ptr, idx, val)
        X = _dense(rows, d, ptr, idx, val)
        cases = {"csr": (ptr, idx, val), "csc": (cptr, cidx, cval),
                 "dense_rowmajor": (None, None, X.reshape(-1)),
                 "dense_colmajor": (None, None, np.ascontiguousarray(X.T).reshape(-1))}
        for layout, arrays in cases.items():
            dp, di, dv = _dev(*arrays)
            ref = g.predict(layout, rows, dp, di, dv).cpu().numpy()
            out = torch.full((rows,), float("nan"), dtype=torch.float32, device=DEV)
            got = g.predict_static(layout, rows, dp, di, dv, out).cpu().numpy()
            assert np.abs(ref - want).max() <= 1e-5 * scale, layout          # snap_predict against the oracle
            assert np.abs(got - want).max() <= 1e-5 * scale, layout          # and the variant as well
            if layout == "csc":
                np.testing.assert_allclose(got, ref, rtol=0, atol=2.0 ** -22 * scale)   # fp64 atomics: last bit
            else:
                assert np.array_equal(got, ref), layout
    g.close()


def test_static_predict_rejects_what_it_cannot_do_without_allocating():
    d = 50
    g = _trained(d, "primal")
    out = torch.zeros(8, dtype=torch.float32, device=DEV)
    ptr, idx, val = _csr(8, d, 5, 3)
    with pytest.raises(snap.SnapError) as e:            # a host matrix would need a device copy
        g.predict_static("csr", 8, ptr, idx, val, out)
    assert e.value.code == -1 and "device memory" in str(e.value)
    # a compressed-column matrix beyond the static buffer of sums: refused, with the limit in the message
    rows = STATIC_ROWS_MAX + 1
    w0 = float(g.model()[0][0])
    cptr = torch.ones(d + 1, dtype=torch.int64, device=DEV)           # one nonzero, (row 0, column 0) = 1, is enough
    cptr[0] = 0
    one_idx = torch.zeros(1, dtype=torch.int32, device=DEV)
    one_val = torch.ones(1, dtype=torch.float32, device=DEV)
    big = torch.zeros(rows, dtype=torch.float32, device=DEV)
    with pytest.raises(snap.SnapError) as e:
        g.predict_static("csc", rows, cptr, one_idx, one_val, big)
    assert e.value.code == -1 and str(STATIC_ROWS_MAX) in str(e.value)
    # at the limit it runs, and so does the row layout beyond it
    big[:] = 7.0
    g.predict_static("csc", STATIC_ROWS_MAX, cptr, one_idx, one_val, big)
    assert float(big[0]) == w0 and float(big[1:STATIC_ROWS_MAX].abs().max()) == 0.0 and float(big[STATIC_ROWS_MAX]) == 7.0
    rptr = torch.ones(rows + 1, dtype=torch.int64, device=DEV)
    rptr[0] = 0
    big[:] = 7.0
    g.predict_static("csr", rows, rptr, one_idx, one_val, big)
    assert float(big[0]) == w0 and float(big[1:].abs().max()) == 0.0
    # invalid indices are reported, nothing is written, and the handle stays usable
    dp, di, dv = _dev(ptr, idx, val)
    bad = di.clone()
    bad[0] = d
    out[:] = 3.0
    with pytest.raises(snap.SnapError) as e:
        g.predict_static("csr", 8, dp, bad, dv, out)
    assert e.value.code == -1 and float(out.min()) == 3.0
    ref = g.predict("csr", 8, dp, di, dv)
    assert torch.equal(g.predict_static("csr", 8, dp, di, dv, out), ref)
    g.close()
