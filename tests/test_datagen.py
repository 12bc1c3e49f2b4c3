"""The seeded generators: shapes, structure and determinism of the synthetic stand-ins."""
import numpy as np
import torch

import datagen


def test_config1_structure():
    p = datagen.uniform_sparse_logistic(n=500, d=100, k=20)
    ptr, idx, val = p.meta["csr"]
    cols = idx.view(500, 20)
    assert torch.all(cols[:, 1:] > cols[:, :-1])                 # distinct, ascending
    assert int(cols.min()) >= 0 and int(cols.max()) < 100
    assert p.layout == "csc" and int(p.ptr[-1]) == 500 * 20 == p.nnz
    # the CSC is the transpose of the CSR
    X = torch.zeros(500, 100)
    X[torch.arange(500).repeat_interleave(20), idx.long()] = 1.0
    Xc = torch.zeros(500, 100)
    colid = torch.repeat_interleave(torch.arange(100), p.ptr[1:] - p.ptr[:-1])
    Xc[p.idx.long(), colid] = p.val
    assert torch.equal(X, Xc)
    for j in range(100):
        r = p.idx[p.ptr[j]:p.ptr[j + 1]]
        assert torch.all(r[1:] > r[:-1])
    assert set(p.y.tolist()) <= {-1.0, 1.0}
    q = datagen.uniform_sparse_logistic(n=500, d=100, k=20)
    assert torch.equal(p.idx, q.idx) and torch.equal(p.y, q.y)
    r = datagen.uniform_sparse_logistic(n=500, d=100, k=20, seed=5)
    assert not torch.equal(p.idx, r.idx)


def test_config2_structure():
    p = datagen.dense_ridge(n=300, d=40)
    A = p.val.view(40, 300)             # column-major n x d
    norms = torch.linalg.norm(A.double(), dim=0)
    assert torch.allclose(norms, torch.ones(300, dtype=torch.float64), atol=1e-6)
    assert abs(float(A.mean())) < 0.01 and p.y.shape == (300,)
    # blocks of rows give the same matrix as one block
    q = datagen.dense_ridge(n=300, d=40, row_block=64)
    assert torch.equal(p.val, q.val) and torch.equal(p.y, q.y)


def test_config3_structure():
    p = datagen.zipf_sparse_svm(n=2000, d=5000, k=50)
    cols = p.idx.view(2000, 50)
    assert torch.all(cols[:, 1:] > cols[:, :-1])
    vals = p.val.view(2000, 50)
    assert torch.all(vals >= 0)
    assert torch.allclose(torch.linalg.norm(vals.double(), dim=1), torch.ones(2000, dtype=torch.float64), atol=1e-6)
    freq = torch.bincount(p.idx.long(), minlength=5000).double()
    assert freq[0] > freq[10] > freq[200] > freq[3000]           # Zipf popularity by rank
    assert set(p.y.tolist()) <= {-1.0, 1.0}
    assert 0.2 < float((p.y > 0).float().mean()) < 0.8


def test_onehot_fields_structure():
    n, d = 20000, 5000
    p = datagen.onehot_fields(n=n, d=d, want_csr=True)
    starts, sizes = p.meta["field_starts"], p.meta["field_sizes"]
    assert len(starts) == 39 and sum(sizes) == d and sizes[:13] == [64] * 13
    assert p.nnz == 39 * n and int(p.ptr[-1]) == 39 * n
    ptr = p.ptr.numpy()
    idx = p.idx.numpy()
    for f in range(39):
        lo, hi = ptr[starts[f]], ptr[starts[f] + sizes[f]]
        assert hi - lo == n                                        # each row once per field
        assert np.array_equal(np.sort(idx[lo:hi]), np.arange(n))
    for j in [0, 5, 832, 833, 900, d - 1]:
        r = idx[ptr[j]:ptr[j + 1]]
        assert np.all(r[1:] > r[:-1])
    # CSR and CSC describe the same matrix
    cptr, cidx, cval = p.meta["csr"]
    tptr, tidx, tval = datagen.csr_to_csc(n, d, cptr, cidx, cval)
    assert torch.equal(tptr, p.ptr) and torch.equal(tidx, p.idx)
    rate = float((p.y > 0).float().mean())
    assert abs(rate - 0.256) < 0.02
    # Zipf head: the first column of a categorical field holds about 1/H of the rows
    f = 20
    c0 = ptr[starts[f] + 1] - ptr[starts[f]]
    H = np.sum(np.arange(1, sizes[f] + 1, dtype=np.float64) ** -1.2)
    assert abs(c0 / n - 1 / H) < 0.02
    q = datagen.onehot_fields(n=n, d=d)
    assert torch.equal(q.idx, p.idx) and torch.equal(q.y, p.y)


def test_pattern_only_problem_has_no_value_array_and_the_same_pattern():
    """pattern_only: no value array at all (val = None stands for "every stored value is 1"); the oracle's
    matrix gets an array of ones for it, everything else is the same problem."""
    import oracle
    a = datagen.onehot_fields(n=3000, d=2000, seed=9)
    b = datagen.onehot_fields(n=3000, d=2000, seed=9, pattern_only=True)
    assert b.val is None and b.nnz == a.nnz == 39 * 3000
    assert torch.equal(a.ptr, b.ptr) and torch.equal(a.idx, b.idx) and torch.equal(a.y, b.y)
    assert b.to("cpu").val is None
    A, B = oracle.Matrix.from_problem(a), oracle.Matrix.from_problem(b)
    assert B.val.dtype == np.float32 and np.array_equal(A.val, B.val) and np.array_equal(A.idx, B.idx)
    w = np.random.default_rng(0).standard_normal(2000)
    assert np.array_equal(A.matvec(w), B.matvec(w))


def test_row_ranges_of_categories_are_consistent():
    a = datagen.onehot_categories(1000, 5000, 7, 15, "cpu")
    b = datagen.onehot_categories(1000, 5000, 7, 15, "cpu", row0=400, nrows=100)
    assert torch.equal(a[400:500], b)
