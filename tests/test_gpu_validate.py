"""The debug mode SYLVIE_VALIDATE=1: precondition checks that run on the device before the
real work and turn a violation into SYLVIE_ERR_INVALID_ARG.  Every bad input here is caught
by the checks, which only read the arrays they are given: nothing out of range is ever
dereferenced."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.fixture
def validate(monkeypatch):
    monkeypatch.setenv("SYLVIE_VALIDATE", "1")


def _wire(n, d):
    from paper_2303_01277_amd import binding as B
    return torch.zeros(n * B.sylvie_wire_row_words(d), dtype=torch.int64, device=DEV)


def test_quantizer_rejects_bad_values_and_indices(validate):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(0)
    d, n = 100, 50
    x = rng.standard_normal((80, d)).astype(np.float32)
    idx = rng.integers(0, 60, n).astype(np.int32)          # rows 60.. are never gathered
    good = _wire(n, d)
    B.sylvie_quantize_1bit_fwd(dev(x), d, d, dev(idx), 0, n, 1, 2, good)
    for bad_value in (np.nan, np.inf, -np.inf, np.float32(2.0 ** 126)):
        y = x.copy()
        y[70, 3] = bad_value                               # not gathered: accepted
        w = _wire(n, d)
        B.sylvie_quantize_1bit_fwd(dev(y), d, d, dev(idx), 0, n, 1, 2, w)
        torch.cuda.synchronize()
        assert torch.equal(w, good)
        y[idx[7], 5] = bad_value                           # gathered: rejected, nothing written
        w = _wire(n, d)
        with pytest.raises(B.SylvieError, match="SYLVIE_VALIDATE"):
            B.sylvie_quantize_1bit_fwd(dev(y), d, d, dev(idx), 0, n, 1, 2, w)
        torch.cuda.synchronize()
        assert not w.any()
    neg = idx.copy()
    neg[11] = -1
    with pytest.raises(B.SylvieError, match="index out of range"):
        B.sylvie_quantize_1bit_bwd(dev(x), d, d, dev(neg), 0, n, 1, 3, _wire(n, d))


def test_unvalidated_call_does_not_wait_or_reject(monkeypatch):
    from paper_2303_01277_amd import binding as B
    monkeypatch.delenv("SYLVIE_VALIDATE", raising=False)
    x = np.ones((4, 64), np.float32)
    x[1, 1] = np.nan                                       # a broken precondition, harmless to memory
    B.sylvie_quantize_1bit_fwd(dev(x), 64, 64, None, 0, 4, 1, 2, _wire(4, 64))
    torch.cuda.synchronize()


def test_wire_reading_aggregation_rejects_bad_operators(validate):
    from paper_2303_01277_amd import binding as B
    d, n_dense, n_wire = 64, 6, 5
    X = dev(np.random.default_rng(1).standard_normal((n_dense, d)).astype(np.float32))
    wire = _wire(n_wire, d)
    Y = torch.zeros((3, d), device=DEV)
    rowptr = dev(np.array([0, 3, 5, 8], np.int64))
    w = dev(np.ones(8, np.float32))

    def call(cols, rp=rowptr):
        B.sylvie_aggregate_csr_fwd_wire(rp, dev(np.array(cols, np.int32)), w, None, None, 3, X, d, d,
                                        n_dense, wire, n_wire, Y, d)

    call([0, 2, 7, 1, 10, 3, 4, 6])                        # dense before wire in every row: fine
    with pytest.raises(B.SylvieError, match="out of order"):
        call([0, 7, 2, 1, 10, 3, 4, 6])                    # wire column 7 before dense column 2
    with pytest.raises(B.SylvieError, match="index out of range"):
        call([0, 2, 11, 1, 10, 3, 4, 6])                   # 11 >= n_dense + n_wire
    with pytest.raises(B.SylvieError, match="index out of range"):
        call([0, 2, 7, -1, 10, 3, 4, 6])
    with pytest.raises(B.SylvieError, match="pointer"):
        call([0, 2, 7, 1, 10, 3, 4, 6], dev(np.array([0, 5, 3, 8], np.int64)))
    torch.cuda.synchronize()


def test_backward_dequantizer_rejects_bad_segments(validate):
    from paper_2303_01277_amd import binding as B
    d, n = 64, 6
    wire = _wire(n, d)
    J = torch.zeros((4, d), device=DEV)
    ids = dev(np.array([0, 2, 3], np.int32))
    ok_ptr = dev(np.array([0, 2, 2, 6], np.int64))
    B.sylvie_dequantize_1bit_bwd(wire, n, d, J, d, ok_ptr, dev(np.array([0, 4, 1, 2, 3, 5], np.int32)), 3, ids)
    with pytest.raises(B.SylvieError, match="index out of range"):
        B.sylvie_dequantize_1bit_bwd(wire, n, d, J, d, ok_ptr, dev(np.array([0, 4, 1, 2, 3, 6], np.int32)), 3, ids)
    with pytest.raises(B.SylvieError, match="out of order"):
        B.sylvie_dequantize_1bit_bwd(wire, n, d, J, d, ok_ptr, dev(np.array([4, 0, 1, 2, 3, 5], np.int32)), 3, ids)
    with pytest.raises(B.SylvieError, match="pointer"):
        B.sylvie_dequantize_1bit_bwd(wire, n, d, J, d, dev(np.array([0, 2, 2, 7], np.int64)),
                                     dev(np.array([0, 4, 1, 2, 3, 5], np.int32)), 3, ids)
    torch.cuda.synchronize()


def test_attention_aggregation_rejects_bad_operators(validate):
    from paper_2303_01277_amd import binding as B
    d, K, n = 64, 4, 3
    X = dev(np.random.default_rng(2).standard_normal((6, d)).astype(np.float32))
    Y = torch.zeros((n, d), device=DEV)
    w = dev(np.ones(8 * K, np.float32))
    good = dev(np.array([0, 3, 5, 8], np.int64))

    def call(cols, rp=good):
        B.sylvie_aggregate_csr_attention(rp, dev(np.array(cols, np.int32)), w, None, K, n, X, d, d, Y, d)

    call([0, 2, 5, 1, 4, 3, 4, 5])
    torch.cuda.synchronize()
    assert bool((Y[0] == X[0] + X[2] + X[5]).all())
    with pytest.raises(B.SylvieError, match="index out of range"):
        call([0, 2, -1, 1, 4, 3, 4, 5])
    with pytest.raises(B.SylvieError, match="SYLVIE_VALIDATE"):
        call([0, 2, 5, 1, 4, 3, 4, 5], rp=dev(np.array([0, 3, 2, 8], np.int64)))       # row pointers descend
