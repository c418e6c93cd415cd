"""The entry point that allocates nothing (domino_colsum_noalloc: partial sums in the library's own device array)
against the entry point it is a variant of (domino_colsum, scratch passed by the caller), through the C ABI."""
import ctypes as C

import pytest

from paper_2409_15241_amd import domino as D

torch = pytest.importorskip("torch")


@pytest.mark.gpu
def test_noalloc_column_sums_equal_those_with_caller_scratch():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    D.load()
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(7)
    st = torch.cuda.Stream(device=dev)
    # two calls in a row on one stream, the second smaller in both directions (ragged: 1000 rows over 64 row
    # ranges, 40 rows = fewer rows than row ranges), then a third with a row stride wider than n, accumulating
    cases = [(1000, 8192, 8192, 0), (40, 264, 264, 0), (333, 1024, 1536, 1)]
    outs_a, outs_b = [], []
    for rows, n, ld, acc in cases:
        m = torch.randn(rows, ld, device=dev, generator=g).to(torch.bfloat16)
        ref = torch.full((n,), 0.5, device=dev, dtype=torch.float32)
        got = ref.clone()
        scratch = torch.empty(64 * n, device=dev, dtype=torch.float32)
        torch.cuda.synchronize()
        D.domino_colsum(m, ld, rows, n, ref, acc, scratch, st)
        D.domino_colsum_noalloc(m, ld, rows, n, got, acc, st)
        outs_a.append((ref, m, rows, n, acc))
        outs_b.append(got)
    torch.cuda.synchronize()
    for (ref, m, rows, n, acc), got in zip(outs_a, outs_b):
        assert torch.equal(ref, got), (rows, n)
        want = m[:, :n].double().sum(0) + (0.5 if acc else 0.0)        # and both are the column sums
        assert float((got.double() - want).abs().max()) <= 1e-4 * max(1.0, float(want.abs().max()))


def test_noalloc_rejects_sizes_beyond_its_array_without_touching_the_gpu():
    lib = D.load()
    assert lib.domino_colsum_noalloc(1, 8200, 4, 8200, 1, 0, None) == D.ERR_UNSUPPORTED
    assert "8192" in D.domino_last_error()
    assert lib.domino_colsum_noalloc(None, 64, 4, 64, 1, 0, None) == D.ERR_NULL_POINTER
    assert lib.domino_colsum_noalloc(1, 64, 4, 60, 1, 0, None) == D.ERR_UNSUPPORTED
