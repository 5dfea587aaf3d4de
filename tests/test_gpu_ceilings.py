"""The plain kernels behind bench.py's mix ceilings really move what they claim: every launch form of the
gather (8 reads : 1 write) and of the scatter (1 read : 8 writes) is checked against numpy on a small case with
a ragged row length and with one that is a whole number of waves."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ceil():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import ceilings
    ceilings.load()          # raises if the kernels were not built
    return ceilings


@pytest.mark.parametrize("rows,cols", [(300, 128), (1000, 72), (20000, 64)])
def test_gather_and_scatter_forms(ceil, rows, cols):
    rng = np.random.default_rng(rows)
    perm = rng.permutation(rows * 8).astype(np.int32)
    table = torch.from_numpy(perm).cuda()
    ceil._check_table(table, rows * 8)
    big = rng.integers(0, 2 ** 31, size=(rows * 8, cols * 4), dtype=np.int32)
    small = rng.integers(0, 2 ** 31, size=(rows, cols * 4), dtype=np.int32)
    want_gather = np.bitwise_or.reduce(big[perm.reshape(rows, 8)], axis=1)
    want_scatter = np.empty_like(big)
    want_scatter[perm] = np.repeat(small, 8, axis=0)
    big_d, small_d = torch.from_numpy(big).cuda(), torch.from_numpy(small).cuda()
    for form in ceil.GATHER_FORMS:
        if form[2] == 3 and cols % 64:
            continue
        print(f"[gather] rows={rows} cols={cols} form={form}", flush=True)
        out = torch.zeros_like(small_d)
        ceil.gather8(form, big_d, table, out, rows, cols)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want_gather), form
    for form in ceil.SCATTER_FORMS:
        print(f"[scatter] rows={rows} cols={cols} form={form}", flush=True)
        out = torch.zeros_like(big_d)
        ceil.scatter8(form, small_d, table, out, rows, cols)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want_scatter), form
