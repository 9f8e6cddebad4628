"""Register-bank conflict scores from the GPU library against the oracle's, exactly."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mixed import mixed_mir  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def gpu_scores(m, rows, n_banks):
    hm = vl.vl_mir_create(m)
    try:
        dev, ld = vl.rows_to_device(rows)
        out = torch.full((rows.shape[0],), -1, dtype=torch.int32, device="cuda")
        vl.vl_bank_conflicts(hm, dev, rows.shape[0], ld, n_banks, out)
        torch.cuda.synchronize()
        return out.cpu().numpy().view(np.uint32)
    finally:
        vl.vl_mir_destroy(hm)


@pytest.mark.parametrize("n_banks", [1, 3, 4, 8, 32, 64])
def test_mixed_shapes(n_banks):
    rng = np.random.default_rng(n_banks)
    m = mixed_mir(0xBB00 + n_banks, n_instr=900, wide_instr=3)
    rows = rng.integers(0, 512, (70, m.n_occ)).astype(np.uint16)
    rows[5] = 65535
    rows[6] = 0
    assert (gpu_scores(m, rows, n_banks) == vlo.bank_conflicts(m, rows, n_banks)).all()


def test_benchmark_kernel_full_size():
    w = gen.config(2)
    k, rows = w.kernels[0], w.rows[0]
    want = vlo.bank_conflicts(k.mir, rows, 4)
    assert (gpu_scores(k.mir, rows, 4) == want).all()
    assert want.min() > 0 and len(np.unique(want)) > 1


def test_argument_errors():
    m = mixed_mir(0xBB99, n_instr=60, wide_instr=0)
    hm = vl.vl_mir_create(m)
    dev, ld = vl.rows_to_device(np.zeros((2, m.n_occ), np.uint16))
    out = torch.full((2,), 9, dtype=torch.int32, device="cuda")
    for args, code in (((0, ld, 4), -2), ((2, m.n_occ - 1, 4), -2), ((2, ld, 0), -3), ((2, ld, 65), -3)):
        with pytest.raises(vl.VlError) as e:
            vl.vl_bank_conflicts(hm, dev, args[0], args[1], args[2], out)
        assert e.value.code == code
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 9).all()
    vl.vl_mir_destroy(hm)
