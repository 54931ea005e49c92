"""The N = 256 sweep of the benchmark definition (four ResNet-18 maps x b in {8, 6, 4, 3, 2}) on a few images per
shape: every cell of tests/sweep_config5.py's table goes through its parity checks against the oracle (container
byte for byte, symbols under the boundary rule, reconstruction <= 1e-4, H <= R < H + 1).  The table at the full
batch size is made by running that script; tests/test_gpu_full_size.py holds whole-tensor parity at N = 256."""
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_every_cell_of_the_sweep_on_a_few_images(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from sweep_config5 import BITS, SHAPES, run

    rows = run(images=5, check_images=5, log=lambda s: None)
    assert len(rows) == len(SHAPES) * len(BITS)
    by_shape = {}
    for r in rows:
        by_shape.setdefault(r["workload"], []).append(r)
    for name, rs in by_shape.items():
        rs.sort(key=lambda r: -r["bits"])
        # fewer bits: a coarser step, a lower rate and a larger error, cell after cell
        for a, b in zip(rs, rs[1:]):
            assert b["delta"] > a["delta"] and b["rate"] <= a["rate"] and b["mse"] >= a["mse"], (name, a, b)
