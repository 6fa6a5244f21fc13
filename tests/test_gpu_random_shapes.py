"""GPU parity on seeded random shapes: the checks of test_gpu_parity.py and test_gpu_packing.py
(same oracle, same bars) on shapes drawn from a fixed seed, so that tile edges, group sizes, block
widths and batch sizes are met in combinations nobody picked by hand.  Every case is valid input."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests import test_gpu_packing as tk          # noqa: E402
from tests import test_gpu_parity as tp           # noqa: E402


def _cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        k = int(rng.integers(0, 8))
        if k == 0:
            c = int(rng.integers(1, 1400)); n = int(rng.integers(1, 3000))
            out.append(("hessian", tp.test_hessian_matches_oracle, (c, n, min(int(rng.integers(1, 4)), n))))
        elif k == 1:
            c = int(rng.integers(2, 900))
            out.append(("cholesky", tp.test_cholesky_inv_matches_oracle, (c, 3 * c + int(rng.integers(0, 500)))))
        elif k == 2:
            out.append(("fit_nu", tp.test_fit_grid_nonuniform,
                        (int(rng.integers(1, 80)), int(rng.integers(1, 3000)), int(rng.integers(2, 5)))))
        elif k == 3:
            group = int(rng.choice([8, 16, 32, 64, 128, 256])); ng = int(rng.integers(1, 6))
            out.append(("fit_aff", tp.test_fit_grid_affine,
                        (int(rng.integers(1, 12)), group * ng, group, int(rng.integers(2, 5)),
                         int(rng.choice([2048, 256, 64, 10])))))
        elif k in (4, 5):
            B = int(rng.choice([32, 64, 128])); mode = str(rng.choice(["nu", "aff"])); bits = int(rng.integers(2, 5))
            r = int(rng.integers(60, 400))
            if mode == "aff":
                group = int(rng.choice([0, 16, 32, 64, 128]))
                gg = group if group else int(rng.integers(200, 500))
                c = gg * int(rng.integers(max(1, 200 // gg), max(2, 600 // gg) + 1)) if group else gg
            else:
                group = 0; c = int(rng.integers(200, 600))
            out.append(("quantize", tp.test_quantize_layer_matches_oracle, (r, c, B, mode, bits, group)))
        else:
            mode, bits, group = [("nu", 4, 0), ("nu", 3, 0), ("nu", 2, 0), ("aff", 4, 128), ("aff", 2, 64),
                                 ("aff", 3, 0), ("aff", 4, 32)][int(rng.integers(0, 7))]
            c = 32 * int(rng.integers(1, 200))
            if group and c % group:
                c = group * max(1, c // group)
            if k == 6:
                out.append(("matmul", tk.test_matmul_from_the_stored_form,
                            (mode, bits, group, int(rng.integers(1, 700)), c, int(rng.integers(1, 140)))))
            else:
                out.append(("matvec", tk.test_matvec_from_the_stored_form,
                            (mode, bits, group, int(rng.integers(1, 300)), c, int(rng.integers(1, 8)))))
    return out


@pytest.mark.parametrize("seed", [2024, 2025])
def test_random_shapes(seed):
    for name, fn, args in _cases(seed, 30):
        print("random shape:", name, args, flush=True)
        fn(*args)
