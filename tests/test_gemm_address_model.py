"""Host-side bounds check of the grouped-GEMM kernels' addressing (tests/gemm_address_model.py) on the shapes that matter:
ragged experts from empty to several row tiles, both K pipelines, gated and plain FFNs, and the one shape whose expert-FFN
GPU test is skipped after a GPU memory fault (48 experts of 0 .. 65 rows, M = 320, H = 64, SwiGLU)."""
import numpy as np
import pytest

import gemm_address_model as G

# rows per expert of the parity case "gate_48_experts" (oracle routing of its seeded input; capacity 65)
ROWS_48 = [65, 0, 0, 3, 0, 1, 0, 0, 2, 0, 65, 0, 56, 0, 0, 31, 3, 65, 0, 65, 2, 1, 7, 0, 0, 2, 0, 18, 0, 65, 11, 65, 65, 0, 65, 0, 0,
           29, 0, 34, 0, 65, 65, 0, 33, 4, 65, 0]
RAGGED_8 = [700, 0, 257, 256, 1, 513, 31, 96]


def offsets(rows):
    return np.concatenate([[0], np.cumsum(rows)])


def test_the_skipped_shape_addresses_nothing_outside_its_tensors():
    tiles = G.run_case(260, 320, 48, 64, 8, 65, offsets(ROWS_48), glu=True)
    live = sum(r > 0 for r in ROWS_48)
    assert tiles == {"fwd1": live, "fwd2": 2 * live, "dhh": live, "dw2": 96, "dxe": 2 * live, "dw1": 192}


@pytest.mark.parametrize("glu", [True, False])
@pytest.mark.parametrize("M,H", [(512, 192), (96, 160), (160, 96), (64, 64), (320, 64), (1024, 448)])
def test_ragged_experts_in_both_k_pipelines(M, H, glu):
    G.run_case(927, M, 8, H, 2, 0, offsets(RAGGED_8), glu=glu)


def test_random_row_counts():
    rng = np.random.default_rng(7)
    for E, k, N in ((5, 2, 300), (64, 6, 150), (256, 1, 700), (16, 4, 2100)):
        rows = rng.multinomial(N * k - int(rng.integers(0, N)), rng.dirichlet(np.full(E, 0.3)))
        G.run_case(N, 128, E, 64, k, 0, offsets(rows), glu=bool(E % 2))


@pytest.mark.parametrize("tensor", ["xe", "w1", "w3", "w2", "dq", "hh", "a1", "a3", "da3", "q", "dxe", "dw1", "dw2", "dw3"])
def test_the_check_is_live(tensor):
    """A tensor 16 bytes short of its size is noticed when the routing fills all N*k rows."""
    rows = [600, 254, 500, 500]
    with pytest.raises(AssertionError, match=tensor):
        G.run_case(927, 512, 4, 192, 2, 0, offsets(rows), glu=True, shrink={tensor: 16})
