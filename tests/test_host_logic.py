"""Host-side logic of the GPU parity tests, checked without a GPU."""
import numpy as np
import pytest

from test_gpu_layer import _stratified_rows


@pytest.mark.parametrize("M,g", [(1, 1), (64, 4), (883, 4), (3404, 4), (16576, 4), (14539, 7), (13363, 8), (500, 1),
                                 (700, 2), (257, 32)])
def test_stratified_rows_cover_every_attention_block_and_gemm_tile(M, g):
    rows = _stratified_rows(M, g, 16, seed=M + g)
    assert rows[0] == 0 and rows[-1] == M - 1 and np.all(np.diff(rows) > 0) and rows.max() < M
    cols = set()
    for r in rows:                                   # the 256-column blocks of (token, head) columns a row touches
        cols.update(range((r * g) // 256, (r * g + g - 1) // 256 + 1))
    assert cols >= set(range((M * g + 255) // 256))
    for tile in (128, 192, 256):                     # every GEMM row tile holds a compared row
        assert set(rows // tile) == set(range((M + tile - 1) // tile)), tile
