"""The row-block evaluation of the oracle that the full-size GPU tests rely on equals the oracle evaluated at once."""
import numpy as np

import oracle
from hgnn_inputs import init_layer_weights, small_mixed_batch
from parity_util import oracle_layer_by_row_blocks, relerr


def test_row_block_evaluation_equals_the_whole_layer():
    b = small_mixed_batch(3, n_mol=4, n_cry=4)
    g = oracle.radius_graph(b.pos, b.graph_off, b.cell, b.pbc, 4.5)
    rng = np.random.default_rng(0)
    H = 16
    W = init_layer_weights(rng, H).astype(np.float64)
    h, v = rng.standard_normal((b.N, H)), rng.standard_normal((b.N, 3))
    gh, gv = rng.standard_normal((b.N, H)), rng.standard_normal((b.N, 3))
    ho, vo, cache = oracle.mp_layer_fwd(h, v, g["dst"], g["col"], g["d2"], g["rvec"], W, 0.1)
    g_h, g_v, gW = oracle.mp_layer_bwd(cache, gh, gv)
    for nblocks in (1, 5, b.N + 3):          # more blocks than rows: empty blocks are skipped
        r = oracle_layer_by_row_blocks(h, v, g, W, 0.1, gh, gv, nblocks)
        assert relerr(r[0], ho) < 1e-13 and relerr(r[1], vo) < 1e-13
        assert relerr(r[2], g_h) < 1e-13 and relerr(r[3], g_v) < 1e-13
        for k in gW:
            assert relerr(r[4][k], gW[k]) < 1e-12, k
