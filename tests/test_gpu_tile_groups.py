"""Products with several tiles per compute unit: an XCD receives its tiles in groups of tile rows.  Shapes whose tile
regions are not a whole number of groups and whose last tile row and column are ragged, one per tile shape of the fast
path, compared with the oracle in full (codes and accumulators bit for bit, Y and dX within the fp32 tolerance).
The contraction is short so that the oracle takes seconds."""
import sys

import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu

# (t, c_in, c_out): 128x192 tiles, 21 x 72, regions of 21 x 9 in groups of 8 rows;
#                   256x256 tiles, 20 x 37, regions of 5 x 19 in groups of 4 rows;
#                   256x288 tiles, 24 x 32, regions of 12 x 8 in groups of 8 rows
_CASES = [(2600, 128, 13824), (5000, 128, 9296), (6000, 128, 9216)]


@pytest.mark.parametrize("t,c_in,c_out", _CASES, ids=["%dx%d" % (c[0], c[2]) for c in _CASES])
def test_ragged_tile_groups(t, c_in, c_out):
    from tests.gpu_harness import Layer, OracleLayer, check_prepare, check_step
    ec = synth.EdgeCase("tile_groups_%d_%d" % (t, c_out), t, c_in, c_out, [5, 100], 16)
    print("tile groups t=%d c_in=%d c_out=%d" % (t, c_in, c_out), flush=True)
    sys.stdout.flush()
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, 90)
    L, R = Layer(W, O, A, B, 1.0, t), OracleLayer(W, O, A, B, 1.0)
    check_prepare(L, R)
    check_step(L, R, X, dY, 0.2, tag="tile groups %d x %d" % (t, c_out))
