"""The chunked formulas the kernels are built from equal the recurrence (fp64, CPU)."""
import numpy as np
import pytest

import chunked_ref
from oracle import ssd_ref
from test_oracle_pins import draw


@pytest.mark.parametrize("Q", [1, 2, 8, 24])
def test_chunked_equals_sequential(Q):
    d = draw(40 + Q, L=24, G=2)
    y, entering, _ = chunked_ref.forward(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], Q, d["init_state"])
    r = ssd_ref.ssd_fwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["init_state"], segment=Q)
    assert np.max(np.abs(y - r["y"])) <= 1e-12 * np.max(np.abs(r["y"]))
    assert np.max(np.abs(entering[:, -1] - r["final_state"])) <= 1e-12 * np.max(np.abs(r["final_state"]))
    assert np.max(np.abs(entering[:, :-1] - r["boundary_states"])) <= 1e-12 * np.max(np.abs(r["boundary_states"]))
    g = chunked_ref.backward(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], Q, entering, d["dfinal_state"])
    o = ssd_ref.ssd_bwd(d["x"], d["dt"], d["A"], d["B"], d["C"], d["D"], d["dy"], d["init_state"], d["dfinal_state"])
    for k in o:
        assert np.max(np.abs(g[k] - o[k])) <= 1e-11 * max(1.0, np.max(np.abs(o[k]))), k
