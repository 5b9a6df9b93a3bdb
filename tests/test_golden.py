import json
import os

import numpy as np

from tests.golden.make_golden import summary


def test_config1_regression_fixture():
    with open(os.path.join(os.path.dirname(__file__), "golden", "config1_oracle.json")) as f:
        ref = json.load(f)
    got = summary()
    assert np.allclose(got["losses"], ref["losses"], rtol=1e-12)
    for k in ref["grad_l2"]:
        assert np.isclose(got["grad_l2"][k], ref["grad_l2"][k], rtol=1e-12)
        assert np.isclose(got["grad_first"][k], ref["grad_first"][k], rtol=1e-10, atol=1e-18)
