"""The oracle against its own frozen outputs (tests/golden/oracle_small_cases.json, written by
tests/golden/make_golden.py from the oracle alone): a change of the oracle's arithmetic shows up here."""
import importlib.util
import json
from pathlib import Path

import numpy as np

GOLDEN = Path(__file__).resolve().parent / "golden"


def test_oracle_reproduces_its_frozen_outputs(oracle):
    spec = importlib.util.spec_from_file_location("make_golden", GOLDEN / "make_golden.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    then = json.loads((GOLDEN / "oracle_small_cases.json").read_text())
    assert now.keys() == then.keys()
    for group in then:
        assert now[group].keys() == then[group].keys()
        for name, fields in then[group].items():
            for key, val in fields.items():
                a, b = np.asarray(now[group][name][key]), np.asarray(val)
                if a.dtype.kind in "iu":
                    np.testing.assert_array_equal(a, b, err_msg=f"{group}/{name}/{key}")
                else:
                    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-300, err_msg=f"{group}/{name}/{key}")
