"""The fp32 oracle must reproduce, bit for bit, the digest stored by tests/golden/make_golden.py
(written by the oracle itself on the development host): guards against drift of its arithmetic
and shows that its pinned operation order gives the same bits on another CPU."""
import importlib.util
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_digest_reproduces():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    with open(os.path.join(HERE, "golden", "oracle_digest.json")) as f:
        want = json.load(f)
    for key, args in (("cfg1", (1,)), ("cfg2_n20000", (2, 20000)), ("cfg1_compact_box", (1, None, True)),
                      ("cfg2_n20000_compact_box", (2, 20000, True))):
        got = mg.digest(*args)
        assert got["inputs"] == want[key]["inputs"], (
            f"{key}: the scene generator drew different inputs on this host (numpy / libm differences), so the "
            "stored digest does not apply; regenerate it with tests/golden/make_golden.py and review the change")
        assert got == want[key]
