"""The oracle against a stored snapshot of its own output.  Kept apart from the pin files:
the snapshot comes from the oracle itself, so it would "notice" every planted mistake of
test_oracle_mutants.py without proving anything about the pins.  CPU only."""


def test_oracle_matches_its_stored_snapshot(golden_dir):
    # guards against accidental edits: the snapshot was written by the oracle itself
    # (tests/golden/make_oracle_snapshot.py), so it pins nothing by itself
    import importlib.util
    import numpy as np
    import json
    import os
    spec = importlib.util.spec_from_file_location("make_oracle_snapshot",
                                                  os.path.join(golden_dir, "make_oracle_snapshot.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(golden_dir, "oracle_snapshot.json")) as f:
        stored = json.load(f)
    now = json.loads(json.dumps(mod.snapshot()))
    assert now.keys() == stored.keys()
    for key, want in stored.items():
        got = now[key]
        if isinstance(want, list) and want and isinstance(want[0], str):      # hexadecimal floats
            a = np.array([float.fromhex(x) for x in got]); b = np.array([float.fromhex(x) for x in want])
            # (the matrix products go through BLAS, whose summation order depends on the machine)
            assert a.shape == b.shape and np.allclose(a, b, rtol=1e-12, atol=0), key
        elif isinstance(want, str):
            assert abs(float.fromhex(got) - float.fromhex(want)) <= 1e-12 * abs(float.fromhex(want)), key
        else:
            assert got == want, key
