"""The oracle against a stored snapshot of its own output.  Kept apart from the pin files:
the snapshot comes from the oracle itself, so it would "notice" every planted mistake of
test_oracle_mutants.py without proving anything about the pins.  CPU only."""


def test_oracle_matches_its_stored_snapshot(golden_dir):
    # guards against accidental edits: the snapshot was written by the oracle itself
    # (tests/golden/make_oracle_snapshot.py), so it pins nothing by itself
    import importlib.util
    import json
    import os
    spec = importlib.util.spec_from_file_location("make_oracle_snapshot",
                                                  os.path.join(golden_dir, "make_oracle_snapshot.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(golden_dir, "oracle_snapshot.json")) as f:
        stored = json.load(f)
    assert json.loads(json.dumps(mod.snapshot())) == stored
