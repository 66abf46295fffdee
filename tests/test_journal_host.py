"""Host logic of the stack driver's resumable journal (no GPU): records survive a reload, a
half-written last line is dropped, and a journal written under another configuration is
refused instead of silently feeding stale choices into a run."""
import json

import pytest

from paper_2602_07899_amd.stack import Journal

CFG = {"stack": "s", "bits": 4, "group": 128, "mode": "passact2", "joint": False, "n_alpha": 20, "seed": 0}


def _rec(layer, name, idx):
    return {"layer": layer, "linear": name, "best_idx": idx, "alpha": idx / 20, "losses": [1.0, 0.5], "joint": None}


def test_journal_round_trip_and_header(tmp_path):
    path = str(tmp_path / "j.jsonl")
    j = Journal(path, config=CFG)
    j.put(_rec(0, "q_proj", 3))
    j.put(_rec(0, "k_proj", 4))
    lines = open(path).read().splitlines()
    assert json.loads(lines[0]) == {"journal_config": CFG} and len(lines) == 3
    k = Journal(path, config=dict(CFG))
    assert set(k.done) == {(0, "q_proj"), (0, "k_proj")} and k.get(0, "k_proj")["best_idx"] == 4
    k.put(_rec(0, "v_proj", 5))
    assert len(open(path).read().splitlines()) == 4          # the header is written once
    assert len(Journal(path, config=CFG).done) == 3


def test_journal_refuses_another_configuration(tmp_path):
    path = str(tmp_path / "j.jsonl")
    Journal(path, config=CFG).put(_rec(0, "q_proj", 3))
    for key, val in (("bits", 3), ("mode", "passact1"), ("joint", True), ("seed", 1)):
        with pytest.raises(ValueError):
            Journal(path, config={**CFG, key: val})
    # a file without a header cannot vouch for its configuration
    bare = str(tmp_path / "bare.jsonl")
    open(bare, "w").write(json.dumps(_rec(0, "q_proj", 3)) + "\n")
    with pytest.raises(ValueError):
        Journal(bare, config=CFG)
    assert len(Journal(bare).done) == 1                      # no configuration given: read as is


def test_journal_drops_a_half_written_tail(tmp_path):
    path = str(tmp_path / "j.jsonl")
    j = Journal(path, config=CFG)
    j.put(_rec(0, "q_proj", 3))
    j.put(_rec(0, "k_proj", 4))
    whole = open(path, "rb").read()
    open(path, "wb").write(whole + b'{"layer": 0, "linear": "v_pr')
    k = Journal(path, config=CFG)
    assert set(k.done) == {(0, "q_proj"), (0, "k_proj")}
    assert open(path, "rb").read() == whole                  # the damaged tail is gone
    k.put(_rec(0, "v_proj", 1))
    assert len(Journal(path, config=CFG).done) == 3
