"""Host logic of the block-streaming driver (no GPU): the per-layer results file and the resume rule."""
import json

import pytest

from paper_2309_15531_amd import stream as ST


def rec(seed, block, layer, bits, group, dim="ic", l_oc=2.0, l_ic=1.0):
    return {"seed": seed, "block": block, "layer": layer, "bits": bits, "group": group, "dim": dim, "L_oc": l_oc, "L_ic": l_ic}


def test_log_round_trip_and_keys(tmp_path):
    p = str(tmp_path / "r.jsonl")
    with ST.ResultsLog(p) as log:
        log.append(rec(3, 0, "q_proj", 3, 128))
        log.append(rec(3, 0, "k_proj", 3, 128, dim="oc"))
        assert len(log) == 2 and log.has(ST.ResultsLog.key(3, 0, "q_proj", 3, 128))
        assert not log.has(ST.ResultsLog.key(3, 0, "q_proj", 4, 128))      # another precision is another key
        assert not log.has(ST.ResultsLog.key(4, 0, "q_proj", 3, 128))      # another seed too
        with pytest.raises(ValueError):
            log.append(rec(3, 0, "q_proj", 3, 128))                        # a key is written once
        with pytest.raises(KeyError):
            log.append({"seed": 3, "block": 1, "layer": "q_proj", "bits": 3})   # no group
    lines = open(p).read().splitlines()
    assert len(lines) == 2 and json.loads(lines[1])["dim"] == "oc"
    with ST.ResultsLog(p) as again:
        assert len(again) == 2 and again.get(ST.ResultsLog.key(3, 0, "k_proj", 3, 128))["dim"] == "oc"


def test_log_drops_a_cut_off_last_record(tmp_path):
    p = str(tmp_path / "r.jsonl")
    with ST.ResultsLog(p) as log:
        log.append(rec(1, 0, "a", 3, 128))
        log.append(rec(1, 0, "b", 3, 128))
    whole = open(p, "rb").read()
    open(p, "ab").write(b'{"seed": 1, "block": 0, "layer": "c", "bi')          # the process died here
    with ST.ResultsLog(p) as log:
        assert len(log) == 2
        log.append(rec(1, 0, "c", 3, 128))
    data = open(p, "rb").read()
    assert data.startswith(whole) and data.count(b"\n") == 3
    assert [json.loads(l)["layer"] for l in data.splitlines()] == ["a", "b", "c"]


def test_pending_layers_order_and_skip(tmp_path):
    with ST.ResultsLog(str(tmp_path / "r.jsonl")) as log:
        names, bits = ["q", "k", "down"], (4, 3)
        todo = ST.pending_layers(log, 7, range(2), names, bits, 128)
        assert todo == [(0, [("q", 4), ("k", 4), ("down", 4), ("q", 3), ("k", 3), ("down", 3)]),
                        (1, [("q", 4), ("k", 4), ("down", 4), ("q", 3), ("k", 3), ("down", 3)])]
        for n in names:
            for b in bits:
                log.append(rec(7, 0, n, b, 128))
        log.append(rec(7, 1, "k", 4, 128))
        todo = ST.pending_layers(log, 7, range(2), names, bits, 128)
        assert todo == [(1, [("q", 4), ("down", 4), ("q", 3), ("k", 3), ("down", 3)])]


class FakeBlockSearch:
    """Stands in for BlockSearch: records the calls, answers with losses derived from the block number."""

    def __init__(self, names, bits_list, group):
        self.names, self.bits_list, self.group = names, bits_list, group
        self.calls, self.slots = [], {}

    def hessians(self, X):
        self.calls.append(("H", X["block"]))

    def launch(self, slot, weights, only=None):
        self.calls.append(("launch", weights["block"], slot))
        assert weights["slot"] == slot
        self.slots[slot] = (weights["block"], list(only))

    def collect(self, slot):
        b, pairs = self.slots.pop(slot)
        self.calls.append(("collect", b, slot))
        return [{"layer": n, "bits": bits, "dim": "ic", "L_oc": 10.0 + b, "L_ic": 1.0 + b} for n, bits in pairs]


def test_run_stream_resumes_where_it_stopped(tmp_path):
    p = str(tmp_path / "r.jsonl")
    names, bits = ["q", "down"], (3,)
    fake = FakeBlockSearch(names, bits, 128)
    stop_after = {"n": 2}

    def on_block(b):
        stop_after["n"] -= 1
        if stop_after["n"] == 0:
            raise KeyboardInterrupt                                      # the run is cut short after two blocks

    with ST.ResultsLog(p) as log:
        with pytest.raises(KeyboardInterrupt):
            ST.run_stream(fake, log, 5, range(4), lambda b, s: {"block": b, "slot": s}, lambda b: {"block": b}, on_block)
    # block b + 1 is queued before block b is collected, and the two result slots alternate
    assert fake.calls[:7] == [("H", 0), ("launch", 0, 0), ("H", 1), ("launch", 1, 1), ("collect", 0, 0),
                              ("H", 2), ("launch", 2, 0)]
    with ST.ResultsLog(p) as log:
        assert len(log) == 4                                             # blocks 0 and 1, two layers each
        fake2 = FakeBlockSearch(names, bits, 128)
        n = ST.run_stream(fake2, log, 5, range(4), lambda b, s: {"block": b, "slot": s}, lambda b: {"block": b})
        assert n == 4 and len(log) == 8
        assert [c for c in fake2.calls if c[0] == "launch"] == [("launch", 2, 0), ("launch", 3, 1)]
        # a third run has nothing to do
        fake3 = FakeBlockSearch(names, bits, 128)
        assert ST.run_stream(fake3, log, 5, range(4), lambda b, s: {"block": b, "slot": s}, lambda b: {"block": b}) == 0
        assert fake3.calls == []
        r = log.get(ST.ResultsLog.key(5, 3, "down", 3, 128))
        assert r["L_oc"] == 13.0 and r["L_ic"] == 4.0 and r["dim"] == "ic" and r["group"] == 128
