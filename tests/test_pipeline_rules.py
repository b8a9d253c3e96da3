"""The speculative pipeline judged by the paper's rules, not by a second implementation.

oracle/pipeline_rules.py restates what sections 4.1 and 5.1-5.3 require of any sender and checks
an action log against it.  Here (a) the checker itself is pinned to the paper's worked example
(the figure of section 5.3) and must reject each way of getting that example wrong; (b) the C++
state machine and the Python model are each judged by it on their own, over every seeded trace;
(c) the patterns the paper names (section 5.1: repetitive, FIFO, LIFO) must be predicted: on a
pure trace of each, once the pattern has shown itself, every swap is served from a ciphertext
prepared ahead of demand; (d) mistakes planted in copies of either implementation (predictor,
IV assignment, NOP padding, validator, discarding) must each be caught by (b) or (c), without
the other implementation being consulted.  Runs without a GPU."""
import ctypes
import os
import shutil
import subprocess
import types

import pytest

import workloads
from oracle import pipeline_rules as rules
from oracle.sequencer_oracle import SequencerOracle

import paper_2411_03357_amd as pgcm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden", "pipeline_worked_example.txt")
SEQ_CPP = os.path.join(ROOT, "paper_2411_03357_amd", "csrc", "pgcm_seq.cpp")
MODEL_PY = os.path.join(ROOT, "oracle", "sequencer_oracle.py")
MIB = 1 << 20
THRESHOLD = 128 * 1024

D1, D2, D3 = (0x1000000, MIB), (0x2000000, MIB), (0x3000000, MIB)


# ---------------------------------------------------------------------------------------------
# (a) the checker against the worked example

def _golden_actions():
    names = {"data1": D1, "data2": D2, "data3": D3}
    out = []
    for l in open(GOLDEN):
        f = l.split()
        if not f or f[0].startswith("#"):
            continue
        out.append(("nop", int(f[1])) if f[0] == "nop" else (f[0], names[f[1]], int(f[2])))
    return out


def _example(after_sync=None, at_req3=(), at_req1=None, extra=()):
    """the figure's situation: the IV stands at 1; data1, data2, data3 are prepared under 1, 2, 3;
    then data3 is asked for, then data1, then comes the synchronisation"""
    g = _golden_actions()
    assert g == [("send", D1, 1), ("nop", 2), ("send", D3, 3), ("drop", D2, 2)]
    steps = [(("out", D1), [("pre", D1, 1)]), (("out", D2), [("pre", D2, 2)]),
             (("out", D3), [("pre", D3, 3)])]
    steps += list(extra)
    steps += [(("req", D3), list(at_req3)),
              (("req", D1), [g[0]] if at_req1 is None else list(at_req1)),
              (("sync",), g[1:] if after_sync is None else list(after_sync))]
    return steps


def _violates(steps, rule, **kw):
    with pytest.raises(rules.RuleViolation) as e:
        rules.check_trace(steps, kw.pop("iv_start", 1), THRESHOLD, **kw)
    assert e.value.rule == rule, str(e.value)


def test_the_worked_example_satisfies_the_rules():
    stats = rules.check_trace(_example(), 1, THRESHOLD, depth=3)
    assert stats == dict(transfers=3, sends=2, nows=0, nops=1, pres=3, drops=1)


def test_each_way_of_getting_the_worked_example_wrong_breaks_its_rule():
    # no NOP: data3 would leave under IV 3 while the receiver expects 2
    _violates(_example(after_sync=[("send", D3, 3), ("drop", D2, 2)]), "W")
    # data3 sent at once under the IV it was made for, out of wire order
    _violates(_example(at_req3=[("send", D3, 3)]), "W")
    # data3 sent under the current IV although it was encrypted under 3
    _violates(_example(at_req3=[("send", D3, 1)]), "V")
    # data3 encrypted again on request although a ciphertext under a later IV is kept
    _violates(_example(at_req3=[("now", D3, 1)], at_req1=[],
                       after_sync=[("now", D1, 2), ("drop", D1, 1), ("drop", D2, 2),
                                   ("drop", D3, 3)]), "E3")
    # data1, kept under the current IV, not sent when asked for
    _violates(_example(at_req1=[]), "E3")
    # the ciphertext of data2, whose IV the wire has passed, kept beyond the synchronisation
    _violates(_example(after_sync=[("nop", 2), ("send", D3, 3)]), "E1")
    # a NOP before the synchronisation (another request of the batch may still fill the gap)
    _violates(_example(at_req1=[("send", D1, 1), ("nop", 2)],
                       after_sync=[("send", D3, 3), ("drop", D2, 2)]), "E4")
    # a NOP that pads the way to nothing
    _violates(_example(after_sync=[("nop", 2), ("send", D3, 3), ("drop", D2, 2), ("nop", 4)]), "E4")
    # the synchronisation encrypts data3 again instead of padding the way to its IV
    _violates(_example(after_sync=[("drop", D3, 3), ("now", D3, 2), ("drop", D2, 2)]), "E5")
    # a small transfer takes the IV a held request's ciphertext waits for
    s1, s2 = (0x5000, 100), (0x6000, 200)
    _violates([(("out", D1), [("pre", D1, 2)]), (("req", D1), []), (("req", s1), [("now", s1, 1)]),
               (("req", s2), [("now", s2, 2)])], "E6")
    # data3 never delivered
    _violates(_example(after_sync=[]), "S")
    # data2 delivered although nobody asked for it
    _violates(_example(after_sync=[("send", D2, 2), ("send", D3, 3)]), "S")
    # data1 written to after it was encrypted, and its old ciphertext sent all the same
    _violates(_example(extra=[(("write", (D1[0] + 5000, 16)), [])]), "V")
    # ... the same write answered correctly: drop, and the request is encrypted on the spot
    ok = _example(extra=[(("write", (D1[0] + 5000, 16)), [("drop", D1, 1)])],
                  at_req1=[("now", D1, 1)],
                  after_sync=[("drop", D2, 2), ("nop", 2), ("send", D3, 3)])
    assert rules.check_trace(ok, 1, THRESHOLD)["nows"] == 1
    # a usable ciphertext thrown away for no reason
    _violates(_example(extra=[(("out", (0x9000000, MIB)), [("drop", D3, 3)])], at_req3=[],
                       after_sync=[("drop", D2, 2), ("now", D3, 2)]), "E2")
    # one IV promised to two ciphertexts
    _violates([(("out", D1), [("pre", D1, 1)]), (("out", D2), [("pre", D2, 1)])], "P")
    # a ciphertext prepared for a chunk nobody has seen
    _violates([(("out", D1), [("pre", D2, 1)])], "P")
    # more kept than the depth allows
    _violates(_example(), "P", depth=2)
    # a small transfer pipelined, or held back
    small = (0x5000, 100)
    _violates([(("out", small), [("pre", small, 1)])], "T")
    _violates([(("req", small), []), (("sync",), [("now", small, 1)])], "T")


# ---------------------------------------------------------------------------------------------
# (b) each implementation judged on its own

PARAMS = (dict(iv_start=7, depth=4, leeway=0), dict(iv_start=0, depth=2, leeway=1),
          dict(iv_start=1 << 40, depth=6, leeway=0, history_limit=5))


def _take_cpp(s):
    return s.take_actions()


def _take_model(s):
    new = s.log[getattr(s, "_taken", 0):]
    s._taken = len(s.log)
    return new


def _judge(make, take, kinds=("repetitive", "fifo", "lifo", "chaos"), seeds=range(25)):
    """every seeded trace through a fresh sender from make(**params); the first violation raises"""
    total = 0
    for kind in kinds:
        for noise in (0.0, 0.3):
            for seed in seeds:
                ev = workloads.swap_trace(kind, seed, noise=noise)
                for kw in PARAMS:
                    steps = rules.steps_of(ev, make(**kw), take)
                    st = rules.check_trace(steps, kw["iv_start"], THRESHOLD, depth=kw["depth"])
                    total += st["transfers"]
    return total


def test_the_cpp_state_machine_keeps_the_rules_on_every_trace():
    assert _judge(pgcm.Sequencer, _take_cpp) > 10000


def test_the_python_model_keeps_the_rules_on_every_trace():
    assert _judge(SequencerOracle, _take_model) > 10000


def test_written_plaintext_is_never_sent_hand_written_trace():
    """prepare, write into the chunk, ask for it (section 5.2): the stale ciphertext is dropped in
    the step of the write, and what is delivered afterwards was encrypted after the write: on the
    spot, or prepared afresh"""
    a, b = (0x4000000, 2 * MIB), (0x5000000, 2 * MIB)
    ev = [("out", a), ("out", b), ("write", (a[0] + MIB, 1)), ("req", a), ("req", b), ("sync",)]
    for make, take in ((pgcm.Sequencer, _take_cpp), (SequencerOracle, _take_model)):
        steps = rules.steps_of(ev, make(iv_start=3, depth=2), take)
        rules.check_trace(steps, 3, THRESHOLD, depth=2)
        assert steps[0][1] == [("pre", a, 3)]
        assert steps[2][1][0] == ("drop", a, 3)
        made = [k for k, (_, acts) in enumerate(steps) for x in acts
                if x[0] in ("pre", "now") and x[1] == a]
        assert made[0] == 0 and len(made) == 2 and made[1] >= 2
        # the same log with the drop taken out is what the validator exists to prevent
        bad = [(e, [x for x in acts if x != ("drop", a, 3)]) for e, acts in steps]
        with pytest.raises(rules.RuleViolation):
            rules.check_trace(bad, 3, THRESHOLD, depth=2)


# ---------------------------------------------------------------------------------------------
# (c) the paper's three patterns are predicted

def _pure_traces():
    layers = [(0x10000000 + i * 4 * MIB, 2 * MIB) for i in (1, 3, 4)]
    rep = []
    for _ in range(6):                       # layers 1, 3, 4 come back round after round
        for c in layers:
            rep += [("req", c), ("sync",)]
    blocks = [(0x20000000 + i * 327680, 327680) for i in range(5)]
    fifo = [("out", c) for c in blocks] + [("sync",)]
    lifo = list(fifo)
    for c in blocks:                         # layer-wise: back in the order they left
        fifo += [("req", c), ("sync",)]
    for c in blocks[::-1]:                   # request-wise: the last to leave is the first back
        lifo += [("req", c), ("sync",)]
    # how many swaps may be served on the critical path before the pattern has shown itself:
    # one round of the repetitive pattern (a chunk must have been seen before), none for FIFO
    # (the oldest swapped-out chunk is the first guess), one for LIFO (the first return shows
    # which end of the swapped-out set the application takes)
    return {"repetitive": (rep, len(layers) + 1), "fifo": (fifo, 0), "lifo": (lifo, 1)}


def _swaps_on_the_critical_path(make, take, events):
    steps = rules.steps_of(events, make(iv_start=0, depth=3), take)
    rules.check_trace(steps, 0, THRESHOLD, depth=3)
    kinds = [a[0] for _, acts in steps for a in acts if a[0] in ("send", "now")]
    assert len(kinds) == sum(e[0] == "req" for e in events)
    return kinds


def _assert_patterns_are_predicted(make, take):
    for name, (events, allowed) in _pure_traces().items():
        kinds = _swaps_on_the_critical_path(make, take, events)
        assert kinds[allowed:] == ["send"] * (len(kinds) - allowed), (name, kinds)


def test_the_cpp_state_machine_predicts_the_papers_patterns():
    _assert_patterns_are_predicted(pgcm.Sequencer, _take_cpp)


def test_the_python_model_predicts_the_papers_patterns():
    _assert_patterns_are_predicted(SequencerOracle, _take_model)


# ---------------------------------------------------------------------------------------------
# (d) planted mistakes

def _caught(make, take):
    """True when the rules or the pattern pins reject the sender"""
    try:
        _assert_patterns_are_predicted(make, take)
        _judge(make, take, seeds=range(8))
    except AssertionError:        # RuleViolation is one
        return True
    return False


CPP_MISTAKES = {
    "predictor takes the wrong end of the swapped-out set":
        ("if (ends == Ends::kFifo) {", "if (ends != Ends::kFifo) {"),
    "repetitive pattern off by one":
        ("if (spoken.find(seen[k + 1]) == spoken.end()) {\n                        *next = seen[k + 1];",
         "if (spoken.find(seen[k]) == spoken.end()) {\n                        *next = seen[k];"),
    "every prediction gets the current IV":
        ("const uint64_t iv = next_iv + leeway;", "const uint64_t iv = iv_cur + leeway;"),
    "no NOP padding at the synchronisation":
        ("while (s->iv_cur < h.second) {", "while (false) {"),
    "validator only sees writes at a chunk's first byte":
        ("if (c.addr < addr + len && addr < c.addr + c.len) {", "if (c.addr == addr) {"),
    "ciphertexts whose IV has passed are kept":
        ("if (e.first < iv_cur && !is_held(e.second)) {",
         "if (e.first + 1000 < iv_cur && !is_held(e.second)) {"),
    "a ciphertext under the current IV counts as too late":
        ("it->second >= s->iv_cur;", "it->second > s->iv_cur;"),
    "held requests are sent at the synchronisation in arrival order":
        ("[](const auto& a, const auto& b) { return a.second < b.second; });\n        std::vector<std::pair<Chunk, uint64_t>> late;",
         "[](const auto& a, const auto& b) { return false; });\n        std::vector<std::pair<Chunk, uint64_t>> late;"),
    "a transfer encrypted on the spot does not release the held request whose IV it reaches":
        ("            ++s->iv_cur;\n            s->release_held();\n            s->drop_passed();\n        } else if",
         "            ++s->iv_cur;\n            s->drop_passed();\n        } else if"),
}


@pytest.mark.parametrize("what", sorted(CPP_MISTAKES))
def test_a_mistake_planted_in_the_cpp_state_machine_is_caught(what, tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    old, new = CPP_MISTAKES[what]
    src = open(SEQ_CPP).read()
    assert src.count(old) == 1, "the planted mistake no longer applies: " + what
    src = src.replace(old, new).replace('#include "../../include/',
                                         '#include "%s/include/' % ROOT)
    path = tmp_path / "seq_mutant.cpp"
    path.write_text(src)
    so = tmp_path / "libseq_mutant.so"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-shared", "-fPIC", str(path), "-o",
                           str(so)])
    lib = ctypes.CDLL(str(so))
    assert _caught(lambda **kw: pgcm.Sequencer(lib=lib, **kw), _take_cpp), what


def test_the_unmodified_cpp_source_built_the_same_way_is_not_caught(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    src = open(SEQ_CPP).read().replace('#include "../../include/', '#include "%s/include/' % ROOT)
    path = tmp_path / "seq_plain.cpp"
    path.write_text(src)
    so = tmp_path / "libseq_plain.so"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-shared", "-fPIC", str(path), "-o",
                           str(so)])
    lib = ctypes.CDLL(str(so))
    assert not _caught(lambda **kw: pgcm.Sequencer(lib=lib, **kw), _take_cpp)


MODEL_MISTAKES = {
    "predictor takes the wrong end of the swapped-out set":
        ('return candidates[0] if self.mode == "fifo" else candidates[-1]',
         'return candidates[-1] if self.mode == "fifo" else candidates[0]'),
    "repetitive pattern off by one":
        ("nxt = flat[k + 1]", "nxt = flat[k]"),
    "every prediction gets the current IV":
        ("iv = next_iv + self.leeway", "iv = self.iv_cur + self.leeway"),
    "no NOP padding at the synchronisation":
        ("            while self.iv_cur < iv:\n                self.log.append((\"nop\", self.iv_cur))\n                self.iv_cur += 1\n            del self.spec[chunk]",
         "            del self.spec[chunk]"),
    "validator only sees writes at a chunk's first byte":
        ("if c[0] < addr + length and addr < c[0] + c[1]:", "if c[0] == addr:"),
    "ciphertexts whose IV has passed are kept":
        ("if v < self.iv_cur and c not in held:", "if v + 1000 < self.iv_cur and c not in held:"),
    "a ciphertext under the current IV counts as too late":
        ("if iv is None or iv < self.iv_cur:", "if iv is None or iv <= self.iv_cur:"),
    "held requests are sent at the synchronisation in arrival order":
        ("ahead = sorted((e for e in self.pending if e[1] >= self.iv_cur), key=lambda e: e[1])",
         "ahead = [e for e in self.pending if e[1] >= self.iv_cur]"),
    "a transfer encrypted on the spot does not release the held request whose IV it reaches":
        ("            self.iv_cur += 1\n            self._release_pending()\n            self._drop_stale()\n        elif iv == self.iv_cur:",
         "            self.iv_cur += 1\n            self._drop_stale()\n        elif iv == self.iv_cur:"),
}


@pytest.mark.parametrize("what", sorted(MODEL_MISTAKES))
def test_a_mistake_planted_in_the_python_model_is_caught(what):
    old, new = MODEL_MISTAKES[what]
    src = open(MODEL_PY).read()
    assert src.count(old) == 1, "the planted mistake no longer applies: " + what
    mod = types.ModuleType("sequencer_mutant")
    exec(compile(src.replace(old, new), "sequencer_mutant.py", "exec"), mod.__dict__)
    assert _caught(mod.SequencerOracle, _take_model), what
