"""The speculative-pipeline state machine (C++, include/pgcm_seq.h) against the plain Python model
written from the paper (oracle/sequencer_oracle.py), the paper's worked example, and the
properties any correct sender must have.  Runs without a GPU."""
import os

import pytest

import workloads
from oracle.sequencer_oracle import SequencerOracle

import paper_2411_03357_amd as pgcm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pipeline_worked_example.txt")


def _replay(events, make):
    s = make()
    for e in events:
        if e[0] == "out":
            s.swap_out(e[1])
        elif e[0] == "req":
            s.request(e[1])
        elif e[0] == "write":
            s.notify_write(e[1])
        else:
            s.sync()
    return s


def _logs(events, **kw):
    cpp = _replay(events, lambda: pgcm.Sequencer(**kw))
    ora = _replay(events, lambda: SequencerOracle(**kw))
    return cpp.take_actions(), [tuple(a) for a in ora.log], cpp.iv_cur, ora.iv_cur


def test_worked_example_of_the_paper():
    """Figure "Tolerate wrong IVs with re-ordering requests and padding NOPs" (section 5.3): the
    IV stands at 1; data1, data2, data3 are pre-encrypted under IVs 1, 2, 3; the application
    asks for data3, then data1, then synchronises."""
    lines = [l.strip() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    names = {"data1": (0x1000000, 1 << 20), "data2": (0x2000000, 1 << 20), "data3": (0x3000000, 1 << 20)}
    expected = []
    for l in lines:
        f = l.split()
        expected.append(("nop", int(f[1])) if f[0] == "nop" else (f[0], names[f[1]], int(f[2])))
    d1, d2, d3 = names["data1"], names["data2"], names["data3"]
    # two earlier rounds teach the predictor the order data1, data2, data3 ...
    warm = []
    for _ in range(2):
        warm += [("req", d1), ("req", d2), ("req", d3), ("sync",)]
    for impl in ("cpp", "oracle"):
        s = pgcm.Sequencer(iv_start=0, depth=3) if impl == "cpp" else SequencerOracle(iv_start=0, depth=3)
        _ = [getattr(s, {"req": "request", "sync": "sync"}[e[0]])(*e[1:]) for e in warm]
        base = s.iv_cur                       # the figure calls this IV "1"
        done = len(s.take_actions()) if impl == "cpp" else len(s.log)
        s.request(d3)
        s.request(d1)
        s.sync()
        log = s.take_actions() if impl == "cpp" else [tuple(a) for a in s.log[done:]]
        shifted = [(a[0], a[1] - base + 1) if a[0] == "nop" else (a[0], a[1], a[2] - base + 1)
                   for a in log]
        # the figure's story: data1 goes out under 1, a NOP takes 2, data3 goes out under 3 and
        # the ciphertext prepared for data2 is invalidated
        story = [a for a in shifted if a[0] in ("send", "nop", "now") or (a[0] == "drop" and a[2] <= 3)]
        assert story == expected, (impl, story)


@pytest.mark.parametrize("kind", ["repetitive", "fifo", "lifo", "chaos"])
@pytest.mark.parametrize("noise", [0.0, 0.3])
def test_cpp_state_machine_equals_the_model(kind, noise):
    for seed in range(25):
        ev = workloads.swap_trace(kind, seed, noise=noise)
        for kw in (dict(iv_start=7, depth=4, leeway=0), dict(iv_start=0, depth=2, leeway=1),
                   dict(iv_start=1 << 40, depth=6, leeway=0, history_limit=5)):
            got, want, iv_c, iv_o = _logs(ev, **kw)
            assert got == want, (kind, seed, kw)
            assert iv_c == iv_o


@pytest.mark.parametrize("kind", ["repetitive", "fifo", "lifo", "chaos"])
def test_sender_invariants(kind):
    for seed in range(25):
        ev = workloads.swap_trace(kind, seed, noise=0.25)
        s = _replay(ev, lambda: pgcm.Sequencer(iv_start=100, depth=4, leeway=1))
        log = s.take_actions()
        # transfers leave under consecutive IVs, none skipped, none reused
        wire = [a for a in log if a[0] in ("send", "now", "nop")]
        assert [a[-1] for a in wire] == list(range(100, 100 + len(wire)))
        assert s.iv_cur == 100 + len(wire)
        # every request is served exactly once (all traces end with a synchronisation)
        asked = sorted(e[1] for e in ev if e[0] == "req")
        served = sorted(a[1] for a in wire if a[0] != "nop")
        assert served == asked
        # a ciphertext is delivered only if it was prepared under that very IV and neither
        # dropped nor delivered since; nothing is prepared twice while still kept
        kept = {}
        for a in log:
            if a[0] == "pre":
                assert a[1] not in kept
                kept[a[1]] = a[2]
            elif a[0] == "send":
                assert kept.pop(a[1]) == a[2]
            elif a[0] == "drop":
                assert kept.pop(a[1]) == a[2]


def test_prediction_pays_off_on_the_patterns_the_paper_names():
    """with a regular pattern and no noise nearly every swap is served from a prepared
    ciphertext; with nothing predictable nearly none is"""
    def hit_rate(kind):
        hits = total = 0
        for seed in range(10):
            ev = workloads.swap_trace(kind, seed, rounds=12)
            log = _replay(ev, lambda: pgcm.Sequencer(depth=4)).take_actions()
            hits += sum(a[0] == "send" for a in log)
            total += sum(a[0] in ("send", "now") for a in log)
        return hits / total
    assert hit_rate("repetitive") > 0.8
    assert hit_rate("fifo") > 0.9
    assert hit_rate("lifo") > 0.5
    assert hit_rate("chaos") < 0.5


def test_iv_bytes_and_argument_checks():
    iv0 = bytes.fromhex("00000000fffffffffffffffe")
    assert pgcm.seq_iv_bytes(iv0, 0) == iv0
    assert pgcm.seq_iv_bytes(iv0, 1) == bytes.fromhex("00000000ffffffffffffffff")
    assert pgcm.seq_iv_bytes(iv0, 2) == bytes.fromhex("000000010000000000000000")
    assert pgcm.seq_iv_bytes(bytes([255] * 12), 1) == bytes(12)
    for n in (0, 5, 1 << 33, (1 << 64) - 1):
        want = ((int.from_bytes(iv0, "big") + n) % (1 << 96)).to_bytes(12, "big")
        assert pgcm.seq_iv_bytes(iv0, n) == want
    with pytest.raises(pgcm.PgcmError):
        pgcm.Sequencer(depth=0)


def test_swapped_out_chunks_below_the_swap_size_are_not_pipelined():
    """only swaps are worth pre-encrypting (section 4.2): a short chunk that leaves the device is
    not tracked, so nothing is encrypted ahead for it and its later request is served on the spot"""
    for make in (lambda: SequencerOracle(iv_start=5, depth=4),
                 lambda: pgcm.Sequencer(iv_start=5, depth=4)):
        s = make()
        s.swap_out((0x1000, 4096))
        s.swap_out((0x9000, 100))
        s.request((0x1000, 4096))
        s.sync()
        log = s.log if hasattr(s, "log") else s.take_actions()
        assert [a[0] for a in log] == ["now"] and log[0][1:] == ((0x1000, 4096), 5)
        s.swap_out((0x100000, 1 << 20))
        log = s.log[1:] if hasattr(s, "log") else s.take_actions()
        assert [a[0] for a in log] == ["pre"]
