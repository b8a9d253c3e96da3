"""Rule checker for logs of the paper's speculative pipelined encryption: test infrastructure.

This module generates nothing.  It is handed what a sender DID (events in, actions out, step by
step) and checks it against what the paper REQUIRES of any such sender, rule by rule.  It knows
no prediction strategy, shares nothing with the C++ state machine or the Python model, and can
therefore judge either of them without consulting the other.

Vocabulary.  An event is ("out", chunk) | ("req", chunk) | ("write", range) | ("sync",) with
chunk = range = (address, bytes).  An action is ("pre", chunk, iv) | ("send", chunk, iv) |
("now", chunk, iv) | ("nop", iv) | ("drop", chunk, iv).  A step is (event, [actions it caused]).

Rules, with the passage each one restates:

 W  wire order (section 4.1, "Swapping sequence and IVs"; section 2.2): both ends count
    transfers, so the transfers that leave (send, now, nop) carry IV_start, IV_start + 1, ..
    with no gap and no reuse.
 S  service (section 5.1, predictor input: requests come in batches closed by a
    synchronisation; order is kept between batches, not inside one): every request is delivered
    exactly once, by a send or a now of that very chunk, no later than the synchronisation that
    closes its batch; nothing is delivered that was not asked for.
 T  small transfers (section 5.1, "Targeting major memory swapping"): a request below the swap
    size is never pipelined: it is answered at once by a now, and no ciphertext is ever
    prepared for such a chunk.
 P  preparation (section 4.3; section 5.1, f's inputs and outputs): a ciphertext is prepared
    only for a chunk the sender has grounds to expect (it was swapped out and has not come back,
    or it came back before), under an IV not yet used on the wire and not promised to another
    kept ciphertext, and a chunk has at most one kept ciphertext; at most `depth` are kept.
 V  validation (section 5.2): a send needs a kept ciphertext made for exactly this address and
    length, under exactly this IV, whose plaintext no write has touched since it was made.  A
    write that overlaps a kept ciphertext's plaintext makes it stale: it may only be dropped,
    and must be before the step ends.
 E  error handling (section 5.3): (E1) a ciphertext whose IV the wire has passed can never be
    sent and is discarded: none survives the step that passed it, except while a held request
    still waits for the synchronisation, and none survives a synchronisation.  (E2) a drop needs
    a reason: its IV has passed, a write overlapped it, or the request that caused the step was
    not predicted (the pipeline is reset).  (E3) a request whose ciphertext is kept under the
    current IV is sent at once, never encrypted again; one whose ciphertext is kept under a
    later IV is held, not encrypted again, unless its chunk is already waiting in this batch;
    a held request ends as a now only if its ciphertext was overtaken or overwritten.
    (E4) a NOP only pads the way to a held request's IV at a synchronisation: NOPs occur only
    in the step of a sync, and every run of them is followed directly by a send.
    (E5) re-ordering inside a batch ("Swap re-ordering"): the held requests of a batch are
    committed in the order of their IVs, whatever order they came in, so every held request
    whose ciphertext the wire has not passed when the synchronisation begins is sent, none of
    them is encrypted again.  (E6) for the same reason no other transfer leaves under the IV a
    held request's ciphertext was made for: when the wire reaches that IV, the held request is
    the one that goes.
"""


class RuleViolation(AssertionError):
    def __init__(self, rule, step, text):
        self.rule, self.step = rule, step
        super().__init__("rule %s, step %d: %s" % (rule, step, text))


def _overlap(a, b):
    return a[0] < b[0] + b[1] and b[0] < a[0] + a[1]


def check_trace(steps, iv_start, threshold, depth=None):
    """steps: list of (event, actions).  Raises RuleViolation at the first broken rule; returns
    a summary dict (transfers, sends, nows, nops, pres, drops) otherwise."""
    iv = iv_start
    kept = {}            # chunk -> dict(iv, stale)
    away = set()         # swapped out, not yet asked for again
    seen = set()         # swaps asked for at some point
    waiting = []         # requests of the open batch not yet delivered: dict(chunk, small,
                         #   had = IV of the usable kept ciphertext when the request came, or
                         #   None; due = that IV was the current one; step)
    stats = dict(transfers=0, sends=0, nows=0, nops=0, pres=0, drops=0)

    for k, (event, actions) in enumerate(steps):
        kind = event[0]
        unpredicted = False
        if kind == "out":
            if event[1][1] >= threshold:
                away.add(event[1])
        elif kind == "write":
            for c, e in kept.items():
                if _overlap(c, event[1]):
                    e["stale"] = True
        elif kind == "req":
            c = event[1]
            small = c[1] < threshold
            had = None
            if not small:
                e = kept.get(c)
                duplicate = any(w["chunk"] == c for w in waiting)
                if e is not None and not e["stale"] and e["iv"] >= iv and not duplicate:
                    had = e["iv"]
                else:
                    unpredicted = True
                seen.add(c)
                away.discard(c)
            waiting.append(dict(chunk=c, small=small, had=had, due=had == iv, step=k))
        elif kind == "sync":
            for w in waiting:
                e = kept.get(w["chunk"])
                w["reorder"] = (w["had"] is not None and e is not None and e["iv"] == w["had"]
                                and not e["stale"] and e["iv"] >= iv)
        else:
            raise ValueError("unknown event %r" % (event,))

        nop_run = False
        dropped = []     # (chunk, iv, was stale) of this step's drops: judged when the step ends
        for a in actions:
            what = a[0]
            if what in ("send", "now", "nop") and a[-1] != iv:
                raise RuleViolation("W", k, "%s under IV %d, the wire is at %d" % (what, a[-1], iv))
            if what in ("now", "nop"):
                for w in waiting:
                    e = kept.get(w["chunk"])
                    if (w["had"] == iv and w["step"] != k and e is not None and e["iv"] == iv
                            and not e["stale"]):
                        raise RuleViolation("E6", k, "%s takes IV %d, for which the held request "
                                            "%r has a ciphertext" % (what, iv, w["chunk"]))
            if nop_run and what not in ("nop", "send"):
                raise RuleViolation("E4", k, "a run of NOPs is followed by %r" % (a,))
            if what == "nop":
                if kind != "sync":
                    raise RuleViolation("E4", k, "NOP outside a synchronisation")
                nop_run = True
                iv += 1
                stats["nops"] += 1
                stats["transfers"] += 1
                continue
            nop_run = False
            c = a[1]
            if what == "pre":
                if c[1] < threshold:
                    raise RuleViolation("T", k, "ciphertext prepared for a small transfer %r" % (c,))
                if c not in away and c not in seen:
                    raise RuleViolation("P", k, "no grounds to expect %r" % (c,))
                if c in kept:
                    raise RuleViolation("P", k, "%r already has a kept ciphertext" % (c,))
                if a[2] < iv:
                    raise RuleViolation("P", k, "prepared under IV %d, the wire is already at %d"
                                        % (a[2], iv))
                if any(e["iv"] == a[2] for e in kept.values()):
                    raise RuleViolation("P", k, "IV %d promised twice" % a[2])
                kept[c] = dict(iv=a[2], stale=False)
                if depth is not None and len(kept) > depth:
                    raise RuleViolation("P", k, "%d ciphertexts kept, depth is %d"
                                        % (len(kept), depth))
                stats["pres"] += 1
            elif what == "drop":
                e = kept.get(c)
                if e is None or e["iv"] != a[2]:
                    raise RuleViolation("E2", k, "drop of %r under IV %d: nothing such is kept"
                                        % (c, a[2]))
                dropped.append((c, a[2], e["stale"]))
                del kept[c]
                stats["drops"] += 1
            elif what == "send":
                cands = [w for w in waiting if w["chunk"] == c]
                if not cands:
                    raise RuleViolation("S", k, "send of %r, which nobody is waiting for" % (c,))
                w = next((w for w in cands if w["had"] == a[2]), cands[0])
                e = kept.get(c)
                if e is None:
                    raise RuleViolation("V", k, "send of %r without a kept ciphertext" % (c,))
                if e["iv"] != a[2]:
                    raise RuleViolation("V", k, "send of %r under IV %d, it was made under %d"
                                        % (c, a[2], e["iv"]))
                if e["stale"]:
                    raise RuleViolation("V", k, "send of %r after its plaintext was written" % (c,))
                del kept[c]
                waiting.remove(w)
                iv += 1
                stats["sends"] += 1
                stats["transfers"] += 1
            elif what == "now":
                cands = [w for w in waiting if w["chunk"] == c]
                if not cands:
                    raise RuleViolation("S", k, "now of %r, which nobody is waiting for" % (c,))
                w = next((w for w in cands if w["step"] == k and w["had"] is None), cands[0])
                if w["small"] and w["step"] != k:
                    raise RuleViolation("T", k, "small transfer %r not answered at once" % (c,))
                if w.get("reorder"):
                    raise RuleViolation("E5", k, "%r encrypted again at the synchronisation "
                                        "although its ciphertext could still be sent in IV order"
                                        % (c,))
                if w["had"] is not None:
                    # encrypted again although a ciphertext was kept for it: allowed only when
                    # that ciphertext has been lost since (overtaken by the wire, or overwritten)
                    e = kept.get(c)
                    if e is not None and e["iv"] == w["had"] and not e["stale"] and e["iv"] >= iv:
                        raise RuleViolation("E3", k, "%r encrypted again although its ciphertext "
                                            "is kept under IV %d" % (c, e["iv"]))
                    if w["step"] == k:
                        raise RuleViolation("E3", k, "%r encrypted on request although its "
                                            "ciphertext was kept under IV %d" % (c, w["had"]))
                waiting.remove(w)
                iv += 1
                stats["nows"] += 1
                stats["transfers"] += 1
            else:
                raise ValueError("unknown action %r" % (a,))
        if nop_run:
            raise RuleViolation("E4", k, "the step ends with a NOP that pads the way to nothing")

        # --- the step is over
        for c, v, stale in dropped:
            if not (stale or v < iv or unpredicted):
                raise RuleViolation("E2", k, "drop of %r (IV %d) without a reason, the wire is "
                                    "at %d" % (c, v, iv))
        for w in waiting:
            if w["step"] != k:
                continue
            # still waiting after its own step: only a swap whose ciphertext lies ahead may be
            if w["small"]:
                raise RuleViolation("T", k, "small transfer %r held back" % (w["chunk"],))
            if w["had"] is None:
                raise RuleViolation("S", k, "%r held although nothing usable is kept for it"
                                    % (w["chunk"],))
            if w["due"]:
                raise RuleViolation("E3", k, "%r was kept under the current IV and was not sent"
                                    % (w["chunk"],))
        held = {w["chunk"] for w in waiting}
        for c, e in kept.items():
            if e["stale"]:
                raise RuleViolation("V", k, "%r was written to and its ciphertext is still kept"
                                    % (c,))
            if e["iv"] < iv and (kind == "sync" or c not in held):
                raise RuleViolation("E1", k, "%r is kept under IV %d, the wire is at %d"
                                    % (c, e["iv"], iv))
        if kind == "sync" and waiting:
            raise RuleViolation("S", k, "%d request(s) not delivered by the synchronisation"
                                % len(waiting))
    return stats


def steps_of(events, sender, take):
    """Replays `events` into `sender` (an object with swap_out / request / notify_write / sync)
    and groups the actions by the event that caused them; take(sender) returns the actions
    emitted since the last call, as tuples."""
    out = []
    for e in events:
        if e[0] == "out":
            sender.swap_out(e[1])
        elif e[0] == "req":
            sender.request(e[1])
        elif e[0] == "write":
            sender.notify_write(e[1])
        else:
            sender.sync()
        out.append((e, [tuple(a) for a in take(sender)]))
    return out
