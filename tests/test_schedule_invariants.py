"""The chunk-to-wavefront schedule the batch calls upload (descriptors, unit map, coarse map,
fold lists), built on the host by pgcm_describe_schedule and checked here without a GPU against
what the kernels assume when they read it:

  * units: every unit belongs to exactly one chunk; a chunk's units are consecutive, cover its
    blocks exactly, and only its first unit may be short;
  * the coarse map never points past the chunk that holds a unit (the kernel only walks forward);
  * partial-set slots: units take slots 0 .. nunits - 1, every fold item writes a slot of its own
    beyond them, and nothing is read before it is written (an item's inputs are units or outputs
    of the level below);
  * fold items tile their level: the sets of a chunk at one level are each folded exactly once,
    32 at a time counted back from the end, so only a chunk's first item may be short;
  * the final step of a chunk reads the 1 .. 32 sets the last level left, which lie
    2^final_power blocks apart, and that power has a table.
"""
import numpy as np
import pytest

import paper_2411_03357_amd as pgcm

KIB, MIB = 1024, 1 << 20
NUM_POWERS = 31   # tables of H^(2^k), k = 0 .. 30


def _check(lens, unit_bytes=0, wave_slots=0):
    s = pgcm.describe_schedule(lens, unit_bytes, wave_slots)
    n = len(lens)
    up = s["unit_power"]
    ub = 1 << up
    if unit_bytes:
        assert 16 << up == unit_bytes
    desc, unit_base = s["desc"], s["unit_base"]
    assert desc.size == n and unit_base.size == n + 1

    # units
    run = 0
    for i, ln in enumerate(lens):
        d = desc[i]
        nblk = (ln + 15) // 16
        nu = (nblk + ub - 1) // ub
        assert int(d["len"]) == ln and int(d["index"]) == i
        assert int(d["nunits"]) == nu and int(d["unit_base"]) == run == int(unit_base[i])
        if nu:
            fb = int(d["first_blocks"])
            assert 1 <= fb <= ub and fb + (nu - 1) * ub == nblk
        run += nu
    assert run == s["nunits"] == int(unit_base[n])
    # every unit in exactly one chunk: unit_base is non-decreasing and ends at the total
    assert np.all(np.diff(unit_base.astype(np.int64)) >= 0)

    # coarse map: entry k serves units 16 k .. 16 k + 15; it must name a chunk at or before the
    # chunk of unit 16 k, and be a valid chunk index, so that the forward walk ends
    assert s["ncoarse"] == (s["nunits"] >> 4) + 1 and s["coarse_map"].size == s["ncoarse"]
    owner = np.repeat(np.arange(n), desc["nunits"].astype(np.int64)) if n else np.zeros(0, int)
    for k, c in enumerate(s["coarse_map"]):
        assert 0 <= int(c) < max(n, 1)
        u = 16 * k
        if u < s["nunits"]:
            assert int(c) <= int(owner[u]), (k, int(c), int(owner[u]))
            # the walk from c reaches the owner: unit_base[owner + 1] > u
            assert int(unit_base[int(owner[u]) + 1]) > u

    # fold items
    items = s["fold_items"]
    assert items.size == s["nfold"] == sum(s["fold_count"])
    written = np.zeros(s["nslots"], bool)
    written[:s["nunits"]] = True          # the bulk kernel writes one set per unit
    level_of = np.full(s["nslots"], -1)
    level_of[:s["nunits"]] = 0
    consumed = np.zeros(s["nslots"], int)
    first = 0
    for level in range(4):
        assert s["fold_first"][level] == first
        cnt = s["fold_count"][level]
        for it in items[first:first + cnt]:
            b, c, o = int(it["in_base"]), int(it["in_count"]), int(it["out_slot"])
            assert 1 <= c <= 32 and b + c <= s["nslots"]
            assert written[b:b + c].all(), "reads a set no earlier launch wrote"
            assert (level_of[b:b + c] == level).all(), "mixes levels"
            assert s["nunits"] <= o < s["nslots"] and not written[o], "output slot taken"
            consumed[b:b + c] += 1
        # a level's launch ends before the next level starts: its outputs become readable now
        for it in items[first:first + cnt]:
            written[int(it["out_slot"])] = True
            level_of[int(it["out_slot"])] = level + 1
        first += cnt
    assert written.all(), "a slot is allocated that nothing writes"

    # per chunk: the chain of levels and the final step
    for i, ln in enumerate(lens):
        d = desc[i]
        nu = int(d["nunits"])
        c, levels = nu, 0
        while c > 32:
            c, levels = (c + 31) // 32, levels + 1
        assert int(d["final_count"]) == c
        assert int(d["final_power"]) == up + 5 * levels < NUM_POWERS
        if nu == 0:
            continue
        fb_, fc = int(d["final_base"]), int(d["final_count"])
        assert (level_of[fb_:fb_ + fc] == levels).all()
        consumed[fb_:fb_ + fc] += 1
        # the chunk's own units are folded by items that only the first of may be short
        if levels:
            base = int(d["unit_base"])
            mine = [it for it in items[:s["fold_count"][0]]
                    if base <= int(it["in_base"]) < base + nu]
            assert sum(int(it["in_count"]) for it in mine) == nu
            assert all(int(it["in_count"]) == 32 for it in mine[1:])
            assert int(mine[0]["in_base"]) == base
    # every set is used exactly once: by one fold item, or by its chunk's final step
    assert (consumed == 1).all()
    # the device workspace holds the image, a counter, per-chunk blocks and every slot
    assert s["workspace_bytes"] >= s["image_bytes"] + 1024 * s["nslots"] + 16 * n
    return s


def test_schedule_of_the_configurations():
    import workloads
    for cfg in (1, 2, 3, 4, 5):
        w = workloads.FULL[cfg]()
        s = _check([int(v) for v in w.lens])
        assert s["path"] == (2 if cfg == 1 else 0)
        if cfg != 1:
            assert s["unit_power"] == 10
    assert _check([100] * 7)["path"] == 1
    assert _check([])["nunits"] == 0


def test_schedule_edge_lengths_and_every_unit_size():
    lens = [0, 1, 15, 16, 17, 1023, 1024, 1025, 16383, 16384, 16385, 0, 3 * 16384 + 7,
            32 * 16384, 32 * 16384 + 1, 33 * 16384, 1024 * 16384 + 5, 5 * MIB + 3, 0]
    _check(lens)
    for unit in [KIB << k for k in range(0, 15)]:
        _check(lens, unit_bytes=unit)
    # a forced unit a chunk cannot be cut into is refused, as the batch calls refuse it
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.describe_schedule([(1 << 36) - 32], unit_bytes=1024)
    assert e.value.status == -3
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.describe_schedule([1 << 36])
    assert e.value.status == -3
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.describe_schedule([5], unit_bytes=1000)
    assert e.value.status == -1
    # the longest chunk there is: 2^22 units, four fold levels
    s = _check([(1 << 36) - 32, 5])
    assert s["fold_count"][3] > 0


def test_schedule_of_random_batches():
    rng = np.random.default_rng(20241103)
    for trial in range(60):
        n = int(rng.integers(1, 40))
        kind = trial % 4
        if kind == 0:      # swap-sized chunks that do not fill the chip: the unit shrinks
            lens = rng.integers(0, 600 * KIB, n)
        elif kind == 1:    # log-uniform, ragged
            lens = np.exp(rng.uniform(np.log(1), np.log(40 * MIB), n)).astype(np.int64)
        elif kind == 2:    # many tiny ones among a few large
            lens = np.where(rng.random(n) < 0.8, rng.integers(0, 2000, n),
                            rng.integers(0, 70 * MIB, n))
        else:              # exact multiples and their neighbours
            lens = (rng.integers(0, 70, n) * 16384 + rng.integers(-1, 2, n)).clip(0)
        lens = [int(v) for v in lens]
        forced = 0 if trial % 3 else int(KIB << int(rng.integers(0, 11)))
        _check(lens, unit_bytes=forced)


def test_unit_choice_follows_the_wavefront_slots_of_the_device():
    """a device with fewer compute units (a partition of the chip) holds fewer wavefronts at
    once, and the unit is chosen for what it holds"""
    lens = [4 * MIB]
    assert 16 << _check(lens)["unit_power"] == 1024                        # 4096 slots
    assert 16 << _check(lens, wave_slots=512)["unit_power"] == 8192        # 32 compute units
    assert 16 << _check(lens, wave_slots=16)["unit_power"] == 16384        # one compute unit
    for slots in (16, 512, 2048, 4096):
        s = _check([320 * KIB] * 9 + [7], wave_slots=slots)
        assert s["nunits"] <= slots or s["unit_power"] == 10
