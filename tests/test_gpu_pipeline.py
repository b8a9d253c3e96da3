"""The speculative pipeline end to end on the GPU: the state machine decides, the batch calls
encrypt, and a receiver that does nothing but count transfers (IV = IV_0 + k, as in the paper's
transport, section 4.1) must accept every delivery and recover every byte."""
import numpy as np
import pytest
import torch

import oracle
import workloads

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


class Sender:
    """carries out the actions of a pgcm.Sequencer with pgcm_encrypt_batch"""

    def __init__(self, key, iv0, seq, memory):
        self.key, self.iv0, self.seq, self.memory = key, iv0, seq, memory
        self.kept = {}      # chunk -> (ciphertext tensor, tag tensor, iv number)
        self.wire = []      # deliveries in order: (chunk or None for a NOP, ciphertext, tag)
        self.nop = torch.zeros(16, dtype=torch.uint8, device="cuda")
        self.bytes_ahead = self.bytes_critical = 0

    def _encrypt(self, items):
        """items: list of (plaintext tensor, iv number) -> list of (ciphertext, tag)"""
        n = len(items)
        ivs = torch.from_numpy(np.frombuffer(
            b"".join(pgcm.seq_iv_bytes(self.iv0, iv) for _, iv in items), np.uint8).copy()).cuda()
        cts = [torch.empty(max(16, (p.numel() + 15) // 16 * 16), dtype=torch.uint8, device="cuda")
               for p, _ in items]
        tags = torch.zeros(16 * n, dtype=torch.uint8, device="cuda")
        pgcm.encrypt_batch(self.key, ivs, None, None, [p.data_ptr() for p, _ in items],
                           [p.numel() for p, _ in items], [c.data_ptr() for c in cts], tags)
        return [(cts[i][:items[i][0].numel()], tags[16 * i:16 * i + 16]) for i in range(n)]

    def run(self):
        # actions are carried out strictly in the order the state machine issued them
        for a in self.seq.take_actions():
            if a[0] == "pre":
                (ct, tag), = self._encrypt([(self.memory[a[1]], a[2])])
                self.kept[a[1]] = (ct, tag, a[2])
                self.bytes_ahead += a[1][1]
            elif a[0] == "send":
                ct, tag, iv = self.kept.pop(a[1])
                assert iv == a[2]
                self.wire.append((a[1], ct, tag))
            elif a[0] == "now":
                (ct, tag), = self._encrypt([(self.memory[a[1]], a[2])])
                self.wire.append((a[1], ct, tag))
                self.bytes_critical += a[1][1]
            elif a[0] == "nop":
                (ct, tag), = self._encrypt([(self.nop[:1], a[1])])
                self.wire.append((None, ct, tag))
            elif a[0] == "drop":
                self.kept.pop(a[1], None)


def _memory_for(events, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    mem = {}
    for e in events:
        if e[0] in ("req", "out") and e[1] not in mem:
            mem[e[1]] = torch.randint(0, 256, (e[1][1],), dtype=torch.uint8, device="cuda", generator=g)
    return mem


def _receive(key, iv0, iv_start, wire):
    """decrypts delivery k under IV_0 + iv_start + k; returns verdicts and plaintexts"""
    n = len(wire)
    ivs = torch.from_numpy(np.frombuffer(
        b"".join(pgcm.seq_iv_bytes(iv0, iv_start + k) for k in range(n)), np.uint8).copy()).cuda()
    outs = [torch.empty(max(16, (ct.numel() + 15) // 16 * 16), dtype=torch.uint8, device="cuda")
            for _, ct, _ in wire]
    srcs = []
    for _, ct, _ in wire:                      # ciphertext views may be unaligned slices: copy
        buf = torch.empty(max(16, (ct.numel() + 15) // 16 * 16), dtype=torch.uint8, device="cuda")
        buf[:ct.numel()] = ct
        srcs.append(buf)
    tags = torch.cat([t for _, _, t in wire]).contiguous()
    ok = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pgcm.decrypt_verify_batch(key, ivs, None, None, [s.data_ptr() for s in srcs],
                              [ct.numel() for _, ct, _ in wire], [o.data_ptr() for o in outs], tags, ok)
    torch.cuda.synchronize()
    return ok.cpu().numpy(), [outs[k][:wire[k][1].numel()] for k in range(n)]


@pytest.mark.parametrize("kind,noise", [("repetitive", 0.3), ("fifo", 0.2), ("lifo", 0.0)])
def test_receiver_that_only_counts_accepts_every_delivery(kind, noise):
    ev = workloads.swap_trace(kind, seed=3, rounds=5, noise=noise)
    rng = np.random.default_rng(99)
    keyb = rng.integers(0, 256, 32, dtype=np.uint8)
    iv0 = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    key = pgcm.expand_key(keyb)
    mem = _memory_for(ev, 5)
    seq = pgcm.Sequencer(iv_start=41, depth=4, leeway=1 if noise else 0)
    snd = Sender(key, iv0, seq, mem)
    asked = []
    for e in ev:
        if e[0] == "out":
            seq.swap_out(e[1])
        elif e[0] == "req":
            seq.request(e[1])
            asked.append(e[1])
        else:
            seq.sync()
        snd.run()
    torch.cuda.synchronize()
    ok, plain = _receive(key, iv0, 41, snd.wire)
    assert ok.tolist() == [1] * len(snd.wire)
    delivered = [c for c, _, _ in snd.wire if c is not None]
    assert sorted(delivered) == sorted(asked)
    for (c, _, _), p in zip(snd.wire, plain):
        if c is not None:
            assert torch.equal(p, mem[c])
    # one delivery cross-checked against the CPU oracle, IV arithmetic included
    k = next(i for i, (c, _, _) in enumerate(snd.wire) if c is not None and c[1] >= 128 * 1024)
    c, ct, tag = snd.wire[k]
    iv = ((int.from_bytes(iv0, "big") + 41 + k) % (1 << 96)).to_bytes(12, "big")
    oct_, otag = oracle.encrypt(keyb, iv, b"", mem[c].cpu().numpy())
    assert ct.cpu().numpy().tobytes() == oct_ and tag.cpu().numpy().tobytes() == otag
    # on regular traffic most bytes were encrypted ahead of demand
    assert snd.bytes_ahead > 0
    if kind != "lifo":
        assert snd.bytes_critical < 0.5 * (snd.bytes_critical + sum(c[1] for c in delivered))
    key.free()


def test_a_replayed_or_reordered_delivery_is_rejected():
    ev = workloads.swap_trace("repetitive", seed=1, rounds=3)
    rng = np.random.default_rng(7)
    keyb = rng.integers(0, 256, 32, dtype=np.uint8)
    iv0 = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    key = pgcm.expand_key(keyb)
    mem = _memory_for(ev, 6)
    seq = pgcm.Sequencer(iv_start=0, depth=3)
    snd = Sender(key, iv0, seq, mem)
    for e in ev:
        seq.request(e[1]) if e[0] == "req" else seq.sync()
        snd.run()
    wire = list(snd.wire)
    wire[1], wire[2] = wire[2], wire[1]        # two deliveries swap places
    wire[4] = wire[0]                          # an old ciphertext is replayed
    ok, _ = _receive(key, iv0, 0, wire)
    assert ok.tolist()[:5] == [1, 0, 0, 1, 0]
    assert all(v == 1 for v in ok.tolist()[5:])
    key.free()


# ------------------------------------------------------------------------------------------
# the same, driven by the library's own pipe object (include/pgcm_pipe.h) instead of Python

class CountingReceiver:
    """the peer: decrypts delivery k straight out of the sender's buffer under IV_0 + start + k,
    on the stream the delivery was made on"""

    def __init__(self, keyb, iv0, iv_start):
        self.key = pgcm.expand_key(keyb)
        self.rx = pgcm.Receiver(self.key, iv0, iv_start)      # the library's counting peer
        self.got = []       # (kind, addr, length, iv, plaintext tensor, ok tensor)

    def deliver(self, kind, addr, length, iv, ct, tag, stream):
        assert self.rx.next_iv == iv
        out = torch.empty(max(16, (length + 15) // 16 * 16), dtype=torch.uint8, device="cuda")
        ok = torch.zeros(1, dtype=torch.uint8, device="cuda")
        self.rx.accept(ct, length, tag, out, ok, stream=stream)
        self.got.append((kind, addr, length, iv, out[:length], ok, None))


@pytest.mark.parametrize("kind,noise", [("repetitive", 0.3), ("fifo", 0.2), ("lifo", 0.0)])
def test_pipe_object_drives_the_batch_calls(kind, noise):
    ev = workloads.swap_trace(kind, seed=4, rounds=5, noise=noise)
    rng = np.random.default_rng(101)
    keyb = rng.integers(0, 256, 32, dtype=np.uint8)
    iv0 = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    key = pgcm.expand_key(keyb)
    mem = _memory_for(ev, 8)
    longest = max(c[1] for c in mem)
    rx = CountingReceiver(keyb, iv0, 17)
    pipe = pgcm.Pipe(key, iv0, rx.deliver, depth=4, iv_start=17, leeway=1 if noise else 0,
                     max_chunk_bytes=longest)
    # the model runs beside it on the same events: same transfers, same order, same IVs
    from oracle.sequencer_oracle import SequencerOracle
    model = SequencerOracle(iv_start=17, depth=4, leeway=1 if noise else 0)
    asked = []
    for e in ev:
        if e[0] == "out":
            pipe.swap_out(mem[e[1]].data_ptr(), e[1][1])
            model.swap_out((mem[e[1]].data_ptr(), e[1][1]))
        elif e[0] == "req":
            pipe.request(mem[e[1]].data_ptr(), e[1][1])
            model.request((mem[e[1]].data_ptr(), e[1][1]))
            asked.append(e[1])
        else:
            pipe.sync()
            model.sync()
    torch.cuda.synchronize()
    by_addr = {t.data_ptr(): c for c, t in mem.items()}
    wire_model = [a for a in model.log if a[0] in ("send", "now", "nop")]
    assert len(rx.got) == len(wire_model)
    for k, ((kd, addr, length, iv, plain, ok, _), m) in enumerate(zip(rx.got, wire_model)):
        assert int(ok.item()) == 1, k
        assert iv == 17 + k and kd == m[0]
        if kd == "nop":
            assert (addr, length) == (0, 1) and m[1] == iv
        else:
            assert (addr, length) == m[1] and m[2] == iv
            assert torch.equal(plain, mem[by_addr[addr]])
    assert sorted(by_addr[g[1]] for g in rx.got if g[0] != "nop") == sorted(asked)
    st = pipe.stats()
    assert st["transfers"] == len(rx.got) and st["nops"] == sum(1 for g in rx.got if g[0] == "nop")
    assert st["ahead_bytes"] == sum(g[2] for g in rx.got if g[0] == "send")
    assert st["critical_bytes"] == sum(g[2] for g in rx.got if g[0] == "now")
    assert st["pre_bytes"] == sum(a[1][1] for a in model.log if a[0] == "pre")
    assert st["dropped_bytes"] == sum(a[1][1] for a in model.log if a[0] == "drop")
    if kind != "lifo":
        assert st["ahead_bytes"] > st["critical_bytes"]
    # argument checks
    with pytest.raises(pgcm.PgcmError) as e:
        pipe.request(mem[asked[0]].data_ptr(), longest + 1)
    assert e.value.status == -3
    with pytest.raises(pgcm.PgcmError) as e:
        pipe.request(mem[asked[0]].data_ptr() + 4, 64)
    assert e.value.status == -2
    # a delivery offered twice: the second copy meets the next IV and is rejected
    kd, addr, length, iv, plain, ok, _ = rx.got[-1]
    stale = torch.zeros(1, dtype=torch.uint8, device="cuda")
    dup = torch.empty(max(16, (length + 15) // 16 * 16), dtype=torch.uint8, device="cuda")
    src = torch.zeros_like(dup)
    src[:length] = plain            # not even ciphertext: any bytes are refused under a new IV
    rx.rx.accept(src, length, torch.zeros(16, dtype=torch.uint8, device="cuda"), dup, stale)
    torch.cuda.synchronize()
    assert int(stale.item()) == 0 and int(dup[:length].max().item() if length else 0) == 0
    assert rx.rx.next_iv == 17 + len(rx.got) + 1
    pipe.destroy()
    rx.rx.destroy()
    rx.key.free()
    key.free()
