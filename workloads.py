"""Seeded synthetic batches shaped like the traffic the paper's systems move.

These inputs stand in for the KV-cache swaps (vLLM), weight offload (FlexGen) and adapter
traffic (PEFT) of the paper's evaluation (section 7.1, "Workloads and metrics"); no model
weights, traces or datasets are used.  This module only draws random inputs and lays them
out; it holds none of the cipher's arithmetic and is the one module that both the CPU
oracle's tests and the GPU library's tests import.

Every chunk is one AES-GCM invocation: its own 96-bit IV, optional AAD, own 128-bit tag.
Chunks live in one packed byte buffer, chunk i at offsets[i] (256-byte aligned).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20241103
ALIGN = 256
MIB = 1 << 20


def iv_sequence(iv0: int, n: int) -> np.ndarray:
    """(n, 12) uint8: IV_i = (iv0 + i) mod 2^96 as a big-endian 96-bit integer.

    The paper's transport starts from an agreed IV and adds one per transfer (section 4.1)."""
    out = np.zeros((n, 12), np.uint8)
    for i in range(n):
        out[i] = np.frombuffer(((iv0 + i) % (1 << 96)).to_bytes(12, "big"), np.uint8)
    return out


@dataclass
class Tamper:
    chunk: int
    where: str   # "ct" or "tag"
    bit: int     # bit index inside that field (bit b of byte b // 8 is 1 << (b % 8))


@dataclass
class Workload:
    name: str
    seed: int
    key: np.ndarray                 # (32,) uint8; (16,) or (24,) after with_cipher
    ivs: np.ndarray                 # (n, 12) uint8; (n, iv_bytes) after with_cipher
    lens: np.ndarray                # (n,) uint64
    offsets: np.ndarray             # (n,) uint64 into the packed payload buffer
    total_bytes: int                # size of the packed buffer
    payload_kind: str               # "u8" | "f16_std1" | "f16_std0.02"
    aad: Optional[np.ndarray] = None       # concatenated AAD bytes, or None for "no AAD at all"
    aad_off: Optional[np.ndarray] = None   # (n + 1,) uint64 offsets into aad
    tampers: List[Tamper] = field(default_factory=list)

    @property
    def n(self) -> int:
        return int(self.lens.size)

    @property
    def payload_bytes(self) -> int:
        return int(self.lens.sum())

    def aad_of(self, i: int) -> bytes:
        if self.aad is None:
            return b""
        return self.aad[int(self.aad_off[i]):int(self.aad_off[i + 1])].tobytes()

    def aad_lens(self) -> Optional[np.ndarray]:
        if self.aad is None:
            return None
        return np.diff(self.aad_off).astype(np.uint32)

    # -- payload ---------------------------------------------------------
    def payload_host(self) -> np.ndarray:
        """the packed buffer as a numpy uint8 array, drawn on the CPU (gaps stay zero)"""
        rng = np.random.default_rng([self.seed, 7])
        buf = np.zeros(self.total_bytes, np.uint8)
        for i in range(self.n):
            ln, off = int(self.lens[i]), int(self.offsets[i])
            if ln == 0:
                continue
            if self.payload_kind == "u8":
                buf[off:off + ln] = rng.integers(0, 256, ln, dtype=np.uint8)
            else:
                std = 1.0 if self.payload_kind == "f16_std1" else 0.02
                vals = (rng.standard_normal((ln + 1) // 2, dtype=np.float32) * std)
                buf[off:off + ln] = vals.astype(np.float16).view(np.uint8)[:ln]
        return buf

    def payload_device(self, device="cuda"):
        """the packed buffer as a torch uint8 tensor drawn on the device with a seeded torch
        generator (values differ from payload_host; read chunks back for a CPU check)"""
        import torch
        g = torch.Generator(device=device)
        g.manual_seed(self.seed * 1000003 + 7)
        if self.payload_kind == "u8":
            # 8 random bytes per int64 draw
            words = (self.total_bytes + 7) // 8
            t = torch.randint(-(1 << 62), 1 << 62, (words,), dtype=torch.int64, device=device,
                              generator=g)
            return t.view(torch.uint8)[:self.total_bytes]
        std = 1.0 if self.payload_kind == "f16_std1" else 0.02
        halves = (self.total_bytes + 1) // 2
        t = torch.empty(halves, dtype=torch.float16, device=device)
        t.normal_(0.0, std, generator=g)
        return t.view(torch.uint8)[:self.total_bytes]

    def chunk(self, buf, i: int):
        off, ln = int(self.offsets[i]), int(self.lens[i])
        return buf[off:off + ln]


def _layout(lens: np.ndarray) -> Tuple[np.ndarray, int]:
    padded = (lens.astype(np.int64) + ALIGN - 1) // ALIGN * ALIGN
    offsets = np.zeros(lens.size, np.uint64)
    if lens.size:
        offsets[1:] = np.cumsum(padded)[:-1].astype(np.uint64)
    return offsets, int(padded.sum()) if lens.size else 0


def _base(cfg: int, seed_shift: int = 0):
    seed = BASE_SEED + cfg + seed_shift
    rng = np.random.default_rng([seed, 1])
    key = rng.integers(0, 256, 32, dtype=np.uint8)
    iv0 = int.from_bytes(rng.integers(0, 256, 12, dtype=np.uint8).tobytes(), "big")
    return seed, rng, key, iv0


def config1(n: int = 64, size: int = 4096) -> Workload:
    """64 chunks x 4096 B, uniform random bytes, counter IVs, no AAD."""
    seed, rng, key, iv0 = _base(1)
    lens = np.full(n, size, np.uint64)
    offsets, total = _layout(lens)
    return Workload("c1_64x4KiB" if (n, size) == (64, 4096) else "c1_%dx%d" % (n, size),
                    seed, key, iv_sequence(iv0, n), lens, offsets, total, "u8")


def config2(n: int = 4096) -> Workload:
    """KV-cache swap shaped like OPT-13B: hidden 5120, 40 layers, fp16, 16-token paged blocks.
    One chunk = K and V of one block of one layer = 2 * 16 * 5120 * 2 B = 327680 B.
    AAD (16 B) = le64(layer) || le64(block id), chunk i -> layer i % 40, block i // 40."""
    seed, rng, key, iv0 = _base(2)
    size = 2 * 16 * 5120 * 2
    lens = np.full(n, size, np.uint64)
    offsets, total = _layout(lens)
    idx = np.arange(n, dtype=np.uint64)
    aad = np.stack([idx % 40, idx // 40], axis=1).astype("<u8").view(np.uint8).reshape(-1).copy()
    aad_off = (np.arange(n + 1, dtype=np.uint64) * 16)
    return Workload("c2_opt13b_kv_%dx320KiB" % n, seed, key, iv_sequence(iv0, n), lens, offsets,
                    total, "f16_std1", aad, aad_off)


def _weights(cfg: int, hidden: int, n: Optional[int], label: str) -> Workload:
    seed, rng, key, iv0 = _base(cfg)
    layer_bytes = 12 * hidden * hidden * 2
    assert layer_bytes % (2 * MIB) == 0
    full = layer_bytes // (2 * MIB)
    n = full if n is None else n
    lens = np.full(n, 2 * MIB, np.uint64)
    offsets, total = _layout(lens)
    return Workload("%s_%dx2MiB" % (label, n), seed, key, iv_sequence(iv0, n), lens, offsets,
                    total, "f16_std0.02")


def config3(n: Optional[int] = None) -> Workload:
    """Weight offload shaped like OPT-66B: one decoder layer, 12 * 9216^2 fp16 parameters
    (2 038 431 744 B) = 972 chunks of 2 MiB, values N(0, 0.02^2), no AAD."""
    return _weights(3, 9216, n, "c3_opt66b_layer")


def config4(n: int = 2000, lo: int = 16 * 1024, hi: int = 8 * MIB) -> Workload:
    """Adapter / mixed traffic: lengths log-uniform in [lo, hi]; 70 % rounded down to a multiple
    of 16 B, 30 % forced off it; AAD length uniform in 0..64 B; uniform random bytes."""
    seed, rng, key, iv0 = _base(4)
    lens = np.floor(np.exp(rng.uniform(np.log(lo), np.log(hi), n))).astype(np.int64)
    ragged = rng.random(n) < 0.30
    tail = rng.integers(1, 16, n)
    lens = lens // 16 * 16
    lens = np.where(ragged, np.minimum(lens + tail, hi - 16 + tail), lens)
    lens = lens.astype(np.uint64)
    offsets, total = _layout(lens)
    alen = rng.integers(0, 65, n)
    aad_off = np.zeros(n + 1, np.uint64)
    aad_off[1:] = np.cumsum(alen)
    aad = rng.integers(0, 256, int(alen.sum()), dtype=np.uint8)
    return Workload("c4_mixed_%d" % n, seed, key, iv_sequence(iv0, n), lens, offsets, total,
                    "u8", aad, aad_off)


def config5(n: Optional[int] = None, frac: float = 0.01) -> Workload:
    """Weight offload shaped like OPT-175B: 12 * 12288^2 fp16 parameters (3 623 878 656 B) =
    1728 chunks of 2 MiB.  round(frac * n) distinct chunks, picked by a seeded permutation, get
    one flipped bit: a seeded coin picks ciphertext or tag, then a uniform bit of that field."""
    w = _weights(5, 12288, n, "c5_opt175b_layer")
    rng = np.random.default_rng([w.seed, 3])
    k = max(1, int(round(frac * w.n))) if w.n else 0
    picks = rng.permutation(w.n)[:k]
    for c in sorted(int(p) for p in picks):
        if rng.random() < 0.5:
            w.tampers.append(Tamper(c, "ct", int(rng.integers(0, 8 * int(w.lens[c])))))
        else:
            w.tampers.append(Tamper(c, "tag", int(rng.integers(0, 128))))
    return w


def ragged_small(seed_shift: int = 0) -> Workload:
    """Edge-case batch: every length class the block structure has (empty, sub-block, exact
    block, block + 1, around the 1 KiB row and 64 KiB segment boundaries), AAD lengths
    0, 1, 15, 16, 17, 64 and some larger."""
    seed, rng, key, iv0 = _base(9, seed_shift)
    lens = [0, 1, 15, 16, 17, 31, 32, 33, 1008, 1023, 1024, 1025, 1040, 4095, 4096, 4097,
            65519, 65535, 65536, 65537, 65552, 66560, 131071, 131072, 131073, 196608 + 5,
            3 * 65536 + 1024 + 16, 1, 0, 16]
    alens = [0, 1, 15, 16, 17, 64, 0, 33, 48, 5, 0, 16, 100, 0, 7, 64, 0, 1, 2, 3, 255, 0, 16,
             32, 0, 0, 9, 0, 13, 0]
    assert len(lens) == len(alens)
    lens = np.array(lens, np.uint64)
    offsets, total = _layout(lens)
    aad_off = np.zeros(len(alens) + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    aad = rng.integers(0, 256, int(sum(alens)), dtype=np.uint8)
    return Workload("ragged_small", seed, key, iv_sequence(iv0, lens.size), lens, offsets, total,
                    "u8", aad, aad_off)


def with_cipher(w: Workload, key_bytes: int, iv_bytes: int) -> Workload:
    """the same batch under another key length (16, 24, 32 bytes) and IV length: a fresh random
    key and n distinct random IVs of iv_bytes bytes each (the paper's transport uses 32 and 12;
    other users of AES-GCM do not)"""
    import dataclasses
    rng = np.random.default_rng([w.seed, 11, key_bytes, iv_bytes])
    key = rng.integers(0, 256, key_bytes, dtype=np.uint8)
    ivs = rng.integers(0, 256, (w.n, iv_bytes), dtype=np.uint8)
    # distinct even when iv_bytes is tiny: the chunk index is written into the leading bytes
    for i in range(w.n):
        tagged = i.to_bytes(4, "big")[-min(4, iv_bytes):]
        ivs[i, :len(tagged)] = np.frombuffer(tagged, np.uint8)
    return dataclasses.replace(w, name="%s_k%d_iv%d" % (w.name, key_bytes, iv_bytes), key=key,
                               ivs=ivs)


FULL = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def mini(cfg: int) -> Workload:
    """Reduced-count versions of the five configurations (same chunk shapes, fewer chunks) that
    the CPU oracle finishes in seconds."""
    if cfg == 1:
        return config1()
    if cfg == 2:
        return config2(n=12)
    if cfg == 3:
        return config3(n=3)
    if cfg == 4:
        return config4(n=24, lo=16 * 1024, hi=1 * MIB)
    if cfg == 5:
        return config5(n=4, frac=0.5)
    raise ValueError(cfg)


# ---------------------------------------------------------------------------------------------
# Swap traces for the speculative-pipeline state machine: lists of events
#   ("out", chunk) | ("req", chunk) | ("write", chunk) | ("sync",)   with chunk = (address, bytes).
# They imitate the swapping patterns the paper names (section 5.1): repetitive weight offloading,
# FIFO layer-wise and LIFO request-wise KV-cache swapping, with small transfers in between.

def swap_trace(kind: str, seed: int = 0, rounds: int = 6, noise: float = 0.0):
    rng = np.random.default_rng([BASE_SEED, 77, seed])
    ev = []
    small = lambda: ("req", (0x7000_0000 + int(rng.integers(0, 1 << 20)) * 64,
                             int(rng.integers(1, 8192))))
    if kind == "repetitive":
        # FlexGen-like: the same offloaded layers come back in the same order every iteration
        layers = [(0x1000_0000 + i * (4 << 20), 2 << 20) for i in sorted(
            rng.choice(24, size=int(rng.integers(3, 9)), replace=False))]
        for _ in range(rounds):
            for i in range(0, len(layers), 2):
                for c in layers[i:i + 2]:
                    ev.append(("req", c))
                    if rng.random() < noise:
                        ev.append(small())
                ev.append(("sync",))
    elif kind in ("fifo", "lifo"):
        # vLLM-like: KV blocks leave in some order and return in the same (FIFO) or the
        # reverse (LIFO) order
        nxt = 0
        for _ in range(rounds):
            n = int(rng.integers(2, 7))
            blocks = [(0x2000_0000 + (nxt + i) * 327680, 327680) for i in range(n)]
            nxt += n
            for c in blocks:
                ev.append(("out", c))
            ev.append(("sync",))
            back = blocks if kind == "fifo" else blocks[::-1]
            for c in back:
                ev.append(("req", c))
                if rng.random() < noise:
                    ev.append(small())
            ev.append(("sync",))
    elif kind == "chaos":
        # nothing predictable: random chunks, repeats inside a batch, writes, stray syncs
        pool = [(0x3000_0000 + i * (1 << 20), int(rng.choice([1 << 19, 1 << 20, 200_000])))
                for i in range(10)]
        for _ in range(rounds * 8):
            r = rng.random()
            c = pool[int(rng.integers(0, len(pool)))]
            if r < 0.45:
                ev.append(("req", c))
            elif r < 0.65:
                ev.append(("out", c))
            elif r < 0.75:
                ev.append(("write", (c[0] + int(rng.integers(0, c[1])), int(rng.integers(1, 4096)))))
            elif r < 0.85:
                ev.append(small())
            else:
                ev.append(("sync",))
        ev.append(("sync",))
    else:
        raise ValueError(kind)
    return ev


def small_transfers(seed_shift: int = 0) -> Workload:
    """Only short chunks (at most 8 KiB: the paper's non-swap traffic and its 1-byte NOPs), every
    length class of the block and row structure, AAD of assorted lengths."""
    seed, rng, key, iv0 = _base(8, seed_shift)
    lens = [1, 0, 15, 16, 17, 32, 33, 100, 1007, 1008, 1009, 1023, 1024, 1025, 1039, 1040, 1041,
            2048, 2049, 4095, 4096, 4097, 5000, 8175, 8176, 8177, 8191, 8192, 7, 64]
    alens = [0, 3, 0, 16, 17, 0, 64, 1, 0, 15, 0, 31, 0, 32, 0, 48, 0, 5, 200, 0, 16, 0, 9, 0, 0, 2,
             0, 20, 0, 0]
    assert len(lens) == len(alens)
    lens = np.array(lens, np.uint64)
    offsets, total = _layout(lens)
    aad_off = np.zeros(len(alens) + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    aad = rng.integers(0, 256, int(sum(alens)), dtype=np.uint8)
    return Workload("small_transfers", seed, key, iv_sequence(iv0, lens.size), lens, offsets,
                    total, "u8", aad, aad_off)
