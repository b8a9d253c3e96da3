"""Lays a workloads.Workload out in device memory and runs it through the GPU library's C ABI
(via the Python binding): used by the tests, the smoke check and the benchmark.  No cipher
arithmetic here."""
import numpy as np
import torch

import paper_2411_03357_amd as pgcm


def expand(w):
    """the workload's key on the GPU: the AES-256 entry point for 32-byte keys, the general one
    otherwise"""
    return pgcm.expand_key(w.key) if w.key.size == 32 else pgcm.expand_key_bytes(w.key)


class DeviceBatch:
    """Device-resident inputs and outputs of one workload: packed payload buffer `plain`, packed
    ciphertext buffer `cipher`, packed decrypt output `back`, ivs, aad, tags, ok, and the host
    descriptor arrays the ABI takes."""

    def __init__(self, w, plain: torch.Tensor, device="cuda", iv_entry=None):
        """iv_entry: call the batch entry points that take an IV length (default: exactly when
        the workload's IVs are not 12 bytes long)"""
        assert plain.dtype == torch.uint8 and plain.numel() == w.total_bytes
        self.w = w
        iv_len = int(w.ivs.shape[1])
        use_iv_entry = iv_len != 12 if iv_entry is None else iv_entry
        assert use_iv_entry or iv_len == 12
        self.iv_bytes = iv_len if use_iv_entry else None
        self.device = device
        self.plain = plain
        # bytes between chunks (alignment padding) are zero in all three buffers, so that whole
        # buffers can be compared
        ends = (w.offsets + w.lens).astype(np.int64)
        nxt = np.append(w.offsets[1:].astype(np.int64), w.total_bytes) if w.n else ends
        for i in np.flatnonzero(nxt > ends):
            plain[int(ends[i]):int(nxt[i])] = 0
        self.cipher = torch.zeros_like(plain)
        self.back = torch.zeros_like(plain)
        self.ivs = torch.from_numpy(w.ivs.reshape(-1).copy()).to(device)
        self.tags = torch.zeros(16 * w.n, dtype=torch.uint8, device=device)
        self.ok = torch.full((w.n,), 0x55, dtype=torch.uint8, device=device)
        self.lens = w.lens.astype(np.uint64)
        self.aad_dev = None
        self.aad_ptrs = None
        self.aad_lens = w.aad_lens()
        if w.aad is not None:
            self.aad_dev = torch.from_numpy(np.concatenate([w.aad, np.zeros(1, np.uint8)])).to(device)
            self.aad_ptrs = (np.uint64(self.aad_dev.data_ptr()) + w.aad_off[:-1]).astype(np.uint64)

    def ptrs(self, buf: torch.Tensor) -> np.ndarray:
        return (np.uint64(buf.data_ptr()) + self.w.offsets).astype(np.uint64)

    def encrypt(self, key, src=None, dst=None, stream=None):
        src = self.plain if src is None else src
        dst = self.cipher if dst is None else dst
        pgcm.encrypt_batch(key, self.ivs, self.aad_ptrs, self.aad_lens, self.ptrs(src), self.lens,
                           self.ptrs(dst), self.tags, stream, iv_bytes=self.iv_bytes)

    def decrypt(self, key, src=None, dst=None, tags=None, stream=None):
        src = self.cipher if src is None else src
        dst = self.back if dst is None else dst
        tags = self.tags if tags is None else tags
        pgcm.decrypt_verify_batch(key, self.ivs, self.aad_ptrs, self.aad_lens, self.ptrs(src),
                                  self.lens, self.ptrs(dst), tags, self.ok, stream,
                                  iv_bytes=self.iv_bytes)

    def measure(self, key, steps, direction=0, stream=None) -> float:
        """host milliseconds for `steps` passes over this batch, enqueued by the library's own
        loop: plain -> cipher -> back (direction 0), plain -> cipher (1), cipher -> back (2)"""
        return pgcm.measure_passes(key, self.ivs, self.aad_ptrs, self.aad_lens,
                                   self.ptrs(self.plain), self.lens, self.ptrs(self.cipher),
                                   self.ptrs(self.back), self.tags, self.ok, steps, direction,
                                   stream, self.iv_bytes or 12)

    def chunk_host(self, buf: torch.Tensor, i: int) -> np.ndarray:
        off, ln = int(self.w.offsets[i]), int(self.w.lens[i])
        return buf[off:off + ln].cpu().numpy()


def apply_tampers(w, cipher: torch.Tensor, tags: torch.Tensor):
    """flips the bits listed in w.tampers, in place, on device copies"""
    for t in w.tampers:
        if t.where == "ct":
            pos = int(w.offsets[t.chunk]) + t.bit // 8
            cipher[pos] ^= (1 << (t.bit % 8))
        else:
            pos = 16 * t.chunk + t.bit // 8
            tags[pos] ^= (1 << (t.bit % 8))
