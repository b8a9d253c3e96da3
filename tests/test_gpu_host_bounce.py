"""Ciphertext kept in pinned host memory: encrypt straight into a host bounce buffer, decrypt
straight out of it, so that a swap crosses PCIe once, as ciphertext (the placement the paper's
transport uses, section 6).  Same bit-exact bar as device-resident ciphertext."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_harness import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("which", ["ragged", "kv"])
def test_ciphertext_in_pinned_host_memory(which):
    w = workloads.ragged_small(seed_shift=3) if which == "ragged" else workloads.mini(2)
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    bounce = torch.zeros(w.total_bytes, dtype=torch.uint8, pin_memory=True)
    b.encrypt(key, dst=bounce)
    torch.cuda.synchronize()
    srcs = [w.chunk(host, i) for i in range(w.n)]
    aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=8)
    bn = bounce.numpy()
    for i in range(w.n):
        assert np.array_equal(w.chunk(bn, i), cts[i]), i
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    # tamper on the host side, then decrypt out of the bounce buffer
    victim = 5 if which == "ragged" else 3
    bn[int(w.offsets[victim])] ^= 1
    b.decrypt(key, src=bounce)
    torch.cuda.synchronize()
    ok = b.ok.cpu().numpy()
    assert [int(i) for i in np.flatnonzero(ok == 0)] == [victim]
    back = b.back.cpu().numpy()
    for i in range(w.n):
        expect = np.zeros_like(srcs[i]) if i == victim else srcs[i]
        assert np.array_equal(w.chunk(back, i), expect), i
    key.free()
