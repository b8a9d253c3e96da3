#!/usr/bin/env python3
"""Throughput of batched AES-256-GCM (encrypt, then decrypt-verify) on one MI355X.

A step is one pass of the whole path over one batch: pgcm_encrypt_batch followed by
pgcm_decrypt_verify_batch of the same chunks, payload resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz, one 32-bit op per lane-clock
LDS_PEAK_GCYCLES = 256 * 2.4               # 256 CUs, one LDS pipe each, 2.4 GHz: port cycles per ns

# Hardware counters of one bulk_kernel launch on the default workload, taken with
# `rocprofv3 --pmc` (summaries and commands: profiles/).  They describe the kernel sources whose
# hash is given; once the sources change they no longer apply and bench.py reports null.
COUNTERS = {
    "sources_sha256": "fe8984312c3d91b1d28d5afbb62eab3deef9dce2e15b2a13524384063f83da38",
    "workload": "c2_opt13b_kv_4096x320KiB",
    "fetch_size_kib": 657226.9,     # FETCH_SIZE per launch
    "fetch_scale": 1310720.0 / 655383.3,   # a 1 310 720 KiB device copy reads 655 383
    "write_size_kib": 1395322.2,    # WRITE_SIZE per launch
    "write_scale": 1310720.0 / 1310720.0,  # the same copy writes 1 310 720.0
    "valu_wave_instructions": 609253376.0,  # SQ_INSTS_VALU per launch
    "lds_wave_instructions": 321931264.0,   # SQ_INSTS_LDS per launch
    "lds_active_cycles": 728154112.0,   # SQ_LDS_IDX_ACTIVE per launch, summed over the 256 CUs
}


def sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for f in ("pgcm_types.h", "pgcm_kernels.h", "pgcm_kernels.hip", "pgcm_host.hip"):
        with open(os.path.join(ROOT, "paper_2411_03357_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def libcrypto_rates(w, seconds=1.0):
    """the host's libcrypto (AES-NI / carry-less multiply), one GCM invocation per 8 MiB: what a
    CPU-side transport like the paper's gets per core and with every core, for context"""
    import threading
    import numpy as np
    import openssl_ref
    size = 8 << 20
    key, iv = w.key.tobytes(), w.ivs[0].tobytes()

    def worker(rates, k):
        data = np.random.default_rng(6 + k).integers(0, 256, size, dtype=np.uint8)
        out = np.empty(size, np.uint8)
        n, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            st = openssl_ref.GcmEncryptStream(key, iv)
            st.update(data, out)             # the foreign call runs without the interpreter lock
            st.tag()
            n += 1
        rates[k] = n * size / (time.perf_counter() - t0) / 1e9

    one = [0.0]
    worker(one, 0)
    threads = min(16, os.cpu_count() or 1)
    rates = [0.0] * threads
    ts = [threading.Thread(target=worker, args=(rates, k)) for k in range(threads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    return {"kind": "libcrypto EVP aes-%d-gcm, encrypt, 8 MiB per invocation" % (8 * len(key)),
            "single_thread_GBps": round(one[0], 2), "all_threads_GBps": round(sum(rates), 2),
            "threads": threads}


def cpu_baseline(w, chunks, threads):
    """the oracle as it stands, timed on this host's cores over a bounded sample of the batch"""
    import numpy as np
    import oracle
    idx = list(range(min(chunks, w.n)))
    sub_lens = [int(w.lens[i]) for i in idx]
    rng = np.random.default_rng(5)
    srcs = [rng.integers(0, 256, ln, dtype=np.uint8) for ln in sub_lens]
    aads = None if w.aad is None else [np.frombuffer(w.aad_of(i), np.uint8) for i in idx]
    t0 = time.perf_counter()
    cts, tags, used = oracle.encrypt_batch(w.key, w.ivs[idx], aads, srcs, nthreads=threads)
    pts, ok, used2 = oracle.decrypt_verify_batch(w.key, w.ivs[idx], aads, cts, tags, threads)
    dt = time.perf_counter() - t0
    assert bool((ok == 1).all())
    nbytes = 2 * sum(sub_lens)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": int(max(used, used2)),
            "kind": "oracle", "nproc": os.cpu_count(), "cpu_model": cpu_model(),
            "sample": "encrypt + decrypt-verify of the first %d chunks (%d B each way) of the same "
                      "batch shape, %.1f s" % (len(idx), sum(sub_lens), dt)}


def pipeline_bench(args):
    """--pipeline: what the speculative pipeline takes off the critical path.  Synthetic swap
    traces (weight offloading, FIFO and LIFO KV swapping) are fed to the library's pipe object
    twice: speculating, and with speculation off (every transfer encrypted when asked for).  For
    every swap the GPU time between the call that put it on the wire and its ciphertext being
    complete is measured with events on the launch stream.  Prints ONE JSON line."""
    import numpy as np
    import torch

    import workloads
    import paper_2411_03357_amd as pgcm

    torch.cuda.set_device(0)
    rng = np.random.default_rng(workloads.BASE_SEED + 500)
    keyb = rng.integers(0, 256, 32, dtype=np.uint8)
    iv0 = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    key = pgcm.expand_key(keyb)
    threshold = 128 * 1024
    out = {}
    for kind in ("repetitive", "fifo", "lifo"):
        ev = workloads.swap_trace(kind, seed=11, rounds=args.steps, noise=0.0)
        chunks = sorted({e[1] for e in ev if e[0] in ("req", "out")})
        g = torch.Generator(device="cuda")
        g.manual_seed(12)
        mem = {c: torch.randint(0, 256, (c[1],), dtype=torch.uint8, device="cuda", generator=g)
               for c in chunks}
        longest = max(c[1] for c in chunks)
        res = {}
        for mode in ("speculative", "on_demand"):
            made = []            # (kind, length, event at the start of the call, event at delivery)
            call_start = [None]

            def deliver(k, addr, length, iv, ct, tag, stream):
                done = torch.cuda.Event(enable_timing=True)
                done.record()
                made.append((k, length, call_start[0], done))

            pipe = pgcm.Pipe(key, iv0, deliver, depth=4, max_chunk_bytes=longest,
                             swap_threshold=threshold if mode == "speculative" else 1 << 62)
            for rep in range(2):                         # the first pass warms up
                made.clear()
                for e in ev:
                    call_start[0] = torch.cuda.Event(enable_timing=True)
                    call_start[0].record()
                    if e[0] == "out":
                        pipe.swap_out(mem[e[1]].data_ptr(), e[1][1])
                    elif e[0] == "req":
                        pipe.request(mem[e[1]].data_ptr(), e[1][1])
                    else:
                        pipe.sync()
                torch.cuda.synchronize()
            swaps = [(k, ln, a.elapsed_time(b) * 1e3) for k, ln, a, b in made
                     if k != "nop" and ln >= threshold]
            st = pipe.stats()
            res[mode] = {"swaps": len(swaps),
                         "critical_us_per_swap": round(sum(t for _, _, t in swaps) / len(swaps), 2),
                         "served_ahead": round(sum(1 for k, _, _ in swaps if k == "send") /
                                               len(swaps), 3),
                         "nops": sum(1 for k, _, _, _ in made if k == "nop"),
                         "pre_bytes_dropped_share": round(
                             st["dropped_bytes"] / st["pre_bytes"], 3) if st["pre_bytes"] else 0.0}
            pipe.destroy()
        out[kind] = res
    key.free()
    spec = sum(out[k]["speculative"]["critical_us_per_swap"] for k in out) / len(out)
    base = sum(out[k]["on_demand"]["critical_us_per_swap"] for k in out) / len(out)
    print(json.dumps({
        "metric": "GPU time on the critical path per swap (call to ciphertext complete), us",
        "value": round(spec, 2), "unit": "us", "higher_is_better": False, "n_gpus": 1,
        "on_demand_value": round(base, 2), "data": "synthetic",
        "config": {"workload": "swap traces: repetitive 2 MiB layers, FIFO and LIFO 320 KiB KV "
                               "blocks, %d rounds each, depth 4" % args.steps},
        "traces": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--key-bytes", type=int, default=32, choices=[16, 24, 32],
                    help="AES key length; the headline (and the paper's transport) is 32")
    ap.add_argument("--iv-bytes", type=int, default=12,
                    help="IV length; the headline (and the paper's transport) is 12")
    ap.add_argument("--unit-bytes", type=int, default=0,
                    help="force the scheduler's unit size (1024 .. 16384); 0: its own choice")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-chunks", type=int, default=0)
    ap.add_argument("--host-bounce", action="store_true",
                    help="keep the ciphertext in pinned host memory (encrypt into / decrypt out of "
                         "a host bounce buffer over PCIe); not the headline configuration")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the payload buffer (a kernel of known "
                         "traffic to scale hardware byte counters by)")
    ap.add_argument("--pipeline", action="store_true",
                    help="measure the speculative pipeline on swap traces instead (its own JSON "
                         "line; --steps is the number of rounds per trace)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this benchmark measures one GPU only (chunks are independent; a multi-GPU "
              "run would just split the chunk list); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.pipeline:
        pipeline_bench(args)
        return

    import numpy as np
    import torch

    import workloads
    import paper_2411_03357_amd as pgcm
    from gpu_harness import DeviceBatch

    torch.cuda.set_device(0)
    w = workloads.FULL[args.config]()
    headline_cipher = args.key_bytes == 32 and args.iv_bytes == 12
    if not headline_cipher:
        w = workloads.with_cipher(w, args.key_bytes, args.iv_bytes)
    key = pgcm.expand_key(w.key) if args.key_bytes == 32 else pgcm.expand_key_bytes(w.key)
    pgcm.set_unit_bytes(key, args.unit_bytes)
    b = DeviceBatch(w, w.payload_device())
    if args.host_bounce:
        b.cipher = torch.zeros(w.total_bytes, dtype=torch.uint8, pin_memory=True)
    payload = w.payload_bytes
    stream = torch.cuda.current_stream()

    def step():
        b.encrypt(key)
        b.decrypt(key)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        scratch = torch.empty_like(b.plain)
        scratch.copy_(b.plain)          # reads and writes w.total_bytes each
        torch.cuda.synchronize()
        del scratch

    # whole-path timing: host clock around K steps, synchronised on both sides.  Inside the timed
    # region the library also records a pair of HIP events around every bulk kernel, on the
    # stream it launches on (no host wait in between); they are read after the region.
    pgcm.set_timing(key, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = 2.0 * payload * args.steps / dt / 1e9
    launches = pgcm.bulk_kernel_ms_history(key, 2 * args.steps)
    pgcm.set_timing(key, False)
    assert len(launches) == min(2 * args.steps, 256) and len(launches) % 2 == 0
    kern = {"enc": launches[0::2], "dec": launches[1::2]}      # a step is encrypt, then decrypt
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain), "round trip failed"

    # per-direction whole-call timing with events on the launch stream; every series starts
    # with untimed calls, because the checks in between leave the GPU idle long enough for its
    # clocks to drop (the first ten launches after 100 ms of idling run up to 20 % slower)
    def timed_calls(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(reps)]
        for _ in range(min(args.warmup, 12)):
            fn(key)
        for s, e in ev:
            s.record(stream)
            fn(key)
            e.record(stream)
        torch.cuda.synchronize()
        return sorted(s.elapsed_time(e) for s, e in ev)

    reps = max(5, min(args.steps, 20))
    enc_ms = timed_calls(b.encrypt, reps)
    dec_ms = timed_calls(b.decrypt, reps)

    # what a plain device copy of the same buffer reaches on this machine, in the same run: the
    # achievable ceiling for a kernel that reads and writes every payload byte once
    copy_ms = None
    if not args.host_bounce:
        copy_ms = timed_calls(lambda _key: b.back.copy_(b.plain), reps)
        b.decrypt(key)                       # b.back holds the decrypted batch again
        torch.cuda.synchronize()

    kern_avg_ms = sum(launches) / len(launches)
    # algorithmic HBM bytes of one launch: every payload byte read once and written once, plus
    # per chunk its IV (12), tag (16), AAD and descriptor (64); what the implementation moves on
    # top of that (1 KiB of partial hash sums per 16 KiB unit) is overhead, not counted here
    aad_total = 0 if w.aad is None else int(w.aad.size)
    algo_bytes = 2 * payload + w.n * (args.iv_bytes + 16 + 64) + aad_total
    achieved = algo_bytes / (kern_avg_ms * 1e-3) / 1e9
    traffic = None
    alu = None
    lds = None
    if (COUNTERS["workload"] == w.name and COUNTERS["sources_sha256"] == sources_sha256()
            and not args.host_bounce and args.unit_bytes == 0):
        traffic = int(1024 * (COUNTERS["fetch_size_kib"] * COUNTERS["fetch_scale"] +
                              COUNTERS["write_size_kib"] * COUNTERS["write_scale"]))
        lane_ops = COUNTERS["valu_wave_instructions"] * 64
        alu_achieved = lane_ops / (kern_avg_ms * 1e-3) / 1e12
        alu = {"bound": "alu", "achieved": round(alu_achieved, 2), "peak": round(VALU_PEAK_TOPS, 2),
               "unit": "T 32-bit lane-ops/s", "frac": round(alu_achieved / VALU_PEAK_TOPS, 4),
               "valu_ops_per_payload_byte": round(lane_ops / payload, 2),
               "lds_lookups_per_payload_byte": round(COUNTERS["lds_wave_instructions"] * 64 / payload, 2)}
        # the resource that binds: cycles in which a CU's LDS pipe is serving lookups (a 64-lane
        # ds_read_b32 holds it for 2 cycles, a ds_read_b128 for 4), against one pipe per CU at
        # the nominal clock
        lds_achieved = COUNTERS["lds_active_cycles"] / (kern_avg_ms * 1e-3) / 1e9
        lds = {"bound": "lds", "achieved": round(lds_achieved, 1), "peak": round(LDS_PEAK_GCYCLES, 1),
               "unit": "G LDS-pipe cycles/s", "frac": round(lds_achieved / LDS_PEAK_GCYCLES, 4),
               "lds_cycles_per_payload_byte": round(COUNTERS["lds_active_cycles"] / payload, 4)}

    # the launch the library's events bracket (the kernel that touches the payload)
    longest = int(w.lens.max())
    if longest <= 1008:
        timed_kernel = "small_kernel (one wavefront per chunk: the whole invocation)"
    elif longest <= 8192 and w.n <= 512:
        timed_kernel = "small_wide_kernel (one workgroup per chunk: the whole invocation)"
    else:
        timed_kernel = "bulk_kernel (CTR keystream + XOR + GHASH)"
    out = {
        "metric": "AES-%d-GCM enc / dec+verify GB/s on 1 MI355X; %% of HBM roofline"
                  % (8 * args.key_bytes),
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": w.name, "chunks": w.n, "payload_bytes": payload,
                   "step": "encrypt batch + decrypt-verify batch", "unit_bytes": args.unit_bytes or pgcm.batch_unit_bytes(w.lens),
                   "key_bytes": args.key_bytes, "iv_bytes": args.iv_bytes,
                   "ciphertext": "pinned host memory" if args.host_bounce else "device memory"},
        "enc_GBps": round(payload / (enc_ms[len(enc_ms) // 2] * 1e-3) / 1e9, 2),
        "dec_verify_GBps": round(payload / (dec_ms[len(dec_ms) // 2] * 1e-3) / 1e9, 2),
        "pct_hbm_roofline": round(100.0 * 2.0 * value / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": timed_kernel,
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes": algo_bytes,
                     "avg_launch_ms": round(kern_avg_ms, 4),
                     "launches_timed": len(launches),
                     "min_launch_ms": round(min(launches), 4),
                     "median_launch_ms": round(sorted(launches)[len(launches) // 2], 4),
                     "max_launch_ms": round(max(launches), 4),
                     "enc_launch_ms": round(sum(kern["enc"]) / len(kern["enc"]), 4),
                     "dec_launch_ms": round(sum(kern["dec"]) / len(kern["dec"]), 4)},
    }
    out["roofline_alu"] = alu
    out["roofline_lds"] = lds
    if copy_ms is not None:
        copy_gbs = 2.0 * w.total_bytes / (copy_ms[len(copy_ms) // 2] * 1e-3) / 1e9
        out["copy_ceiling"] = {"kind": "device-to-device copy of the payload buffer (HBM read + "
                                       "write), median of %d" % reps,
                               "traffic_GBps": round(copy_gbs, 1),
                               "bulk_kernel_frac_of_copy": round(achieved / copy_gbs, 4)}
    import hashlib
    h = hashlib.sha256()
    for arr in (w.key, w.ivs, w.lens, w.aad if w.aad is not None else np.zeros(0, np.uint8)):
        h.update(np.ascontiguousarray(arr).tobytes())
    out["inputs_sha256"] = h.hexdigest()    # key, IVs, lengths, AAD (the payload is seeded too)
    if not args.no_cpu_baseline:
        chunks = args.cpu_chunks or max(1, int(40e6 // max(1, int(w.lens.mean()))))
        threads = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(w, chunks, threads)
        out["cpu_libcrypto"] = libcrypto_rates(w)
    key.free()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
