#!/usr/bin/env python3
"""Throughput of batched AES-256-GCM (encrypt, then decrypt-verify) on one MI355X.

A step is one pass of the whole path over one batch: pgcm_encrypt_batch followed by
pgcm_decrypt_verify_batch of the same chunks, payload resident in HBM.  Prints ONE JSON line.

`value` and `roofline` are quoted on the KV-cache swap shape (configuration 2); `configs` holds
the same measurement for all five configurations.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--only] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
# 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz, one 32-bit op per lane-clock: a wavefront instruction
# whose operands are all vector registers occupies its SIMD for two cycles (measured: 1.77 such
# instructions per clock per CU; one with a scalar-register operand takes four).  The same
# count as the published 157.3 TFLOP/s of FP32 vector rate at two flops per lane-clock.
VALU_PEAK_TOPS = 256 * 128 * 2.4e9 / 1e12
LDS_PEAK_GCYCLES = 256 * 2.4               # 256 CUs, one LDS pipe each, 2.4 GHz: port cycles per ns

# Hardware counters of one bulk_kernel launch on the default workload, taken with
# `rocprofv3 --pmc` (summaries and commands: profiles/).  They describe the kernel sources
# (pgcm_kernels.hip and the two headers it includes) whose hash is given; once those change the
# counters no longer apply and bench.py reports null.
COUNTERS = {
    "sources_sha256": "23d93b85df471d2e331f0279dbec7481c4e09c6246208d02277e6dbc7621b70a",
    "workload": "c2_opt13b_kv_4096x320KiB",
    "fetch_size_kib": 657146.8,     # FETCH_SIZE per launch
    "fetch_scale": 1310720.0 / 655383.0,   # a 1 310 720 KiB device copy reads 655 383
    "write_size_kib": 1395456.0,    # WRITE_SIZE per launch
    "write_scale": 1310720.0 / 1310720.0,  # the same copy writes 1 310 720.0
    "valu_wave_instructions": 588482560.0,  # SQ_INSTS_VALU per launch
    "lds_wave_instructions": 321832960.0,   # SQ_INSTS_LDS per launch
    "lds_active_cycles": 728154112.0,   # SQ_LDS_IDX_ACTIVE per launch, summed over the 256 CUs
    "gui_active_cycles": 24682199.5 / 8,  # GRBM_GUI_ACTIVE per launch (summed over the 8 XCDs) ...
    "pmc_launch_ms": 1.5139392,           # ... and the launch's duration in that same run
}


def sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for f in ("pgcm_types.h", "pgcm_kernels.h", "pgcm_kernels.hip"):
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


def bitsliced_bench(args):
    """--bitsliced: the cost of the one alternative to table-driven AES rounds, measured.  The
    bitsliced kernel writes the counter-mode keystream for as many blocks as the KV-cache swap
    shape has (no payload is read, nothing is hashed: the round function alone plus the store);
    the table-driven bulk kernel of the batch calls is timed beside it on that shape, doing the
    whole of AES-GCM.  Prints ONE JSON line."""
    import re
    import torch

    import workloads
    import paper_2411_03357_amd as pgcm
    from device_batch import DeviceBatch

    torch.cuda.set_device(0)
    w = workloads.config2()
    key = pgcm.expand_key(w.key)
    nblocks = w.payload_bytes // 16
    out = torch.empty(16 * nblocks, dtype=torch.uint8, device="cuda")
    iv = w.ivs[0].tobytes()
    for _ in range(3):
        pgcm.bitsliced_keystream(key, iv, 0, nblocks, out)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(max(3, args.steps // 10))]
    for s, e in ev:
        s.record()
        pgcm.bitsliced_keystream(key, iv, 0, nblocks, out)
        e.record()
    torch.cuda.synchronize()
    ms = sorted(s.elapsed_time(e) for s, e in ev)
    bs_ms = ms[len(ms) // 2]
    del out
    # the table-driven kernel on the same number of blocks (whole AES-GCM: keystream, XOR, GHASH)
    b = DeviceBatch(w, w.payload_device())
    b.measure(key, 5, direction=1)
    pgcm.set_timing(key, True)
    b.measure(key, 20, direction=1)
    table_ms = sorted(pgcm.bulk_kernel_ms_history(key, 20))[10]
    pgcm.set_timing(key, False)
    key.free()
    gen = open(os.path.join(ROOT, "paper_2411_03357_amd", "csrc", "pgcm_bitsliced_gen.h")).read()
    sbox = int(re.search(r"kSboxInstructions = (\d+)", gen).group(1))
    mix = int(re.search(r"kMixColumnInstructions = (\d+)", gen).group(1))
    per_round = 16 * sbox + 4 * mix                   # wavefront instructions per 2048 blocks
    print(json.dumps({
        "metric": "bitsliced AES-256 counter-mode keystream on 1 MI355X, GB/s (measurement of the "
                  "alternative round function; not the batch path)",
        "value": round(16 * nblocks / (bs_ms * 1e-3) / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
        "higher_is_better": True, "data": "synthetic", "dtype": "u32 bit planes",
        "config": {"workload": "%d counter blocks (the block count of %s), keystream only"
                               % (nblocks, w.name)},
        "bitsliced_kernel_ms": round(bs_ms, 4),
        "table_driven_bulk_kernel_ms": round(table_ms, 4),
        "table_driven_GBps_whole_gcm": round(w.payload_bytes / (table_ms * 1e-3) / 1e9, 2),
        "sbox_instructions": sbox, "mixcolumn_addkey_instructions_per_column": mix,
        "valu_instructions_per_round_per_64_blocks": round(per_round / 32.0, 2),
        "note": "dynamic instruction counts (SQ_INSTS_VALU) are in profiles/"}))


def latency_bench(args):
    """--latency: time of ONE call on batches that do not fill the chip (the paper's swaps come a
    few chunks at a time, section 5.1): encrypt calls and encrypt + decrypt-verify passes enqueued
    back to back by the library's own loop, microseconds per call.  Prints ONE JSON line."""
    import numpy as np
    import torch

    import workloads
    import paper_2411_03357_amd as pgcm
    from device_batch import DeviceBatch

    torch.cuda.set_device(0)
    kib, mib = 1024, 1 << 20
    cases = [("1 x 1 B", [1]), ("1 x 4 KiB", [4096]), ("64 x 4 KiB", [4096] * 64),
             ("1 x 320 KiB", [320 * kib]), ("16 x 320 KiB", [320 * kib] * 16),
             ("1 x 2 MiB", [2 * mib]), ("4 x 2 MiB", [2 * mib] * 4), ("1 x 8 MiB", [8 * mib]),
             ("256 x 320 KiB", [320 * kib] * 256), ("1 x 64 MiB", [64 * mib])]
    reps = max(50, args.steps * 3)
    out = {}
    for name, lens in cases:
        rng = np.random.default_rng(1)
        lens = np.array(lens, np.uint64)
        off, total = workloads._layout(lens)
        w = workloads.Workload("latency", 1, rng.integers(0, 256, 32, dtype=np.uint8),
                               workloads.iv_sequence(5, lens.size), lens, off, total, "u8")
        key = pgcm.expand_key(w.key)
        b = DeviceBatch(w, w.payload_device())
        row = {}
        for label, one_launch in (("us_per_encrypt_call", True), ("several_kernels", False)):
            pgcm.set_one_launch(key, one_launch)
            b.measure(key, 50, direction=1)
            row[label] = round(min(b.measure(key, reps, direction=1) for _ in range(3)) /
                               reps * 1e3, 2)
        pgcm.set_one_launch(key, True)
        b.measure(key, 20)
        row["us_per_pass"] = round(b.measure(key, reps) / reps * 1e3, 2)
        row["GBps_encrypt"] = round(w.payload_bytes / row["us_per_encrypt_call"] / 1e3, 1)
        out[name] = row
        key.free()
    print(json.dumps({
        "metric": "time of one encrypt call on a batch that does not fill the chip, us "
                  "(back to back on one stream)",
        "value": out["1 x 320 KiB"]["us_per_encrypt_call"], "unit": "us",
        "higher_is_better": False, "n_gpus": 1, "data": "synthetic", "dtype": "u8",
        "config": {"workload": "1 x 320 KiB (one KV-cache block of the OPT-13B shape); the other "
                               "batches in `batches`", "calls_timed": reps},
        "batches": out}))


def measure_workload(pgcm, torch, w, args, steps, warmup, headline):
    """One workload through the library's own timing loop.  Returns (results dict, batch, key);
    the caller frees them.  steps passes (encrypt + decrypt-verify) are timed by the host clock,
    synchronised on both sides, with a pair of events around every bulk kernel; then each
    direction alone."""
    import numpy as np
    from device_batch import DeviceBatch, apply_tampers

    key = pgcm.expand_key(w.key) if w.key.size == 32 else pgcm.expand_key_bytes(w.key)
    pgcm.set_unit_bytes(key, args.unit_bytes)
    if args.matrix_hash:
        pgcm.set_matrix_hash(key, True)
    b = DeviceBatch(w, w.payload_device())
    if args.host_bounce:
        b.cipher = torch.zeros(w.total_bytes, dtype=torch.uint8, pin_memory=True)
    payload = w.payload_bytes
    pgcm.reserve(key, w.n, payload, torch.cuda.current_stream())
    b.measure(key, warmup)
    if headline and args.calibrate_copy:
        scratch = torch.empty_like(b.plain)
        scratch.copy_(b.plain)          # reads and writes w.total_bytes each
        torch.cuda.synchronize()
        del scratch

    pgcm.set_timing(key, True)
    ms = b.measure(key, steps)
    launches = pgcm.bulk_kernel_ms_history(key, 2 * steps)
    pgcm.set_timing(key, False)
    assert len(launches) == min(2 * steps, 256) and len(launches) % 2 == 0
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain), "round trip failed"
    # the same passes without the event pairs: the events' hand-overs cost the GPU a few
    # microseconds per call, which is nothing to a batch that fills the chip and a third of a
    # pass of the small-transfer path
    plain_steps = max(5, min(steps, 20))
    b.measure(key, min(warmup, 12))     # the checks above let the clocks drop
    ms_plain = b.measure(key, plain_steps) / plain_steps

    # each direction alone, again by the library's loop; a series starts with untimed passes
    # because the checks in between leave the GPU idle long enough for its clocks to drop.
    # Decrypt-verify runs on the workload's own ciphertext: with its tampering where it has any
    # (the rejected chunks are wiped inside the timed calls)
    reps = max(5, min(steps, 20))
    b.measure(key, min(warmup, 12), direction=1)
    enc_ms = b.measure(key, reps, direction=1) / reps
    rejected = sorted({t.chunk for t in w.tampers})
    if rejected:
        apply_tampers(w, b.cipher, b.tags)
    b.measure(key, min(warmup, 12), direction=2)
    dec_ms = b.measure(key, reps, direction=2) / reps
    if rejected:
        ok = b.ok.cpu().numpy()
        assert sorted(np.flatnonzero(ok == 0).tolist()) == rejected, "verdicts"

    kern_avg_ms = sum(launches) / len(launches)
    # algorithmic HBM bytes of one launch: every payload byte read once and written once, plus
    # per chunk its IV, tag (16), AAD and descriptor (64); what the implementation moves on
    # top of that (1 KiB of partial hash sums per 16 KiB unit) is overhead, not counted here
    aad_total = 0 if w.aad is None else int(w.aad.size)
    algo_bytes = 2 * payload + w.n * (int(w.ivs.shape[1]) + 16 + 64) + aad_total
    achieved = algo_bytes / (kern_avg_ms * 1e-3) / 1e9
    res = {"workload": w.name, "chunks": w.n, "payload_bytes": payload,
           "value": round(2.0 * payload * steps / (ms * 1e-3) / 1e9, 2), "unit": "GB/s",
           "steps": steps, "ms_per_step": round(ms / steps, 4),
           "ms_per_step_without_launch_events": round(ms_plain, 4),
           "value_without_launch_events": round(2.0 * payload / (ms_plain * 1e-3) / 1e9, 2),
           "enc_GBps": round(payload / (enc_ms * 1e-3) / 1e9, 2),
           "dec_verify_GBps": round(payload / (dec_ms * 1e-3) / 1e9, 2),
           "chunks_rejected_in_dec_verify": len(rejected),
           "unit_bytes": args.unit_bytes or pgcm.batch_unit_bytes(w.lens),
           "avg_launch_ms": round(kern_avg_ms, 4),
           "roofline_frac": round(achieved / HBM_PEAK_GBS, 4)}
    detail = {"launches": launches, "algo_bytes": algo_bytes, "achieved": achieved,
              "kern_avg_ms": kern_avg_ms, "reps": reps}
    return res, detail, b, key


def timed_kernel_name(w):
    longest = int(w.lens.max())
    if longest <= 1008:
        return "small_kernel (one wavefront per chunk: the whole invocation)"
    if longest <= 8192 and w.n <= 512:
        return "small_wide_kernel (one workgroup per chunk: the whole invocation)"
    return "bulk_kernel (CTR keystream + XOR + GHASH)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="the workload `value` and `roofline` are quoted on (default: the KV-cache "
                         "swap shape); the other four are measured too, into `configs`")
    ap.add_argument("--only", action="store_true", help="measure --config alone")
    ap.add_argument("--key-bytes", type=int, default=32, choices=[16, 24, 32],
                    help="AES key length; the headline (and the paper's transport) is 32")
    ap.add_argument("--iv-bytes", type=int, default=12,
                    help="IV length; the headline (and the paper's transport) is 12")
    ap.add_argument("--unit-bytes", type=int, default=0,
                    help="force the scheduler's unit size (1024 .. 16384); 0: its own choice")
    ap.add_argument("--matrix-hash", action="store_true",
                    help="GHASH row multiplication on the matrix cores instead of the LDS table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-chunks", type=int, default=0)
    ap.add_argument("--host-bounce", action="store_true",
                    help="keep the ciphertext in pinned host memory (encrypt into / decrypt out of "
                         "a host bounce buffer over PCIe); not the headline configuration")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the payload buffer (a kernel of known "
                         "traffic to scale hardware byte counters by)")
    ap.add_argument("--latency", action="store_true",
                    help="time single calls on small batches instead (its own JSON line)")
    ap.add_argument("--bitsliced", action="store_true",
                    help="measure the bitsliced round function beside the table-driven one "
                         "instead (its own JSON line)")
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
    if args.bitsliced:
        bitsliced_bench(args)
        return
    if args.latency:
        latency_bench(args)
        return

    import numpy as np
    import torch

    import workloads
    import paper_2411_03357_amd as pgcm

    torch.cuda.set_device(0)

    def workload(cfg):
        w = workloads.FULL[cfg]()
        if not (args.key_bytes == 32 and args.iv_bytes == 12):
            w = workloads.with_cipher(w, args.key_bytes, args.iv_bytes)
        return w

    w = workload(args.config)
    res, det, b, key = measure_workload(pgcm, torch, w, args, args.steps, args.warmup, True)
    payload = w.payload_bytes
    launches, achieved, kern_avg_ms = det["launches"], det["achieved"], det["kern_avg_ms"]
    kern = {"enc": launches[0::2], "dec": launches[1::2]}      # a pass is encrypt, then decrypt

    # what a plain device copy of the same buffer reaches on this machine, in the same run: the
    # achievable ceiling for a kernel that reads and writes every payload byte once
    copy_gbs = None
    if not args.host_bounce:
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(det["reps"])]
        for _ in range(5):
            b.back.copy_(b.plain)
        for s, e in ev:
            s.record()
            b.back.copy_(b.plain)
            e.record()
        torch.cuda.synchronize()
        copy_ms = sorted(s.elapsed_time(e) for s, e in ev)
        copy_gbs = 2.0 * w.total_bytes / (copy_ms[len(copy_ms) // 2] * 1e-3) / 1e9

    traffic = None
    alu = None
    lds = None
    if (COUNTERS["workload"] == w.name and COUNTERS["sources_sha256"] == sources_sha256()
            and not args.host_bounce and args.unit_bytes == 0 and not args.matrix_hash):
        traffic = int(1024 * (COUNTERS["fetch_size_kib"] * COUNTERS["fetch_scale"] +
                              COUNTERS["write_size_kib"] * COUNTERS["write_scale"]))
        # The clock the chip ran at under this kernel, measured in the counter run:
        # GRBM_GUI_ACTIVE (cycles of the graphics clock while the launch was in flight) over the
        # launch's duration in that run.  Boxes of the pool differ in the clock they sustain, so
        # the fractions "at the measured clock" are taken inside the counter run alone (busy
        # cycles over elapsed cycles of the same launch), not against this run's kernel time.
        cycles = COUNTERS["gui_active_cycles"]
        clock_ghz = cycles / (COUNTERS["pmc_launch_ms"] * 1e-3) / 1e9
        lane_ops = COUNTERS["valu_wave_instructions"] * 64
        alu_achieved = lane_ops / (kern_avg_ms * 1e-3) / 1e12
        alu = {"bound": "alu", "achieved": round(alu_achieved, 2), "peak": round(VALU_PEAK_TOPS, 2),
               "unit": "T 32-bit lane-ops/s", "frac": round(alu_achieved / VALU_PEAK_TOPS, 4),
               "measured_clock_GHz": round(clock_ghz, 3),
               "frac_at_measured_clock": round(lane_ops / (256 * 128 * cycles), 4),
               "valu_ops_per_payload_byte": round(lane_ops / payload, 2),
               "lds_lookups_per_payload_byte": round(COUNTERS["lds_wave_instructions"] * 64 / payload, 2)}
        # the resource that binds: cycles in which a CU's LDS pipe is serving lookups (a 64-lane
        # ds_read_b32 holds it for 2 cycles, a ds_read_b128 for 4), against one pipe per CU
        lds_achieved = COUNTERS["lds_active_cycles"] / (kern_avg_ms * 1e-3) / 1e9
        lds = {"bound": "lds", "achieved": round(lds_achieved, 1), "peak": round(LDS_PEAK_GCYCLES, 1),
               "unit": "G LDS-pipe cycles/s", "frac": round(lds_achieved / LDS_PEAK_GCYCLES, 4),
               "measured_clock_GHz": round(clock_ghz, 3),
               "frac_at_measured_clock": round(COUNTERS["lds_active_cycles"] / (256 * cycles), 4),
               "lds_cycles_per_payload_byte": round(COUNTERS["lds_active_cycles"] / payload, 4)}

    out = {
        "metric": "AES-%d-GCM enc / dec+verify GB/s on 1 MI355X; %% of HBM roofline"
                  % (8 * args.key_bytes),
        "value": res["value"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": w.name, "chunks": w.n, "payload_bytes": payload,
                   "step": "encrypt batch + decrypt-verify batch, enqueued by the library's own "
                           "loop (pgcm_measure_passes)",
                   "unit_bytes": res["unit_bytes"],
                   "row_hash": "matrix cores" if args.matrix_hash else "LDS table",
                   "key_bytes": args.key_bytes, "iv_bytes": args.iv_bytes,
                   "ciphertext": "pinned host memory" if args.host_bounce else "device memory"},
        "enc_GBps": res["enc_GBps"],
        "dec_verify_GBps": res["dec_verify_GBps"],
        "pct_hbm_roofline": round(100.0 * 2.0 * res["value"] / HBM_PEAK_GBS, 2),
        "roofline": {"bound": "hbm", "kernel": timed_kernel_name(w),
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes": det["algo_bytes"],
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
    if copy_gbs is not None:
        out["copy_ceiling"] = {"kind": "device-to-device copy of the payload buffer (HBM read + "
                                       "write), median of %d" % det["reps"],
                               "traffic_GBps": round(copy_gbs, 1),
                               "bulk_kernel_frac_of_copy": round(achieved / copy_gbs, 4)}
    import hashlib
    h = hashlib.sha256()
    for arr in (w.key, w.ivs, w.lens, w.aad if w.aad is not None else np.zeros(0, np.uint8)):
        h.update(np.ascontiguousarray(arr).tobytes())
    out["inputs_sha256"] = h.hexdigest()    # key, IVs, lengths, AAD (the payload is seeded too)
    key.free()
    del b
    torch.cuda.empty_cache()

    # the other workloads, same measurement with fewer passes, so that one line covers all five
    configs = {str(args.config): res}
    if not args.only and not args.host_bounce:
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                continue
            wc = workload(cfg)
            steps = min(args.steps, 200 if cfg == 1 else 30)
            rc, _, bc, kc = measure_workload(pgcm, torch, wc, args, steps, min(args.warmup, 10),
                                             False)
            rc["timed_kernel"] = timed_kernel_name(wc)
            configs[str(cfg)] = rc
            kc.free()
            del bc
            torch.cuda.empty_cache()
    res["timed_kernel"] = timed_kernel_name(w)
    out["configs"] = {k: configs[k] for k in sorted(configs)}

    if not args.no_cpu_baseline:
        chunks = args.cpu_chunks or max(1, int(600e6 // max(1, int(w.lens.mean()))))   # about 15 s
        threads = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(w, chunks, threads)
        out["cpu_libcrypto"] = libcrypto_rates(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
