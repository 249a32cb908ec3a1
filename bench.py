#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

A step is one decode step of the whole stack: for every layer, kv_append of
the step's K/V rows followed by decode_attn over everything stored so far.
The headline workload is the all-resident 32-layer stack (32 heads x 128,
batch 32, prompt 512, 512 generated tokens, contiguous fp16 KV); an offloaded
leg (paged KV, half of the layers streamed from pinned host memory) is timed
after it and reported under "offload" in the same JSON line, and the same
shape with the offloaded half taken block by block and streamed in chunks
under "offload_blocks".

Prints ONE JSON line.  `value` is decode tokens/s with all inputs already in
HBM (resident layers) or pinned host memory (offloaded layers) when the timed
region starts.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
PCIE5_X16_GBPS = 64.0       # nominal, one direction

# HBM traffic of the split kernel, from two rocprofv3 --pmc runs of this file's headline workload
# (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch, mean over the timed launches), each scaled by what the
# same counter read for the plain copy kernel of known size in the same run.  Reads are kept as a ratio to
# the algorithmic KV bytes of the same launches: the kernel re-reads nothing, and what exceeds 1 is the
# rounding of every sequence to whole 16-key tiles plus q, so the ratio carries over to any number of steps
# of the workload.  Writes (outputs, partial results, the appended rows) are a fixed number of bytes per
# launch of that batch.  Both are valid only for the kernel source they were taken on: if okv_kernels.hip
# has changed since, `traffic` is reported as null.
TRAFFIC_RECORD = {
    "workload": "cfg2",
    "kernel_sha256": "5a1747b6fb410b0ef77cd8abb128a8735718c45a69c02285b23bd970a05856b3",
    "fetch_kib": 199121.0, "fetch_scale": 2.0000, "algorithmic_bytes": 402915328,   # context 737..800
    "write_kib": 768.0, "write_scale": 1.0000,
}


def recorded_traffic(workload, bytes_per_launch):
    """HBM bytes per launch from the recorded counters, or None if they do not apply."""
    import hashlib
    rec = TRAFFIC_RECORD
    src = os.path.join(ROOT, "paper_2504_11816_amd", "csrc", "okv_kernels.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    if not rec["kernel_sha256"] or sha != rec["kernel_sha256"] or workload != rec["workload"]:
        return None
    fetch_ratio = rec["fetch_kib"] * 1024 * rec["fetch_scale"] / rec["algorithmic_bytes"]
    return fetch_ratio * bytes_per_launch + rec["write_kib"] * 1024 * rec["write_scale"]


def log(msg):
    print(msg, file=sys.stderr, flush=True)


_SETTLE = {"big_release": False, "seconds": 6.0}


def settle(leg, seconds=None):
    """A pause before a leg's timed region when the process has given tens of GiB of device memory back since
    it last paused (closing the previous leg's buffers): for several seconds after such a release steps with
    copies in them run 2-3 % slower (the same leg, in the same process: 618-624 ms a step right away, 607 from
    the sixth second on or after a pause of 8 s) -- something is still busy with the memory.  A serving process
    does not do that; the headline leg runs first and never waits."""
    import torch
    torch.cuda.synchronize()
    seconds = _SETTLE["seconds"] if seconds is None else min(seconds, _SETTLE["seconds"])
    waited = 0.0
    if _SETTLE["big_release"] and seconds > 0:
        log(f"[bench] {leg}: waiting {seconds:.0f} s for the device to settle after the previous leg's release")
        time.sleep(seconds)
        waited = seconds
    _SETTLE["big_release"] = False
    return waited


def released():
    """Called when a leg has closed its buffers."""
    import torch
    torch.cuda.empty_cache()
    _SETTLE["big_release"] = True


def fixed_inputs(st, seed):
    """q / k_new / v_new per layer, drawn once and reused every step, plus outputs."""
    import torch
    from paper_2504_11816_amd import synth
    dev = st.device
    q = [synth.randn_f16_torch((st.B, st.H, st.d), synth.stream_seed(seed, synth.TENSOR_Q, l), dev) for l in range(st.L)]
    k = [synth.randn_f16_torch((st.B, st.G, st.d), synth.stream_seed(seed, synth.TENSOR_KNEW, l), dev) for l in range(st.L)]
    v = [synth.randn_f16_torch((st.B, st.G, st.d), synth.stream_seed(seed, synth.TENSOR_VNEW, l), dev) for l in range(st.L)]
    out = [torch.empty((st.B, st.H, st.d), dtype=st.out_torch_dtype, device=dev) for _ in range(st.L)]
    torch.cuda.synchronize()
    return q, k, v, out


def kv_bytes_of_steps(ctx0, steps, G, d, L):
    """Algorithmic KV bytes read over `steps` decode steps that start from
    ctx0 stored tokens: sum over steps, layers and sequences of n_b * 2*G*d*2."""
    ctx0 = np.asarray(ctx0, dtype=np.int64)
    per_tok = 2 * G * d * 2
    total = 0
    for s in range(1, steps + 1):
        total += int((ctx0 + s).sum()) * per_tok * L
    return total


def timed_steps(st, ctx0, table, inputs, steps, warmup, running=False):
    """W untimed steps, state reset, then exactly K timed steps.  running: the K steps follow the warm-up
    steps as later steps of one generation follow earlier ones (the warm-up starts W tokens earlier, so the
    timed steps see the same contexts); the copy pipeline is then in its running state on both sides of
    the timed region: the first step finds its first copies done, the last one leaves those of the step
    after it in flight, and K steps move exactly K times the offloaded bytes."""
    import torch
    bound = st.bind_step(*inputs)          # every layer of a step goes out in one call (okv_decode_step)
    st.set_batch(ctx0 - warmup if running else ctx0, table)
    for _ in range(warmup):
        st.step_bound(bound)
    st.synchronize()
    if not running:
        st.set_batch(ctx0, table)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step_bound(bound)
    st.synchronize()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def kernel_time(st, ctx0, table, inputs, steps, per_step=False):
    """Same K steps again with the split-K kernels bracketed by HIP events on the
    compute stream: summed bracket time (s) and number of launches.  per_step: one
    bracket around each step's launches, which then run back to back as in the
    timed region (all layers resident); else one bracket per launch, which leaves
    the GPU idle for a few microseconds before every kernel."""
    bound = st.bind_step(*inputs)
    st.set_batch(ctx0, table)
    st.ctx.okv_profile_enable(2 if per_step else 1)
    for _ in range(steps):
        st.step_bound(bound)
    ms, n = st.ctx.okv_profile_read()
    st.ctx.okv_profile_enable(0)
    return ms * 1e-3, n


_CPU_JOB = {}


def _cpu_pairs(pairs):
    """Worker of cpu_baseline: the oracle on a run of (sequence, head) pairs of the layer in _CPU_JOB."""
    from oracle import attention as oa
    j = _CPU_JOB
    for (b, h) in pairs:
        oa.decode_attn(j["q"], j["pool"], j["layout"], j["ctx"], j["H"], sample=[(b, h)])
    return len(pairs)


def cpu_baseline(st, ctx_now, q_layers, budget_s=15.0):
    """The fp64 oracle, as it stands, on this host's cores: the (b, h) pairs of the same workload, layer
    after layer, shared out over one worker process per core of the affinity mask (each worker runs the
    oracle single-threaded), until the time budget is used."""
    import multiprocessing as mp
    from threadpoolctl import threadpool_limits
    cores = len(os.sched_getaffinity(0))
    layout = st.layout()
    pairs = [(b, h) for b in range(st.B) for h in range(st.H)]
    per_task = max(1, len(pairs) // (cores * 8))
    tasks = [pairs[i:i + per_task] for i in range(0, len(pairs), per_task)]
    done, tokens, dt, layers = 0, 0, 0.0, 0
    with threadpool_limits(limits=1):
        for layer in range(st.L):
            # not timed: the oracle starts from host memory; the workers are forked after the layer's data is
            # in place and inherit it (they never touch the GPU and leave without running exit handlers)
            _CPU_JOB.update(q=q_layers[layer].cpu().numpy(), pool=st.read_pool(layer), layout=layout, ctx=ctx_now, H=st.H)
            pool = mp.get_context("fork").Pool(cores)
            try:
                layers += 1
                t0 = time.perf_counter()
                for n in pool.imap_unordered(_cpu_pairs, tasks):
                    done += n
                dt += time.perf_counter() - t0
            finally:
                # the workers end by themselves once the queue is closed; terminate() would signal them, and a
                # signal handler that a profiler has installed in the parent is inherited by them
                pool.close()
                pool.join()
            tokens += int(sum(int(ctx_now[b]) for (b, h) in pairs))
            if dt > budget_s:
                break
    _CPU_JOB.clear()
    # one (b, h) pair of one layer is 1 / (H * L) of a generated token's attention
    tok_rate = done / dt / (st.H * st.L)
    kv_gbps = tokens * 2 * st.d * 2 * (st.G / st.H) / dt / 1e9
    return {"value": tok_rate, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "kv_gbps": kv_gbps,
            "sample": f"{done} (sequence, head) pairs = {layers} whole layer(s) at context {int(np.mean(ctx_now))}, "
                      f"{dt:.1f} s of numpy fp64 on {cores} worker processes (one per core, single-threaded each), "
                      f"scaled to {st.H} heads x {st.L} layers"}


def run_resident(args, workload=None, steps=None, warmup=None, with_cpu=None, layers=None):
    """An all-resident workload of synth.WORKLOADS: `steps` decode steps of the whole stack, timed end to
    end, then once more with the split-K launches of every step bracketed by HIP events."""
    import torch
    from paper_2504_11816_amd import synth
    from paper_2504_11816_amd.harness import Stack
    workload = workload or args.workload
    w = dict(synth.WORKLOADS[workload])
    steps = steps if steps else (args.steps if args.steps else w["steps"])
    warmup = args.warmup if warmup is None else warmup
    with_cpu = (not args.no_cpu) if with_cpu is None else with_cpu
    L, H, G, d, B, T = w["L"], w["H"], w["G"], w["d"], w["B"], w["T"]
    layers = args.layers if layers is None else layers
    if layers:
        L = min(L, layers)
    if w["ragged"]:
        ctx_first = synth.ragged_ctx_lens(B, w["ragged"][0], w["ragged"][1], args.seed)
    else:
        ctx_first = np.full(B, w["ctx"], dtype=np.int32)
    # Fewer steps than the workload's own generation length: the steps in the MIDDLE of the generation, whose
    # mean context is the workload's mean (the time of a step is linear in its context, so tokens/s over
    # them is what the whole generation gives); the first steps would be its cheapest ones.
    first_step = (w["steps"] - steps) // 2 if (not w["ragged"] and 0 < steps < w["steps"]) else 0
    ctx_first = ctx_first + first_step
    ctx0 = ctx_first - 1                                   # stored before the first timed step
    cap = int(ctx0.max()) + max(steps, warmup) + 1
    log(f"[bench] {workload}: L={L} H={H} G={G} d={d} B={B} T={T} ctx {int(ctx_first.min())}..{int(ctx_first.max())} "
        f"steps={steps} capacity={cap}")
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=cap, out_dtype=0, split_tokens=args.split_tokens)
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(args.seed, synth.TENSOR_POOL, l))
    table = None
    if T:
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                           max_blocks_per_seq=st.max_blocks)
    inputs = fixed_inputs(st, args.seed)
    log("[bench] pools filled; timing")
    settled = settle(workload, 2.0)                      # no copies in these steps: the effect is under 1 % here
    dt = timed_steps(st, ctx0, table, inputs, steps, warmup)
    split = st.ctx.okv_get_split_tokens()
    n_items = len(st.ctx.okv_worklist(from_device=False))
    kv_bytes = kv_bytes_of_steps(ctx0, steps, G, d, L)
    log(f"[bench] {steps} steps in {dt * 1e3:.1f} ms, split {split}")
    k_s, k_n = kernel_time(st, ctx0, table, inputs, steps, per_step=True)
    log(f"[bench] split-K kernel: {k_n} launches, {k_s / max(k_n, 1) * 1e6:.1f} us average")
    res = {
        "workload": workload,
        "tokens_per_s": B * steps / dt, "ms_per_step": dt / steps * 1e3, "kv_gbps": kv_bytes / dt / 1e9,
        "hbm_frac": kv_bytes / dt / 1e9 / HBM_PEAK_GBPS,
        "kernel_gbps": kv_bytes / k_s / 1e9, "kernel_frac": kv_bytes / k_s / 1e9 / HBM_PEAK_GBPS,
        "kernel_avg_us": k_s / max(k_n, 1) * 1e6, "kernel_launches": k_n,
        "kernel_time_includes_merge_pass": n_items > B, "settle_s": settled,
        "kv_bytes_per_launch": kv_bytes / max(k_n, 1), "split_tokens": split, "work_items": n_items, "steps": steps,
        "B": B, "L": L, "H": H, "G": G, "d": d, "T": T, "first_step": first_step + 1, "workload_steps": w["steps"],
        "ctx_desc": (f"{int(ctx_first.max())}..{int(ctx_first.max()) + steps - 1}" if not w["ragged"] else
                     f"ragged {int(ctx_first.min())}..{int(ctx_first.max())} at the first step (mean "
                     f"{float(ctx_first.mean()):.0f}, sum {int(ctx_first.sum())}), +1 per step"),
    }
    log(f"[bench] {workload}: {res['tokens_per_s']:.0f} tokens/s, {res['kv_gbps']:.0f} GB/s of KV end to end "
        f"({100 * res['hbm_frac']:.1f}% of HBM peak), kernels alone {100 * res['kernel_frac']:.1f}%")
    cpu = None
    if with_cpu:
        log("[bench] timing the CPU oracle on a sample")
        mid = ctx0 + steps                                  # lengths as the run left them
        cpu = cpu_baseline(st, mid, inputs[0], args.cpu_seconds)
    st.close()
    del st
    released()
    return res, cpu


def run_latency(args, reps=200):
    """The small single-layer workload (8 heads x 64, batch 4, context 256: 2 MiB of KV, which sits in
    cache): latency only.  Every step is issued and waited for on its own; the median over `reps` steps is
    reported, for contiguous and for paged pools, with the time the step's kernels take on the GPU beside
    it (HIP events around the launches of a step: the rest is what the host spends issuing them)."""
    import torch
    from paper_2504_11816_amd import synth
    from paper_2504_11816_amd.harness import Stack
    w = dict(synth.WORKLOADS["cfg1"])
    L, H, G, d, B = w["L"], w["H"], w["G"], w["d"], w["B"]
    out = {"workload": f"cfg1: {L} layer, {H} heads x {d}, batch {B}, context {w['ctx']}", "reps": reps}
    for name, T in (("contiguous", 0), ("paged", 16)):
        ctx0 = np.full(B, w["ctx"] - 1, dtype=np.int32)
        st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=w["ctx"] + 16, out_dtype=0)
        st.fill_pool(0, synth.stream_seed(args.seed, synth.TENSOR_POOL, 0))
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                           max_blocks_per_seq=st.max_blocks) if T else None
        inputs = fixed_inputs(st, args.seed)
        bound = st.bind_step(*inputs)
        lat, gpu = [], []
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(reps + 20):
            st.set_batch(ctx0, table)                      # every repetition is the same step: 256 keys attended
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record(st.compute_stream)
            st.step_bound(bound)
            e1.record(st.compute_stream)
            st.synchronize()
            t1 = time.perf_counter()
            if i >= 20:
                lat.append((t1 - t0) * 1e6)
                gpu.append(e0.elapsed_time(e1) * 1e3)
        out[name] = {"step_latency_us_median": float(np.median(lat)), "step_latency_us_p10": float(np.percentile(lat, 10)),
                     "step_latency_us_p90": float(np.percentile(lat, 90)), "gpu_time_us_median": float(np.median(gpu)),
                     "work_items": len(st.ctx.okv_worklist(from_device=False)), "kernels_per_step": 3 if len(st.ctx.okv_worklist(from_device=False)) > B else 2}
        log(f"[bench] cfg1 {name}: step latency {out[name]['step_latency_us_median']:.1f} us median "
            f"({out[name]['step_latency_us_p10']:.1f}..{out[name]['step_latency_us_p90']:.1f}), on the GPU {out[name]['gpu_time_us_median']:.1f} us")
        st.close()
        del st
    released()
    return out


def run_probe(nbytes=1 << 30, reps=5):
    """Plain 16-byte-per-lane copy and read kernels over 1 GiB: what a kernel with no
    arithmetic reaches on this GPU, and the known-size dispatches HBM counters are scaled by."""
    import torch
    from paper_2504_11816_amd import binding
    dev = torch.device("cuda:0")
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream()               # no stream of torch's pool: see harness.new_stream
    torch.cuda.synchronize()
    out = {"bytes": nbytes}
    for name, fn, moved in (("copy", lambda: binding.okv_probe_copy(dst, src, nbytes, st.cuda_stream), 2 * nbytes),
                            ("read", lambda: binding.okv_probe_read(src, nbytes, sink, st.cuda_stream), nbytes)):
        fn()
        st.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(reps):
            fn()
        e1.record(st)
        st.synchronize()
        out[name + "_gbps"] = moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    log(f"[bench] plain kernels on 1 GiB: copy {out['copy_gbps']:.0f} GB/s (read+write), read {out['read_gbps']:.0f} GB/s")
    return out


# Offloaded legs.  cfg5's full batch (192 sequences, 240 GiB of pinned KV) does not fit
# the host memory a single-GPU machine may use; its per-sequence shape (context 4096, 60 % of
# the layers on the host) is run at batch 48 unless --offload-batch says otherwise.
OFFLOAD_DEFAULT_BATCH = {"cfg3": 64, "cfg5": 48}


def overlap_figures(res, t_step_ms, t_copy_plain_ms, t_copy_pipelined_ms, t_compute_ms):
    """overlap = 1 - (t_step - t_copy_only) / t_compute_only with the two halves measured alone: 1 when a
    step costs no more than its copies, 0 when the attention adds to them in full (Eq. 6 of the paper's
    model), below 0 when a step loses more than its whole attention time to something else.  Given twice:
    against the copies run back to back on one stream with nothing between them, and against the copy half
    issued as the pipeline issues it (two copy streams, a wait for the buffer's release before and a record
    after every copy), which is the half a step really contains.  The copy half is the faster of two replays (a
    replay differs by +-1 ms from one to the next, a tenth of the attention time of the whole-layer leg) and the
    figure is capped at 1: a step cannot cost less than its copies, `overlap_uncapped` says what the noise made
    of it."""
    res["t_step_ms"] = t_step_ms
    res["t_compute_only_ms"] = t_compute_ms
    res["t_copy_only_ms"] = t_copy_pipelined_ms
    res["t_copy_back_to_back_ms"] = t_copy_plain_ms
    res["overlap_uncapped"] = 1.0 - (t_step_ms - t_copy_pipelined_ms) / max(t_compute_ms, 1e-9)
    res["overlap"] = min(1.0, res["overlap_uncapped"])
    res["overlap_vs_back_to_back_copies"] = 1.0 - (t_step_ms - t_copy_plain_ms) / max(t_compute_ms, 1e-9)
    res["copy_protocol_cost_ms"] = t_copy_pipelined_ms - t_copy_plain_ms
    return res


def host_memory_gib():
    """(MemTotal, MemAvailable) of this box in GiB."""
    vals = {}
    with open("/proc/meminfo") as f:
        for line in f:
            k, v = line.split(":")
            if k in ("MemTotal", "MemAvailable"):
                vals[k] = int(v.split()[0]) / 2 ** 20
    return vals.get("MemTotal", 0.0), vals.get("MemAvailable", 0.0)


def pinnable_gib(want_gib, step_gib=4):
    """How much pinned, device-mapped host memory this process can get, up to want_gib: hipHostMalloc in
    pieces of step_gib until it is refused, then everything is given back.  (On the benchmark boxes the
    refusal comes at about 70 GiB whatever the 288 GiB of RAM: a limit of the container, not of the host.)"""
    from paper_2504_11816_amd.harness import PinnedHalfBuffer
    got, bufs = 0, []
    try:
        while got + step_gib <= want_gib:
            bufs.append(PinnedHalfBuffer(step_gib << 29))
            got += step_gib
    except MemoryError:
        pass
    for b in bufs:
        b.free()
    return float(got)


def cfg5_batch():
    """The batch the offline workload (batch 192, context 4096, 20 of 32 layers on the host) is run at: its own
    if the host share (241 GiB at batch 192) can be pinned, else the largest multiple of 8 whose host share
    fits 95 % of what this process can pin (measured just before the leg)."""
    from paper_2504_11816_amd import synth
    w = synth.WORKLOADS["cfg5"]
    total, avail = host_memory_gib()
    n_off = -(-w["c_off"][0] * w["L"] // w["c_off"][1])
    per_seq_gib = n_off * synth.blocks_needed(w["ctx"] + 8, w["T"]) * w["T"] * 2 * w["G"] * w["d"] * 2 / 2 ** 30
    full = w["B"] * per_seq_gib
    can_pin = pinnable_gib(min(full + 4, 0.8 * avail))
    B = min(w["B"], int(0.95 * can_pin / per_seq_gib) // 8 * 8)
    return max(8, B), {"host_ram_gib": total, "host_ram_available_gib": avail, "pinnable_gib_measured": can_pin,
                      "full_batch": w["B"], "full_batch_pinned_gib": full}


def run_offload(args, name=None, B=None, steps=None, warmup=None):
    """Paged KV, part of the layers in pinned host memory, streamed per layer."""
    import torch
    from paper_2504_11816_amd import binding, synth
    from paper_2504_11816_amd.harness import Stack
    name = name or args.offload_workload
    w = dict(synth.WORKLOADS[name])
    L, H, G, d, T = w["L"], w["H"], w["G"], w["d"], w["T"]
    B = B or args.offload_batch or OFFLOAD_DEFAULT_BATCH[name]
    steps = steps or args.offload_steps or (6 if name == "cfg3" else 3)
    warmup = (2 if name == "cfg3" else 1) if warmup is None else warmup
    ctx0 = np.full(B, w["ctx"] - 1, dtype=np.int32)
    cap = w["ctx"] + steps + warmup
    on_host, n_off = binding.kv_offload_plan(L, w["c_off"][0], w["c_off"][1])
    n_staging = args.staging or 2
    log(f"[bench] offload leg {name}: B={B} ctx={w['ctx']} T={T} host layers {n_off}/{L} steps={steps} staging buffers {n_staging}")
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=cap, on_host=on_host, out_dtype=0,
               n_staging=n_staging)
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(args.seed, synth.TENSOR_POOL, l))
    table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                       max_blocks_per_seq=st.max_blocks)
    inputs = fixed_inputs(st, args.seed)
    host_layer = int(np.flatnonzero(on_host)[0])
    link = binding.okv_measure_h2d(st.staging[0], st.pools[host_layer], min(st.pool_bytes, 2 << 30), 10,
                                   st.h2d_stream.cuda_stream)
    log(f"[bench] host-to-device link: {link:.1f} GB/s (plain hipMemcpyAsync, pinned, median of 10)")
    settle(f"offload leg {name}")
    dt = timed_steps(st, ctx0, table, inputs, steps, warmup, running=True)
    per_tok = 2 * G * d * 2
    link_bytes = sum(int((ctx0 + s).sum()) * per_tok * n_off for s in range(1, steps + 1))
    kv_bytes = kv_bytes_of_steps(ctx0, steps, G, d, L)
    # the two halves alone: every layer's attention kernels (one step), and one step's copies
    k_s, k_n = kernel_time(st, ctx0, table, inputs, 1)
    st.set_batch(ctx0, table)
    copy_ms = st.ctx.okv_time_copies(False, 1)
    copy_pipe_ms = min(st.ctx.okv_time_copies(True, steps), st.ctx.okv_time_copies(True, steps))
    res = {
        "workload": name, "B": B, "ctx": w["ctx"], "host_layers": int(n_off), "layers": L, "steps": steps,
        "tokens_per_s": B * steps / dt, "ms_per_step": dt / steps * 1e3, "kv_gbps": kv_bytes / dt / 1e9,
        "link_gbps_measured": link, "link_gbps_nominal": PCIE5_X16_GBPS,
        "link_gbps_achieved": link_bytes / dt / 1e9, "link_frac": link_bytes / dt / 1e9 / link,
        "attn_kernel_ms_per_step": k_s * 1e3, "attn_kernel_gbps": kv_bytes / steps / k_s / 1e9,
        "copy_only_ms_per_step": copy_ms,
        "pinned_gib": n_off * st.pool_bytes / 2 ** 30, "staging_buffers": n_staging,
        "staging_gib": n_staging * st.pool_bytes / 2 ** 30,
    }
    # What a step costs beyond its copies run back to back, set against the attention it contains:
    # below 1 means compute is (partly) hidden; the per-copy dependency latency of the two-stream
    # protocol (~0.8 ms per layer copy in the copy trace) is in this figure too.
    res["step_minus_copies_ms"] = res["ms_per_step"] - copy_ms
    overlap_figures(res, res["ms_per_step"], copy_ms, copy_pipe_ms, res["attn_kernel_ms_per_step"])
    log(f"[bench] offload leg {name}: {res['ms_per_step']:.1f} ms/step, link {res['link_gbps_achieved']:.1f} GB/s "
        f"= {100 * res['link_frac']:.1f}% of measured; copies alone {copy_ms:.1f} ms back to back, {copy_pipe_ms:.1f} ms "
        f"as the pipeline issues them; attention kernels alone {res['attn_kernel_ms_per_step']:.1f} ms/step "
        f"({res['attn_kernel_gbps']:.0f} GB/s); overlap {res['overlap']:.2f} ({res['overlap_vs_back_to_back_copies']:.2f} against back-to-back copies)")
    st.close()
    del st
    released()
    return res


def run_offload_blocks(args):
    """The same shape with the offload share taken block by block: in every layer the
    oldest blocks of each sequence (C_off of the blocks the batch can grow into) are in
    pinned host memory and streamed in chunks; the staging buffers hold one chunk each."""
    import torch
    from paper_2504_11816_amd import binding, synth
    from paper_2504_11816_amd.harness import Stack
    name = args.offload_workload
    w = dict(synth.WORKLOADS[name])
    L, H, G, d, T = w["L"], w["H"], w["G"], w["d"], w["T"]
    B = args.offload_batch or OFFLOAD_DEFAULT_BATCH[name]
    steps, warmup = args.offload_steps or (4 if name == "cfg3" else 2), 1
    ctx0 = np.full(B, w["ctx"] - 1, dtype=np.int32)
    cap = w["ctx"] + steps + warmup
    need = B * synth.blocks_needed(cap, T)
    n_res, n_host = binding.okv_plan_block_split(need, w["c_off"][0], w["c_off"][1])
    shape = binding.make_config(n_layers=L, n_q_heads=H, n_kv_heads=G, head_dim=d, block_tokens=T, max_batch=B,
                                max_blocks_per_seq=synth.blocks_needed(cap, T), blocks_per_layer=need)
    block_bytes = binding.okv_block_bytes(shape)
    chunk_blocks = max(1, (args.chunk_mib << 20) // block_bytes)
    n_staging = args.staging or 2
    log(f"[bench] block-granular leg {name}: B={B} ctx={w['ctx']} T={T} host blocks {n_host}/{need} per layer, "
        f"chunks of {chunk_blocks} blocks ({chunk_blocks * block_bytes / 2 ** 20:.0f} MiB), {n_staging} staging buffers")
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=cap, out_dtype=0, n_staging=n_staging,
               blocks_per_layer=need, resident_blocks=n_res, chunk_blocks=chunk_blocks, hot_tails=not args.no_tails)
    # link rate first (it overwrites the start of layer 0's HBM part, which is filled afterwards)
    probe_bytes = min(st.dev_part[0].numel() * 2, st.host_part[0].numel() * 2, 2 << 30)
    link = binding.okv_measure_h2d(st.dev_part[0], st.host_part[0], probe_bytes, 10, st.h2d_stream.cuda_stream)
    log(f"[bench] host-to-device link: {link:.1f} GB/s ({probe_bytes / 2 ** 20:.0f} MiB copies)")
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(args.seed, synth.TENSOR_POOL, l))
    table = synth.classed_block_table([st.cap_tokens] * B, T, n_res, n_host, n_host, args.placement, args.seed + 1,
                                      max_blocks_per_seq=st.max_blocks)
    inputs = fixed_inputs(st, args.seed)
    settle(f"block-granular leg {name}")
    dt = timed_steps(st, ctx0, table, inputs, steps, warmup, running=True)
    # what crosses the link per step: every host block of every layer (all of them hold keys:
    # the oldest blocks of a sequence are full)
    host_tokens = int(((table >= n_res).sum(axis=1) * T).sum())
    assert all(int((table[b] >= n_res).sum()) * T <= int(ctx0[b]) for b in range(B)) or args.placement != "prefix"
    link_bytes = host_tokens * 2 * G * d * 2 * L * steps
    kv_bytes = kv_bytes_of_steps(ctx0, steps, G, d, L)
    k_s, k_n = kernel_time(st, ctx0, table, inputs, 1)
    st.set_batch(ctx0, table)
    copy_ms = st.ctx.okv_time_copies(False, 1)
    copy_pipe_ms = min(st.ctx.okv_time_copies(True, steps), st.ctx.okv_time_copies(True, steps))
    res = {
        "workload": name, "placement": args.placement, "B": B, "ctx": w["ctx"], "layers": L, "steps": steps,
        "host_blocks_per_layer": int(n_host), "blocks_per_layer": int(need),
        "host_share_of_keys": host_tokens / float((ctx0 + 1).sum()),
        "chunk_mib": chunk_blocks * block_bytes / 2 ** 20, "copies_per_step": len(st.ctx_units()) * L,
        "tokens_per_s": B * steps / dt, "ms_per_step": dt / steps * 1e3, "kv_gbps": kv_bytes / dt / 1e9,
        "link_gbps_measured": link, "link_gbps_achieved": link_bytes / dt / 1e9,
        "link_frac": link_bytes / dt / 1e9 / link,
        "attn_kernel_ms_per_step": k_s * 1e3, "attn_launches_per_step": k_n,
        "copy_only_ms_per_step": copy_ms, "step_minus_copies_ms": dt / steps * 1e3 - copy_ms,
        "pinned_gib": L * st.host_part[0].numel() * 2 / 2 ** 30,
        "staging_buffers": n_staging, "staging_gib": n_staging * st.staging_bytes / 2 ** 30,
        "split_tokens": st.ctx.okv_get_split_tokens(),
    }
    overlap_figures(res, res["ms_per_step"], copy_ms, copy_pipe_ms, res["attn_kernel_ms_per_step"])
    log(f"[bench] block-granular leg {name}: {res['ms_per_step']:.1f} ms/step, link {res['link_gbps_achieved']:.1f} GB/s "
        f"= {100 * res['link_frac']:.1f}% of measured; copies alone {copy_ms:.1f} ms back to back, {copy_pipe_ms:.1f} ms as the "
        f"pipeline issues them; attention alone {res['attn_kernel_ms_per_step']:.1f} ms/step in {k_n} launches; "
        f"overlap {res['overlap']:.2f}; staging {res['staging_gib']:.2f} GiB")
    st.close()
    del st
    released()
    return res


def run_prefill(args):
    """The prefill side of the offloaded shape: the K/V rows of a whole prompt batch are
    stored layer by layer, half of the layers into pinned host memory.  Timed twice: the
    stores alone, and next to a stand-in for the layer's computation (a plain read kernel
    over a buffer sized to take about as long as a layer's write-out), to show that a layer
    costs the longer of the two rather than their sum."""
    import torch
    from paper_2504_11816_amd import binding, synth
    from paper_2504_11816_amd.harness import Stack
    name = args.offload_workload
    w = dict(synth.WORKLOADS[name])
    L, H, G, d, T = w["L"], w["H"], w["G"], w["d"], w["T"]
    B = args.offload_batch or OFFLOAD_DEFAULT_BATCH[name]
    P = w["ctx"]
    on_host, n_off = binding.kv_offload_plan(L, w["c_off"][0], w["c_off"][1])
    log(f"[bench] prefill leg {name}: B={B} prompt={P} T={T} host layers {n_off}/{L}")
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=P + 16, on_host=on_host, out_dtype=0, n_staging=args.staging or 2)
    if args.prefill_table == "ordered":                  # a sequence's blocks are neighbours in the pool
        table = synth.identity_block_table([st.cap_tokens] * B, T, max_blocks_per_seq=st.max_blocks)
    else:
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                           max_blocks_per_seq=st.max_blocks)
    rows = B * P
    layer_bytes = rows * 2 * G * d * 2
    # two sets of row buffers, used alternately: the projection of layer l + 2 may only
    # overwrite a set once the store of layer l has left it (okv_prefill_release)
    bufs = [(synth.randn_f16_torch((rows, G, d), synth.stream_seed(args.seed, synth.TENSOR_KNEW, i), st.device),
             synth.randn_f16_torch((rows, G, d), synth.stream_seed(args.seed, synth.TENSOR_VNEW, i), st.device))
            for i in range(2)]
    host_layer = int(np.flatnonzero(on_host)[0])
    link = binding.okv_measure_d2h(st.pools[host_layer], bufs[0][0], min(layer_bytes // 2, 2 << 30), 10,
                                   st.h2d_stream.cuda_stream)
    log(f"[bench] device-to-host link: {link:.1f} GB/s (plain hipMemcpyAsync, pinned, median of 10)")
    # the stand-in computation: a read of `work` bytes takes about one host layer's write-out
    sink = torch.zeros(4, dtype=torch.int32, device=st.device)
    scratch = torch.empty(args.standin_gib << 30, dtype=torch.uint8, device=st.device)
    cs = st.compute_stream.cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.okv_probe_read(scratch, scratch.numel(), sink, cs)
    st.compute_stream.synchronize()
    e0.record(st.compute_stream)
    for _ in range(8):
        binding.okv_probe_read(scratch, scratch.numel(), sink, cs)
    e1.record(st.compute_stream)
    st.compute_stream.synchronize()
    read_ms = e0.elapsed_time(e1) / 8
    want_ms = layer_bytes / (link * 1e9) * 1e3 * n_off / L      # so that compute and write-out are about level
    reads_per_layer = max(1, int(round(want_ms / read_ms)))

    plan = {}
    settle("prefill leg")

    def one_pass(with_compute):
        st.set_batch([0] * B, table)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        c = st.ctx
        c.okv_prefill_begin([P] * B)
        plan.update(c.okv_prefill_plan())
        for l in range(L):
            k_rows, v_rows = bufs[l % 2]
            if l >= 2:
                c.okv_prefill_release(l - 2)                   # this layer's "projection" overwrites the set of layer l - 2
            if with_compute:
                for _ in range(reads_per_layer):
                    binding.okv_probe_read(scratch, scratch.numel(), sink, cs)
            c.kv_append_bulk(l, k_rows, v_rows)
        c.okv_prefill_end()
        st.synchronize()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    one_pass(False)                                            # warm-up (first touch of the pinned pools)
    t_store = one_pass(False)
    t_both = one_pass(True)
    t_compute = L * reads_per_layer * read_ms * 1e-3
    host_bytes = n_off * layer_bytes
    hbm_bytes = (L - n_off) * layer_bytes
    res = {
        "workload": name, "B": B, "prompt": P, "layers": L, "host_layers": int(n_off),
        "tokens_per_s": B * P / t_store, "ms_stores_alone": t_store * 1e3,
        "link_gbps_measured": link, "link_gbps_achieved": host_bytes / t_store / 1e9,
        "link_frac": host_bytes / t_store / 1e9 / link,
        "standin_compute_ms": t_compute * 1e3, "ms_with_compute": t_both * 1e3,
        "max_of_the_two_ms": max(t_compute, t_store) * 1e3, "sum_of_the_two_ms": (t_compute + t_store) * 1e3,
        "host_gib": host_bytes / 2 ** 30, "hbm_gib": hbm_bytes / 2 ** 30,
        "block_table": args.prefill_table,
        "route": "staging + hipMemcpyAsync" if plan.get("staged_groups") else "kernel through the mapped pointer",
        "copies_per_host_layer": plan.get("copies", 0),
    }
    log(f"[bench] prefill leg {name}: stores alone {res['ms_stores_alone']:.1f} ms = {res['link_gbps_achieved']:.1f} GB/s to the host "
        f"({100 * res['link_frac']:.1f}% of measured); stand-in compute alone {res['standin_compute_ms']:.1f} ms; together "
        f"{res['ms_with_compute']:.1f} ms (max {res['max_of_the_two_ms']:.1f}, sum {res['sum_of_the_two_ms']:.1f}); "
        f"route: {res['route']}, {res['copies_per_host_layer']} copies per host layer")
    st.close()
    del st, bufs, scratch
    released()
    return res


def run_layers(args):
    """Whole decoder layers in the decode stage: the headline stack (32 layers, hidden 4096,
    feed-forward 16384, batch 32, context 513 upwards) with random weights; per step every
    layer reads its 402 MB of weights and its share of the KV cache once.  Also times each
    linear product alone."""
    import torch
    from paper_2504_11816_amd import binding, synth
    from paper_2504_11816_amd.harness import BoundLayers, LayerScratch, LayerWeights, Stack
    w = dict(synth.WORKLOADS[args.decoder_workload])
    L, H, G, d, B, T = w["L"], w["H"], w["G"], w["d"], w["B"], w["T"]
    if args.layers:
        L = min(L, args.layers)
    h1, h2 = H * d, 4 * H * d
    steps, warmup = args.layer_steps, 4
    if w["ragged"]:
        ctx0 = synth.ragged_ctx_lens(B, w["ragged"][0], w["ragged"][1], args.seed) - 1
    else:
        ctx0 = np.full(B, w["ctx"] - 1, dtype=np.int32)
    st = Stack(L=L, H=H, G=G, d=d, B=B, T=T, cap_tokens=int(ctx0.max()) + steps + warmup + 1, out_dtype=0)
    for l in range(L):
        st.fill_pool(l, synth.stream_seed(args.seed, synth.TENSOR_POOL, l))
    table = None
    if T:
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                           max_blocks_per_seq=st.max_blocks)
    weights = [LayerWeights(h1, h2, args.seed, l, st.device, kv_cols=G * d) for l in range(L)]
    scratch = LayerScratch(B, h1, h2, G, d, st.device)
    x0 = synth.randn_f16_torch((B, h1), synth.stream_seed(args.seed, synth.TENSOR_Q), st.device)
    x = x0.clone()

    bound = BoundLayers(st, weights, scratch)      # one call into the library per step (okv_decoder_step)

    def run(n):
        for _ in range(n):
            x.copy_(x0)                    # keep the activations at the scale of the inputs (random weights amplify)
            bound.step(x)
    settle("decoder layers")
    st.set_batch(ctx0, table)
    with torch.cuda.stream(st.compute_stream):
        run(warmup)
        st.synchronize()
        st.set_batch(ctx0, table)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)
        st.synchronize()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    kv_bytes = kv_bytes_of_steps(ctx0, steps, G, d, L)
    w_bytes = sum(wt.bytes_read_per_step() for wt in weights) * steps
    # each product alone, back to back over the layers' own matrices in turn (two rounds): with L layers the
    # weights come from HBM as they do in a step, not from the memory-side cache a single matrix would sit in;
    # at the leg's own batch and at 32, 64, 128 and 192 rows (more than 128 rows take two launches, each reading
    # the weights again: the rate below counts the matrix once)
    cs = st.compute_stream

    def products_alone(m, sc):
        out = {}
        for name, fn, nbytes in (
                (f"qkv {h1 + 2 * G * d}x{h1}", lambda wt: binding.okv_linear_qkv(sc.a, wt.packed["wqkv"], wt.bqkv, sc.q, sc.k, sc.v, m, h1, G * d, h1, cs.cuda_stream, sc.ws, sc.ws_bytes), (h1 + 2 * G * d) * h1 * 2),
                ("out 4096x4096", lambda wt: binding.okv_linear(sc.t, wt.packed["wo"], wt.t["bo"], sc.z, sc.y, m, h1, h1, False, cs.cuda_stream, sc.ws, sc.ws_bytes), h1 * h1 * 2),
                ("ffn1 16384x4096", lambda wt: binding.okv_linear(sc.z, wt.packed["w1"], wt.t["b1"], None, sc.u, m, h2, h1, True, cs.cuda_stream, sc.ws, sc.ws_bytes), h1 * h2 * 2),
                ("ffn2 4096x16384", lambda wt: binding.okv_linear(sc.u, wt.packed["w2"], wt.t["b2"], sc.z, sc.y, m, h1, h2, False, cs.cuda_stream, sc.ws, sc.ws_bytes), h1 * h2 * 2)):
            for wt in weights:
                fn(wt)
            cs.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(cs)
            for _ in range(2):
                for wt in weights:
                    fn(wt)
            e1.record(cs)
            cs.synchronize()
            us = e0.elapsed_time(e1) / (2 * len(weights)) * 1e3
            out[name] = {"us": us, "weight_gbps": nbytes / us / 1e3, "hbm_frac": nbytes / us / 1e3 / HBM_PEAK_GBPS}
        return out

    alone = products_alone(B, scratch)
    by_rows = {}
    for m in (32, 64, 128, 192):
        sc = scratch if m == B else LayerScratch(m, h1, h2, G, d, st.device)
        for t in (sc.a, sc.t, sc.z, sc.u):
            t.normal_()
        by_rows[str(m)] = alone if m == B else products_alone(m, sc)
        del sc
    res = {
        "workload": f"{L} decoder layers ({args.decoder_workload} shape: {H} query / {G} KV heads x {d}), hidden {h1}, feed-forward {h2}, batch {B}, "
                    + (f"context {w['ctx']}..{w['ctx'] + steps - 1}" if not w["ragged"] else
                       f"ragged contexts {int(ctx0.min()) + 1}..{int(ctx0.max()) + 1} (+1 per step)") + ", random weights",
        "steps": steps, "tokens_per_s": B * steps / dt, "ms_per_step": dt / steps * 1e3,
        "weight_gb_per_step": w_bytes / steps / 1e9, "kv_gb_per_step": kv_bytes / steps / 1e9,
        "hbm_gbps": (w_bytes + kv_bytes) / dt / 1e9, "hbm_frac": (w_bytes + kv_bytes) / dt / 1e9 / HBM_PEAK_GBPS,
        "linear_alone": alone,
        "linear_alone_by_rows": by_rows,
    }
    log(f"[bench] decoder layers: {res['ms_per_step']:.2f} ms/step, {res['tokens_per_s']:.0f} tokens/s, "
        f"{res['hbm_gbps']:.0f} GB/s of weights + KV ({100 * res['hbm_frac']:.1f}% of HBM peak); products alone: "
        + ", ".join(f"{k} {v['us']:.1f} us = {v['weight_gbps']:.0f} GB/s" for k, v in alone.items()))
    st.close()
    del st, weights, scratch, bound
    released()
    return res


def run_model(args, off):
    """The paper's prediction model on this GPU's own numbers (§IV-D, §IV-F): the decode
    attention time per layer is measured at several batch sizes, the calibration line
    CTCF(t) = alpha t + beta is fitted by least squares against the theoretical time
    (attention flops over the published FP16 matrix peak, as the paper does with vendor
    figures), checked on batch sizes left out of the fit, and then used with the measured
    link rate to predict the offloaded leg's step time, which is compared with the measurement."""
    import torch
    from paper_2504_11816_amd import infersave as isv, synth
    from paper_2504_11816_amd.harness import Stack
    w = dict(synth.WORKLOADS["cfg3"])
    H, G, d, T = w["H"], w["G"], w["d"], w["T"]
    ctx, layers, steps = w["ctx"], 4, 3
    h1 = H * d
    flops = 2.5e15                                            # MI355X dense FP16 matrix peak
    fit_b, hold_b = [8, 16, 32, 64, 96], [12, 24, 48, 80]
    times = {}
    for B in sorted(fit_b + hold_b):
        st = Stack(L=layers, H=H, G=G, d=d, B=B, T=T, cap_tokens=ctx + 16, out_dtype=0)
        for l in range(layers):
            st.fill_pool(l, synth.stream_seed(args.seed, synth.TENSOR_POOL, l))
        table = synth.shuffled_block_table([st.cap_tokens] * B, T, st.blocks_per_layer, args.seed + 1,
                                           max_blocks_per_seq=st.max_blocks)
        inputs = fixed_inputs(st, args.seed)
        ctx0 = np.full(B, ctx - 1, dtype=np.int32)
        kernel_time(st, ctx0, table, inputs, 1)              # warm-up
        k_s, k_n = kernel_time(st, ctx0, table, inputs, steps, per_step=True)
        times[B] = k_s / k_n                                  # seconds per layer and step
        st.close()
        del st
        released()
    theory = {B: isv.isv_attention_flops_decode(B, ctx + (steps - 1) / 2, h1) / flops for B in times}
    alpha, beta, fit_err = isv.isv_ctcf_fit([theory[B] for B in fit_b], [times[B] for B in fit_b])
    hold_err = float(np.mean([abs(alpha * theory[B] + beta - times[B]) / times[B] for B in hold_b]))
    res = {
        "theory": "4 BS context h1 flops per layer over 2.5 PFLOP/s", "context": ctx, "fit_batches": fit_b,
        "holdout_batches": hold_b, "alpha": alpha, "beta_us": beta * 1e6, "fit_mean_rel_err": fit_err,
        "holdout_mean_rel_err": hold_err,
        "measured_us_per_layer": {str(B): times[B] * 1e6 for B in sorted(times)},
    }
    log(f"[bench] CTCF on decode attention at context {ctx}: alpha {alpha:.1f}, beta {beta * 1e6:.1f} us; mean error "
        f"{100 * fit_err:.1f}% on the fitted batch sizes, {100 * hold_err:.1f}% on the held-out ones")
    if off:
        # the offloaded leg: per layer max(CTCF(compute), transfer) with the measured link rate (overlap),
        # and the paper's compute + transfer (Eq. 6) beside it
        B, L = off["B"], off["layers"]
        c_off = off["host_layers"] / L
        model = isv.IsvModel(0.0, h1, 4 * h1, L, 2)
        # a one-token task at the leg's context: (c_off 2 (L_in + 1) + L_out) h1 prec BS / BW with L_in + 1 = context
        work = isv.IsvWorkload(B, off["ctx"] - 1, 2)
        t_attn = isv.isv_attention_flops_decode(B, off["ctx"], h1) / flops
        full = isv.isv_predict(model, work, isv.IsvInstance(288e9, 1.0, flops, off["link_gbps_measured"] * 1e9,
                                                            off["link_gbps_measured"] * 1e9, 1, 0, 1, 0), c_off, True)
        t_trans = full["t_trans_dec"]
        cd = alpha * t_attn + beta
        overlap_ms = L * max(cd, t_trans) * 1e3
        summed_ms = L * (cd + t_trans) * 1e3
        res["offload_prediction"] = {
            "c_off": c_off, "t_trans_per_layer_ms": t_trans * 1e3, "ctcf_attention_per_layer_ms": cd * 1e3,
            "predicted_ms_per_step_overlap": overlap_ms, "predicted_ms_per_step_eq6_sum": summed_ms,
            "measured_ms_per_step": off["ms_per_step"],
            "rel_err_overlap": abs(overlap_ms - off["ms_per_step"]) / off["ms_per_step"],
        }
        log(f"[bench] model on the offloaded leg: predicted {overlap_ms:.1f} ms/step with overlap ({summed_ms:.1f} as the "
            f"sum of Eq. 6), measured {off['ms_per_step']:.1f}")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (0 = the workload's own count)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3_resident", "cfg4", "gqa8", "gqa16", "kv8", "kv4", "kv2"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--split-tokens", type=int, default=0,
                    help="resident leg: upper bound on the keys of one work item (0 = the library chooses)")
    ap.add_argument("--layers", type=int, default=0,
                    help="run only this many layers of the stack (counter runs: per-launch figures do not "
                         "depend on the depth); 0 = the workload's own depth")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--no-offload", action="store_true", help="skip every offloaded leg")
    ap.add_argument("--no-layers", action="store_true", help="skip the whole-layer offloaded leg")
    ap.add_argument("--offload-workload", default="cfg3", choices=["cfg3", "cfg5"])
    ap.add_argument("--offload-steps", type=int, default=0)
    ap.add_argument("--offload-batch", type=int, default=0)
    ap.add_argument("--staging", type=int, default=0, help="staging buffers (1..4); 0 = 2")
    ap.add_argument("--no-blocks", action="store_true", help="skip the block-granular offloaded leg")
    ap.add_argument("--no-tails", action="store_true",
                    help="block-granular leg: store every appended row through the mapped pointer instead of keeping "
                         "the newest blocks in HBM")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the legs of the other named workloads (cfg2 in full, cfg4, cfg1)")
    ap.add_argument("--no-cfg5", action="store_true", help="skip the offline large-batch offloaded leg")
    ap.add_argument("--settle", type=float, default=6.0,
                    help="seconds a leg with copies waits before its timed region when the leg before it has just "
                         "released its buffers (legs without copies wait 2 s at most); 0 = never")
    ap.add_argument("--no-model", action="store_true", help="skip the prediction-model leg")
    ap.add_argument("--no-decoder", action="store_true", help="skip the whole-decoder-layer leg")
    ap.add_argument("--layer-steps", type=int, default=32, help="decoder-layer leg: decode steps to time")
    ap.add_argument("--decoder-workload", default="cfg2", choices=["cfg2", "cfg3_resident", "cfg4", "gqa8"],
                    help="decoder-layer leg: the stack and batch it runs on (all resident)")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill-side store leg")
    ap.add_argument("--prefill-table", default="ordered", choices=["ordered", "shuffled"],
                    help="prefill leg: how the block table hands out blocks")
    ap.add_argument("--standin-gib", type=int, default=8,
                    help="prefill leg: bytes one kernel of the stand-in computation reads")
    ap.add_argument("--chunk-mib", type=int, default=256, help="block-granular leg: size of a streamed chunk")
    ap.add_argument("--placement", default="prefix", choices=["prefix", "sequence", "scatter"],
                    help="block-granular leg: which blocks of a sequence live on the host")
    ap.add_argument("--probe", action="store_true",
                    help="also run the plain copy / read kernels on 1 GiB (the yardstick for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; there is no multi-GPU path (--gpus 1 only)")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    _SETTLE["seconds"] = args.settle
    res, cpu = run_resident(args)
    probe = run_probe() if args.probe else None
    # the other named workloads, each at its own size whatever --steps says
    extra = {}
    if not args.no_configs:
        if not (args.workload == "cfg2" and res["steps"] >= 512 and not args.layers):
            extra["cfg2_full"], _ = run_resident(args, "cfg2", steps=512, with_cpu=False, layers=0)
        extra["cfg4"], _ = run_resident(args, "cfg4", steps=20, with_cpu=False, layers=0)
        extra["cfg1"] = run_latency(args)
        # 8, 4 and 2 KV heads at the same KV bytes per layer: what the pool layout's slabs of several tiles buy
        extra["few_kv_heads"] = {w: run_resident(args, w, steps=8, with_cpu=False, layers=0)[0] for w in ("kv8", "kv4", "kv2")}
    off = None if (args.no_offload or args.no_layers) else run_offload(args)
    off_blocks = None if (args.no_offload or args.no_blocks) else run_offload_blocks(args)
    if not (args.no_offload or args.no_cfg5):
        B5, why = cfg5_batch()
        leg = run_offload(args, "cfg5", B=B5, steps=2, warmup=1)
        leg.update(why)
        leg["note"] = (f"batch {B5} of the workload's {why['full_batch']}: at the full batch the host share is "
                       f"{why['full_batch_pinned_gib']:.0f} GiB of pinned memory; this box has {why['host_ram_gib']:.0f} GiB of RAM "
                       f"but hipHostMalloc is refused beyond {why['pinnable_gib_measured']:.0f} GiB (measured just before the leg); "
                       f"the per-sequence shape, the plan (20 of 32 layers on the host) and the depth are the workload's own")
        extra["cfg5_shape"] = leg
    prefill = None if (args.no_offload or args.no_prefill) else run_prefill(args)
    model = None if args.no_model else run_model(args, off)
    layers = None if args.no_decoder else run_layers(args)
    part = "" if res["steps"] >= res["workload_steps"] else (
        f" (steps {res['first_step']}..{res['first_step'] + res['steps'] - 1} of its {res['workload_steps']}: the middle of the "
        f"generation, where the mean context is the workload's mean)")
    line = {
        "metric": "decode_attn_tokens_per_s", "value": res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": res["steps"], "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}{part}: {res['L']} layers, {res['H']} q heads / {res['G']} kv heads x {res['d']}, "
                               f"batch {res['B']}, context {res['ctx_desc']}, fp16 KV "
                               f"{'paged T=%d' % res['T'] if res['T'] else 'contiguous'}, all resident",
                   "split_tokens": res["split_tokens"],
                   "arithmetic": "fp16 K/V/q and softmax weights into the matrix cores, fp32 accumulation and softmax"},
        "kv_gbps": res["kv_gbps"], "hbm_frac": res["kv_gbps"] / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": res["kernel_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": res["kernel_gbps"] / HBM_PEAK_GBPS,
                     "traffic": recorded_traffic(args.workload, res["kv_bytes_per_launch"]),
                     "kernel": "attn_split_mfma_kernel",
                     "avg_us": res["kernel_avg_us"],
                     "launches": res["kernel_launches"], "bytes_per_launch": res["kv_bytes_per_launch"]},
        "cpu_baseline": cpu,
        "offload": off,
        "offload_blocks": off_blocks,
        "prefill_store": prefill,
        "model": model,
        "decoder_layers": layers,
    }
    line.update(extra)
    if probe:
        line["probe"] = probe
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
