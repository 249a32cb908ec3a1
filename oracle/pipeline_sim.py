"""Replay of a copy / append / attend op trace on a fake copy engine (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

When part of the KV cache lives in host memory it has to be brought back to
the GPU, layer by layer, before the attention of that layer can run (paper
§II-B, §IV-C Case 2).  The library does this through a small number of
staging buffers fed by a copy stream while a compute stream appends and
attends.  It can emit, without touching a GPU, the exact sequence of
operations it would enqueue; this module replays such a sequence with
arbitrary (random) durations and checks that no ordering of completions
allowed by the stream/event semantics can read or overwrite the wrong data.

Trace format: a list of 6-tuples (kind, step, layer, buf, copy_idx, wait_idx)
  kind 0 COPY     copy stream:    wait consumed[wait_idx] (if >= 0), copy host
                                  pool of `layer` into staging `buf`, then
                                  signal ready[copy_idx]
  kind 1 APPEND   compute stream: wait ready[wait_idx] (if >= 0); write this
                                  step's K/V of `layer` into staging `buf`
                                  and into the host pool (buf < 0: resident
                                  layer, no staging involved)
  kind 2 ATTN     compute stream: attention of `layer` reading staging `buf`
                                  (or the resident pool when buf < 0)
  kind 3 RELEASE  compute stream: signal consumed[copy_idx]
Stream semantics: each stream runs its ops in issue order, one at a time; a
wait holds the stream until the event has fired; an event fires when every
op issued to its stream before the signal has finished.  Waiting on an event
whose signal has not been issued yet does not wait at all, so a trace that
does so is rejected.
"""
import random

COPY, APPEND, ATTN, RELEASE = 0, 1, 2, 3


class Hazard(Exception):
    pass


def replay(trace, on_host, seed=0, copy_scale=1.0, compute_scale=1.0):
    """Simulate the trace; raise Hazard on the first violation, else return
    a dict with the makespan and the busy time of the copy stream."""
    rng = random.Random(seed)
    free = {"copy": 0.0, "compute": 0.0}
    ready, consumed = {}, {}
    ops = []                                  # (kind, step, layer, buf, copy_idx, start, finish)
    for (kind, step, layer, buf, cidx, widx) in trace:
        if kind == COPY:
            stream, dur = "copy", copy_scale * rng.uniform(0.5, 1.5)
            gate = 0.0
            if widx >= 0:
                if widx not in consumed:
                    raise Hazard(f"copy {cidx} waits on consumed[{widx}] before it was signalled")
                gate = consumed[widx]
        elif kind == APPEND:
            stream, dur = "compute", compute_scale * rng.uniform(0.01, 0.1)
            gate = 0.0
            if widx >= 0:
                if widx not in ready:
                    raise Hazard(f"append waits on ready[{widx}] before its copy was issued")
                gate = ready[widx]
            if on_host[layer] and widx < 0:
                raise Hazard(f"append of host layer {layer} does not wait for its copy")
        elif kind == ATTN:
            stream, dur, gate = "compute", compute_scale * rng.uniform(0.5, 1.5), 0.0
        elif kind == RELEASE:
            stream, dur, gate = "compute", 0.0, 0.0
        else:
            raise Hazard(f"unknown op kind {kind}")
        start = max(free[stream], gate)
        finish = start + dur
        free[stream] = finish
        if kind == COPY:
            ready[cidx] = finish
        if kind == RELEASE:
            consumed[cidx] = finish
        ops.append((kind, step, layer, buf, cidx, start, finish))

    # ---- data checks -----------------------------------------------------
    copies = [o for o in ops if o[0] == COPY]
    appends = {(o[1], o[2]): o for o in ops if o[0] == APPEND}
    n_steps = 1 + max((o[1] for o in ops if o[0] in (APPEND, ATTN)), default=-1)
    n_layers = len(on_host)
    for step in range(n_steps):
        for layer in range(n_layers):
            att = [o for o in ops if o[0] == ATTN and o[1] == step and o[2] == layer]
            if len(att) != 1:
                raise Hazard(f"step {step} layer {layer}: {len(att)} attention ops")
            att = att[0]
            app = appends.get((step, layer))
            if app is None or app[6] > att[5]:
                raise Hazard(f"step {step} layer {layer}: attention without a finished append")
            if not on_host[layer]:
                if att[3] >= 0 or app[3] >= 0:
                    raise Hazard(f"resident layer {layer} uses a staging buffer")
                continue
            buf = att[3]
            if buf < 0 or app[3] != buf:
                raise Hazard(f"step {step} host layer {layer}: append/attention buffers differ")
            into = [c for c in copies if c[3] == buf]
            before = [c for c in into if c[6] <= att[5]]
            if not before:
                raise Hazard(f"step {step} layer {layer}: staging {buf} read before any copy finished")
            src = max(before, key=lambda c: c[6])
            if src[2] != layer:
                raise Hazard(f"step {step} layer {layer}: staging {buf} holds layer {src[2]}")
            if step > 0:
                prev = appends[(step - 1, layer)]
                if src[5] < prev[6]:
                    raise Hazard(f"step {step} layer {layer}: copy read the host pool before "
                                 f"the previous step's append had landed")
            if app[5] < src[6]:
                raise Hazard(f"step {step} layer {layer}: append wrote staging before the copy ended")
            for c in into:
                if c is src:
                    continue
                if c[5] < att[6] and c[6] > src[6]:
                    raise Hazard(f"step {step} layer {layer}: staging {buf} overwritten by copy "
                                 f"{c[4]} while still in use")
    busy = sum(c[6] - c[5] for c in copies)
    return {"makespan": max(free.values()), "copy_busy": busy,
            "copy_span": (max((c[6] for c in copies), default=0.0)
                          - min((c[5] for c in copies), default=0.0))}
