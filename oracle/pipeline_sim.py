"""Replay of a copy / append / attend op trace on a fake copy engine (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

When part of the KV cache lives in host memory it has to be brought back to
the GPU before the attention that reads it can run (paper §II-B, §IV-C
Case 2).  The library does this through a small number of staging buffers fed
by copy streams while a compute stream attends.  The unit that is streamed is
a *chunk*: either a whole layer's pool (then the layer has one chunk) or a
run of consecutive blocks of the layer's host pool (then a layer has several
chunks and, possibly, a share of blocks that never leaves HBM).  The library
can emit, without touching a GPU, the exact sequence of operations it would
enqueue; this module replays such a sequence with arbitrary (random)
durations and checks that no ordering of completions allowed by the
stream/event semantics can read or overwrite the wrong data.

Trace format: a list of 7-tuples (kind, step, layer, chunk, buf, copy_idx, wait_idx)
  kind 0 COPY     copy stream:    wait consumed[wait_idx] (if >= 0), copy chunk
                                  `chunk` of the host pool of `layer` into
                                  staging `buf`, then signal ready[copy_idx]
  kind 1 APPEND   compute stream: this step's K/V rows of `layer` are handed to
                                  the attention launches of the layer that
                                  follow (nothing is enqueued)
  kind 2 ATTN     compute stream: wait ready[wait_idx] (if >= 0); attention of
                                  `layer` over the keys held in chunk `chunk`,
                                  read from staging `buf` (chunk = -1, buf = -1:
                                  the keys whose blocks stay in HBM).  The
                                  launch that meets a sequence's newest
                                  position stores the step's rows into the
                                  pool it reads and, for a staged chunk, into
                                  that chunk of the host pool.
  kind 3 RELEASE  compute stream: signal consumed[copy_idx]
  kind 4 MERGE    compute stream: combine the layer's partial results
Stream semantics: each stream runs its ops in issue order, one at a time; a
wait holds the stream until the event has fired; an event fires when every
op issued to its stream before the signal has finished.  Waiting on an event
whose signal has not been issued yet does not wait at all, so a trace that
does so is rejected.  Copies into different staging buffers are taken to be
on different streams (the library uses two copy streams, by buffer parity:
an ordering between buffers that the replay does not assume can only make the
library safer than what is checked here).
"""
import random

COPY, APPEND, ATTN, RELEASE, MERGE = 0, 1, 2, 3, 4


class Hazard(Exception):
    pass


def _union_length(intervals):
    total, end = 0.0, None
    for lo, hi in sorted(intervals):
        if end is None or lo > end:
            total += hi - lo
            end = hi
        elif hi > end:
            total += hi - end
            end = hi
    return total


def replay(trace, host_chunks, has_resident=None, seed=0, copy_scale=1.0, compute_scale=1.0):
    """Simulate the trace; raise Hazard on the first violation, else return a
    dict with the makespan and the busy time of the copy engine.

    host_chunks[l]   number of streamed chunks of layer l (0: all of it in HBM)
    has_resident[l]  1 if layer l has keys in HBM (default: layers without chunks)
    """
    n_layers = len(host_chunks)
    if has_resident is None:
        has_resident = [1 if host_chunks[l] == 0 else 0 for l in range(n_layers)]
    rng = random.Random(seed)
    free = {"compute": 0.0}
    ready, consumed = {}, {}
    ops = []              # dicts: kind, step, layer, chunk, buf, cidx, widx, start, finish, pos
    for pos, (kind, step, layer, chunk, buf, cidx, widx) in enumerate(trace):
        gate = 0.0
        if kind == COPY:
            stream, dur = f"copy{buf}", copy_scale * rng.uniform(0.5, 1.5)
            if widx >= 0:
                if widx not in consumed:
                    raise Hazard(f"copy {cidx} waits on consumed[{widx}] before it was signalled")
                gate = consumed[widx]
        elif kind == APPEND:
            stream, dur = "compute", 0.0
        elif kind == ATTN:
            stream, dur = "compute", compute_scale * rng.uniform(0.5, 1.5)
            if widx >= 0:
                if widx not in ready:
                    raise Hazard(f"attention waits on ready[{widx}] before its copy was issued")
                gate = ready[widx]
        elif kind == RELEASE:
            stream, dur = "compute", 0.0
        elif kind == MERGE:
            stream, dur = "compute", compute_scale * rng.uniform(0.01, 0.1)
        else:
            raise Hazard(f"unknown op kind {kind}")
        start = max(free.get(stream, 0.0), gate)
        finish = start + dur
        free[stream] = finish
        if kind == COPY:
            ready[cidx] = finish
        if kind == RELEASE:
            consumed[cidx] = finish
        ops.append(dict(kind=kind, step=step, layer=layer, chunk=chunk, buf=buf, cidx=cidx, widx=widx,
                        start=start, finish=finish, pos=pos))

    # ---- data checks -----------------------------------------------------
    copies = [o for o in ops if o["kind"] == COPY]
    by_cidx = {}
    for c in copies:
        if c["cidx"] in by_cidx:
            raise Hazard(f"copy index {c['cidx']} used twice")
        by_cidx[c["cidx"]] = c
    n_steps = 1 + max((o["step"] for o in ops if o["kind"] in (APPEND, ATTN)), default=-1)
    attn_of = {}
    for o in ops:
        if o["kind"] == ATTN:
            key = (o["step"], o["layer"], o["chunk"])
            if key in attn_of:
                raise Hazard(f"step {o['step']} layer {o['layer']} chunk {o['chunk']}: attended twice")
            attn_of[key] = o
    for step in range(n_steps):
        for layer in range(n_layers):
            app = [o for o in ops if o["kind"] == APPEND and o["step"] == step and o["layer"] == layer]
            mer = [o for o in ops if o["kind"] == MERGE and o["step"] == step and o["layer"] == layer]
            if len(app) != 1 or len(mer) != 1:
                raise Hazard(f"step {step} layer {layer}: {len(app)} appends, {len(mer)} merges")
            app, mer = app[0], mer[0]
            want = ([-1] if has_resident[layer] else []) + list(range(host_chunks[layer]))
            have = sorted(c for (s, l, c) in attn_of if s == step and l == layer)
            if have != sorted(want):
                raise Hazard(f"step {step} layer {layer}: attention over chunks {have}, expected {want}")
            for chunk in want:
                att = attn_of[(step, layer, chunk)]
                if not (app["pos"] < att["pos"] < mer["pos"]):
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: attention not between "
                                 f"the layer's append and merge")
                if chunk < 0:
                    if att["buf"] >= 0 or att["widx"] >= 0:
                        raise Hazard(f"step {step} layer {layer}: HBM-resident keys read through staging")
                    continue
                buf = att["buf"]
                if buf < 0:
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: no staging buffer")
                mine = by_cidx.get(att["widx"])
                if mine is None:
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: attention does not wait for a copy")
                if mine["buf"] != buf or mine["layer"] != layer or mine["chunk"] != chunk:
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: waits for copy {mine['cidx']} "
                                 f"of layer {mine['layer']} chunk {mine['chunk']} into staging {mine['buf']}")
                into = [c for c in copies if c["buf"] == buf]
                before = [c for c in into if c["finish"] <= att["start"]]
                if not before:
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: staging {buf} read before any copy finished")
                src = max(before, key=lambda c: c["finish"])
                if src is not mine:
                    raise Hazard(f"step {step} layer {layer} chunk {chunk}: staging {buf} holds copy "
                                 f"{src['cidx']} instead of {mine['cidx']}")
                if step > 0:
                    prev = attn_of[(step - 1, layer, chunk)]
                    if src["start"] < prev["finish"]:
                        raise Hazard(f"step {step} layer {layer} chunk {chunk}: copy read the host pool "
                                     f"before the previous step's rows had landed")
                for c in into:
                    if c is src:
                        continue
                    if c["start"] < att["finish"] and c["finish"] > src["finish"]:
                        raise Hazard(f"step {step} layer {layer} chunk {chunk}: staging {buf} overwritten "
                                     f"by copy {c['cidx']} while still in use")
    spans = [(c["start"], c["finish"]) for c in copies]
    return {"makespan": max(free.values()), "copy_busy": _union_length(spans),
            "copy_span": (max((c["finish"] for c in copies), default=0.0)
                          - min((c["start"] for c in copies), default=0.0))}
