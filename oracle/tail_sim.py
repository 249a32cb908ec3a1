"""A model of block-granular offload with the sequences' newest blocks kept in HBM (oracle side).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

Paper §IV-C keeps a share of the KV cache in host memory and §IV-D moves it to the GPU for every decode
step; which appended rows travel back when is left open.  The library's reading: a row appended to a block
of the HOST pool goes into a slot in HBM (two slots per sequence and layer, block j uses slot j % 2) and
into the staged copy that the step attends; the block is written to the host pool once, after the step
that fills it.  A staged copy is a snapshot of the host pool taken when its copy ran, which may be as
early as one step before its use, so it can lack rows; before a chunk is attended the rows
[tail_from, n - 1) of every sequence's newest and second-newest block are copied into it from their slots
if the plan says the chunk needs it.

This module replays that protocol on sets of row positions: no data, no arithmetic of the method.  It
takes the per-step decisions (which chunks to patch, which sequences' blocks to write out) from a plan
function -- the library's, or expected_plan below, which states the rule in the words above -- and checks
that every chunk's attention sees exactly the rows its blocks hold, that a slot is never reused before its
block was written out, and that the host pool is complete after a final write-out.
"""
import numpy as np


def expected_plan(table, T, n_after, tail_from, resident, chunk, n_chunks):
    """(patch_chunk [n_chunks], fills_block [B]) for the step after which the sequences hold n_after keys."""
    B = len(n_after)
    patch = np.zeros(n_chunks, dtype=np.uint8)
    fills = np.zeros(B, dtype=np.uint8)
    for b in range(B):
        n, t0 = int(n_after[b]), int(tail_from[b])
        newest = (n - 1) // T
        for j in (newest - 1, newest):
            if j < 0 or (j + 1) * T <= t0:            # no position of this block was appended by this batch
                continue
            blk = int(table[b][j])
            if blk >= resident:
                patch[(blk - resident) // chunk] = 1
        if n % T == 0 and t0 < n and int(table[b][n // T - 1]) >= resident:
            fills[b] = 1
    return patch, fills


class ProtocolError(AssertionError):
    pass


def replay(table, T, ctx_before, resident, chunk, n_chunks, steps, plan, lag=1, rng=None):
    """Run `steps` decode steps of the model.  plan(n_after, tail_from) -> (patch_chunk, fills_block).
    lag: how old the snapshot a staged chunk holds may be, in steps (1: the copy ran before the previous
    step's write-out; 0: after it); with rng every chunk draws its own lag in [0, lag].
    Raises ProtocolError on the first violation; returns the number of (chunk, step) attentions checked."""
    table = np.asarray(table)
    B = table.shape[0]
    n = np.asarray(ctx_before, dtype=np.int64).copy()
    tail_from = n.copy()

    def chunk_of(blk):
        return (blk - resident) // chunk

    # rows (positions inside the sequence) that the host pool holds, per (sequence, block index)
    host = {}
    for b in range(B):
        for j in range((int(n[b]) + T - 1) // T):
            if table[b][j] >= resident:
                host[(b, j)] = set(range(j * T, min((j + 1) * T, int(n[b]))))
    slots = [[(None, set()), (None, set())] for _ in range(B)]
    states = [{k: set(v) for k, v in host.items()}]           # states[t]: the host pool before step t
    checked = 0
    for s in range(steps):
        n += 1
        patch, fills = plan(n.copy(), tail_from.copy())
        new_rows = {}
        for b in range(B):
            p = int(n[b]) - 1
            j = p // T
            if table[b][j] < 0:
                raise ProtocolError(f"step {s}: sequence {b} has no block for position {p}")
            if table[b][j] >= resident:
                held, rows = slots[b][j % 2]
                if held != j:
                    if held is not None:
                        want = set(range(max(held * T, int(tail_from[b])), (held + 1) * T))
                        if not want <= host.get((b, held), set()):
                            raise ProtocolError(f"step {s}: slot of sequence {b} reused before block {held} was written out")
                    slots[b][j % 2] = (j, set())
                new_rows[b] = (j, p)
        for c in range(n_chunks):
            age = lag if rng is None else int(rng.integers(0, lag + 1))
            snap = states[max(0, len(states) - 1 - age)]
            staged = {k: set(v) for k, v in snap.items() if chunk_of(table[k[0]][k[1]]) == c}
            if patch[c]:
                for b in range(B):
                    newest = (int(n[b]) - 1) // T
                    for j in (newest - 1, newest):
                        if j < 0 or table[b][j] < resident or chunk_of(table[b][j]) != c:
                            continue
                        lo, hi = max(j * T, int(tail_from[b])), min((j + 1) * T, int(n[b]) - 1)
                        if lo >= hi:
                            continue
                        held, rows = slots[b][j % 2]
                        if held != j or not set(range(lo, hi)) <= rows:
                            raise ProtocolError(f"step {s} chunk {c}: rows [{lo}, {hi}) of sequence {b} are not in their slot")
                        staged.setdefault((b, j), set()).update(range(lo, hi))
            for b, (j, p) in new_rows.items():               # the attention launch stores the step's row itself
                if chunk_of(table[b][j]) == c:
                    staged.setdefault((b, j), set()).add(p)
            for b in range(B):
                for j in range((int(n[b]) + T - 1) // T):
                    if table[b][j] >= resident and chunk_of(table[b][j]) == c:
                        want = set(range(j * T, min((j + 1) * T, int(n[b]))))
                        if staged.get((b, j), set()) != want:
                            missing = sorted(want - staged.get((b, j), set()))
                            raise ProtocolError(f"step {s} chunk {c}: sequence {b} block {j} lacks rows {missing[:4]}")
                        checked += 1
        for b, (j, p) in new_rows.items():
            slots[b][j % 2][1].add(p)
        for b in range(B):
            if fills[b]:
                if int(n[b]) % T:
                    raise ProtocolError(f"step {s}: write-out of sequence {b} asked for although no block is full")
                j = int(n[b]) // T - 1
                lo = max(j * T, int(tail_from[b]))
                held, rows = slots[b][j % 2]
                if table[b][j] < resident or held != j or not set(range(lo, (j + 1) * T)) <= rows:
                    raise ProtocolError(f"step {s}: write-out of block {j} of sequence {b} reads a slot that does not hold it")
                host.setdefault((b, j), set()).update(range(lo, (j + 1) * T))
        states.append({k: set(v) for k, v in host.items()})
    # the final write-out of what is left in the slots, then the pools must be complete
    for b in range(B):
        j = (int(n[b]) - 1) // T
        if n[b] > 0 and table[b][j] >= resident:
            lo = max(j * T, int(tail_from[b]))
            held, rows = slots[b][j % 2]
            if lo < int(n[b]):
                if held != j or not set(range(lo, int(n[b]))) <= rows:
                    raise ProtocolError(f"final write-out: slot of sequence {b} does not hold block {j}")
                host.setdefault((b, j), set()).update(range(lo, int(n[b])))
    for b in range(B):
        for j in range((int(n[b]) + T - 1) // T):
            if table[b][j] >= resident:
                want = set(range(j * T, min((j + 1) * T, int(n[b]))))
                if host.get((b, j), set()) != want:
                    raise ProtocolError(f"after the final write-out the host pool lacks rows of sequence {b} block {j}")
    return checked
