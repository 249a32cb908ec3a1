"""The model of "newest blocks stay in HBM" (oracle/tail_sim.py): accepts the rule as stated for every
placement and staging age, and notices each way of getting it wrong."""
import numpy as np
import pytest

from oracle import tail_sim
from paper_2504_11816_amd import synth


def case(seed, policy, T=16, B=7, cap=160, share=(3, 5), chunk=4):
    rng = np.random.default_rng(seed)
    need = B * (cap // T)
    n_host = -(-need * share[0] // share[1])
    resident = need - n_host + 2
    table = synth.classed_block_table([cap] * B, T, resident, n_host + 3, n_host, policy, seed + 1, max_blocks_per_seq=cap // T)
    ctx = rng.integers(0, cap - 70, size=B).astype(np.int32)
    n_chunks = -(-(n_host + 3) // chunk)
    return table, T, ctx, resident, chunk, n_chunks


def plan_of(table, T, resident, chunk, n_chunks):
    return lambda n, t0: tail_sim.expected_plan(table, T, n, t0, resident, chunk, n_chunks)


@pytest.mark.parametrize("policy", ["prefix", "sequence", "scatter"])
def test_the_stated_rule_serves_every_chunk_its_rows(policy):
    for seed in range(6):
        table, T, ctx, resident, chunk, n_chunks = case(seed, policy)
        for lag, rng in ((0, None), (1, None), (1, np.random.default_rng(seed))):
            checked = tail_sim.replay(table, T, ctx, resident, chunk, n_chunks, 66, plan_of(table, T, resident, chunk, n_chunks), lag, rng)
            assert checked > 0 or policy == "prefix"


def test_hand_case():
    # one sequence, blocks of 16, every block on the host in chunks of 2 blocks; 14 keys at the start
    table = np.array([[0, 1, 2, 3]], dtype=np.int32)
    plan = plan_of(table, 16, 0, 2, 2)
    patch, fills = plan(np.array([15]), np.array([14]))       # the step that stores position 14
    assert patch.tolist() == [1, 0] and fills.tolist() == [0]
    patch, fills = plan(np.array([16]), np.array([14]))       # ... position 15: block 0 is full
    assert patch.tolist() == [1, 0] and fills.tolist() == [1]
    patch, fills = plan(np.array([17]), np.array([14]))       # block 1 is the newest, block 0 the one before: both in chunk 0
    assert patch.tolist() == [1, 0] and fills.tolist() == [0]
    patch, fills = plan(np.array([33]), np.array([14]))       # newest block 2 (chunk 1), the one before is block 1 (chunk 0)
    assert patch.tolist() == [1, 1]
    patch, fills = plan(np.array([49]), np.array([14]))       # newest block 3, before it block 2: chunk 1 only
    assert patch.tolist() == [0, 1]
    patch, fills = plan(np.array([32]), np.array([32]))       # 32 keys, all of them there when the batch was described
    assert patch.tolist() == [0, 0] and fills.tolist() == [0]
    assert tail_sim.replay(table, 16, [14], 0, 2, 2, 40, plan, lag=1) > 0


def test_planted_mistakes_are_noticed():
    table, T, ctx, resident, chunk, n_chunks = case(3, "scatter")
    good = plan_of(table, T, resident, chunk, n_chunks)
    tail_sim.replay(table, T, ctx, resident, chunk, n_chunks, 50, good, 1)

    def never_patch(n, t0):
        p, f = good(n, t0)
        return np.zeros_like(p), f

    def newest_block_only(n, t0):                            # forgets the block before the newest
        B = len(n)
        p = np.zeros(n_chunks, dtype=np.uint8)
        for b in range(B):
            j = (int(n[b]) - 1) // T
            if table[b][j] >= resident and (j + 1) * T > t0[b]:
                p[(table[b][j] - resident) // chunk] = 1
        return p, good(n, t0)[1]

    def never_write_out(n, t0):
        p, f = good(n, t0)
        return p, np.zeros_like(f)

    def write_out_a_step_late(n, t0):
        p, _ = good(n, t0)
        _, f = good(n - 1, t0)
        return p, f

    for bad in (never_patch, newest_block_only, never_write_out, write_out_a_step_late):
        with pytest.raises(tail_sim.ProtocolError):
            tail_sim.replay(table, T, ctx, resident, chunk, n_chunks, 50, bad, 1)
    # a staged copy older than the protocol allows (two write-outs behind) is not covered by the patch either
    with pytest.raises(tail_sim.ProtocolError):
        for seed in range(8):
            t2, T2, c2, r2, ch2, nc2 = case(seed, "sequence")
            tail_sim.replay(t2, T2, c2, r2, ch2, nc2, 70, plan_of(t2, T2, r2, ch2, nc2), lag=18)
