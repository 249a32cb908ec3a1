"""GPU parity for pool layouts whose slabs hold several 16-token tiles (fewer KV heads than fill 32 KiB with one
tile: St > 1).  Outputs against the fp64 oracle at the usual tolerance, appended rows and the pools bit for bit,
also through the slots that keep the newest blocks of offloaded sequences in HBM."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import kv_layout
from paper_2504_11816_amd import binding

from gpu_util import build_stack, make_inputs, run_and_check
from test_gpu_block_classes import classed_stack, oracle_outputs, poison_staging

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


SHAPES = [(32, 4, 128, 64), (32, 2, 128, 64), (16, 1, 128, 128), (16, 8, 64, 32), (8, 2, 128, 256), (32, 4, 128, 0),
          (4, 1, 64, 0), (24, 3, 64, 64)]
# (H, G, d, T): 2, 4, 8, 2, 4 tiles per slab; contiguous pools of 2 and 16; three KV heads (24 KiB runs)


@pytest.mark.parametrize("H,G,d,T", SHAPES)
def test_outputs_and_appended_rows(H, G, d, T):
    ctx = np.array([0, 15, 16, 63, 64, 130, 300, 511], dtype=np.int32)
    st = build_stack(L=2, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=528, seed=950)
    tiles = binding.okv_slab_tiles(G, d, T if T else st.max_ctx)
    say(f"slabs H={H} G={G} d={d} T={T}: {tiles} tiles per slab")
    assert tiles > 1 and tiles == kv_layout.slab_tiles(G, d, T if T else st.max_ctx)
    want = [st.read_pool(l) for l in range(2)]
    n = ctx.copy()
    for step in range(3):
        q, k, v, out = make_inputs(st, 952, step, st.device)
        st.step(q, k, v, out)
        st.synchronize()
        n += 1
        for l in range(2):
            kv_layout.append_scatter(want[l], st.layout(), n, k[l].cpu().numpy(), v[l].cpu().numpy())
            np.testing.assert_array_equal(st.read_pool(l).view(np.uint16), want[l].view(np.uint16))
    run_and_check(st, n_steps=2, seed=954)
    st.close()


@pytest.mark.parametrize("G,d,T", [(2, 128, 64), (4, 128, 32), (1, 64, 256)])
def test_newest_blocks_in_hbm_with_slabs_of_several_tiles(G, d, T):
    # the kernel that moves rows between the slots and the staged chunks or the host pool finds a row's
    # position from its place in the block: here with 4, 2 and 16 tiles per slab
    say(f"slabs: tails G={G} d={d} T={T}")
    from gpu_util import assert_close
    H, L = 2 * G, 2
    ctx = np.array([0, T - 1, T, 2 * T - 3, T // 2], dtype=np.int32)
    st = classed_stack(L=L, H=H, G=G, d=d, T=T, ctx_before=ctx, cap_tokens=4 * T, c_off=Fraction(3, 5), chunk_blocks=3,
                       policy="scatter", seed=961, workspace_items=5 * 8)
    assert st.hot_tails and binding.okv_slab_tiles(G, d, T) > 1
    st.tail_blocks.fill_(0xFF)
    poison_staging(st)
    want = [st.read_pool(l) for l in range(L)]
    layout = st.layout()
    n = ctx.copy()
    for step in range(T + 6):
        q, k, v, out = make_inputs(st, 963, step, st.device)
        st.step(q, k, v, out)
        st.synchronize()
        n += 1
        for l in range(L):
            kv_layout.append_scatter(want[l], layout, n, k[l].cpu().numpy(), v[l].cpu().numpy())
            if step % 5 == 0 or step >= T:
                ref = oracle_outputs(want[l], layout, q[l].cpu().numpy(), n, H, G)
                assert_close(out[l].float().cpu().numpy().reshape(-1, d), ref.reshape(-1, d), f"step {step} layer {l}")
    for l in range(L):
        np.testing.assert_array_equal(st.read_pool(l).view(np.uint16), want[l].view(np.uint16))
    st.close()
