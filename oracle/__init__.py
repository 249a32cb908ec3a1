"""CPU oracle for offloaded-KV decode attention.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory: it exists so that the tests, the smoke check and the CPU-baseline
leg of the benchmark have a slow, plain, obviously-correct statement of what
the GPU path must compute.  It shares no code with the HIP library and never
calls it.  Floating point is fp64 on the exact values of the fp16 inputs.

Modules
  attention     softmax(q K^T / sqrt(d)) V for one decode step, contiguous or
                paged KV, MHA or grouped query heads
  kv_layout     element offsets of a K/V row in a contiguous or paged pool and
                the scatter that one append performs
  offload_plan  which layers leave the GPU for an offload ratio C_off
  kv_bytes      the paper's size / flop / transfer-time formulas
  worklist      the tiling a split-K work list has to satisfy
  pipeline_sim  replay of a copy/attend op trace on a fake copy engine
  tail_sim      replay of "newest blocks stay in HBM" on sets of row positions

Every function here is pinned by a CPU test (tests/test_oracle_*.py) to a
closed form, an invariant, a library routine on a special case or brute
force; none is "parity unpinned".
"""
