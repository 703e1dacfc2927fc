"""CPU oracle for the level-batched Child-Sum Tree-LSTM forward.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product: only the test
suite, the smoke check and the benchmark's CPU-baseline leg may import it.  It
shares no code with the HIP library and never imports it.

Contents
  schedule_oracle.py   heights / level buckets / permutation / child CSR, plus
                       an independent brute-force height routine for tiny trees;
                       schedule_typed: the same table filed by (depth, signature)
  treelstm_oracle.py   node-by-node postorder evaluation in fp64 (numpy)
  treelstm_typed_oracle.py   the same with one cell (weight set) per signature
  treelstm_oracle.c    the same definition in plain C (fp64), one tree at a
                       time; used where the numpy version is too slow
  treelstm_backward_oracle.py   reverse-mode gradients of the same forest, node by
                       node in fp64, and the activations a training forward keeps
  cache_oracle.py      fingerprint of a parent array (the key of the schedule cache) and
                       the cache's replacement policy
  build.py             compiles the C file with gcc

Pins (tests/test_oracle_*.py): brute-force heights, chain / star / perfect
k-ary closed forms, stable-argsort CSR, leaf closed form, chain == library
LSTM, star with U_f = 0 == library LSTM cell on summed child states, saturated
forget gates select children by the sign of their own h, zero-weight closed
form c = i*u*subtree_size, relabelling and forest-vs-single-tree invariance,
numpy oracle vs C oracle; for the gradient oracle: autograd of an independently
written torch forward, a library LSTM differentiated by the library, central
differences of the forward oracle, a one-leaf closed form; for the fingerprint:
the published SplitMix64 stream, hand arithmetic, sensitivity to single edits.  Launch-count tables of the paper (Table 1, Table 2)
need its dataset: parity unpinned, nothing here reproduces them.
"""
