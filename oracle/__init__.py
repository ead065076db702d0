"""CPU ORACLE -- test infrastructure only.

A plain, slow, independent implementation of what the tree-attention hot path computes, written
from the paper's definitions.  Only tests, the smoke check and the bench's cpu_baseline leg may
import this package; the product path never does.  It shares no code with the HIP library.

  meta.py              DFS serialisation (Eq. 8), node ranges, path counts g_n and K, position ids
                       (Eq. 9, partition offset eq. pos_offset_child), loss weights g/K (Eq. 4),
                       visibility bounds, the three statements of the attention mask.
  branch_attention.c   per-branch causal attention forward/backward + scatter-sum (Eq. 1, 5, 6).
  attention.py         ctypes front end of the C file; dense-mask attention for tiny inputs.
  loss.py              log-softmax / gather / weighting in fp64; Eq. 1 and Eq. 4 forms of the loss.
  build.py             compiles branch_attention.c with gcc (fp64 and fp32 arithmetic variants).

Pins: see tests/test_oracle_*.py.  No function here is "parity unpinned".
"""
