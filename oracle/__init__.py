"""CPU oracle for decoupled data-parallel training with stale gradients.

TEST INFRASTRUCTURE ONLY. This package is the slow, plain reference that the HIP
library is checked against; it is imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product path. It shares no code with the
HIP library and does not import it.

Everything is fp64 on the CPU (torch CPU tensors are used as an array library:
matmul/einsum/indexing; no autograd, no nn modules).

Pins (tests/test_oracle_*.py): finite differences, brute-force loops on tiny shapes,
torch.autograd on the same functions, reduction to plain SGD for K=1/W=1, equality
of the W-replica mean with the concatenated-batch gradient, agreement of the
pipelined recurrence with the definition form evaluated at the skewed weight
vector, warm-up invariants and the consensus lemma for P = (1/S) 1 1^T.

Parity unpinned: absolute loss curves, accuracy and per-mini-batch times of the
paper's experiment section (they need CIFAR-10 and the authors' network/hardware).
"""
