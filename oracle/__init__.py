"""CPU oracle for one pipeline stage's training step and for the partition solver.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
HIP library is checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product package never does,
and nothing here imports the product package.

Everything is written out from the definitions: convolution as a sum over
kernel taps of a shifted input times a weight slice, batch normalisation with
batch statistics, the exact adjoints for the backward pass, the SGD-momentum
recurrence, and for the solver the dynamic programme of the paper's section
"Dynamic Model Partition".  Arithmetic is float64 by default (dtype is an
argument so the same code can be timed in float32).
"""
