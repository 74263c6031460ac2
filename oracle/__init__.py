"""CPU oracle for the ahead-of-time multi-stream DAG executor.

TEST INFRASTRUCTURE ONLY. Nothing in the product package imports this; only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg do. It shares no
code with the HIP library: both sides read the same workload descriptions
(package ``workloads``) and nothing else.

Three results are defined here, all written from the paper (Nimble,
arXiv 2012.02732):

* ``forward``  - the tensors a DAG computes. The method only changes *when*
  tasks run (Section 4.1), so this is the plain definition: nodes evaluated in
  ascending id (a topological order), each operator by its textbook formula,
  fp32 storage, fp64 arithmetic inside an operator.
* ``schedule`` - Algorithm 1 (Section 4.2) followed step by step, plus the
  synchronisation plan of Appendix A, with every free choice fixed.
* ``backward`` - (module ``backward``; no HIP counterpart yet) the gradients of a
  DAG and a plain SGD update, the computation a recorded training iteration
  (Section 5) would have to reproduce; pinned by central differences of an fp64
  forward pass and by torch.autograd on CPU.

Parity status: operator formulas are pinned against closed forms, pure-Python
brute force and torch.nn.functional on CPU; the schedule is pinned by the
paper's theorems (Theorem 3 closed form, Theorem 4 by brute force over all
partitions, Lemma 1, Lemma 4), by brute-force maximum antichains and by
hand-derived vectors. The particular maximum matching picked among equally
good ones (tie-break order) is a convention: "parity unpinned" for that choice
alone.
"""
