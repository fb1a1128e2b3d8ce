"""fp64 CPU oracle of the swap-rewritten CNN training step.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the CPU-baseline leg
of the benchmark may import this package; it shares no code with the HIP path.

ops       layer arithmetic (textbook definitions; the paper fixes none)
graph     computational graph and topological ordering (Section 3)
rewrite   swap-out / swap-in rewriting and control-edge strategies (Sections 4, 5.1)
model     graph of a workload: forward layers plus reverse-mode backward vertices (Section 3.3)
evaluate  runs a graph vertex by vertex (swap operations are identities, Eq. 2 and Eq. 5)

Parity unpinned: the tensor and operation counts the paper reports for its
TensorFlow graphs (317, 2397, 2779 tensors; 634/687 and 3895/4052 added
operations) and its batch-size and images/s figures depend on graphs and
hardware that are not available; nothing here is pinned to them.
"""
