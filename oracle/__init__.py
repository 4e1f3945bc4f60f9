"""CPU oracle for the paged-KV decode and KV-reclamation path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 / exact-integer definitions of
what the GPU library computes, written from the paper's problem statement
(Section 2.3 "Challenges", Section 3, Section 5) and from the textbook
definition of softmax attention.  Nothing here is imported by the product
package, and nothing here imports it; the two share no code.  Only the test
suite, the smoke check and the CPU-baseline leg of the benchmark call it.

Modules
-------
attention : fp64 decode attention over a contiguous copy of the paged KV
plan      : split of a decode batch into work items and bounded slices
reclaim   : relocation of live blocks out of a range + block-table rewrite
policy    : selective handle choice (Algorithm 1), MIAD headroom, cooldown gate

Pins (see tests/): attention is pinned by a pure-Python scalar brute force, by
a library fp64 scaled-dot-product routine, by closed forms and invariances;
reclamation by a dictionary-based simulator and by conservation invariants;
Algorithm 1 by exhaustive enumeration of its greedy choice on small instances.
The pairing rule of relocation (i-th live source, ascending, goes to the i-th
free destination, ascending) and the pool layout are choices of this library,
not of the paper: for them parity is oracle-defined (pinned only by the
brute-force simulator and the invariants), i.e. "parity unpinned" by the paper.
"""
