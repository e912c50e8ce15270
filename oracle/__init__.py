"""CPU oracle for the per-edge-bucket training step of Legend (arXiv 2505.09258).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 restatement of
what the bucket step computes, written from the paper (Sec. 2.1, Eq. 1, Sec. 3,
Sec. 4 Alg. 1/2, Sec. 6) and from the readings listed in the design notes.  It
shares no code with the HIP library and must never be imported by the product
package: only the tests, the smoke check and the benchmark's CPU-baseline leg
call it.

Pins (see tests/test_oracle_*.py): splitmix64 published vectors, big-integer
mulhi, closed forms on hand-built 3-node graphs, float64 finite differences,
torch.autograd on Eq. 1 written out directly, dense torch.optim.Adagrad, the
n = 6 worked example of Sec. 4 and the state counts of Table 6.

The whole-bucket result has no printed worked example in the paper: its parity
is pinned only through the pins of its parts.
"""
