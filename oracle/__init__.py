"""CPU oracle: TEST INFRASTRUCTURE, not part of the product.

A plain, slow, fp64 numpy implementation of the three GNN layers exactly as
the paper defines them, in the ORIGINAL operator order (Scatter -> ApplyEdge ->
ReduceScatter -> Aggregate, every per-edge tensor materialised, everything
stashed for the backward pass).  It exists only so that tests, the smoke check
and the benchmark's cpu_baseline leg have something independent to compare the
HIP library with.  It shares no code with the HIP path and neither imports the
other; only `tests/`, `__graft_entry__.smoke()` and `bench.py`'s cpu_baseline
leg may import it.

Modules
  segments   per-destination reductions over a CSR edge list (library reduceat)
  gat        GAT layer, forward and backward      (App. A.2 "GAT", Sec. 4 Eq. 1)
  edgeconv   EdgeConv layer, forward and backward (App. A.2 "EdgeConv")
  gmm        MoNet / GMMConv layer                (App. A.2 "GMMConv")
  plan       integer tables: CSC transpose, degree buckets, degree order
  cost_model closed-form operation / IO counts    (Sec. 4, Sec. 5 examples)

Parity pins (see tests/test_oracle_*.py): dense-adjacency brute force, scipy
sparse special cases, closed forms, finite differences, torch-autograd on the
dense formula.  Parts the paper leaves open (LeakyReLU slope, head layout,
diagonal GMM covariance, pseudo-coordinate source) follow the readings listed
in the design document and are "parity unpinned" by the paper itself.
"""
