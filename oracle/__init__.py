"""CPU oracle for the partition-wise full-graph GNN layer path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the bench's
CPU-baseline leg.  The product package never imports it, and it never imports the product
package.  It shares no code with the HIP path.

* ``oracle.fullgraph``  - full-graph GCN / SAGE-mean forward, loss, backward (plain C, fp64).
* ``oracle.partition``  - partition assignment rules, boundary lists by set arithmetic, and a
  naive partition-wise evaluator used to pin the "any k gives the full-graph result"
  invariant.
"""
