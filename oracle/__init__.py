"""Plain CPU oracle for packed-tree Broadcast / AllReduce.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product (the HIP library and its Python
binding) never imports it and shares no code with it.

Parity status: every function is pinned in tests/test_oracle_*.py except the
exact number of trees MWU returns before pruning and the exact optimum of the
tree-count minimisation, which depend on constants the paper does not state
("parity unpinned" for those two figures only).
"""
