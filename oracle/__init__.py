"""CPU oracle for the HAP per-device hot path.  TEST INFRASTRUCTURE ONLY.

Plain numpy in float64, written from the paper's definitions (Sec. 3.2 cost
model, Sec. 5.1 load balancing and rounding, Fig. "semantics" MatMul sharding
rules, Sec. 2.3.2 / Fig. "sfb" sufficient-factor broadcasting, Sec. 6
parameter slicing, Sec. 7.6 uneven placement of MoE experts, Sec. 2.3.1 All-Gather
data movement, Sec. 4 program synthesis on small graphs).  It shares no code with the HIP library and never imports
it.  Only tests, the smoke check and the benchmark's cpu_baseline leg may use
this package; the product path must never route through it.

Pin status: every function here is pinned by tests/test_oracle_*.py (closed
forms, brute force on tiny inputs, finite differences, identities the paper
states).  No function is "parity unpinned".
"""
