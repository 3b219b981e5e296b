"""CPU oracle: TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It is independent of the HIP path: no shared kernels, headers,
helpers or tables.  `ref` wraps the plain C loops of sparsert_oracle.c;
`plan_ref` restates the inspector's integer plan specification in NumPy.
"""
