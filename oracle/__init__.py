"""CPU oracle for the relational-GNN layer path (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the HIP package.
"""
