"""CPU oracle for the MoE layer — test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this.
It shares nothing with the HIP path and does not import the product package.
"""
