"""CPU oracle for the QuEST quantized-linear hot path (arXiv 2502.05003).

TEST INFRASTRUCTURE ONLY.  Plain double-precision statements of what the paper defines,
used by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of bench.py.  The
product package never imports this directory, and this directory never imports the product.
"""
