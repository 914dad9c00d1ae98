"""CPU oracle for one training step under the out-of-core hybrid method.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this package; the HIP library and its Python binding never
do, and this package imports nothing from them.
"""
