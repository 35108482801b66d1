"""Slow, plain CPU reference implementations used only to check the HIP path.

Test infrastructure: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The library package never imports it.
"""
