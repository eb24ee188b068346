"""Fused lazy-array DAG evaluation on MI355X (deferred-execution NumPy scheme).

``paper_1901_03771_amd.lazy``      thin ctypes binding over the C-ABI library
``paper_1901_03771_amd.workloads`` seeded synthetic inputs and user programs

Nothing is loaded at import time; the binding loads the HIP library on first
use and raises if it is missing.
"""
