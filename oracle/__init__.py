"""CPU oracle for the MLMC gradient-compression hot path.

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow, written-from-the-paper definition of what
the HIP library computes.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import it; the product package never does, and the two share no code.
"""
