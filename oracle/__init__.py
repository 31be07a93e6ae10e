"""Plain CPU oracle for the Medusa static-tree verify path (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
