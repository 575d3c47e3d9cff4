"""Plain CPU oracle for the hot path (TEST INFRASTRUCTURE ONLY).

Imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
leg -- never by the product package.
"""
