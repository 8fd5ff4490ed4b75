"""CPU oracle of the MoE layer forward.  TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and the benchmark's reported
``cpu_baseline`` leg may import this package; the product path never does, and
this package imports nothing from the product path.
"""
