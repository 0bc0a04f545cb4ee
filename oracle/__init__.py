"""CPU oracle of the per-block mixed-precision Adam step and of the swapping planner.

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg import
this package; it shares no code with the HIP library."""
