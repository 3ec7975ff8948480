"""CPU oracle for ragged per-head decode attention and its work planner.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this package;
only the tests, the smoke check and the benchmark's CPU-baseline leg do.  It
shares no code with the HIP path.
"""
