"""fp64 CPU oracle of the GR-KAN group-wise rational function.

TEST INFRASTRUCTURE ONLY: used by tests, the smoke check and the bench's
CPU-baseline leg; never by the GPU product path.
"""
