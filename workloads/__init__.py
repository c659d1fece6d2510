"""Seeded synthetic workloads (shapes, bucket layouts, values, groupings).

Input generation only: shared by the CPU oracle's tests and the GPU path's
tests and benchmark; contains none of the arithmetic of the method."""
