"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This package only draws random tensors of the workloads' shapes and rounds
them to the storage type; it holds none of the method's arithmetic and imports
neither the oracle nor the HIP binding.
"""
