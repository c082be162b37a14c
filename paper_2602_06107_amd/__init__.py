"""MI355X-native OBRS hot path (Jackpot): HIP kernels behind a C-ABI library plus a thin binding.

``paper_2602_06107_amd.obrs`` is the binding (loads the built HIP library and fails loudly if it
is missing); ``paper_2602_06107_amd.workloads`` holds the seeded synthetic input generators.
"""
__all__ = ["obrs", "workloads"]
