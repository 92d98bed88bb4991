"""MI355X-native hot path of SCAR's checkpoint strategies (partial recovery and
prioritized checkpoints, Sections 4.1-4.3 of "Fault Tolerance in Iterative-Convergent
Machine Learning").

`paper_1810_07354_amd.scar` is the Python face of the C-ABI library (HIP kernels for
gfx950); `paper_1810_07354_amd.workloads` makes the seeded synthetic parameter stores.
Nothing here falls back to a CPU path: using `scar` without the built library raises.
"""

__all__ = ["scar", "workloads"]
