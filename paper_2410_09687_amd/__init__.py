"""MI355X-native MoIN hot path: nearest-centroid sequence routing and the
sequence-routed multi-adapter LoRA linear layer, behind the C-ABI ``libmoin``.

``paper_2410_09687_amd.moin`` is the thin binding (argument marshalling
only); ``paper_2410_09687_amd.workloads`` draws the seeded synthetic inputs.
Importing the package loads nothing native; the shared library is opened on
the first call and a missing library is a hard error, never a fallback.
"""
__all__ = ["moin", "workloads"]
