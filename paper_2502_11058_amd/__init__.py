"""MI355X-native partial-synchronisation + local-update step of DreamDDP's partial local SGD.

`workloads` (shapes and seeded inputs) is importable without a GPU; `binding` loads the HIP library.
"""
__all__ = ["workloads", "binding"]
