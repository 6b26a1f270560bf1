"""Batched NotebookOS policy replay on AMD MI355X (gfx950).

``replay`` is the ctypes binding of the HIP library (``nbos_replay_create`` /
``nbos_replay_run`` / ``nbos_replay_stats``); ``tracegen`` makes seeded synthetic
traces. Importing the package loads nothing; the binding loads the shared
library on first use and raises if it has not been built.
"""
__all__ = ["replay", "tracegen"]
