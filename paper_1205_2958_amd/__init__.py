"""b-bit minwise-hash signature engine for MI355X (gfx950).

``paper_1205_2958_amd.minhash`` is the thin binding over the C-ABI library
(``include/minhash.h``); ``paper_1205_2958_amd.workloads`` draws the seeded
synthetic inputs.  Importing the package loads nothing native; the binding
loads ``libminhash.so`` on first use and raises if it is missing.
"""

__all__ = ["minhash", "workloads"]
