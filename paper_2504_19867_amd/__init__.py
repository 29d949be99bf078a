"""semi-PD hot path on MI355X: ctypes binding of the C-ABI library libsemipd.so.

`from paper_2504_19867_amd import semipd` loads the in-tree shared library (build it with
`python paper_2504_19867_amd/build.py`); there is no fallback when it is missing.
"""
from . import semipd  # noqa: F401
