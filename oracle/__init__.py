"""fp64 CPU oracle of the semi-PD hot path: TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with paper_2504_19867_amd (the HIP path) and
neither imports the other.
"""
from . import attention, allocator  # noqa: F401
