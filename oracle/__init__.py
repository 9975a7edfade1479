"""CPU oracle of the CRISP hybrid-sparse path -- test infrastructure only.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the HIP library's package.
"""
from .binding import *  # noqa: F401,F403
