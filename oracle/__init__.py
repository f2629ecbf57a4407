"""CPU oracle for the QUIK linear layer -- test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It never imports the GPU package and shares no code with it.
"""
from .quik_oracle import *  # noqa: F401,F403
