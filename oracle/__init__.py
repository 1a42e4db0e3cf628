"""CPU oracle for the variant-selection path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It shares nothing with the GPU library.
"""
from .binding import Oracle, build_oracle, load_oracle  # noqa: F401
