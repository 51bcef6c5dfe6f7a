"""CPU oracle of the AET-SGD client/round/server loop.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.
"""
from .oracle import Oracle, build, load  # noqa: F401
