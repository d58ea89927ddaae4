"""Plain CPU oracle (fp64 reference plus fp32 mode) for the tests, the smoke
check and the benchmark's cpu_baseline leg.  Nothing on the product path may
import this package."""
