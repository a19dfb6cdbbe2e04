"""CPU oracle (test infrastructure, not the product) for the GPT-NeoX decode
block.  Only tests, the smoke check and the benchmark's cpu_baseline leg import
this package; it never imports the HIP library's binding."""
from .neox_oracle import Oracle, load  # noqa: F401
