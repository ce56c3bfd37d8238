"""TEST INFRASTRUCTURE ONLY - slow, plain CPU statement of what the resharding
path computes.  Imported by tests, the smoke check and the benchmark's
cpu_baseline leg; never by the product, and it never imports the product."""
from . import dataset, reshard, spec  # noqa: F401
