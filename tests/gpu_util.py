"""GPU test helpers: the host<->device marshalling and the layer driver live in the package
(paper_2605_19218_amd/torch_harness.py) so that the benchmark and the smoke test use the same ones."""
from paper_2605_19218_amd.torch_harness import (D, DEV, Pipeline, bf16_ulp, rk_dtype, to_dev, to_host,  # noqa: F401
                                                torch_dtype)
