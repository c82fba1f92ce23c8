"""MI355X-native hot path of the two-stage DDCCANet feature extractor (arXiv 2209.13027).

`binding.Context` wraps the C ABI declared in include/ddcca.h; `workloads` holds the
seeded synthetic inputs; `pipeline` chains the four calls of the path.
"""
from . import workloads  # noqa: F401
