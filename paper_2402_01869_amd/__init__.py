"""MI355X (gfx950) hot path of InferCept's intercept handling: mixed-batch paged attention and
KV-block pack / unpack behind a C ABI (include/infercept_hot.h).

`binding` marshals arguments into libinfercept_hot.so; `workloads` draws seeded synthetic inputs;
`build` compiles the library.  The library is loaded on first use and there is no CPU fallback.
"""
from . import workloads  # noqa: F401  (numpy only)
from . import binding    # noqa: F401  (loads the shared library lazily)

__all__ = ["binding", "workloads"]
