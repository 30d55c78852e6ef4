"""Seeded synthetic inputs for the stitched-decode workloads.

This package is *data only*: a counter-based random number generator, the
decoder shapes and the five workload recipes.  It holds none of the method's
arithmetic (no normalisation, rotary embedding, attention, entropy or routing
code) so that both the CPU oracle and the HIP path can be fed the very same
buffers without sharing any compute code.
"""

from .rng import uniform01, normal, randint, uniform23, stream_key  # noqa: F401
from .shapes import (  # noqa: F401
    ModelShape, TINY_S, TINY_L, S15, M7, M14, M32, SHAPES,
    kv_bytes_per_token, weight_bytes_read_per_step, weight_bytes_resident,
)
from .recipes import (  # noqa: F401
    Workload, WORKLOADS, ModelWeights, make_weights, make_prompt, logit_scale,
    pick_tau, RouterWeights, make_router_weights,
)
