"""fp64 CPU oracle for AdaS-Attn, the token-selective FFN and the attention backward -- test infrastructure only.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the HIP package.
"""
from .adaspark_oracle import (  # noqa: F401
    Shape,
    build,
    num_cubes,
    cube_map,
    cube_pool,
    relevance,
    top_p,
    top_k,
    cube_select,
    cube_select_topk,
    cube_select_shared,
    group_mean_query,
    sparse_attn,
    dense_attn,
    num_threads,
)
from . import adaspark_ffn_oracle as ffn  # noqa: F401,E402  (AdaS-FFN, Sec. 3.3)
from . import adaspark_bwd_oracle as bwd  # noqa: F401,E402  (backward of Eq. 3, selection constant)
