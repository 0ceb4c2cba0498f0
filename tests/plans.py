"""Which kernel instantiation each call of the library would launch, over a grid of descriptors.

The library answers that itself (mglu_describe_plan runs the launchers' own dispatch, host only), so
the enumeration here cannot drift from the code.  `enumerate_plans` returns, for every instantiation
the grid reaches, the cheapest descriptor that selects it; the CPU suite checks that the grid reaches
every kernel compiled into libmglu.so, the GPU suite runs one oracle-parity case per instantiation.
"""
import itertools

import torch

from paper_2506_23225_amd import api, build

DTYPES = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
CALLS = ("forward", "forward_variant", "projections", "linear", "swiglu", "forward_routed")
ROUTE_K = (1, 2, 4, 16)    # sizes the routed kernel for 2, 4, 8 or 16 selected masks (with the token count)
MASK_COUNTS = (1, 2, 4, 8, 16)
# token counts on both sides of every hand-over: the resident kernel's 16, the panel kernel's token
# blocks (17-64), the tiled kernel's 64-, 96- and 128-token tiles in one, two and many rows
TOKENS = (1, 3, 16, 17, 33, 40, 49, 64, 65, 80, 96, 100, 130, 200, 257, 390, 520, 1030, 2100)
# (d_model, d_ff): small ragged; wide enough for the panel kernel's 8-block workgroups and the resident
# kernel's large-launch flavour (ragged tail, odd chunk count); wide with a short reduction (cheap tall
# tiles); a long reduction that no longer fits LDS for 16 tokens, narrow and wide
SHAPES = ((264, 100), (1024, 25616), (136, 28672), (256, 14400), (8192, 64), (384, 4112), (2048, 25616))


def enumerate_plans():
    """{plan name: (cost, dtype name, call, n_masks, tokens, d_model, d_ff, route_k)} -- cheapest case per plan."""
    build.build(force=False)   # host-only query, but the library has to exist (compiles only if it is absent or stale)
    best = {}
    for dname, call, n_m, T, (h, d) in itertools.product(DTYPES, CALLS, MASK_COUNTS, TOKENS, SHAPES):
        if call in ("linear", "swiglu") and n_m != 1:
            continue
        if call == "projections" and T > 64:
            continue   # a debug view of the decode kernels' sums; its outputs are (1 + 2 n_m) fp32 planes
        desc = api.make_desc(T, h, d, n_m, DTYPES[dname])
        cost = T * h * d * (1 + n_m)
        for k in (ROUTE_K if call == "forward_routed" else (0,)):
            if k > n_m:
                continue
            try:
                plan = api.mglu_describe_plan(desc, call, k)
            except api.MgluError as e:
                if call == "forward_routed" and e.status == 2:
                    continue   # more than 16 tokens, or x beyond the routed kernel's LDS budget
                raise
            if plan not in best or cost < best[plan][0]:
                best[plan] = (cost, dname, call, n_m, T, h, d, k)
    return best
