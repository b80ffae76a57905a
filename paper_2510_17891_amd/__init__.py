"""MI355X-native rollout generation: paged-KV batched decode with a fused Gumbel-max sampler.

The product is the C library declared in include/rl.h (sources in csrc/); `binding` marshals arguments.
"""
from . import binding  # noqa: F401
from .binding import Rollout, RLError, lib  # noqa: F401
from .rollout_loop import generate_groups, group_page_need  # noqa: F401
