"""kt: per-GPU gradient bucket pack / weighted reduce / unpack for MI355X.

The work is done by libkt.so (hand-written HIP for gfx950 behind a C ABI, see
include/kt.h); ``binding`` marshals arguments, ``workloads`` describes the
synthetic gradient sets.
"""
from . import binding, workloads  # noqa: F401
from .binding import (Plan, KtError, kt_plan_shares, kt_plan_group_weights, kt_replan_shares,  # noqa: F401
                      kt_sampler_epoch)
