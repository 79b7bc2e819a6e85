"""MI355X-native hot path of SPACE auto-correct decoding (arxiv 2402.11809).

`binding` wraps the C ABI of libspace_hip.so one to one; `layout` builds block layouts
(Eq. 2) on the host; `runtime` holds the thin generate loop of Algorithm 1 on top of them.
Nothing here computes any part of the step: it all runs in the HIP kernels.
"""
from .layout import BlockLayoutSpec, paper_layout, first_step_layout, prefill_layout, grouped_layout  # noqa: F401
