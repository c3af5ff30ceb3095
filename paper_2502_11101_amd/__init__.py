"""MI355X-native CacheFocus prefill path: re-positioned cached-KV attention,
per-document attention mass, pruning and position allocation (HIP, gfx950).

``paper_2502_11101_amd.binding`` wraps the C-ABI library ``libcachefocus.so``;
``paper_2502_11101_amd.workloads`` draws the synthetic inputs.
"""

__all__ = ["binding", "workloads"]
