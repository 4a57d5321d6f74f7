"""Fused logit-lens projection and steering kernels for MI355X (gfx950).

`binding` wraps every entry point of the C-ABI library (include/ll.h): ll_workspace_bytes, ll_project,
ll_project_ex (through ll_project's bias / topk_softmax arguments), ll_project_timed (timed=True),
ll_project_static and ll_project_static_pass_rows, ll_steer_workspace_bytes, ll_steer_vector,
ll_steer_inject, ll_steer_inject_raw, ll_steer_sweep_workspace_bytes, ll_steer_sweep and
ll_steer_sweep_topk (k=...), ll_capture_append, ll_error_string and
ll_last_hip_error (inside LLError).  `workloads` draws the seeded synthetic inputs; `serialize`
writes the paper's JSON output.  Nothing is loaded at import time: the shared library is opened
on first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "workloads", "serialize"]
