"""Fused logit-lens projection and steering kernels for MI355X (gfx950).

`binding` wraps the C-ABI library (ll_project, ll_steer_vector,
ll_steer_inject); `workloads` draws the seeded synthetic inputs.  Nothing is
loaded at import time: the shared library is opened on first use and its
absence is an error, never a fallback.
"""
__all__ = ["binding", "workloads"]
