"""MI355X (gfx950) decode-step hot path of STEP: paged GQA decode attention, the step scorer and
refcounted prune/free, as hand-written HIP kernels behind the C-ABI library libstep.

Importing the package loads nothing; `paper_2601_09093_amd.binding` loads libstep.so on first use
and raises if it is missing (there is no CPU fallback).
"""
__all__ = ["binding", "workloads"]
