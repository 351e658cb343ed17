"""MI355X-native block-level kernel scheduling (slicing, preemptible persistent workers,
two-stream priority scheduler).  The HIP library is loaded by `.binding`; there is no
CPU fallback.  `python -m paper_2410_07381_amd.build` compiles it in-tree."""

__all__ = ["binding", "build"]
