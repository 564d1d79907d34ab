"""MI355X-native checkpoint-selection solver (gfx950 HIP kernels behind a C ABI).

``paper_2502_12499_amd.binding`` marshals torch device tensors into the three
library calls (``ckpt_eval_peak``, ``ckpt_solve_cubic``, ``ckpt_solve_linear``);
``paper_2502_12499_amd.inputs`` holds the seeded synthetic chain generators.
"""
__all__ = ["binding", "inputs"]
