"""Batched activation-checkpoint dynamic program for MI355X (gfx950).

Thin Python binding over the C ABI declared in include/ckpt_dp.h; every step of
the solve runs in the HIP library (libckpt_dp.so, built in-tree by
paper_2302_02599_amd/build.py).  There is no CPU fallback: loading fails loudly
when the library is missing.
"""
from .binding import (CKPT_INF, CkptError, Solution, ckpt_block_indices, ckpt_block_indices_batched,  # noqa: F401
                      ckpt_budget_sweep, ckpt_check_inputs, ckpt_discretize, ckpt_discretize_sweep, ckpt_init,
                      ckpt_linearize, ckpt_row_index, ckpt_row_pitch, ckpt_schedule, ckpt_schedule_batched,
                      ckpt_schedule_workspace_bytes, ckpt_select_plan, ckpt_simulate_batched, ckpt_solve_batched,
                      ckpt_solve_batched_noalloc, ckpt_solve_batched_opts, ckpt_solve_profiled, ckpt_table_elems, ckpt_table_rows,
                      ckpt_workspace_bytes, lib_path, load_library, solve)
