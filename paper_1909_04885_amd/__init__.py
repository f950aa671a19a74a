"""MI355X (gfx950) implementation of the CoCoA round for generalised linear models.

`binding.ChicleRound` is a thin ctypes layer over `libchicle_round.so` (C ABI declared in
`include/chicle_round.h`); every step of the round runs in that library's HIP kernels.  PyTorch is
used only to allocate device memory and to supply the HIP stream.
"""
from .binding import (ChicleError, ChicleRound, balance, library_path, load_library,  # noqa: F401
                      next_solver_count, projected_iteration_time, rebalance, scale_in, scale_out)
