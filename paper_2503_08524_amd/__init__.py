"""MI355X (gfx950) implementation of the decode hot path of Position-Aware Depth
Decay Decoding (D^3).  The work is done by hand-written HIP kernels behind a C
ABI (include/d3.h, built into libd3.so); this package only marshals arguments.
"""
from .binding import (D3Error, Decoder, d3_plan_depth, d3_plan_depth_linear, d3_plan_from_table, d3_workspace_size,
                      library_path, load_library)

__all__ = ["D3Error", "Decoder", "d3_plan_depth", "d3_plan_depth_linear", "d3_plan_from_table", "d3_workspace_size", "library_path", "load_library"]
