"""MI355X-native per-rank tensor-parallel linear layer (1D / 2D-SUMMA / 2.5D / 3D): a thin ctypes
binding over libtplinear.so.  Importing this package does not load the library; the first call
does, and fails loudly if it has not been built (python -m paper_2110_14883_amd.build)."""
from .binding import (  # noqa: F401
    EPI_BIAS, EPI_BIAS_GELU, EPI_NONE, MODE_1D_COL, MODE_1D_ROW, MODE_2D, MODE_2P5D, MODE_3D, MODE_3D_GATHERED,
    PASS_DW, PASS_DW_PARTIALS, PASS_DX, PASS_DX_PARTIALS, PASS_FWD, Grid, TpError, lib, tp_block_map, tp_dgelu, tp_linear_bwd,
    tp_linear_fwd, tp_linear_workspace_size, tp_bias_act, tp_linear_bwd_partials, tp_partials_map, tp_bias_grad, plan_opts, tp_strerror,
    tp_linear_fwd_static, tp_static_scratch_bytes, tp_bias_grad_workspace_size,
)
