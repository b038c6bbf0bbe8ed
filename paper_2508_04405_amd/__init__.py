"""MI355X-native W6A6 / W6A8 quantized linear layer (GEMM + decode GEMV).

`binding` is the thin ctypes layer over the C ABI in include/flexq.h; `synth`
draws the seeded synthetic inputs; `build` compiles the HIP sources; `dev` (not
imported here) binds the development library of include/flexq_dev.h for tests
and measurement tables.
"""
from .binding import (FlexQError, Layer, gemm_w6a6, gemm_w6a8, gemv_tiles, gemv_w6a6, gemv_w6a8,  # noqa: F401
                      gemv_w6a8_noalloc, layer_linears, layout_version, linear_g128, load, make_workspace,
                      pack_w6, packed_bytes, quant_act, quant_act_g128, quant_act_tiles, quant_w6,
                      rmsnorm_quant, swiglu_quant, unpack_w6, untile_act, workspace_bytes)
