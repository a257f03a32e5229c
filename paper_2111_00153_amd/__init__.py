"""RMSMP row-wise mixed-scheme quantized GEMM for MI355X: Python binding of librmsmp.so."""
from .binding import *  # noqa: F401,F403
from .binding import (conv2d_launcher, gemm_launcher, ConvDesc, Epilogue, Packed, RmsmpError, make_epilogue, pack_u4, unpack_u4,  # noqa: F401
                      EXPORTS, FIXED4, POT4, FIXED8, OUT_INT32, OUT_FP32, OUT_U4)
