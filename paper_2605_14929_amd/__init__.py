"""MI355X-native pair search of "Scaled Outer Product": thin Python binding over libsop_hip.so.

Every step of the search runs in the HIP kernels of the shared library; this package only loads
it, marshals arguments and hands PyTorch device pointers and streams across the C boundary.
There is no CPU fallback: importing works anywhere, calling needs the built library and a GPU.
"""
from .binding import (  # noqa: F401
    SopError, lib, lib_path, Context, ScaleFmt, WeightFmt, Outputs,
    sop_check_alphabet, sop_atom_nf, sop_atom_sh, sop_atom_negate, sop_atom_bof, sop_lloyd_1d, sop_dd_fit, sop_dd_fit_grid, sop_weight_grid, sop_layer_shift,
    F32, BF16, SEL_WSE, SEL_COS, SEL_MSE, SCALE_ABSMAX, SCALE_ARGMAX, fmt_by_name, build_alphabet,
)
