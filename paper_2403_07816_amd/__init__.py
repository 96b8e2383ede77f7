"""MI355X-native MoE feed-forward layer of Branch-Train-MiX: Python binding of
the C-ABI HIP library (see include/btx_moe.h).  The shared library is loaded
on first use, so importing the package (e.g. for `synth`) needs no GPU."""
