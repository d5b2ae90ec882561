"""MI355X-native lognormal neural-gradient compression (stats -> threshold / FP-n format ->
stochastic prune + FP-n quantize).  Thin Python binding over the C interface in `include/lgn.h`;
every step of the path runs in the HIP kernels of `liblgn.so`.  PyTorch is used for device
memory and streams only."""
from .binding import *  # noqa: F401,F403
